"""Batched decode step as the paper states Eq. 1: over a batch B.

TEST INFRASTRUCTURE ONLY.  A batch is one C-oracle context per sequence (own KV cache and
position), stepped block by block so that the exit decision after backbone block l can look
at every sequence:

    D(l) = 1[ min_{b in B} s_b(l) > tau ],   s_b(l) = cos(h_b(l-1), h_b(l))        (Eq. 1)

rule "batch_min": the whole batch leaves the backbone together at the first l in [L_s, L-1]
with D(l) = 1 (Eq. 1 as printed).  rule "per_sequence": every sequence for itself, s_b(l) >
tau (the benchmark's ragged batch; with one sequence both rules coincide).  A forced exit
position overrides the threshold for its sequence, as in the single-sequence oracle.  After a
sequence has left the backbone its remaining blocks run as river twins writing the shared
cache slots, and the original final norm + LM head give its logits.
"""
from __future__ import annotations

import numpy as np

from . import river_oracle as ro


def batch_step(oracles, tokens, tau: float, min_exit: int, rule: str = "batch_min", forced=None):
    """One decode step for all sequences.  Returns (next_tokens, exit_positions, sims [B, L],
    hidden [L+1, B, d], logits [B, V])."""
    cfg = oracles[0].cfg
    L, B = cfg.n_layers, len(oracles)
    tau = float(np.float32(tau))                       # tau is a single-precision configuration field
    forced = [None] * B if forced is None else list(forced)
    h = [o.embed(t) for o, t in zip(oracles, tokens)]
    hidden = np.zeros((L + 1, B, cfg.d_model))
    hidden[0] = np.array(h)
    sims = np.full((B, L), np.nan)
    exited = [f == 0 for f in forced]
    e = [0 if x else L for x in exited]
    for l in range(1, L + 1):
        nxt = []
        for b, o in enumerate(oracles):
            hb = o.block(l, o.pos, exited[b], h[b])
            if not exited[b]:
                a, c = np.ascontiguousarray(h[b]), np.ascontiguousarray(hb)
                sims[b, l - 1] = ro.lib().orc_cosine(ro._ptr(a), ro._ptr(c), cfg.d_model)
            nxt.append(hb)
        if min_exit <= l < L:
            live = [b for b in range(B) if not exited[b]]
            all_pass = all(sims[b, l - 1] > tau for b in live)
            for b in live:
                if forced[b] is not None:
                    go = forced[b] == l
                else:
                    go = all_pass if rule == "batch_min" else sims[b, l - 1] > tau
                if go:
                    exited[b], e[b] = True, l
        h = nxt
        hidden[l] = np.array(h)
    toks, logits = [], []
    for b, o in enumerate(oracles):
        toks.append(o.head(h[b]))
        logits.append(o.logits())
        o.advance()
    return toks, e, sims, hidden, np.array(logits)
