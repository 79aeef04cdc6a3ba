"""Pins for the batched form of Eq. 1 (oracle/batch_oracle.py).

With one sequence, or with the per-sequence rule, a batched step must be the single-sequence
oracle bit for bit.  With the batch-min rule the exit position is pinned by brute force: the
similarities of every sequence on its dense (never-exit) trajectory are computed by
independent single-sequence runs, the first block whose minimum over the batch exceeds tau is
found in plain numpy, and the batched step must then equal single-sequence steps forced at
that position."""
import numpy as np
import pytest

from oracle import batch_oracle as bo
from oracle import river_oracle as ro
from paper_2604_18396_amd import configs, inputs

TINY_BF16 = configs.TINY.with_(name="tiny-bf16", dtype=configs.DTYPE_BF16)
PROMPTS = [(5, 11), (9, 12), (3, 13), (12, 14)]          # (length, seed): ragged positions


def fresh(cfg, w, river):
    os_, toks = [], []
    for n, seed in PROMPTS:
        o = ro.Oracle(cfg, w, river)
        toks.append(o.prefill(inputs.make_prompt(cfg.vocab, n, seed)))
        os_.append(o)
    return os_, toks


@pytest.mark.parametrize("cfg0", [configs.TINY, TINY_BF16], ids=lambda c: c.name)
@pytest.mark.parametrize("tau", [0.675, 0.52])
def test_per_sequence_rule_is_the_single_sequence_oracle(cfg0, tau):
    cfg = cfg0.with_(tau=tau)
    w = inputs.make_weights(cfg, configs.C1.seed_weights)
    river = ro.quantize_river(cfg, w)
    A, toks_a = fresh(cfg, w, river)
    Bs, toks_b = fresh(cfg, w, river)
    assert toks_a == toks_b
    seen = set()
    for step in range(6):
        forced = [None, 3 if step % 2 else None, None, cfg.n_layers if step == 2 else None]
        nt, e, sims, hidden, logits = bo.batch_step(A, toks_a, tau, cfg.min_exit_layer, "per_sequence", forced)
        for b, o in enumerate(Bs):
            t1, e1, s1 = o.decode_step(toks_b[b], forced[b])
            assert (t1, e1) == (nt[b], e[b])
            np.testing.assert_array_equal(s1, sims[b])
            np.testing.assert_array_equal(o.hidden(), hidden[:, b])
            np.testing.assert_array_equal(o.logits(), logits[b])
            np.testing.assert_array_equal(o.kcache(), A[b].kcache())
            toks_b[b] = t1
        toks_a = nt
        seen |= set(e)
    assert len(seen) > 1
    # one sequence: the batch-min rule is the same thing
    o1, o2 = ro.Oracle(cfg, w, river), ro.Oracle(cfg, w, river)
    t = o1.prefill([4, 5, 6]); o2.prefill([4, 5, 6])
    for _ in range(4):
        nt, e, sims, _, logits = bo.batch_step([o1], [t], tau, cfg.min_exit_layer, "batch_min")
        t2, e2, s2 = o2.decode_step(t)
        assert (nt[0], e[0]) == (t2, e2)
        np.testing.assert_array_equal(logits[0], o2.logits())
        t = t2


@pytest.mark.parametrize("tau", [0.3, 0.5, 0.55, 0.62, 0.7, 0.9])
def test_batch_min_rule_against_brute_force(tau):
    cfg = configs.TINY.with_(tau=tau)
    L, Ls = cfg.n_layers, cfg.min_exit_layer
    w = inputs.make_weights(cfg, configs.C1.seed_weights)
    river = ro.quantize_river(cfg, w)
    A, toks = fresh(cfg, w, river)
    exits_seen = set()
    for step in range(5):
        # brute force: dense similarities of every sequence from independent single-sequence runs
        dense_s = []
        for b, (n, seed) in enumerate(PROMPTS):
            o = ro.Oracle(cfg.with_(tau=1.0), w, river)
            o.prefill(inputs.make_prompt(cfg.vocab, n, seed))
            for k in range(step):                       # replay this sequence's history as it happened
                o.decode_step(history[k][0][b], history[k][1])
            _, _, s = o.decode_step(toks[b])
            dense_s.append(s)
        dense_s = np.array(dense_s)                      # [B, L]
        e_star = L
        for l in range(Ls, L):
            if dense_s[:, l - 1].min() > np.float32(tau):
                e_star = l
                break
        nt, e, sims, hidden, logits = bo.batch_step(A, toks, tau, Ls, "batch_min")
        assert e == [e_star] * len(PROMPTS)              # the whole batch leaves together
        np.testing.assert_allclose(sims[:, :e_star], dense_s[:, :e_star], rtol=0, atol=0)
        assert np.all(np.isnan(sims[:, e_star:]))
        # and the step equals single-sequence steps forced at e_star
        for b, (n, seed) in enumerate(PROMPTS):
            o = ro.Oracle(cfg, w, river)
            o.prefill(inputs.make_prompt(cfg.vocab, n, seed))
            for k in range(step):
                o.decode_step(history[k][0][b], history[k][1])
            t1, e1, _ = o.decode_step(toks[b], e_star)
            assert (t1, e1) == (nt[b], e_star)
            np.testing.assert_array_equal(o.logits(), logits[b])
        if step == 0:
            history = []
        history.append((list(toks), e_star))
        toks = nt
        exits_seen.add(e_star)
    if tau == 0.3:
        assert exits_seen == {Ls}
    if tau == 0.9:
        assert exits_seen == {L}
    # the batch rule is never shallower than any sequence's own rule would be
