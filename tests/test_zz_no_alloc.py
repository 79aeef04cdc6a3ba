"""river_create_static (the entry point for callers that cannot allocate device memory)
against river_create: same kernels, activations and barrier counters in the library's static
device array.  Two contexts in a row on the same array, the second with a smaller model,
must reproduce the ordinary contexts bit for bit (tokens, exit positions, similarities,
hidden states, logits, KV cache) and stay within the parity bar of the CPU oracle."""
import sys

import numpy as np
import pytest

from oracle import river_oracle as ro
from paper_2604_18396_amd import binding, configs, inputs

pytestmark = pytest.mark.gpu

MID = configs.ModelConfig("mid-bf16", 3, 1024, 8, 2, 128, 2816, 1002, 500000.0, 1e-5,
                          configs.DTYPE_BF16, 192, 1, 2.0)
TINY_BF16 = configs.TINY.with_(name="tiny-bf16", dtype=configs.DTYPE_BF16, min_exit_layer=1)


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run(cfg, dw, dr, prompt, sched, static, mode):
    g = binding.River(cfg, dw, dr, exec_mode=mode, static_scratch=static)
    tok = g.prefill(prompt)
    out = {"tokens": [tok], "exits": [], "sims": [], "hidden": [], "logits": []}
    for e in sched:
        tok, eg, sg = g.decode_step(tok, e)
        out["tokens"].append(tok); out["exits"].append(eg); out["sims"].append(sg)
        out["hidden"].append(g.hidden()); out["logits"].append(g.logits())
    n = len(prompt) + len(sched)
    out["k"], out["v"] = g.kcache()[:, :n].copy(), g.vcache()[:, :n].copy()
    g.close()
    return out


def check(cfg, prompt_len, sched, seed, mode):
    w = inputs.make_weights(cfg, seed, gain_std=0.05)
    dw = binding.upload_weights(w)
    dr = binding.quantize_river(cfg, dw)
    prompt = inputs.make_prompt(cfg.vocab, prompt_len, seed + 1)
    say(f"no-alloc entry point: {cfg.name} mode={mode} prompt {prompt_len}")
    a = run(cfg, dw, dr, prompt, sched, False, mode)
    b = run(cfg, dw, dr, prompt, sched, True, mode)
    assert a["tokens"] == b["tokens"] and a["exits"] == b["exits"] == list(sched)
    for key in ("sims", "hidden", "logits"):
        for x, y in zip(a[key], b[key]):
            np.testing.assert_array_equal(x, y)
    np.testing.assert_array_equal(a["k"], b["k"])
    np.testing.assert_array_equal(a["v"], b["v"])
    # and against the oracle, to the parity bar (teacher-forced with the static run's tokens)
    tol = 2e-2 if cfg.dtype == configs.DTYPE_BF16 else 1e-4
    o = ro.Oracle(cfg, w, ro.quantize_river(cfg, w))
    tok = o.prefill(prompt)
    for i, e in enumerate(sched):
        assert b["tokens"][i] == tok
        tok, eo, _ = o.decode_step(tok, e)
        ho = o.hidden()
        for l in range(cfg.n_layers + 1):
            assert np.abs(b["hidden"][i][l] - ho[l]).max() / np.abs(ho[l]).max() <= tol
        lo = o.logits()
        assert np.abs(b["logits"][i] - lo).max() / np.abs(lo).max() <= tol
    o.close()


def test_static_scratch_contexts_match_ordinary_ones_twice_in_a_row():
    check(MID, 130, [1, 3, 2, 3, 1, 2], 71, binding.EXEC_PERSISTENT)
    # second call on the same static array, smaller model and input: nothing of the first
    # context's contents may leak into it
    check(TINY_BF16, 9, [4, 1, 2, 3], 73, binding.EXEC_PERSISTENT)
    check(TINY_BF16.with_(name="tiny-fp32", dtype=configs.DTYPE_F32), 5, [2, 4, 1], 75, binding.EXEC_KERNELS)


def test_static_scratch_limits():
    cfg = TINY_BF16.with_(tau=2.0)
    w = inputs.make_weights(cfg, 3)
    dw = binding.upload_weights(w)
    g = binding.River(cfg, dw, None, static_scratch=True)
    with pytest.raises(binding.RiverError) as ei:          # one live static context per device
        binding.River(cfg, dw, None, static_scratch=True)
    assert ei.value.code == binding.RIVER_ESTATE
    ordinary = binding.River(cfg, dw, None)                 # ordinary contexts are not affected
    assert ordinary.prefill([1, 2, 3]) == g.prefill([1, 2, 3])
    ordinary.close()
    g.close()
    # a configuration whose step-transient data exceed the 8 MiB array is refused, nothing runs
    big = cfg.with_(n_layers=600, max_seq=4)
    wb = dict(dw)
    wb["layers"] = [dw["layers"][0]] * 600
    with pytest.raises(binding.RiverError) as ei:
        binding.River(big, wb, None, static_scratch=True)
    assert ei.value.code == binding.RIVER_ENOSPC and "8388608" in str(ei.value)
    g = binding.River(cfg, dw, None, static_scratch=True)   # the array is free again
    assert 0 <= g.prefill([1, 2, 3]) < cfg.vocab
    g.close()
