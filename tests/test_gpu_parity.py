"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Bars (from the benchmark spec): exit positions and token ids bit-exact under teacher
forcing except at steps whose similarity lies within 1e-3 of tau; hidden states and
logits within max relative error 1e-4 (fp32) / 2e-2 (bf16), where the relative error of a
vector is |a-b|_inf / |b|_inf with b the oracle's."""
import sys

import numpy as np
import pytest
import torch

import helpers
from helpers import grid_model
from oracle import river_oracle as ro
from paper_2604_18396_amd import binding, configs, inputs

pytestmark = pytest.mark.gpu

TOL = {configs.DTYPE_F32: 1e-4, configs.DTYPE_BF16: 2e-2}
BAND = 1e-3
MODES = [binding.EXEC_KERNELS, binding.EXEC_PERSISTENT]
MODE_IDS = ["kernels", "persistent"]

TINY_BF16 = configs.TINY.with_(name="tiny-bf16", dtype=configs.DTYPE_BF16)
TINY_BOTH = [configs.TINY, TINY_BF16]


def needs_mode(cfg, mode):
    """The one-launch mode is switched off for fp32 in the library (river_create refuses it):
    its fp32 instantiation once faulted on the GPU at the mid shape and no cause could be
    shown, so that combination stays off the GPU; fp32 is covered in the kernels mode."""
    if mode == binding.EXEC_PERSISTENT and cfg.dtype == configs.DTYPE_F32:
        pytest.skip("one-launch mode is bf16-only: unexplained GPU fault of its fp32 instantiation")
# spans several wavefront tiles with ragged tails: 2816 columns = 1 full + 1 partial
# 2048-code wave load, vocab not a multiple of the 4-row task, 3 splits of attention
MID = configs.ModelConfig("mid-bf16", 3, 1024, 8, 2, 128, 2816, 1002, 500000.0, 1e-5,
                          configs.DTYPE_BF16, 192, 1, 2.0)
MID_F32 = MID.with_(name="mid-fp32", dtype=configs.DTYPE_F32, n_q_heads=16, n_kv_heads=2, head_dim=64)
MID_F32_HD128 = MID.with_(name="mid-fp32-hd128", dtype=configs.DTYPE_F32)     # fp32 cache rows of 128 elements


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def relerr(a, b):
    return float(np.abs(np.asarray(a, np.float64) - b).max() / max(np.abs(b).max(), 1e-30))


def check_token(cfg, tg, to, lo, what):
    """Greedy token against the oracle's.  fp32: must be equal.  bf16: logits are only
    required to agree within TOL * max|logit|, so two logits closer than that cannot be
    ordered reliably; a different token is accepted only then, and every use is counted
    and printed (the total appears in the terminal summary)."""
    if tg == to:
        return
    gap = (lo[to] - lo[tg]) / max(np.abs(lo).max(), 1e-30)
    assert cfg.dtype == configs.DTYPE_BF16, f"{what}: fp32 token {tg} vs oracle {to} (gap {gap:.3e})"
    assert gap <= TOL[cfg.dtype], f"{what}: token {tg} vs oracle {to} (gap {gap:.3e})"
    helpers.NEAR_TIES.append(f"{what}: token {tg} vs oracle {to}, oracle logit gap {gap:.3e} of max|logit|")
    say(f"NEAR-TIE accepted: {helpers.NEAR_TIES[-1]}")


class Pair:
    """Oracle and HIP context on the same weights; each side quantises its own river."""

    def __init__(self, cfg, weights, mode, with_river=True, oracle=None, prefill_gemm_min_tokens=0, river=None):
        """river: a river quantised elsewhere, [{matrix: (codes, scale, zero)}] of CPU tensors,
        handed to both sides as data."""
        self.cfg = cfg
        self.o = oracle or ro.Oracle(cfg, weights, river if river is not None else
                                     (ro.quantize_river(cfg, weights) if with_river else None))
        self.dw = binding.upload_weights(weights)
        if river is not None:
            self.dr = [{m: tuple(t.cuda() for t in blk[m]) for m in blk} for blk in river]
        else:
            self.dr = binding.quantize_river(cfg, self.dw) if with_river else None
        self.g = binding.River(cfg, self.dw, self.dr, exec_mode=mode,
                               prefill_gemm_min_tokens=prefill_gemm_min_tokens)

    def prefill(self, prompt, exit_layer=None):
        to = self.o.prefill(prompt, exit_layer)
        tg = self.g.prefill(prompt, exit_layer)
        self.compare_state("prefill")
        check_token(self.cfg, tg, to, self.o.logits(), "prefill")
        return to

    def compare_state(self, what):
        tol = TOL[self.cfg.dtype]
        ho, hg = self.o.hidden(), self.g.hidden()
        for l in range(self.cfg.n_layers + 1):
            err = relerr(hg[l], ho[l])
            assert err <= tol, f"{what}: hidden state h({l}) rel err {err:.3e} > {tol}"
        err = relerr(self.g.logits(), self.o.logits())
        assert err <= tol, f"{what}: logits rel err {err:.3e} > {tol}"

    def step(self, token, forced=None, what="step"):
        """Teacher-forced step: both sides consume `token`.  Returns the oracle's outputs."""
        cfg = self.cfg
        to, eo, so = self.o.decode_step(token, forced)
        tg, eg, sg = self.g.decode_step(token, forced)
        if forced is None and eg != eo:
            # allowed only if a similarity that decided lies within the band around tau
            k = min(eg, eo)
            assert abs(so[k - 1] - np.float32(cfg.tau)) < BAND, \
                f"{what}: exit {eg} vs oracle {eo}, s={so[k - 1]} not near tau={cfg.tau}"
            self.g.rewind(self.g.pos - 1)            # replay with the oracle's decision
            tg, eg, sg = self.g.decode_step(token, eo)
        assert eg == eo, f"{what}: exit position {eg} vs oracle {eo}"
        ne = eo if eo > 0 else 0
        # Exit positions must agree except where s lies within BAND of tau, so the two sides'
        # similarities must themselves agree within BAND (bf16); fp32 is held to 2e-5.
        np.testing.assert_allclose(sg[:ne], so[:ne], rtol=0, atol=BAND if cfg.dtype else 2e-5,
                                   err_msg=f"{what}: similarities")
        assert np.all(np.isnan(sg[ne:])) and np.all(np.isnan(so[ne:]))
        self.compare_state(what)
        check_token(cfg, tg, to, self.o.logits(), what)
        return to, eo, so

    def compare_cache(self, n_pos):
        ko, vo = self.o.kcache(), self.o.vcache()
        kg, vg = self.g.kcache(), self.g.vcache()
        tol = TOL[self.cfg.dtype]
        for name, a, b in (("K", kg, ko), ("V", vg, vo)):
            assert np.all(np.isfinite(a[:, :n_pos])), f"{name} cache has unwritten slots"
            for l in range(self.cfg.n_layers):
                err = relerr(a[l, :n_pos], b[l, :n_pos])
                assert err <= tol, f"{name} cache layer {l + 1}: rel err {err:.3e}"

    def close(self):
        self.g.close()
        self.o.close()


def run_teacher_forced(pair, prompt, steps, forced=None, label=""):
    tok = pair.prefill(prompt)
    exits = []
    for i in range(steps):
        f = None if forced is None else int(forced[i])
        tok, e, _ = pair.step(tok, f, what=f"{label} step {i}")
        exits.append(e)
    return exits


# ---------------------------------------------------------------- quantiser

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["fp32", "bf16"])
def test_river_construction_bit_exact(dtype):
    say(f"quantiser parity {dtype}")
    g = torch.Generator().manual_seed(5)
    for rows, cols, group in [(64, 256, 64), (50, 688, 64), (33, 4096, 64), (7, 2816, 128)]:
        w = (torch.randn(rows, cols, generator=g) * 0.02).to(dtype)
        w[0, :64] = 0.25                                   # a constant group
        co, so, zo = ro.quantize_w4(w, group)
        cg, sg, zg = binding.river_quantize_w4(w.cuda(), group)
        torch.cuda.synchronize()
        assert torch.equal(cg.cpu(), co), (rows, cols, group)
        assert torch.equal(sg.cpu().view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                           so.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))
        assert torch.equal(zg.cpu().view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                           zo.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))


# ------------------------------------------------------------- tiny configs

@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("tau", [0.9, 0.675, 0.52])
@pytest.mark.parametrize("cfg0", TINY_BOTH, ids=lambda c: c.name)
def test_c1_threshold_mode(mode, tau, cfg0):
    needs_mode(cfg0, mode)
    say(f"C1 threshold {cfg0.name} tau={tau} mode={mode}")
    cfg = cfg0.with_(tau=tau)
    w = inputs.make_weights(cfg, configs.C1.seed_weights)
    pair = Pair(cfg, w, mode)
    prompt = inputs.make_prompt(cfg.vocab, configs.C1.prompt_len, configs.C1.seed_prompt)
    exits = run_teacher_forced(pair, prompt, configs.C1.decode_steps, label=f"C1 tau={tau}")
    if tau == 0.9:
        assert set(exits) == {cfg.n_layers}
    else:
        assert len(set(exits)) > 1
    pair.compare_cache(configs.C1.prompt_len + configs.C1.decode_steps)
    pair.close()


@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("cfg0", [configs.TINY, TINY_BF16], ids=lambda c: c.name)
def test_forced_mixed_schedule_all_depths(mode, cfg0):
    needs_mode(cfg0, mode)
    say(f"forced schedule {cfg0.name} mode={mode}")
    cfg = cfg0.with_(min_exit_layer=0)
    w = inputs.make_weights(cfg, 21)
    pair = Pair(cfg, w, mode)
    sched = [0, 4, 1, 2, 3, 3, 0, 2, 4, 1, 1, 4]
    exits = run_teacher_forced(pair, inputs.make_prompt(cfg.vocab, 5, 22), len(sched), sched, cfg0.name)
    assert exits == sched
    pair.compare_cache(5 + len(sched))
    pair.close()


@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("cfg0", TINY_BOTH, ids=lambda c: c.name)
def test_never_exit_equals_dense_bitwise(mode, cfg0):
    """tau >= 1 and exit forced at L run no river block: logits identical to a context
    that has no river at all."""
    needs_mode(cfg0, mode)
    say(f"never-exit {cfg0.name} mode={mode}")
    cfg = cfg0
    w = inputs.make_weights(cfg, configs.C1.seed_weights)
    dw = binding.upload_weights(w)
    dr = binding.quantize_river(cfg, dw)
    prompt = inputs.make_prompt(cfg.vocab, 16, configs.C1.seed_prompt)
    outs = []
    for c, river, forced in ((cfg.with_(tau=1.0), dr, None), (cfg.with_(tau=-2.0), dr, cfg.n_layers),
                             (cfg.with_(tau=2.0), None, None)):
        g = binding.River(c, dw, river, exec_mode=mode)
        tok = g.prefill(prompt)
        logs = []
        for _ in range(6):
            tok, e, _ = g.decode_step(tok, forced)
            assert e == cfg.n_layers
            logs.append(g.logits())
        outs.append(np.array(logs))
        g.close()
    np.testing.assert_array_equal(outs[0], outs[2])
    np.testing.assert_array_equal(outs[1], outs[2])


@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("cfg0", [configs.TINY, TINY_BF16], ids=lambda c: c.name)
def test_lossless_river_equals_dense(mode, cfg0):
    """Block matrices on the 4-bit grid: the twin equals the backbone, so any schedule
    reproduces the dense run (traversal + shared cache slots, no quantisation error)."""
    needs_mode(cfg0, mode)
    say(f"lossless river {cfg0.name} mode={mode}")
    cfg = cfg0.with_(min_exit_layer=1)
    w = grid_model(cfg, 31)
    dw = binding.upload_weights(w)
    dr = binding.quantize_river(cfg, dw)
    prompt = inputs.make_prompt(cfg.vocab, 6, 32)
    sched = [1, 3, 2, 4, 1, 2, 3, 1]
    runs = []
    for forced in ([cfg.n_layers] * len(sched), sched):
        g = binding.River(cfg, dw, dr, exec_mode=mode)
        tok = g.prefill(prompt)
        hs = []
        for f in forced:
            tok, e, _ = g.decode_step(tok, f)
            assert e == f
            hs.append(g.hidden())
        runs.append(np.array(hs))
        g.close()
    # fp32: the same arithmetic up to summation order.  bf16: the 4-bit phases take their
    # input vector in half precision (weight-only 4-bit, 16-bit activations), the backbone
    # in fp32, so the two runs differ by that rounding.
    tol = 1e-5 if cfg.dtype == configs.DTYPE_F32 else 4e-3
    for a, b in zip(runs[1], runs[0]):
        for l in range(cfg.n_layers + 1):
            assert relerr(a[l], b[l].astype(np.float64)) <= tol


@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("cfg0", TINY_BOTH, ids=lambda c: c.name)
def test_kv_canary_every_slot_written(mode, cfg0):
    """Intrinsic KV integrity: with the cache pre-filled with NaN, every slot (l, p < pos)
    is finite after the run (backbone or river wrote it) and no slot beyond pos was touched."""
    needs_mode(cfg0, mode)
    say(f"KV canary {cfg0.name} mode={mode}")
    cfg = cfg0.with_(tau=0.52)
    w = inputs.make_weights(cfg, configs.C1.seed_weights)
    pair = Pair(cfg, w, mode)
    pair.g.fill_cache(0xFF)
    prompt = inputs.make_prompt(cfg.vocab, 16, configs.C1.seed_prompt)
    exits = run_teacher_forced(pair, prompt, 20, label="canary")
    assert min(exits) < cfg.n_layers
    n = 36
    pair.compare_cache(n)
    assert np.all(np.isnan(pair.g.kcache()[:, n:])) and np.all(np.isnan(pair.g.vcache()[:, n:]))
    assert np.all(pair.o.written()[:, :n] == 1)
    pair.close()


# ------------------------------------------------- several tiles, ragged tails

@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("cfg", [MID, MID_F32, MID_F32_HD128], ids=lambda c: c.name)
def test_mid_shape_ragged_tiles(mode, cfg):
    needs_mode(cfg, mode)
    say(f"mid shape {cfg.name} mode={mode}")
    w = inputs.make_weights(cfg, 77)
    pair = Pair(cfg, w, mode)
    prompt = inputs.make_prompt(cfg.vocab, 130, 78)          # every wavefront of the attention workgroups busy, ragged
    sched = [1, 3, 2, 3, 1, 2, 3, 3, 1, 2]
    exits = run_teacher_forced(pair, prompt, len(sched), sched, cfg.name)
    assert exits == sched
    pair.compare_cache(130 + len(sched))
    pair.close()


@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("cfg0", [configs.TINY, TINY_BF16], ids=lambda c: c.name)
def test_long_context_many_splits(mode, cfg0):
    """Attention over 1100+ cached positions: 4 splits of about 276 positions (two chunks
    per workgroup), merged by the consumer."""
    needs_mode(cfg0, mode)
    say(f"long context {cfg0.name} mode={mode}")
    cfg = cfg0.with_(max_seq=1200, tau=0.675)
    w = inputs.make_weights(cfg, configs.C1.seed_weights)
    pair = Pair(cfg, w, mode)
    prompt = inputs.make_prompt(cfg.vocab, 1100, 91)
    run_teacher_forced(pair, prompt, 6, label="long")
    pair.compare_cache(1106)
    pair.close()


MANY_HEADS = configs.ModelConfig("many-heads-bf16", 2, 512, 128, 32, 64, 1024, 512, 10000.0, 1e-5,
                                 configs.DTYPE_BF16, 1200, 1, 2.0)


@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("cfg", [MANY_HEADS, MANY_HEADS.with_(name="many-heads-fp32", dtype=configs.DTYPE_F32)],
                         ids=lambda c: c.name)
def test_many_heads_several_chunks_per_workgroup(mode, cfg):
    """128 query heads leave room for two splits only, so at 1100 positions a workgroup walks
    550 of them: both chunks in flight, then the first one issued again (the loop of the
    attention phase that the other shapes never take), one item per workgroup."""
    needs_mode(cfg, mode)
    say(f"many heads {cfg.name} mode={mode}")
    w = inputs.make_weights(cfg, 5)
    pair = Pair(cfg, w, mode)
    prompt = inputs.make_prompt(cfg.vocab, 1100, 6)
    sched = [1, 2, 2, 1]
    exits = run_teacher_forced(pair, prompt, len(sched), sched, cfg.name)
    assert exits == sched
    pair.compare_cache(1100 + len(sched))
    pair.close()


# ------------------------------------------------------------ API behaviour

def test_async_steps_and_records_match_sync():
    say("async records")
    cfg = TINY_BF16.with_(tau=0.675)                 # bf16: the one-launch mode
    w = inputs.make_weights(cfg, configs.C1.seed_weights)
    dw = binding.upload_weights(w)
    dr = binding.quantize_river(cfg, dw)
    prompt = inputs.make_prompt(cfg.vocab, 16, configs.C1.seed_prompt)
    g = binding.River(cfg, dw, dr)
    tok = g.prefill(prompt)
    sync = []
    for _ in range(24):
        tok, e, s = g.decode_step(tok)
        sync.append((tok, e, s.copy()))
    h_sync, l_sync = g.hidden(), g.logits()
    g.close()
    g = binding.River(cfg, dw, dr)
    g.prefill(prompt)
    for _ in range(24):
        g.decode_step(None, None, sync=False)      # consumes the device-side token, no host sync
    toks, es, sims = g.read_records(24)
    assert list(toks) == [t for t, _, _ in sync]
    assert list(es) == [e for _, e, _ in sync]
    np.testing.assert_array_equal(sims, np.array([s for _, _, s in sync]))
    # determinism: same seed, same bits
    np.testing.assert_array_equal(g.hidden(), h_sync)
    np.testing.assert_array_equal(g.logits(), l_sync)
    g.close()


@pytest.mark.parametrize("cfg0", TINY_BOTH, ids=lambda c: c.name)
def test_one_token_prompt_and_rewind_replay(cfg0):
    """A prompt of a single token; then a rewind by three positions followed by the same
    steps gives the same bits as the first pass (the rewritten cache slots hold the same
    values) and still matches the oracle, which is rewound the same way."""
    say(f"short prompt + rewind {cfg0.name}")
    cfg = cfg0.with_(tau=0.675)
    w = inputs.make_weights(cfg, configs.C1.seed_weights)
    pair = Pair(cfg, w, None)
    tok = pair.prefill([7])
    toks, hs = [tok], []
    for i in range(6):
        tok, e, _ = pair.step(tok, what=f"pass 1 step {i}")
        toks.append(tok)
        hs.append(pair.g.hidden())
    pair.g.rewind(4)                 # positions 4, 5, 6 are decoded again
    pair.o.rewind(4)
    tok = toks[3]
    for i in range(3, 6):
        tok, e, _ = pair.step(tok, what=f"pass 2 step {i}")
        assert tok == toks[i + 1]
        np.testing.assert_array_equal(pair.g.hidden(), hs[i])
    pair.compare_cache(7)
    pair.close()


def test_error_paths_through_the_abi():
    say("error paths")
    cfg = configs.TINY.with_(max_seq=8)
    w = inputs.make_weights(cfg, 3)
    dw = binding.upload_weights(w)
    dr = binding.quantize_river(cfg, dw)
    g = binding.River(cfg, dw, dr)
    with pytest.raises(binding.RiverError) as ei:
        g.decode_step(1)
    assert ei.value.code == binding.RIVER_ESTATE                 # decode before prefill
    with pytest.raises(binding.RiverError) as ei:
        g.prefill([cfg.vocab])
    assert ei.value.code == binding.RIVER_EINVAL
    with pytest.raises(binding.RiverError) as ei:
        g.prefill(list(range(9)))
    assert ei.value.code == binding.RIVER_ENOSPC
    g.prefill([1, 2, 3, 4, 5, 6, 7])
    with pytest.raises(binding.RiverError) as ei:
        g.decode_step(1, 1)                                      # below L_s
    assert ei.value.code == binding.RIVER_EINVAL
    g.decode_step(1)
    with pytest.raises(binding.RiverError) as ei:
        g.decode_step(1)                                         # cache full
    assert ei.value.code == binding.RIVER_ENOSPC
    with pytest.raises(binding.RiverError):
        g.rewind(99)
    g.rewind(3)
    assert g.pos == 3
    g.close()
    dense = binding.River(cfg.with_(tau=0.1), dw, None)
    dense.prefill([1, 2])
    with pytest.raises(binding.RiverError) as ei:
        dense.decode_step(1)                                     # could exit but has no river
    assert ei.value.code == binding.RIVER_ESTATE
    dense.close()


def test_barrier_wait_is_bounded():
    """A spin limit of one poll makes device-wide waits give up at once: the kernel must
    still run to completion and the host must report the time-out, not hang."""
    say("bounded barrier wait")
    cfg = TINY_BF16
    w = inputs.make_weights(cfg, 3)
    dw = binding.upload_weights(w)
    g = binding.River(cfg.with_(tau=2.0), dw, None, exec_mode=binding.EXEC_PERSISTENT, spin_limit=1)
    try:
        g.prefill([1, 2, 3, 4])
        timed_out = False
    except binding.RiverError as e:
        timed_out = e.code == binding.RIVER_EHIP
    # with one poll per wait at least one of the 21 barriers per token gives up
    assert timed_out
    with pytest.raises(binding.RiverError):
        g.decode_step(1)
    g.close()
    # a fresh context on the same device works afterwards
    g = binding.River(cfg.with_(tau=2.0), dw, None, exec_mode=binding.EXEC_PERSISTENT)
    assert 0 <= g.prefill([1, 2, 3, 4]) < cfg.vocab
    g.close()


# ------------------------------------------- long context: 5 to 8 attention splits

LONG = configs.ModelConfig("long-hd128-bf16", 2, 512, 8, 2, 128, 1408, 1002, 500000.0, 1e-5,
                           configs.DTYPE_BF16, 4208, 1, 2.0)
LONG_F32 = LONG.with_(name="long-hd128-fp32", dtype=configs.DTYPE_F32)


@pytest.mark.parametrize("cfg", [LONG, LONG_F32], ids=lambda c: c.name)
def test_long_context_5_to_8_splits_head_dim_128(cfg):
    """Contexts of 2305 .. 4203 positions at head_dim 128: the host picks 5, 6, 7 and 8
    attention splits (one per 512 positions above 2048), every workgroup walks more than
    two chunks (bf16: 3 chunks of 256 positions, fp32: 5 of 128), and the consumer merges
    up to eight partials.  One 4200-token prompt, then the sequence is rewound to shorter
    lengths on both sides (slots beyond the length are never read), three teacher-forced
    steps with backbone and river blocks at each length."""
    w = inputs.make_weights(cfg, 61)
    river = ro.quantize_river(cfg, w)
    prompt = inputs.make_prompt(cfg.vocab, 4200, 62)
    modes = MODES if cfg.dtype == configs.DTYPE_BF16 else [binding.EXEC_KERNELS]
    for mode in modes:
        say(f"long context {cfg.name} mode={mode}: oracle prefill of {len(prompt)} tokens")
        pair = Pair(cfg, w, mode, oracle=ro.Oracle(cfg, w, river))
        tok = pair.prefill(prompt)
        for length, splits in ((4200, 8), (3328, 7), (2816, 6), (2304, 5)):
            pair.g.rewind(length)
            pair.o.rewind(length)
            assert min(8, -(-(length + 1) // 512)) == splits
            for i, e in enumerate((1, 2, 2)):
                tok, eo, _ = pair.step(tok, e, what=f"{cfg.name} mode {mode} length {length} step {i}")
            say(f"  length {length} ({splits} splits) ok")
        pair.compare_cache(4203)
        pair.close()


# ------------------------------------------------------------ non-unit norm gains

@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("cfg0", [configs.TINY, TINY_BF16, MID, MID_F32_HD128], ids=lambda c: c.name)
def test_non_unit_norm_gains(mode, cfg0):
    """Norm gains 1 + N(0, 0.1^2): the gain multiply of the fused RMSNorm prologue (embedding
    row, hidden state and half-precision layouts, final norm) in backbone and river blocks."""
    needs_mode(cfg0, mode)
    say(f"norm gains {cfg0.name} mode={mode}")
    cfg = cfg0.with_(min_exit_layer=0)
    w = inputs.make_weights(cfg, 83, gain_std=0.1)
    assert float((w["layers"][0]["attn_norm"].float() - 1).abs().max()) > 0.05
    pair = Pair(cfg, w, mode)
    L = cfg.n_layers
    sched = [0, L, 1, L - 1, 2 % L, 0]
    exits = run_teacher_forced(pair, inputs.make_prompt(cfg.vocab, 9, 84), len(sched), sched, cfg0.name)
    assert exits == sched
    pair.compare_cache(9 + len(sched))
    pair.close()


# ------------------------------------------------ sequence-level exit in the prefill

@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("ep", [0, 2, 3])
@pytest.mark.parametrize("cfg0", [configs.TINY, TINY_BF16, MID], ids=lambda c: c.name)
def test_prefill_at_unified_exit_depth(mode, ep, cfg0):
    """Prefill phase with sequence-level exit: every prompt position runs e_p backbone blocks
    and river twins above; then token-level steps over that cache."""
    needs_mode(cfg0, mode)
    say(f"prefill depth {ep} {cfg0.name} mode={mode}")
    cfg = cfg0.with_(min_exit_layer=0)
    ep = min(ep, cfg.n_layers)
    w = inputs.make_weights(cfg, 87, gain_std=0.05)
    pair = Pair(cfg, w, mode)
    n = 37
    tok = pair.prefill(inputs.make_prompt(cfg.vocab, n, 88), ep)
    for i, e in enumerate((cfg.n_layers, 1, 0, 2)):
        tok, eo, _ = pair.step(tok, e, what=f"after prefill at {ep}, step {i}")
    pair.compare_cache(n + 4)
    pair.close()


def test_prefill_outputs_and_argument_checks():
    say("prefill outputs")
    cfg = TINY_BF16
    w = inputs.make_weights(cfg, 3)
    dw = binding.upload_weights(w)
    dr = binding.quantize_river(cfg, dw)
    g = binding.River(cfg, dw, dr)
    out = torch.full((cfg.vocab,), float("nan"), dtype=torch.float32, device="cuda")
    tok = g.prefill([5, 6, 7], None, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), g.logits())
    assert int(out.argmax()) == tok
    with pytest.raises(binding.RiverError) as ei:
        g.prefill([5, 6, 7], 1)                                  # below L_s = 2
    assert ei.value.code == binding.RIVER_EINVAL
    with pytest.raises(binding.RiverError) as ei:
        g.prefill([5, 6, 7], cfg.n_layers + 1)
    assert ei.value.code == binding.RIVER_EINVAL
    g.close()
    dense = binding.River(cfg.with_(tau=2.0), dw, None)
    with pytest.raises(binding.RiverError) as ei:
        dense.prefill([5, 6, 7], 2)                              # needs the river
    assert ei.value.code == binding.RIVER_ESTATE
    # outputs asked for without out_token: refused before anything is enqueued
    dense.prefill([5, 6, 7])
    import ctypes as C
    e = C.c_int32()
    rc = binding.load().river_decode_step(dense._h, None, None, None, C.byref(e), None)
    assert rc == binding.RIVER_EINVAL and dense.pos == 3
    dense.close()


def test_barrier_slot_pool_reuse_and_exhaustion():
    """Contexts take one of 64 barrier slots per device: 70 contexts created and destroyed one
    after the other reuse slots; the 65th simultaneous context is refused with RIVER_ENOSPC."""
    import gc
    say("barrier slot pool")
    gc.collect()
    cfg = TINY_BF16.with_(tau=2.0, max_seq=8)
    w = inputs.make_weights(cfg, 3)
    dw = binding.upload_weights(w)
    for i in range(70):
        g = binding.River(cfg, dw, None)
        if i % 23 == 0:
            assert 0 <= g.prefill([1, 2, 3]) < cfg.vocab
        g.close()
    held = []
    with pytest.raises(binding.RiverError) as ei:
        for i in range(65):
            held.append(binding.River(cfg, dw, None))
    assert ei.value.code == binding.RIVER_ENOSPC and "64" in str(ei.value)
    assert len(held) == 64
    ref = held[0].prefill([1, 2, 3])
    assert held[63].prefill([1, 2, 3]) == ref                    # the last slot works like the first
    for g in held:
        g.close()
    g = binding.River(cfg, dw, None)                             # slots are free again
    assert g.prefill([1, 2, 3]) == ref
    g.close()


# ------------------------------------------------------- prefill on the matrix cores

GEMM_SHAPES = [MID,
               configs.ModelConfig("pf-hd64-bf16", 2, 512, 16, 4, 64, 1024, 1002, 10000.0, 1e-5,
                                   configs.DTYPE_BF16, 400, 0, 2.0),
               configs.ModelConfig("pf-g128-bf16", 2, 256, 4, 4, 128, 640, 300, 500000.0, 1e-5,
                                   configs.DTYPE_BF16, 400, 0, 2.0, river_group=128)]


@pytest.mark.parametrize("n_prompt", [1, 33, 130, 300])
@pytest.mark.parametrize("cfg0", GEMM_SHAPES, ids=lambda c: c.name)
def test_gemm_prefill_matches_oracle(cfg0, n_prompt):
    """The MFMA prefill (forced for every prompt length) at full depth, at a unified depth in
    the middle and with every block as its river twin: hidden states and logits of the last
    prompt position, the K/V cache of every block and position (ragged last 128-row tile,
    several key tiles, the causal diagonal), then token-level steps over that cache."""
    cfg = cfg0.with_(min_exit_layer=0, max_seq=400)
    w = inputs.make_weights(cfg, 93, gain_std=0.05)
    river = ro.quantize_river(cfg, w)
    prompt = inputs.make_prompt(cfg.vocab, n_prompt, 94)
    for ep in (cfg.n_layers, 1, 0):
        say(f"GEMM prefill {cfg.name} prompt {n_prompt} depth {ep}")
        pair = Pair(cfg, w, None, oracle=ro.Oracle(cfg, w, river), prefill_gemm_min_tokens=1)
        tok = pair.prefill(prompt, ep)
        pair.compare_cache(n_prompt)
        for i, e in enumerate((cfg.n_layers, 0, 1)):
            tok, _, _ = pair.step(tok, e, what=f"{cfg.name} after GEMM prefill at {ep}, step {i}")
        pair.compare_cache(n_prompt + 3)
        pair.close()


def test_gemm_prefill_in_chunks_equals_serial_prefill_closely():
    """A prompt longer than one chunk (1024 rows): positions of later chunks attend to the
    cache the earlier chunks wrote.  Compared with the per-position prefill of the same
    library (same cache slots, tolerance of the half-precision operands) and, through
    test_long_context_5_to_8_splits_head_dim_128, with the oracle."""
    cfg = LONG.with_(max_seq=2600)
    w = inputs.make_weights(cfg, 95)
    dw = binding.upload_weights(w)
    dr = binding.quantize_river(cfg, dw)
    prompt = inputs.make_prompt(cfg.vocab, 2500, 96)
    outs = []
    for min_tokens in (-1, 1):
        g = binding.River(cfg, dw, dr, prefill_gemm_min_tokens=min_tokens)
        tok = g.prefill(prompt, 1)
        outs.append((tok, g.hidden(), g.logits(), g.kcache()[:, :2500].copy(), g.vcache()[:, :2500].copy()))
        g.close()
    for a, b in zip(outs[1][1:], outs[0][1:]):
        assert relerr(a, np.asarray(b, np.float64)) <= 5e-3


# ------------------------------------------------------------ backbone offloading

@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
def test_backbone_offloading_reads_deep_blocks_from_pinned_host_memory(mode):
    """Backbone Offloading (method section; appendix on memory): the matrices of backbone
    blocks above a depth cutoff live in pinned host memory instead of HBM; the river stays
    resident.  Tokens that stay below the cutoff never touch them; tokens that go deeper read
    them in place.  Results must equal the all-in-HBM context bit for bit and match the oracle."""
    cfg = MID.with_(min_exit_layer=0)
    say(f"backbone offloading mode={mode}")
    w = inputs.make_weights(cfg, 77, gain_std=0.05)
    pair = Pair(cfg, w, mode)
    off = binding.offload_backbone(pair.dw, 1)                  # blocks 2 and 3 out of HBM
    assert not off["layers"][2]["wq"].is_cuda and off["layers"][2]["wq"].is_pinned()
    assert off["layers"][0]["wq"].is_cuda and off["layers"][2]["attn_norm"].is_cuda
    g2 = binding.River(cfg, off, pair.dr, exec_mode=mode, prefill_gemm_min_tokens=-1)
    prompt = inputs.make_prompt(cfg.vocab, 12, 78)
    tok = pair.prefill(prompt, 1)                               # prefill at depth 1: no offloaded block is read
    assert g2.prefill(prompt, 1) == pair.g.prefill(prompt, 1)
    for i, e in enumerate([1, 0, 3, 1, 2, 3]):
        t2, e2, s2 = g2.decode_step(tok, e)
        tok, eo, so = pair.step(tok, e, what=f"offloading step {i}")
        np.testing.assert_array_equal(g2.hidden(), pair.g.hidden())
        np.testing.assert_array_equal(g2.logits(), pair.g.logits())
        assert e2 == eo
    g2.close()
    pair.close()


# ------------------------------------------------------------------ FP16 KV cache

@pytest.mark.parametrize("mode", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("cfg0", [TINY_BF16, MID, MANY_HEADS], ids=lambda c: c.name)
def test_fp16_kv_cache(mode, cfg0):
    """KV cache in IEEE half (the paper's cache type) under bf16 weights: decode attention at
    both head sizes, the per-position and the MFMA prefill, several splits; cache compared as
    half values with the oracle's."""
    say(f"fp16 KV cache {cfg0.name} mode={mode}")
    cfg = cfg0.with_(min_exit_layer=0, kv_dtype=configs.KV_F16, max_seq=700)
    w = inputs.make_weights(cfg, 97, gain_std=0.05)
    L = cfg.n_layers
    for n_prompt, gemm in ((9, -1), (600, 1)):
        if gemm == 1 and cfg.d_ffn % 64:
            gemm = -1
        pair = Pair(cfg, w, mode, prefill_gemm_min_tokens=gemm)
        tok = pair.prefill(inputs.make_prompt(cfg.vocab, n_prompt, 98), L if n_prompt == 9 else 1)
        for i, e in enumerate((L, 0, 1, L - 1)):
            tok, _, _ = pair.step(tok, e, what=f"fp16 cache {cfg.name} prompt {n_prompt} step {i}")
        pair.compare_cache(n_prompt + 4)
        kg = pair.g.kcache()[:, :n_prompt + 4]
        assert np.array_equal(kg, kg.astype(np.float16).astype(np.float32))
        pair.close()


def foreign_river(cfg, weights, group):
    """A river produced by another quantiser than the library's: integer zero points (as GPTQ- and
    AWQ-style formats store them), scale = (max - min) / 15 of the group rounded to the weight
    dtype, code = clamp(round(w / scale) + zero).  Input data for both sides."""
    out = []
    for blk in weights["layers"]:
        q = {}
        for m in ro.MATRICES:
            w = blk[m].to(torch.float32).numpy()
            rows, cols = w.shape
            g = w.reshape(rows, cols // group, group)
            mn, mx = g.min(-1), g.max(-1)
            scale = torch.from_numpy(np.where(mx > mn, (mx - mn) / 15.0, 1.0).astype(np.float32)).to(blk[m].dtype)
            sc = scale.to(torch.float32).numpy()
            zero = np.clip(np.rint(-mn / sc), 0, 15)
            codes = np.clip(np.rint(g / sc[..., None]) + zero[..., None], 0, 15).astype(np.uint8).reshape(rows, cols)
            packed = torch.from_numpy((codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8))
            q[m] = (packed.contiguous(), scale.contiguous(), torch.from_numpy(zero.astype(np.float32)).to(blk[m].dtype).contiguous())
        out.append(q)
    return out


@pytest.mark.parametrize("mode", MODES)
def test_river_quantised_elsewhere_integer_zero_points(mode):
    """The river arrays are plain data: a river from another quantiser (integer zero points,
    group 128) goes through prefill (MFMA GEMMs and per position) and decode on both sides."""
    cfg = MID.with_(name="mid-foreign-river", river_group=128, max_seq=96)
    weights = inputs.make_weights(cfg, 77, gain_std=0.1)
    river = foreign_river(cfg, weights, 128)
    for min_tokens in (0, -1):                          # MFMA prefill / per-position prefill
        say(f"foreign river, mode {mode}, prefill_gemm_min_tokens {min_tokens}")
        pair = Pair(cfg, weights, mode, prefill_gemm_min_tokens=min_tokens, river=river)
        tok = pair.prefill(inputs.make_prompt(cfg.vocab, 40, 78), 2)
        for step, forced in enumerate([1, 3, 2, 1]):
            tok, _, _ = pair.step(tok, forced, f"foreign river step {step}")
        pair.compare_cache(44)
        pair.close()
