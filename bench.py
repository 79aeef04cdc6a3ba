#!/usr/bin/env python3
"""Decode throughput of the early-exit path on one MI355X, with its HBM roofline.

A "step" is one decode step: one token through the whole hot path (embedding, L blocks
as backbone or river twin with KV written to the shared cache, exit test, final norm +
LM head + argmax).  Default workload: the 8B-shape bf16 configuration with a 512-token
prompt and a seeded forced exit schedule (about half of the tokens leave the backbone
in its first half); a dense (no-exit) run and an all-river run of the same shape are timed
alongside (the three columns of the paper's speed table).  All
inputs are synthetic and resident in HBM before the timed region starts.

Prints ONE JSON line.  --gpus above 1 is refused: this build is single-GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published peak
MEASURED = os.path.join(ROOT, "paper_2604_18396_amd", "measured_traffic.json")


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def timed_steps(g, torch, forced, k):
    """Queue k decode steps back to back (device-side token hand-over, no host sync) and
    time them with events on the stream the kernels run on."""
    stream = torch.cuda.current_stream()
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record(stream)
    for i in range(k):
        g.decode_step(None, None if forced[i] is None else int(forced[i]), sync=False)
    end.record(stream)
    torch.cuda.synchronize()
    return start.elapsed_time(end)        # ms


def cpu_baseline(cfg, weights, sched, budget_steps, budget_seconds=25.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the workload:
    at most budget_steps decode steps (and at most the schedule's length, and about
    budget_seconds) of the same shape and exit schedule after a 4-token prompt."""
    from oracle import river_oracle as ro
    from paper_2604_18396_amd import inputs
    t0 = time.time()
    river = ro.quantize_river(cfg, weights)
    o = ro.Oracle(cfg.with_(max_seq=64), weights, river)
    prompt = inputs.make_prompt(cfg.vocab, 4, 4242)
    tok = o.prefill(prompt)
    log(f"oracle ready (quantise + 4-token prompt) in {time.time() - t0:.1f}s")
    t1 = time.time()
    n = 0
    for i in range(min(int(budget_steps), len(sched), 56)):
        tok, e, _ = o.decode_step(tok, int(sched[i]))
        n += 1
        if time.time() - t1 > budget_seconds:
            break
    dt = time.time() - t1
    o.close()
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": n / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{n} decode steps of the same shape and exit schedule after a 4-token "
                      f"prompt (context 5..{4 + n}); fp64 C oracle with OpenMP"}


def phase_trace(ctx_len):
    """Per-phase timeline of the one-launch kernel at the 8B shape from the diagnostics build
    (device clock stamps at every device-wide barrier): for a dense and an all-river token, per
    phase the time until the first / median / last workgroup arrives at the barrier behind it
    and the time that barrier then takes.  Needs libriver_trace.so
    (python3 -c "from paper_2604_18396_amd import build; build.build(trace=True)")."""
    from paper_2604_18396_amd import build
    os.environ["RIVER_LIB_PATH"] = build.TRACE_LIB
    import numpy as np
    import torch
    from paper_2604_18396_amd import binding, byte_model, configs, inputs
    cfg = configs.LLAMA_8B.with_(max_seq=ctx_len + 64, min_exit_layer=0)
    one = cfg.with_(n_layers=1)
    w1 = inputs.make_weights(one, 7)                      # one block's weights stand for all 32 (timing only)
    dw1 = binding.upload_weights(w1)
    dw = {k: dw1[k] for k in ("tok_emb", "final_norm", "lm_head")}
    dw["layers"] = [dw1["layers"][0]] * cfg.n_layers
    dr = binding.quantize_river(one, dw1) * cfg.n_layers
    g = binding.River(cfg, dw, dr, exec_mode=binding.EXEC_PERSISTENT)
    g.prefill(list(range(1, ctx_len + 1)))
    L = cfg.n_layers
    names = ["QKV", "attention", "O-proj", "gate/up", "down"]
    mats = [("wq", "wk", "wv"), (), ("wo",), ("w_gate", "w_up"), ("w_down",)]
    print(f"# phase timeline of k_step_persistent<1>, 8B shape, context {ctx_len}, mean over blocks 2..{L}, microseconds")
    for which, fe in (("dense token (backbone blocks)", L), ("all-river token (4-bit twins)", 0)):
        for _ in range(4):
            g.decode_step(None, fe, sync=False)
        g.decode_step(None, fe, sync=True)
        t = g.trace(256).astype(np.int64)                # [5L, 2, 256], 10 ns ticks
        A, R = t[:, 0, :], t[:, 1, :]
        print(f"## {which}: whole token {(A[-1].max() - R[0].min()) / 100:.1f} us (first release to last arrival, head excluded)")
        print(f"#  {'phase':10s} {'MB read':>8s} {'first done':>10s} {'median':>8s} {'last done':>9s} {'barrier':>8s} {'span':>7s} {'at 8 TB/s':>9s}")
        total = 0.0
        for p in range(5):
            first, med, last, bar = [], [], [], []
            for l in range(1, L):
                b = l * 5 + p
                start = R[b - 1].max()
                first.append(A[b].min() - start); med.append(np.median(A[b]) - start)
                last.append(A[b].max() - start); bar.append(R[b].max() - A[b].max())
            f = lambda v: float(np.mean(v)) / 100
            mb = 0.0
            for m in mats[p]:
                r_, c_ = configs.matrix_shape(cfg, m)
                mb += (r_ * c_ * 2 if fe == L else r_ * c_ // 2 + 4 * r_ * (c_ // cfg.river_group)) / 1e6
            if p == 1:
                mb = byte_model.kv_bytes_per_position(cfg) / L * (ctx_len + 5) / 1e6
            span = f(last) + f(bar)
            total += span
            print(f"   {names[p]:10s} {mb:8.1f} {f(first):10.2f} {f(med):8.2f} {f(last):9.2f} {f(bar):8.2f} {span:7.2f} {mb / 8.0:9.2f}")
        print(f"   per block {total:.1f} us")
    g.close()


def calibrate_copy(mib, iters):
    """A plain device copy of known size, for scaling the rocprofv3 FETCH_SIZE / WRITE_SIZE
    counters: run `rocprofv3 --pmc FETCH_SIZE -- python3 bench.py --calibrate-copy 1024`."""
    import torch
    n = mib << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(iters):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"calibration_copy_mib": mib, "launches": iters}), flush=True)


def bench_batch(args, wl, torch, np, binding, byte_model, configs, inputs):
    """Ragged batch (C5): B sequences per step, exit positions drawn independently per sequence
    and step, both weight sets read wherever the batch straddles a block.  value = aggregate
    tokens/s over the B sequences.  Alongside: all sequences at full depth (dense), and all
    sequences sharing one exit position per step (what a whole-batch rule like Eq. 1's minimum
    over the batch buys: one weight set per block)."""
    K, W, B = args.steps, args.warmup, wl.batch
    cfg = wl.model.with_(max_seq=wl.prompt_len + W + K + 8)
    L = cfg.n_layers
    t0 = time.time()
    weights = inputs.make_weights(cfg, wl.seed_weights)
    log(f"weights generated on the host in {time.time() - t0:.1f}s")
    dw = binding.upload_weights(weights)
    dr = binding.quantize_river(cfg, dw)
    g = binding.River(cfg, dw, dr, max_batch=B)
    prompts = [inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed_prompt + b) for b in range(B)]
    scheds = np.stack([inputs.make_exit_schedule(L, W + K, wl.seed_exits + b) for b in range(B)], axis=1)  # [W+K, B]

    def prefill_all():
        t = time.time()
        for b in range(B):
            g.prefill(prompts[b], seq=b)
        torch.cuda.synchronize()
        return time.time() - t

    def run(sched):
        for i in range(W):
            g.decode_batch(B, None, sched[i], sync=False)
        stream = torch.cuda.current_stream()
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        start.record(stream)
        for i in range(W, W + K):
            g.decode_batch(B, None, sched[i], sync=False)
        end.record(stream)
        torch.cuda.synchronize()
        _, exits = g.read_batch_records(min(K, 1024), B)
        assert [list(map(int, e)) for e in exits] == [list(map(int, e)) for e in sched[W + K - len(exits):]], \
            "exit schedule not honoured"
        return start.elapsed_time(end)

    log(f"prefill of {B} x {wl.prompt_len} tokens in {prefill_all():.2f}s")
    ms_ragged = run(scheds)
    prefill_all()
    ms_dense = run(np.full_like(scheds, L))
    prefill_all()
    uniform = np.repeat(scheds[:, :1], B, axis=1)
    ms_uniform = run(uniform)
    g.close()
    ctx0 = wl.prompt_len + W

    def mean_bytes(sched):
        return float(np.mean([byte_model.batch_step_bytes(cfg, [int(e) for e in sched[W + i]], [ctx0 + i + 1] * B)
                              for i in range(K)]))

    def leg(ms, sched):
        by = mean_bytes(sched)
        gbs = by / (ms * 1e-3 / K) / 1e9
        return {"value": B * K / (ms * 1e-3), "unit": "tokens/s", "ms_per_step": ms / K,
                "algorithmic_bytes_per_step": by, "achieved_GBps": gbs, "frac": gbs / HBM_PEAK_GBS}

    r, dn, un = leg(ms_ragged, scheds), leg(ms_dense, np.full_like(scheds, L)), leg(ms_uniform, uniform)
    # HBM bytes per step from the rocprofv3 counter runs recorded beside the package
    traffic, traffic_detail = None, None
    if os.path.exists(MEASURED):
        traffic_detail = json.load(open(MEASURED)).get(f"{wl.name}:batched")
        if traffic_detail:
            traffic = traffic_detail["fetch_bytes_per_launch"] + traffic_detail["write_bytes_per_launch"]
            traffic_detail = dict(traffic_detail,
                                  source="NOT measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                         "runs summarised under profiles/ (see its note for the step count "
                                         "and the algorithmic bytes of that run)")
    out = {
        "metric": "decode tokens/s @batch1 (8B shape) w/ early exit; HBM GB/s as % of peak",
        "value": r["value"], "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "shape": cfg.name, "prompt_len": wl.prompt_len, "batch": B,
                   "exit_schedule": "forced, independent per sequence: 1/2 U{L/4..L/2} + 1/2 U{L/2+1..L-1}",
                   "mean_exit_position": float(np.mean(scheds[W:])), "exec_mode": "batched kernels",
                   "note": "aggregate over the batch; this workload is NOT the batch-1 headline metric"},
        "roofline": {"bound": "hbm", "achieved": r["achieved_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": r["frac"], "traffic": traffic, "kernel": "all kernels of a batched step "
                     "(k_bd_gemm dominates)", "algorithmic_bytes_per_launch": r["algorithmic_bytes_per_step"],
                     "traffic_detail": traffic_detail},
        "dense": dn, "uniform_exit": dict(un, note="every sequence of a step leaves at the same position "
                                                   "(one weight set per block), the effect of a whole-batch rule"),
    }
    if not args.no_cpu_baseline:
        try:
            from oracle import river_oracle as ro
            t0 = time.time()
            river = ro.quantize_river(cfg, weights)
            os_ = []
            for b in range(min(B, 8)):
                o = ro.Oracle(cfg.with_(max_seq=16), weights, river)
                os_.append((o, o.prefill(prompts[b][:2])))
            log(f"oracle ready in {time.time() - t0:.1f}s")
            t1, n = time.time(), 0
            for i in range(2):
                for b, (o, tok) in enumerate(os_):
                    tok, _, _ = o.decode_step(tok, int(scheds[i, b]))
                    os_[b] = (o, tok)
                    n += 1
                if time.time() - t1 > 20:
                    break
            dt = time.time() - t1
            out["cpu_baseline"] = {"value": n / dt, "unit": "tokens/s",
                                   "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                                   "kind": "oracle", "sample": f"{n} single-sequence decode steps (the batch's "
                                   "sequences one after the other, 2-token prompts); fp64 C oracle with OpenMP"}
        except Exception as exc:          # noqa: BLE001
            out["cpu_baseline"] = None
            out["cpu_baseline_error"] = f"{type(exc).__name__}: {exc}"
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="C3-8b-bf16-ctx512")
    ap.add_argument("--mode", default="persistent", choices=["persistent", "kernels"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=24)
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="only run a plain device copy of MIB MiB three times (counter calibration)")
    ap.add_argument("--offload-from", type=int, default=0, metavar="BLOCK",
                    help="Backbone Offloading: keep the matrices of backbone blocks above BLOCK in pinned host "
                         "memory (read in place over the host link); 0 = everything in HBM")
    ap.add_argument("--phase-trace", type=int, default=0, metavar="CTX",
                    help="only print the per-phase barrier timeline of the diagnostics build at context CTX")
    args = ap.parse_args()
    if args.phase_trace:
        phase_trace(args.phase_trace)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only; --gpus must be 1 "
              "(no collectives or sharding exist in it).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_18396_amd import binding, byte_model, configs, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        calibrate_copy(args.calibrate_copy, 3)
        return
    wl = configs.WORKLOADS[args.workload]
    if wl.batch > 1:
        bench_batch(args, wl, torch, np, binding, byte_model, configs, inputs)
        return
    K, W = args.steps, args.warmup
    cfg = wl.model.with_(max_seq=wl.prompt_len + W + K + 8)
    L = cfg.n_layers

    t0 = time.time()
    weights = inputs.make_weights(cfg, wl.seed_weights)
    log(f"weights generated on the host in {time.time() - t0:.1f}s")
    t0 = time.time()
    dw = binding.upload_weights(weights)
    dr = binding.quantize_river(cfg, dw)
    torch.cuda.synchronize()
    log(f"uploaded + river built on the GPU in {time.time() - t0:.1f}s")
    resident = byte_model.backbone_param_bytes(cfg) + L * byte_model.block_bytes_river(cfg)
    if args.offload_from:
        dw = binding.offload_backbone(dw, args.offload_from)
        resident -= (L - args.offload_from) * (byte_model.block_bytes_backbone(cfg) - 2 * cfg.d_model * 2)
        log(f"backbone blocks {args.offload_from + 1}..{L} offloaded to pinned host memory; "
            f"{resident / 2**30:.2f} GiB of parameters resident in HBM")
    mode = binding.EXEC_PERSISTENT if args.mode == "persistent" else binding.EXEC_KERNELS
    # tau = 1: Eq. 1 never fires (s <= 1, strict '>'), so the threshold-mode leg below runs
    # the whole backbone with the exit test taken after every block; forced legs ignore tau
    g = binding.River(cfg.with_(tau=1.0), dw, dr, exec_mode=mode)
    prompt = inputs.make_prompt(cfg.vocab, wl.prompt_len, wl.seed_prompt)
    t0 = time.time()
    g.prefill(prompt)
    log(f"prefill of {wl.prompt_len} tokens in {time.time() - t0:.2f}s")
    sched = inputs.make_exit_schedule(L, W + K, wl.seed_exits)

    # river run: W warm-up steps, then exactly K timed steps
    for i in range(W):
        g.decode_step(None, int(sched[i]), sync=False)
    ms_river = timed_steps(g, torch, sched[W:], K)
    toks, exits, _ = g.read_records(K)
    assert list(exits) == [int(e) for e in sched[W:]], "exit schedule not honoured"
    # dense run at the same shape and the same context lengths
    g.rewind(wl.prompt_len)
    dense = np.full(W + K, L, dtype=np.int32)
    for i in range(W):
        g.decode_step(None, L, sync=False)
    ms_dense = timed_steps(g, torch, dense[W:], K)
    # the same dense steps with Eq. 1 deciding (tau = 1 never exits): every workgroup reduces
    # the similarity partials after every backbone block; the difference to the forced dense
    # run is the cost of the exit decision on the critical path
    g.rewind(wl.prompt_len)
    for i in range(W):
        g.decode_step(None, None, sync=False)
    ms_thr = timed_steps(g, torch, [None] * K, K)
    _, exits_thr, _ = g.read_records(K)
    assert set(int(e) for e in exits_thr) == {L}, "tau = 1 must never exit"
    g.close()
    # all-river run ("Full-Quant." of the paper's speed table: every block as its 4-bit twin,
    # exit position 0), same shape and context lengths; needs L_s = 0, hence its own context
    g0 = binding.River(cfg.with_(min_exit_layer=0), dw, dr, exec_mode=mode)
    g0.prefill(prompt)
    zeros = np.zeros(W + K, dtype=np.int32)
    for i in range(W):
        g0.decode_step(None, 0, sync=False)
    ms_fq = timed_steps(g0, torch, zeros[W:], K)
    g0.close()

    ctx0 = wl.prompt_len + W                      # positions attended by timed step i: ctx0 + i + 1
    bytes_river = [byte_model.step_bytes(cfg, int(sched[W + i]), ctx0 + i + 1) for i in range(K)]
    bytes_dense = [byte_model.step_bytes(cfg, L, ctx0 + i + 1) for i in range(K)]
    bytes_fq = [byte_model.step_bytes(cfg, 0, ctx0 + i + 1) for i in range(K)]
    tok_s = K / (ms_river * 1e-3)
    tok_s_dense = K / (ms_dense * 1e-3)
    gbs = float(np.mean(bytes_river)) / (ms_river * 1e-3 / K) / 1e9
    gbs_dense = float(np.mean(bytes_dense)) / (ms_dense * 1e-3 / K) / 1e9
    tok_s_fq = K / (ms_fq * 1e-3)
    gbs_fq = float(np.mean(bytes_fq)) / (ms_fq * 1e-3 / K) / 1e9

    # HBM bytes per launch from the rocprofv3 counter runs recorded beside the package
    traffic, traffic_detail = None, None
    if os.path.exists(MEASURED):
        traffic_detail = json.load(open(MEASURED)).get(f"{args.workload}:{args.mode}")
        if traffic_detail:
            traffic = traffic_detail["fetch_bytes_per_launch"] + traffic_detail["write_bytes_per_launch"]
            traffic_detail = dict(traffic_detail,
                                  source="NOT measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                         "runs summarised under profiles/ (see its note for the step count "
                                         "and the algorithmic bytes of that run)")

    out = {
        "metric": "decode tokens/s @batch1 (8B shape) w/ early exit; HBM GB/s as % of peak",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_river / K, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.dtype == 1 else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "shape": cfg.name, "prompt_len": wl.prompt_len,
                   "exit_schedule": "forced, 1/2 U{L/4..L/2} + 1/2 U{L/2+1..L-1}",
                   "mean_exit_position": float(np.mean(sched[W:])), "exec_mode": args.mode,
                   "batch": 1, "offload_from": args.offload_from,
                   "resident_parameter_GiB": resident / 2**30},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "k_step_persistent<1, false>" if args.mode == "persistent" else "all step kernels",
                     "algorithmic_bytes_per_launch": float(np.mean(bytes_river)),
                     "traffic_detail": traffic_detail},
        "dense": {"value": tok_s_dense, "unit": "tokens/s", "ms_per_step": ms_dense / K,
                  "achieved_GBps": gbs_dense, "frac": gbs_dense / HBM_PEAK_GBS},
        "full_quant": {"value": tok_s_fq, "unit": "tokens/s", "ms_per_step": ms_fq / K,
                       "achieved_GBps": gbs_fq, "frac": gbs_fq / HBM_PEAK_GBS,
                       "note": "every block as its 4-bit river twin (exit position 0)"},
        "threshold_dense": {"value": K / (ms_thr * 1e-3), "unit": "tokens/s", "ms_per_step": ms_thr / K,
                            "note": "Eq. 1 decides with tau = 1 (never exits): dense steps with the exit "
                                    "test on the critical path of every block"},
        "exit_decision_us_per_block": (ms_thr - ms_dense) / K * 1e3 / (L - 1),
        "exit_decision_us_per_token": (ms_thr - ms_dense) / K * 1e3,
        "speedup_vs_dense": tok_s / tok_s_dense,
        "full_quant_speedup_vs_dense": tok_s_fq / tok_s_dense,
        "paper_context": "River-LLM reports 1.53x-2.16x over its 16-bit backbone on one NVIDIA A40 "
                         "(Llama3.1-8B: 25.3 -> 45.0 tokens/s on GSM8K); other hardware, not a target",
    }
    if not args.no_cpu_baseline:
        # the GPU figures above are printed whatever happens in the CPU leg
        try:
            out["cpu_baseline"] = cpu_baseline(cfg, weights, sched[W:], args.cpu_steps)
        except Exception as exc:          # noqa: BLE001
            out["cpu_baseline"] = None
            out["cpu_baseline_error"] = f"{type(exc).__name__}: {exc}"
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
