#!/usr/bin/env python3
"""Benchmark of the pruning stage on one MI355X.

A step = one pass of the whole hot path (asap_score, asap_select, asap_merge, asap_compact_kv)
over one batch of synthetic input already resident in HBM.  The K/V compaction runs on a second
stream next to the similarity and merge kernels (its positions come from asap_positions right
after the selection); the step ends when both streams are done.  Default workload: C6, the
2304-visual-token, batch-16, bf16 configuration (LLaVA-NeXT-7B shaped) the metric is quoted on.

Prints ONE JSON line: whole-job images/s, ms per step, the roofline of the dominant kernel
(per-kernel durations measured with HIP events recorded by the library on the launch stream,
in a second pass of the same K steps right after the timed one, so that the events do not
slow the timed region), the whole-stage HBM fraction, and the fp64 oracle timed on the host
cores on a bounded sample of the same workload.

    python bench.py [--steps K] [--warmup W] [--workload C6] [--no-cpu-baseline] [--copy-calibration]
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

HBM_PEAK = 8.0e12          # B/s, MI355X HBM3E
MFMA_PEAK = {"bf16": 2.5e15, "f32": 157.3e12}

def measured_traffic(workload: str, kernels) -> tuple:
    """HBM bytes per launch and kernel as rocprofv3's FETCH_SIZE / WRITE_SIZE counters saw them in an
    earlier run of this script: read from the committed summary profiles/bench_<workload>_hbm_traffic.txt
    (its header holds the commands and the calibration against a plain copy).  The figures are only used
    when that summary lists exactly the kernels this run launched; otherwise (a kernel was added, renamed
    or dropped since the counters were taken) none is reported.  Returns (dict or None, source, note)."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_hbm_traffic.txt")
    rel = os.path.relpath(path, ROOT)
    if not os.path.exists(path):
        return None, rel, "no counter summary for this workload"
    table = {}
    for line in open(path):
        parts = line.split()
        if len(parts) >= 6 and parts[0].startswith("k_"):
            try:
                table[parts[0].split("<")[0]] = float(parts[-1]) * 1e6
            except ValueError:
                pass
    if set(table) != set(kernels):
        return None, rel, ("the summary lists other kernels than this run launched: "
                           f"only there {sorted(set(table) - set(kernels))}, only here {sorted(set(kernels) - set(table))}")
    return table, rel, "counter run of an earlier build of the same kernel list, not of this run"


def esize(dt: str) -> int:
    return 2 if dt == "bf16" else 4


def algorithmic_bytes(cfg, mean_text: float, n_layers: int) -> dict:
    """Compulsory bytes (each input read once, each output written once) per kernel and for the
    whole stage, and the similarity flops."""
    B, H, Hkv, d, D, P, V, k = cfg.B, cfg.H, cfg.Hkv, cfg.d, cfg.D, cfg.P, cfg.V, cfg.k
    eq, eh, ek = esize(cfg.qk_dtype), esize(cfg.h_dtype), esize(cfg.kv_dtype)
    T = mean_text
    q_vis, k_vis, q_txt = B * H * V * d * eq, B * Hkv * V * d * eq, B * H * T * d * eq
    vis_h = B * V * D * eh
    out_rows = B * (P + k + T)
    per_kernel = {
        "k_qsum": q_vis,
        "k_qsplit": 8 * B * H * d + 16 * B * Hkv * d,
        "k_mass_mfma": k_vis + 12 * B * V,
        "k_attn_stats": k_vis + q_txt + 8 * B * V,
        "k_attn_colsum": k_vis + q_txt + 4 * B * H * V,
        "k_mass_finish": 20 * B * V,
        "k_rowstats_logits": 4 * B * H * V + 8 * B * V,
        "k_colsum_logits": 8 * B * H * V,
        "k_score": 4 * B * H * V + 16 * B * V,
        "k_select": 12 * B * V,
        "k_score_select": 4 * B * H * V + 16 * B * V + 8 * B * V,
        "k_positions": 4 * B * k + 4 * B * (P + k + cfg.Tmax),
        "k_sim": vis_h + 8 * B * (V - k),
        "k_merge": vis_h + B * (P + T) * D * eh + out_rows * D * eh,
        "k_compact": 2 * 2 * n_layers * Hkv * out_rows * d * ek,
    }
    per_kernel["k_compact_paged"] = per_kernel["k_compact"]
    # K/V rows of prefix and text: moved by k_score_select_kv when the stage runs that kernel, and then
    # not by k_compact (the caller of this function moves the bytes over when it sees that kernel)
    per_kernel["kv_fixed_rows"] = 2 * 2 * n_layers * Hkv * B * (P + T) * d * ek
    per_kernel["k_score_select_kv"] = per_kernel["k_score_select"] + per_kernel["kv_fixed_rows"]
    per_kernel["k_compact_fixed"] = per_kernel["kv_fixed_rows"]       # deep caches: those rows start at once
    # f32 keys: the first text-row sweep leaves its logits and k_colsum_rows reads them (the caller of
    # this function adds them to k_attn_stats when it sees that kernel); bytes of work, not compulsory ones
    per_kernel["stored_logits"] = 4 * B * H * T * V
    per_kernel["k_colsum_rows"] = per_kernel["stored_logits"] + 4 * B * H * V
    stage = (q_vis + k_vis + q_txt + 12 * B * V) + 12 * B * V + (vis_h + 8 * B * (V - k)) \
        + (vis_h + B * (P + T) * D * eh + out_rows * D * eh) + per_kernel["k_compact"]
    return {"per_kernel": per_kernel, "stage": stage, "sim_flops": 2.0 * B * (V - k) * k * D}


def cpu_baseline(inp, cfg, budget_s: float = 12.0, route: str = "absorb", lse_extra=None,
                 score_rows: str = "all") -> dict:
    """The oracle as it stands, timed on the host on the first few images of the batch."""
    import numpy as np
    from oracle import asap_oracle as O          # only this leg touches the oracle
    from paper_2603_14549_amd import synth
    try:
        from threadpoolctl import threadpool_info
        pools = threadpool_info()
        threads = max([i.get("num_threads", 1) for i in pools] or [1])
        blas = ", ".join(sorted({f"{i.get('internal_api', '?')} {i.get('version', '')}".strip() for i in pools}))
    except Exception:
        threads, blas = os.cpu_count() or 1, "unknown"
    cpu_model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu_model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    done, t_total = 0, 0.0
    while t_total < budget_s and done < 16 * cfg.B:
        t0 = time.perf_counter()
        b = done % cfg.B
        ref = O.stage(synth.to_f64(inp["q"][b], cfg.qk_dtype), synth.to_f64(inp["k"][b], cfg.qk_dtype),
                      synth.to_f64(inp["hidden"][b], cfg.h_dtype), int(inp["text_len"][b]), cfg.P, cfg.V,
                      cfg.Tmax, cfg.k, linear_mass=True, route=route,
                      lse_extra=None if lse_extra is None else lse_extra[b].astype(np.float64),
                      score_rows=score_rows)
        for l in range(cfg.L_kv):
            for cache in (inp["k_cache"][l], inp["v_cache"][l]):
                O.gather_kv(cache[b], ref["pos_out"], ref["new_len"])
        t_total += time.perf_counter() - t0
        done += 1
    return {"value": done / t_total, "unit": "images/s", "cores": int(threads), "kind": "oracle",
            "cpu_model": cpu_model, "os_cpu_count": os.cpu_count(), "blas": blas, "blas_threads": int(threads),
            "sample": f"{done} single-image oracle stages cycling over the {cfg.B} images of workload {cfg.name} "
                      f"(fp64 NumPy, sum-of-queries form of Eq. 2, K/V gather included, {t_total:.1f} s)",
            "ms_per_image": 1e3 * t_total / done}


def bench_library_gemm(args, cfg):
    """Reference point, not part of the product: the vendor GEMM library (through torch.bmm) on the
    similarity product's shape with dense, already gathered operands -- no row gather, no norms, no
    arg-max -- and with torch's row arg-max added.  Says what fraction of the MFMA peak a plain GEMM of
    this shape reaches on the same GPU."""
    import torch
    dt = torch.bfloat16 if cfg.h_dtype == "bf16" else torch.float32
    M, K, N = cfg.V - cfg.k, cfg.D, cfg.k
    a = torch.randn(cfg.B, M, K, device="cuda").to(dt)
    b = torch.randn(cfg.B, N, K, device="cuda").to(dt)
    big = torch.randn(8192, 8192, device="cuda").to(dt)

    def timed(f):
        for _ in range(args.warmup):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps

    flops = 2.0 * cfg.B * M * K * N
    t_gemm = timed(lambda: torch.bmm(a, b.transpose(1, 2)))
    t_argmax = timed(lambda: torch.bmm(a, b.transpose(1, 2)).max(dim=2))
    t_big = timed(lambda: big @ big)
    peak = MFMA_PEAK[cfg.h_dtype]
    print(json.dumps({
        "metric": "vendor-library GEMM on the similarity shape (reference)", "unit": "us", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "dtype": cfg.h_dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.B} x [{M} x {K}] x [{K} x {N}]"},
        "bmm_us": 1e6 * t_gemm, "bmm_frac_of_mfma_peak": flops / t_gemm / peak,
        "bmm_plus_row_argmax_us": 1e6 * t_argmax,
        "gemm_8192_cubed_us": 1e6 * t_big, "gemm_8192_cubed_frac_of_mfma_peak": 2.0 * 8192 ** 3 / t_big / peak}))


def bench_front_end(args, cfg):
    """asap_score_from_hidden (Eq. 2 from the hidden states, the fused front end) against asap_score on the
    same workload: the whole scoring call both ways, and the kernels of each."""
    import numpy as np
    import torch
    from paper_2603_14549_amd import binding, harness, synth
    inp = synth.make_inputs(cfg, with_kv=False)
    ctx = binding.Context(0)
    st = harness.DeviceStage(inp, ctx=ctx)
    P, V = cfg.P, cfg.V
    wq = harness.to_device(synth.quantise(np.ascontiguousarray(inp["Wq"].T), cfg.h_dtype), cfg.h_dtype)
    ws = torch.empty(binding.asap_front_end_workspace_bytes(st.p), dtype=torch.uint8, device="cuda")
    q_vis, q_txt, k_vis = st.q[:, :, P:P + V], st.q[:, :, P + V:], st.k[:, :, P:P + V]
    b = st.buf
    calls = {
        "asap_score": lambda: ctx.asap_score(st.p, q_vis, q_txt, k_vis, st.text_len, None, b.s_raw, b.s_hat, b.score,
                                             b.workspace),
        "asap_score_from_hidden": lambda: ctx.asap_score_from_hidden(st.p, st.hidden, wq, cfg.rope_theta, None, q_txt,
                                                                     k_vis, st.text_len, None, b.s_raw, b.s_hat,
                                                                     b.score, ws),
    }
    res = {}
    for name, run in calls.items():
        for _ in range(args.warmup):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run()
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / args.steps
        ctx.asap_timing_enable(min(8192, 12 * args.steps))
        for _ in range(args.steps):
            run()
        torch.cuda.synchronize()
        timing = ctx.asap_timing_collect()
        ctx.asap_timing_enable(0)
        res[name] = {"ms_per_call": ms, "kernels_us": {k: round(1e3 * v[0] / v[1], 1) for k, v in timing.items()}}
    eh, eq = esize(cfg.h_dtype), esize(cfg.qk_dtype)
    print(json.dumps({
        "metric": "scoring call: visual queries given vs taken from the hidden states", "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "dtype": cfg.h_dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B}, {cfg.V} visual tokens, hidden {cfg.D}, {cfg.H} heads x {cfg.d}"},
        "bytes_read_visual_queries_MB": cfg.B * cfg.H * cfg.V * cfg.d * eq / 1e6,
        "bytes_read_visual_hidden_MB": cfg.B * cfg.V * cfg.D * eh / 1e6,
        "extra_multiply_adds_G": 2.0 * cfg.B * cfg.d * cfg.V * cfg.D / 1e9,
        **res}))


def bench_attention(args, cfg):
    """asap_attention on the workload's shapes: q, k from the generator, random values; one launch set
    (bias, transpose, attention) per step.  Flops = 4 d per (query, key) pair the mask lets through."""
    import numpy as np
    import torch
    from paper_2603_14549_amd import binding, harness, synth
    inp = synth.make_inputs(cfg, with_kv=False)
    ctx = binding.Context(0)
    stage = harness.DeviceStage(inp, ctx=ctx)
    buf = stage.run()
    vals = torch.randn(cfg.B, cfg.Hkv, cfg.N, cfg.d, device="cuda").to(stage.q.dtype)
    out = torch.empty(cfg.B, cfg.H, cfg.N, cfg.d, dtype=stage.q.dtype, device="cuda")
    ws = torch.empty(binding.asap_attention_workspace_bytes(stage.p), dtype=torch.uint8, device="cuda")
    run = lambda: ctx.asap_attention(stage.p, stage.q, stage.k, vals, buf.s_hat, out, ws)
    steps, warmup = args.steps, args.warmup
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ctx.asap_timing_enable(min(8192, 4 * steps))
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    timing = ctx.asap_timing_collect()
    ctx.asap_timing_enable(0)
    N, V = cfg.N, cfg.V
    pairs = N * (N + 1) // 2 + V * (V - 1) // 2
    flops = 4.0 * cfg.d * pairs * cfg.H * cfg.B
    ms, n = timing["k_attention"]
    k_s = 1e-3 * ms / n
    peak = MFMA_PEAK[cfg.qk_dtype]
    print(json.dumps({
        "metric": "SG-BiMask attention forward, images/sec per layer", "value": cfg.B * steps / elapsed,
        "unit": "images/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": 1e3 * elapsed / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.qk_dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B}, N={N} ({cfg.P}+{V}+{cfg.Tmax}), {cfg.H}/{cfg.Hkv} heads x {cfg.d}, "
                               f"mask=keybias"},
        "roofline": {"kernel": "k_attention", "bound": "mfma", "achieved": flops / k_s / 1e12, "peak": peak / 1e12,
                     "unit": "TFLOP/s", "frac": flops / k_s / peak, "traffic": None},
        "kernels": {k: {"avg_us": round(1e3 * v[0] / v[1], 1)} for k, v in timing.items()}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C6")
    ap.add_argument("--route", choices=["absorb", "paper"], default="absorb",
                    help="absorb (default, the headline workload): pruned -> kept routing; paper: Sec. 4.2 as "
                         "written, routing inside the kept set + refill (threshold 0.8)")
    ap.add_argument("--attention", action="store_true",
                    help="measure asap_attention (one layer's forward under the Eq. 4-5 mask) on the workload's "
                         "shapes instead of the pruning stage; prints its own JSON line")
    ap.add_argument("--front-end", action="store_true",
                    help="time asap_score_from_hidden (Eq. 2 from the hidden states) against asap_score on the "
                         "workload; prints its own JSON line")
    ap.add_argument("--library-gemm", action="store_true",
                    help="reference point only: time the vendor GEMM library (torch.bmm) on the similarity "
                         "product's shape with dense operands, and an 8192^3 GEMM; prints its own JSON line")
    ap.add_argument("--lse-extra", action="store_true",
                    help="full-row softmax timing path (Eq. 5 over the whole row): pass a seeded log-sum-exp of "
                         "every text row's non-visual logits, which the score kernels fold into the denominators")
    ap.add_argument("--paged-kv", type=int, default=0, metavar="PAGE_SIZE",
                    help="keep the K/V caches as pools of PAGE_SIZE-token pages with block tables and compact them "
                         "with asap_compact_kv_paged (0 = contiguous caches, the headline workload)")
    ap.add_argument("--last-token", action="store_true",
                    help="rank the visual tokens by the last text token's row alone (score_rows = ASAP_ROWS_LAST)")
    ap.add_argument("--rotate", type=int, default=0, metavar="SETS",
                    help="also time the stage cycling over SETS (>= 2) copies of the inputs and outputs at different "
                         "addresses, so that no step finds its data in the caches (the small workloads fit the "
                         "256 MB last-level cache and their default, warm figure profits from it)")
    ap.add_argument("--hidden-row-pad", type=int, default=0, metavar="ELEMENTS",
                    help="store the rows of the input hidden states this many elements further apart than their "
                         "length (the stage takes strided views; rows a power of two bytes apart all start in the "
                         "same memory channel)")
    ap.add_argument("--in-flight", type=int, default=0, metavar="BATCHES",
                    help="also time BATCHES (>= 2) independent copies of the batch in flight at once, each with a "
                         "context and a stream of its own (a serving loop that does not wait for one batch before "
                         "it submits the next); reported beside `value`, which stays one batch at a time")
    ap.add_argument("--graph", action="store_true",
                    help="also time replays of the stage call captured into a HIP graph")
    ap.add_argument("--one-stream", action="store_true",
                    help="asap_stage with two_streams = 0: the K/V compaction follows the merge on the caller's stream")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="accepted for the counter runs documented in profiles/: the 1 GiB device copies that "
                         "calibrate FETCH_SIZE / WRITE_SIZE are part of every run now")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU (the pruning stage of one GPU's share of the batch); "
              "images are independent, so N GPUs would each run this same stage on B/N images. "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2603_14549_amd import binding, harness, synth

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    binding.load()
    cfg = synth.CONFIGS[args.workload]
    if args.attention:
        return bench_attention(args, cfg)
    if args.library_gemm:
        return bench_library_gemm(args, cfg)
    if args.front_end:
        return bench_front_end(args, cfg)
    t0 = time.perf_counter()
    inp = synth.make_inputs(cfg)
    gen_s = time.perf_counter() - t0
    ctx = binding.Context(0)
    paper = args.route == "paper"
    overrides = dict(route=binding.ASAP_ROUTE_PAPER, sim_threshold=0.8) if paper else {}
    lse_extra = None
    if args.lse_extra:
        lse_extra = np.random.default_rng(cfg.seed + 1000).normal(2.0, 2.0, size=(cfg.B, cfg.H, cfg.Tmax)) \
            .astype(np.float32)
    stage = harness.DeviceStage(inp, ctx=ctx, lse_extra=lse_extra, page_size=args.paged_kv or None,
                                last_token=args.last_token, hidden_row_pad=args.hidden_row_pad,
                                overlap=False if args.one_stream else "auto", **overrides)
    torch.cuda.synchronize()

    # The measurement legs that need no wall clock come first: K steps with the library's per-kernel HIP
    # events on, and the copy yardstick.  The GPU has idled while the inputs were generated, and for the
    # first ten milliseconds or so of load after an idle spell this box runs the same steps up to a tenth
    # slower than it sustains (the per-step times of a cold run show it); the timed pass below should
    # measure the sustained state also when it is only a few milliseconds long (--steps 20).
    launches_per_step = 18
    ctx.asap_timing_enable(min(8192, launches_per_step * args.steps))
    for _ in range(args.steps):
        stage.run_async()
    torch.cuda.synchronize()
    timing = ctx.asap_timing_collect()
    ctx.asap_timing_enable(0)

    # what a plain device-to-device copy of 1 GiB reaches on this machine (bytes read + bytes written per
    # second), as a second yardstick beside the nominal peak; with --copy-calibration the copies also
    # serve to scale the traffic counters of a rocprofv3 run
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_bw = 5 * 2.0 * (1 << 30) / (c0.elapsed_time(c1) * 1e-3)
    del src, dst

    # W warm-up steps, then exactly K steps on the wall clock
    for _ in range(args.warmup):
        stage.run_async()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        stage.run_async()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    images_per_s = cfg.B * args.steps / elapsed

    rotated = None
    if args.rotate >= 2:
        sets = [stage] + [harness.DeviceStage(inp, ctx=ctx, lse_extra=lse_extra, page_size=args.paged_kv or None,
                                              last_token=args.last_token, hidden_row_pad=args.hidden_row_pad,
                                              overlap=False if args.one_stream else "auto", **overrides)
                          for _ in range(args.rotate - 1)]
        for i in range(args.warmup):
            sets[i % len(sets)].run_async()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            sets[i % len(sets)].run_async()
        torch.cuda.synchronize()
        rot_ms = 1e3 * (time.perf_counter() - t0) / args.steps
        rotated = {"sets": len(sets), "ms_per_step": rot_ms, "images_per_s": cfg.B / (rot_ms * 1e-3),
                   "note": "same steps cycling over copies of all inputs and outputs at different addresses"}
        del sets

    in_flight = None
    if args.in_flight >= 2:
        copies = [stage] + [harness.DeviceStage(inp, ctx=binding.Context(0), lse_extra=lse_extra,
                                                page_size=args.paged_kv or None, last_token=args.last_token,
                                                hidden_row_pad=args.hidden_row_pad,
                                                overlap=False if args.one_stream else "auto", **overrides)
                            for _ in range(args.in_flight - 1)]
        lanes = [torch.cuda.Stream() for _ in copies]       # default priority

        def submit(rounds):
            for _ in range(rounds):
                for st, lane in zip(copies, lanes):
                    with torch.cuda.stream(lane):
                        st.run_async()
        torch.cuda.synchronize()
        submit(max(args.warmup // len(copies), 2))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rounds = max(args.steps // len(copies), 1)
        submit(rounds)
        torch.cuda.synchronize()
        f_ms = 1e3 * (time.perf_counter() - t0) / (rounds * len(copies))
        in_flight = {"batches": len(copies), "ms_per_batch": f_ms, "images_per_s": cfg.B / (f_ms * 1e-3),
                     "note": "independent batches submitted round-robin to streams and contexts of their own; "
                             "their kernels share the GPU as the hardware schedules them"}
        del copies[1:]

    graph_replay = None
    if args.graph and not stage.call_by_call:
        # the stage records kernels and event record / wait pairs only, so it can be captured; replays are
        # timed like the eager steps (launch-bound shapes, single images above all, are where it may pay)
        cap_stream = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(cap_stream):
            stage.run_async()
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=cap_stream):
                stage.run_async()
        torch.cuda.synchronize()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = 1e3 * (time.perf_counter() - t0) / args.steps
        graph_replay = {"ms_per_step": g_ms, "images_per_s": cfg.B / (g_ms * 1e-3),
                        "note": "the same stage call captured once into a HIP graph and replayed"}
        del graph

    # a further pass: every step bracketed by its own pair of events on the caller's stream (the stage ends
    # with the second stream joined), for the spread; the pairs cost a few microseconds per step, which is
    # why `value` comes from the unbracketed pass above
    n_spread = min(args.steps, 200)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_spread + 1)]
    marks[0].record()
    for i in range(n_spread):
        stage.run_async()
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_step = np.sort(np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(n_spread)]))
    step_spread = {"p10": float(per_step[int(0.1 * (n_spread - 1))]), "median": float(np.median(per_step)),
                   "p90": float(per_step[int(0.9 * (n_spread - 1))]), "steps": n_spread,
                   "note": "per-step event pairs on the caller's stream"}

    # last pass, only when the K/V compaction runs beside k_sim: a few steps on one stream with the
    # per-kernel events on, for the duration of k_sim when nothing shares the memory system with it
    sim_alone = None
    if stage.two_streams and not stage.call_by_call:
        n_alone = min(args.steps, 5)
        ctx.asap_timing_enable(launches_per_step * n_alone)
        for _ in range(n_alone):
            ctx.asap_stage(stage.p, stage.io, binding.ASAP_STREAMS_ONE)
        torch.cuda.synchronize()
        alone = ctx.asap_timing_collect()
        sim_alone = alone.get("k_sim") or alone.get("k_sim_f32")
        ctx.asap_timing_enable(0)

    mean_text = float(np.mean(inp["text_len"]))
    alg = algorithmic_bytes(cfg, mean_text, cfg.L_kv)
    sim_name = "k_sim_f32" if "k_sim_f32" in timing else "k_sim"      # f32 hidden states have a kernel of their own
    alg["per_kernel"]["k_sim_f32"] = alg["per_kernel"]["k_sim"]
    if paper:
        # kept x kept search; the merge reads the k final rows and the rows they absorb (counted from the run)
        eh = esize(cfg.h_dtype)
        n_src = int((stage.buf.assign.flatten()[:cfg.B * cfg.k] >= 0).sum())
        kept_rows = cfg.B * cfg.k * cfg.D * eh
        old_sim, old_merge = alg["per_kernel"]["k_sim"], alg["per_kernel"]["k_merge"]
        alg["per_kernel"]["k_sim"] = alg["per_kernel"]["k_sim_f32"] = kept_rows + 8 * cfg.B * cfg.k
        alg["per_kernel"]["k_merge"] = old_merge - cfg.B * cfg.V * cfg.D * eh + kept_rows + n_src * cfg.D * eh
        alg["per_kernel"]["k_paper_plan"] = 12 * cfg.B * cfg.k + 4 * cfg.B * cfg.V
        alg["stage"] += (alg["per_kernel"]["k_sim"] - old_sim) + (alg["per_kernel"]["k_merge"] - old_merge) \
            + alg["per_kernel"]["k_paper_plan"]
        alg["sim_flops"] = 2.0 * cfg.B * cfg.k * cfg.k * cfg.D
    if "k_score_select_kv" in timing or "k_compact_fixed" in timing:     # prefix and text rows of K/V went earlier
        alg["per_kernel"]["k_compact"] -= alg["per_kernel"]["kv_fixed_rows"]
    if "k_colsum_rows" in timing:
        alg["per_kernel"]["k_attn_stats"] += alg["per_kernel"]["stored_logits"]
    kernels = {}
    for name, (ms, n) in timing.items():
        avg_us = 1e3 * ms / n
        per_launch_bytes = alg["per_kernel"].get(name, 0) * args.steps / n      # several launches per step share it
        kernels[name] = {"avg_us": round(avg_us, 2), "launches_per_step": n / args.steps,
                         "alg_MB": round(per_launch_bytes / 1e6, 2),
                         "GBps": round(per_launch_bytes / (avg_us * 1e-6) / 1e9, 1)}
    step_kernel_us = sum(1e3 * ms / args.steps for ms, _ in timing.values())
    # The dominant kernel is looked for on the main stream: the K/V compaction kernels run beside k_select,
    # k_sim and k_merge on the second stream, so their elapsed time is the time they share the memory
    # system, not a cost of their own.
    on_main = {k: v for k, v in timing.items()
               if not (stage.two_streams and k.startswith("k_compact"))}
    dominant = max(on_main, key=lambda k: on_main[k][0])
    d_ms, d_n = timing[dominant]
    d_avg_s = 1e-3 * d_ms / d_n
    variant = paper or args.paged_kv or args.last_token or args.lse_extra       # counters exist for the default run only
    measured, traffic_source, traffic_note = (None, None, "no counter run for this variant") if variant else \
        measured_traffic(cfg.name, list(timing))
    traffic = None if measured is None else measured.get(dominant)
    if dominant == sim_name and cfg.V > cfg.k:
        flops = alg["sim_flops"] * args.steps / d_n
        peak = MFMA_PEAK[cfg.h_dtype]
        roofline = {"kernel": dominant, "bound": "mfma", "achieved": flops / d_avg_s / 1e12, "peak": peak / 1e12,
                    "unit": "TFLOP/s", "frac": flops / d_avg_s / peak, "traffic": traffic,
                    "traffic_source": traffic_source, "traffic_note": traffic_note}
        if cfg.h_dtype == "f32":
            roofline["arithmetic"] = "six bf16 matrix products per f32 product (three bf16 pieces per operand)"
            roofline["issued_frac_of_bf16_peak"] = 6.0 * flops / d_avg_s / MFMA_PEAK["bf16"]
    else:
        nbytes = alg["per_kernel"].get(dominant, 0) * args.steps / d_n
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": nbytes / d_avg_s / 1e9, "peak": HBM_PEAK / 1e9,
                    "unit": "GB/s", "frac": nbytes / d_avg_s / HBM_PEAK, "traffic": traffic,
                    "traffic_source": traffic_source, "traffic_note": traffic_note}
    sim = timing.get(sim_name)
    sim_roofline = None
    if sim:
        s_avg = 1e-3 * sim[0] / sim[1]
        sim_roofline = {"bound": "mfma", "achieved": alg["sim_flops"] / s_avg / 1e12,
                        "peak": MFMA_PEAK[cfg.h_dtype] / 1e12, "unit": "TFLOP/s",
                        "frac": alg["sim_flops"] / s_avg / MFMA_PEAK[cfg.h_dtype]}
    if sim_roofline is not None and cfg.h_dtype == "f32":
        # the library has no fp32 matrix-core path for this product any more: every f32 operand is cut into
        # three bf16 pieces and six of the nine piece products are formed on the bf16 matrix cores
        sim_roofline["arithmetic"] = ("f32 operands as three bf16 pieces, six bf16 matrix products per f32 product; "
                                      "peak and frac are those of fp32 matrix instructions, the precision delivered")
        sim_roofline["issued_frac_of_bf16_peak"] = 6.0 * alg["sim_flops"] / s_avg / MFMA_PEAK["bf16"]
    if sim_roofline is not None and sim_alone:
        a_avg = 1e-3 * sim_alone[0] / sim_alone[1]
        sim_roofline["alone"] = {"avg_us": round(1e6 * a_avg, 2), "achieved": alg["sim_flops"] / a_avg / 1e12,
                                 "frac": alg["sim_flops"] / a_avg / MFMA_PEAK[cfg.h_dtype],
                                 "note": "same kernel in a single-stream run of the stage"}
    stage_roofline = {"bound": "hbm", "alg_MB": round(alg["stage"] / 1e6, 1),
                      "achieved": alg["stage"] / (ms_per_step * 1e-3) / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                      "frac": alg["stage"] / (ms_per_step * 1e-3) / HBM_PEAK,
                      "sum_kernel_us": round(step_kernel_us, 1)}
    # what the memory system really moved per step (counter runs of the default route): the keys are swept
    # three times where the algorithmic figure counts them once
    if measured:
        moved = sum(measured.get(name, 0.0) * n / args.steps for name, (_, n) in timing.items())
        stage_roofline["traffic_MB"] = round(moved / 1e6, 1)
        stage_roofline["traffic_frac"] = moved / (ms_per_step * 1e-3) / HBM_PEAK
        stage_roofline["traffic_vs_copy"] = moved / (ms_per_step * 1e-3) / copy_bw
        stage_roofline["traffic_source"] = traffic_source
    stage_roofline["measured_copy_GBps"] = round(copy_bw / 1e9, 1)

    out = {
        "metric": "pruning-stage images/sec at %d visual tokens" % cfg.V,
        "value": images_per_s, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "us_per_image": 1e3 * ms_per_step / cfg.B, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.h_dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={cfg.B}, {cfg.P} prefix + {cfg.V} visual + {cfg.Tmax} text tokens, "
                               f"hidden {cfg.D}, {cfg.H}/{cfg.Hkv} heads x {cfg.d}, keep {cfg.k}, "
                               f"qk/hidden/kv dtypes {cfg.qk_dtype}/{cfg.h_dtype}/{cfg.kv_dtype}, "
                               f"{cfg.L_kv} K/V layers, mask=keybias, route={args.route}"
                               f"{' (t=0.8)' if paper else ''}, mu=1"
                               f"{', softmax over the full row (lse_extra)' if args.lse_extra else ''}"
                               f"{', ranked by the last text token' if args.last_token else ''}"
                               f"{f', K/V in pages of {args.paged_kv} tokens' if args.paged_kv else ''}",
                   "input_generation_s": round(gen_s, 1)},
        "roofline": roofline,
        "step_ms": step_spread,
        "stage_roofline": stage_roofline,
        "similarity_gemm": sim_roofline,
        "kernels": kernels,
    }
    if rotated is not None:
        out["rotated_inputs"] = rotated
    if graph_replay is not None:
        out["graph_replay"] = graph_replay
    if in_flight is not None:
        out["in_flight"] = in_flight
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, cfg, route=args.route, lse_extra=lse_extra,
                                           score_rows="last" if args.last_token else "all")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
