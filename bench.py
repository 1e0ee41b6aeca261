#!/usr/bin/env python3
"""Benchmark of the MXFP4+ hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic Llama-3.1-8B MLP-shaped data (gate/up projection,
4096 tokens):  quantize the bf16 activations to MXFP4+  ->  W4A4 GEMM against the MXFP4+ weights (E2M3 image build of
both operands + block-scaled MFMA kernel, fp32 output)  ->  de-convert the activations back to bf16.  Weights are
quantized once before the timed region (they are static); everything else, including the image build of the weights,
is inside it.  Inputs are resident in HBM when timing starts.

Order of a run: `--settle-ms` of untimed steps (the chip's clocks need tens of milliseconds of load to settle; reported
as `settle_ms` / `settle_steps`), then `--warmup` untimed steps, then exactly `--steps` timed steps.

Prints ONE JSON line.  `value` = 2*M*N*K / (time of the whole step): every stage is in the denominator, only the
useful GEMM flops are in the numerator.  Every timed figure besides `value` carries median and min next to the mean.
`--extras` adds the format comparisons, the other configurations and the measured ceilings (minutes of GPU work less:
about 10 s); `--only X` is a profiling aid that runs one stage per step.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP4_TFLOPS = 10100.0     # MI355X dense MXFP4 MFMA, published
PEAK_HBM_GBPS = 8000.0
METRIC = "MXFP4+ GEMM TFLOP/s (Llama-8B linear shapes); quantize GB/s; % roofline"

WORKLOADS = {
    # name: (synth config, weight name)
    "prefill_mlp": ("prefill_mlp", "wgate"),
    "prefill_mlp_down": ("prefill_mlp_down", "wdown"),
    "prefill_attn": ("prefill_attn", "wqo"),
    "prefill_attn_kv": ("prefill_attn", "wkv"),
    "large70b": ("large70b", "w"),
    "decode": ("decode", "w"),
}
ONLY = ["all", "quantize", "quantize_w", "quantize_t", "quantize_image", "prepack", "convert", "gemm", "gemm_e2m1w", "gemm_e4m3", "gemm_pp_exact",
        "gemm_fp6p", "gemm_w4a16", "gemm_decode_large", "gemm_decode_large_four_bit", "gemm_bf16a", "dequantize", "copy"]


def stats(samples):
    import numpy as np
    s = np.asarray(samples, dtype=np.float64)
    return {"mean": float(s.mean()), "median": float(np.median(s)), "min": float(s.min()), "n": int(s.size)}


def product_kernel_name(M, N):
    """The kernel mxp_gemm_prepacked launches for two E2M3 images of this shape (the library's routing, restated for the label)."""
    if M <= 16 and (N + 31) // 32 < 256:
        return "gemm_skinny16_kernel"
    if M <= 64 or (M <= 128 and (N + 255) // 256 < 64):
        return "gemm_skinny_kernel"
    if ((M + 127) // 128) * ((N + 127) // 128) <= 256:
        return "gemm_block_kernel"
    return "gemm_kernel_dma"


def traffic_from_profiles(workload, out_dtype):
    """HBM-side bytes per GEMM launch, from the committed rocprofv3 --pmc summary (None if there is no matching line)."""
    path = os.path.join(ROOT, "profiles", "gemm_kernel_dma_%s.md" % workload)
    try:
        for line in open(path):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH") and ("out=" + out_dtype) in line:
                return float(line.split("=")[-1].strip())
    except OSError:
        pass
    return None


def cpu_baseline(a_bits, w_bits, budget_s=25.0):
    """The CPU oracle (as it stands) on a bounded sample of the same workload: quantize + fp64 GEMM + de-conversion.
    The sample is the whole workload when the oracle finishes it inside the budget; otherwise all weight rows against a
    subset of activation rows that holds both rows next to every 256-row tile edge, filled up from the front."""
    import numpy as np
    import oracle

    M, K = a_bits.shape
    N = w_bits.shape[0]
    threads = oracle.num_threads()
    m0, n0 = min(64, M), min(2048, N)
    t = time.perf_counter()
    qa = oracle.quantize(a_bits[:m0], oracle.MXFP4P)
    qw = oracle.quantize(w_bits[:n0], oracle.MXFP4P)
    oracle.gemm(qa, oracle.MXFP4P, qw, oracle.MXFP4P)
    rate = m0 * n0 * K / max(time.perf_counter() - t, 1e-4)
    m = int(max(8, min(M, budget_s * rate / (N * K))))
    if m >= M:
        rows = np.arange(M)
        what = "the whole workload"
    else:
        edges = [r for e in range(0, M + 1, 256) for r in (e - 1, e) if 0 <= r < M]
        rows = np.unique(np.concatenate([np.asarray(edges[: max(m // 2, 2)], dtype=np.int64), np.arange(M)]))
        keep = np.isin(rows, edges[: max(m // 2, 2)])
        rows = np.concatenate([rows[keep], rows[~keep][: max(m - int(keep.sum()), 0)]])
        what = "%d of %d activation rows (both rows at every 256-row tile edge first, then rows from the front) x all %d weight rows" % (rows.size, M, N)
    t = time.perf_counter()
    qa = oracle.quantize(np.ascontiguousarray(a_bits[rows]), oracle.MXFP4P)
    qw = oracle.quantize(w_bits, oracle.MXFP4P)
    oracle.gemm(qa, oracle.MXFP4P, qw, oracle.MXFP4P)
    oracle.dequantize(qa, oracle.MXFP4P)
    dt = time.perf_counter() - t
    return {"value": 2.0 * rows.size * N * K / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": "oracle quantize + fp64 gemm + dequantize on %s, K = %d: %.1f s" % (what, K, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-ms", type=float, default=250.0,
                    help="untimed steps run for this long before the warm-up: from idle the clocks need ~40 ms of load to "
                         "settle (a step takes ~20 %% longer until then)")
    ap.add_argument("--workload", default="prefill_mlp", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--extras", action="store_true", help="also time the other formats, configurations and the measured ceilings")
    ap.add_argument("--out-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--only", default="all", choices=ONLY,
                    help="profiling aid: run just one stage per step (the JSON line is then not a benchmark result)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives exist in the method's hot path); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_14557_amd import mxp, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    mxp.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    cfg, wname = WORKLOADS[args.workload]
    a_bits, ws = synth.make(cfg)
    w_bits = ws[wname]
    M, K = a_bits.shape
    N = w_bits.shape[0]

    def to_dev(x):
        return torch.from_numpy(x.view(np.int16)).view(torch.bfloat16).to(dev)

    A, W = to_dev(a_bits), to_dev(w_bits)
    out_dt = torch.float32 if args.out_dtype == "f32" else torch.bfloat16
    # static weights: quantized once, outside the timed region
    qw = mxp.quantize(W, mxp.MXFP4P)
    # every buffer the step touches is allocated once
    qa = (torch.empty((M, K // 2), dtype=torch.uint8, device=dev), torch.empty((M, K // 32), dtype=torch.uint8, device=dev),
          torch.empty((M, K // 32), dtype=torch.uint8, device=dev))
    img_a = torch.empty(mxp.image_bytes(M, K), dtype=torch.uint8, device=dev)
    # few rows (decode): the MXFP4+ weights stay 4-bit (E2M1 image with residual bytes); otherwise the E2M3 image
    few_rows = M <= 64
    img_w = torch.empty(mxp.image_bytes_e2m1r(N, K) if few_rows else mxp.image_bytes(N, K), dtype=torch.uint8, device=dev)
    w_kind = mxp.IMAGE_E2M1R if few_rows else mxp.IMAGE_E2M3
    D = torch.empty((M, N), dtype=out_dt, device=dev)
    back = torch.empty((M, K), dtype=torch.bfloat16, device=dev)

    def convert():
        # activations: one pass writes the canonical MXFP4+ arrays and the GEMM image; weights: canonical -> image
        if few_rows:
            mxp.quantize_image(A, mxp.MXFP4P, out=img_a, q_out=qa)
            mxp.prepack_e2m1r(qw, out=img_w)
        else:
            mxp.convert_operands(A, mxp.MXFP4P, qa, img_a, qw, mxp.MXFP4P, img_w)

    def product():
        mxp.gemm_prepacked(M, N, K, img_a, img_w, out=D, b_kind=w_kind)

    def step(ev=None, gemm_ev=None):
        if ev is not None:
            ev[0].record()
        convert()
        if ev is not None:
            ev[1].record()
        if gemm_ev is not None:
            gemm_ev[0].record()
        product()
        if gemm_ev is not None:
            gemm_ev[1].record()
        if ev is not None:
            ev[2].record()
        mxp.dequantize(qa, mxp.MXFP4P, out=back)
        if ev is not None:
            ev[3].record()

    if args.only != "all":
        from paper_2510_14557_amd import bench_extras
        fn = bench_extras.only_stage(args.only, locals())
        for _ in range(max(args.warmup, 3)):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "workload": args.workload, "ms_per_call": (time.perf_counter() - t0) * 1e3 / args.steps,
                          "note": "profiling aid, not a benchmark line"}))
        return

    # settle: untimed steps until the clocks have had `settle_ms` of load
    t0 = time.perf_counter()
    settle_steps = 0
    while (time.perf_counter() - t0) * 1e3 < args.settle_ms:
        for _ in range(25):
            step()
        torch.cuda.synchronize()
        settle_steps += 25
    settle_ms = (time.perf_counter() - t0) * 1e3
    for _ in range(args.warmup):
        step()
    # Timed region: K steps; the only instrumentation inside it is a HIP event pair around the GEMM launch on every 5th
    # step, recorded on the stream the kernels are launched on (torch's current stream).  An event record stops the
    # next dispatch from overlapping the previous kernel's tail (a few us per record), hence not on every step.
    gemm_events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] if s % 5 == 0 else None for s in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(gemm_ev=gemm_events[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gemm_st = stats([e[0].elapsed_time(e[1]) for e in gemm_events if e is not None])
    gemm_ms = gemm_st["mean"]

    # Per-stage breakdown from a second, fully instrumented pass (not part of `value`: the extra events add ~10 us/step).
    n_prof = max(min(args.steps, 100), 20)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(n_prof)]
    for s in range(n_prof):
        step(ev=events[s])
    torch.cuda.synchronize()
    stage_names = ("convert_a_and_w", "gemm", "dequantize")
    stage_st = {n: stats([events[s][i].elapsed_time(events[s][i + 1]) for s in range(n_prof)]) for i, n in enumerate(stage_names)}

    def groups(fn, inner, n_groups, warm=1):
        """`n_groups` samples of the per-call time of `fn`, each from `inner` calls back to back between one event pair."""
        for _ in range(warm * inner):
            fn()
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_groups)]
        for g in range(n_groups):
            evs[g][0].record()
            for _ in range(inner):
                fn()
            evs[g][1].record()
        torch.cuda.synchronize()
        return stats([e[0].elapsed_time(e[1]) / inner for e in evs])

    # the product kernel alone, launches back to back (no dispatch gaps): the figure a kernel trace shows
    gemm_b2b = groups(product, 20, 10, warm=5)

    # Standalone mxp_quantize (canonical outputs only), launches back to back over rotating source copies whose total
    # exceeds the 256 MB Infinity Cache: the weight matrix (3 copies) and the activation tensor (12 copies).
    def timed_quantize(src_bits, copies, inner, n_groups):
        srcs = [to_dev(src_bits) for _ in range(copies)]
        q = mxp.quantize(srcs[0], mxp.MXFP4P)
        it = [0]

        def fn():
            mxp.quantize_into(srcs[it[0] % copies], mxp.MXFP4P, *q)
            it[0] += 1
        return groups(fn, inner, n_groups)

    del W
    q_w = timed_quantize(w_bits, 3, 6, 8)
    q_a = timed_quantize(a_bits, 12, 12, 8)

    flops = 2.0 * M * N * K
    q_bytes = lambda r: r * K * 2.5625                       # bf16 in + nibbles + scale + index
    gbps = lambda nbytes, st: {k: (nbytes / (v * 1e-3) / 1e9 if k != "n" else v) for k, v in
                               (("mean", st["mean"]), ("median", st["median"]), ("best", st["min"]), ("n", st["n"]))}
    conv_bytes = M * K * (2.5625 + 0.78125) + N * K * (0.5625 + (0.5625 if few_rows else 0.78125))
    line = {
        "metric": METRIC,
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_ms": settle_ms,
        "settle_steps": settle_steps,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "mxfp4+ (E2M1 elements, E2M3 block max, E8M0 scales), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": args.workload, "M": M, "N": N, "K": K, "A": "bf16 N(0,1) + outlier channels x50",
                   "W": {"prefill_mlp": "bf16 N(0,0.02) + 0.1% Student-t(3)", "prefill_mlp_down": "bf16 N(0,0.02) + 0.1% Student-t(3)",
                         "large70b": "bf16 N(0,0.015)"}.get(args.workload, "bf16 N(0,0.02)"),
                   "out_dtype": args.out_dtype,
                   "step": "convert(A: bf16 -> canonical + image; W: canonical -> image; one launch) -> scaled-MFMA GEMM -> dequantize(A)"},
        "roofline": {"bound": "mfma", "achieved": flops / (gemm_ms * 1e-3) / 1e12, "peak": PEAK_FP4_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / (gemm_ms * 1e-3) / 1e12 / PEAK_FP4_TFLOPS,
                     "traffic": traffic_from_profiles(args.workload, args.out_dtype),
                     "kernel": product_kernel_name(M, N), "kernel_ms": gemm_ms, "kernel_ms_median": gemm_st["median"],
                     "kernel_ms_min": gemm_st["min"], "kernel_samples": gemm_st["n"],
                     "kernel_ms_back_to_back": gemm_b2b,
                     "frac_back_to_back": flops / (gemm_b2b["mean"] * 1e-3) / 1e12 / PEAK_FP4_TFLOPS,
                     "note": "kernel_ms = mean over HIP event pairs around the launch on every 5th timed step (includes the "
                             "dispatch gap an event record opens); kernel_ms_back_to_back = the same launch 20x between "
                             "one event pair, 10 groups, after the timed region; traffic = FETCH_SIZE*2.0 + WRITE_SIZE "
                             "bytes per launch from profiles/"},
        "stages_ms": stage_st,
        "convert_GBps": gbps(conv_bytes, stage_st["convert_a_and_w"]),
        "dequantize_GBps": gbps(M * K * (0.5625 + 2.0), stage_st["dequantize"]),
        # mxp_quantize on the workload's two tensors (bytes = bf16 in + codes + scale + index bytes out)
        "quantize_GBps": gbps(q_bytes(N), q_w)["mean"],
        "quantize_frac_hbm": gbps(q_bytes(N), q_w)["mean"] / PEAK_HBM_GBPS,
        "quantize": {"W bf16 [%d x %d], 3 copies in rotation" % (N, K): dict(gbps(q_bytes(N), q_w), ms=q_w),
                     "A bf16 [%d x %d], 12 copies in rotation" % (M, K): dict(gbps(q_bytes(M), q_a), ms=q_a),
                     "frac_hbm_W": gbps(q_bytes(N), q_w)["mean"] / PEAK_HBM_GBPS,
                     "frac_hbm_A": gbps(q_bytes(M), q_a)["mean"] / PEAK_HBM_GBPS},
    }
    if few_rows:                                          # few rows: bound by reading the weight image once
        wbytes = float(img_w.numel())
        line["roofline"].update({"bound": "hbm", "achieved": wbytes / (gemm_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                 "frac": wbytes / (gemm_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                                 "frac_back_to_back": wbytes / (gemm_b2b["mean"] * 1e-3) / 1e9 / PEAK_HBM_GBPS})
    if args.extras:
        from paper_2510_14557_amd import bench_extras
        line.update(bench_extras.run(locals()))
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(a_bits, w_bits)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
