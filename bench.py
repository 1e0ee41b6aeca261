#!/usr/bin/env python3
"""Benchmark of the MXFP4+ hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic Llama-3.1-8B MLP-shaped data (gate/up projection,
4096 tokens):  quantize the bf16 activations to MXFP4+  ->  W4A4 GEMM against the MXFP4+ weights (E2M3 image build of
both operands + block-scaled MFMA kernel, fp32 output)  ->  de-convert the activations back to bf16.  Weights are
quantized once before the timed region (they are static); everything else, including the image build of the weights,
is inside it.  Inputs are resident in HBM when timing starts.

Prints ONE JSON line.  `value` = 2*M*N*K / (time of the whole step): every stage is in the denominator, only the
useful GEMM flops are in the numerator.
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

WORKLOADS = {
    # name: (synth config, weight name)
    "prefill_mlp": ("prefill_mlp", "wgate"),
    "prefill_mlp_down": ("prefill_mlp_down", "wdown"),
    "prefill_attn": ("prefill_attn", "wqo"),
    "large70b": ("large70b", "w"),
    "decode": ("decode", "w"),
}


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


def cpu_baseline(a_bits, w_bits, budget_s=40.0):
    """The CPU oracle on a bounded sample of the same workload: quantize + fp64 GEMM of a row subset."""
    import numpy as np
    import oracle

    K = a_bits.shape[1]
    threads = oracle.num_threads()
    # calibrate on a small piece, then size the sample for about budget_s of CPU work
    m0, n0 = min(64, a_bits.shape[0]), min(2048, w_bits.shape[0])
    t = time.perf_counter()
    qa = oracle.quantize(a_bits[:m0], oracle.MXFP4P)
    qw = oracle.quantize(w_bits[:n0], oracle.MXFP4P)
    oracle.gemm(qa, oracle.MXFP4P, qw, oracle.MXFP4P)
    dt = max(time.perf_counter() - t, 1e-4)
    rate = m0 * n0 * K / dt
    macs = budget_s * rate
    n = int(min(w_bits.shape[0], max(2048, macs / (a_bits.shape[0] * K))))
    m = int(max(8, min(a_bits.shape[0], macs / (n * K))))
    t = time.perf_counter()
    qa = oracle.quantize(a_bits[:m], oracle.MXFP4P)
    qw = oracle.quantize(w_bits[:n], oracle.MXFP4P)
    oracle.gemm(qa, oracle.MXFP4P, qw, oracle.MXFP4P)
    oracle.dequantize(qa, oracle.MXFP4P)
    dt = time.perf_counter() - t
    return {"value": 2.0 * m * n * K / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": "oracle quantize+gemm+dequantize on A[%d x %d] x W[%d x %d]^T (first rows of the same tensors), %.1f s"
                      % (m, K, n, K, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The chip needs about 40 ms of sustained load before its clocks settle (step time falls from ~220 us over the first
    # 20 steps to a steady ~180 us after ~200): the defaults time steady state.  500 steps are about 0.1 s of GPU work.
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--workload", default="prefill_mlp", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed steps and the per-stage pass (no format comparisons, decode shapes or probes): "
                         "the run whose kernel trace holds nothing but the step's own kernels")
    ap.add_argument("--out-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--only", default="all", choices=["all", "quantize", "quantize_t", "quantize_image", "prepack", "gemm", "gemm_e4m3", "gemm_fp6p", "gemm_w4a16", "gemm_decode_large", "gemm_decode_large_four_bit", "dequantize", "copy"],
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
    WT = W.t().contiguous() if args.only == "quantize_t" else None     # the weights as stored [K][N]
    del W
    # every buffer the step touches is allocated once
    qa = (torch.empty((M, K // 2), dtype=torch.uint8, device=dev), torch.empty((M, K // 32), dtype=torch.uint8, device=dev),
          torch.empty((M, K // 32), dtype=torch.uint8, device=dev))
    img_a = torch.empty(mxp.image_bytes(M, K), dtype=torch.uint8, device=dev)
    # few rows (decode): the MXFP4+ weights stay 4-bit (E2M1 image with residual bytes); otherwise the E2M3 image
    few_rows = M <= 64 and args.only == "all"
    img_w = torch.empty(mxp.image_bytes_e2m1r(N, K) if few_rows else mxp.image_bytes(N, K), dtype=torch.uint8, device=dev)
    w_kind = mxp.IMAGE_E2M1R if few_rows else mxp.IMAGE_E2M3
    D = torch.empty((M, N), dtype=out_dt, device=dev)
    back = torch.empty((M, K), dtype=torch.bfloat16, device=dev)

    stages = ("quantize_a", "prepack_w", "gemm", "dequantize")
    if args.only == "copy":
        copy_src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        copy_dst = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)

    if args.only == "gemm_e4m3":       # the MXFP4++ product (Sec. 4.3) on the same tensors, E4M3 images
        img_a8 = mxp.prepack_e4m3(mxp.quantize(A, mxp.MXFP4PP), mxp.MXFP4PP)
        W8 = to_dev(w_bits)
        img_w8 = mxp.prepack_e4m3(mxp.quantize(W8, mxp.MXFP4PP), mxp.MXFP4PP)
        del W8
    if args.only == "gemm_fp6p":       # MXFP6+ activations x MXFP6 weights (Sec. 4.2 formats): two K segments, incl. both prepacks
        W6 = to_dev(w_bits)
        qa6, qw6 = mxp.quantize(A, mxp.MXFP6P), mxp.quantize(W6, mxp.MXFP6)
        del W6
        ws6 = torch.empty(mxp.gemm_workspace_bytes(M, N, K, mxp.MXFP6P, mxp.MXFP6), dtype=torch.uint8, device=dev)
    if args.only == "gemm_w4a16":      # conversion-based product at the benchmark shape (tiled kernel)
        W16 = to_dev(w_bits)
        qw16 = mxp.quantize(W16, mxp.MXFP4P)
        del W16
    if args.only in ("gemm_decode_large", "gemm_decode_large_four_bit"):   # 8 rows against a 70B-sized layer, random codes
        Nl, Kl = 28672, 8192
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        ql = (torch.randint(0, 256, (Nl, Kl // 2), dtype=torch.uint8, device=dev, generator=gen),
              torch.randint(120, 134, (Nl, Kl // 32), dtype=torch.uint8, device=dev, generator=gen),
              torch.randint(0, 32, (Nl, Kl // 32), dtype=torch.uint8, device=dev, generator=gen))
        img_wl = mxp.prepack(ql, mxp.MXFP4P) if args.only == "gemm_decode_large" else mxp.prepack_e2m1r(ql)   # E2M3 image / 4-bit image
        img_al = mxp.prepack(tuple(t[:8].contiguous() for t in ql), mxp.MXFP4P)
        Dl = torch.empty((8, Nl), dtype=torch.float32, device=dev)
        del ql

    def step_only():
        if args.only == "gemm_e4m3":
            mxp.gemm_prepacked(M, N, K, img_a8, img_w8, out=D, a_kind=mxp.IMAGE_E4M3, b_kind=mxp.IMAGE_E4M3)
        elif args.only == "gemm_w4a16":
            mxp.gemm_w4a16(A, qw16, mxp.MXFP4P, out=D)
        elif args.only == "gemm_fp6p":
            mxp.gemm(qa6, mxp.MXFP6P, qw6, mxp.MXFP6, out=D, workspace=ws6)
        elif args.only == "gemm_decode_large":
            mxp.gemm_prepacked(8, Nl, Kl, img_al, img_wl, out=Dl)
        elif args.only == "gemm_decode_large_four_bit":
            mxp.gemm_prepacked(8, Nl, Kl, img_al, img_wl, out=Dl, b_kind=mxp.IMAGE_E2M1R)
        elif args.only == "quantize":
            mxp.quantize_into(A, mxp.MXFP4P, *qa)
        elif args.only == "quantize_t":
            mxp.quantize_t(WT, mxp.MXFP4P)
        elif args.only == "quantize_image":
            mxp.quantize_image(A, mxp.MXFP4P, out=img_a, q_out=qa)
        elif args.only == "prepack":
            mxp.prepack(qw, mxp.MXFP4P, out=img_w)
        elif args.only == "gemm":
            mxp.gemm_prepacked(M, N, K, img_a, img_w, out=D)
        elif args.only == "copy":
            # plain device copy of a known size (256 MiB): the reference that scales the FETCH_SIZE / WRITE_SIZE counters
            copy_dst.copy_(copy_src)
        else:
            mxp.dequantize(qa, mxp.MXFP4P, out=back)

    def step(ev=None, gemm_ev=None):
        # activations: one pass writes the canonical MXFP4+ arrays and the GEMM image; weights: canonical -> image
        if ev is not None:
            ev[0].record()
        mxp.quantize_image(A, mxp.MXFP4P, out=img_a, q_out=qa)
        if ev is not None:
            ev[1].record()
        if few_rows:
            mxp.prepack_e2m1r(qw, out=img_w)
        else:
            mxp.prepack(qw, mxp.MXFP4P, out=img_w)
        if ev is not None:
            ev[2].record()
        if gemm_ev is not None:
            gemm_ev[0].record()
        mxp.gemm_prepacked(M, N, K, img_a, img_w, out=D, b_kind=w_kind)
        if gemm_ev is not None:
            gemm_ev[1].record()
        if ev is not None:
            ev[3].record()
        mxp.dequantize(qa, mxp.MXFP4P, out=back)
        if ev is not None:
            ev[4].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.only != "all":
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_only()
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "ms_per_call": (time.perf_counter() - t0) * 1e3 / args.steps,
                          "note": "profiling aid, not a benchmark line"}))
        return
    # Timed region: K steps; the only instrumentation inside it is a HIP event pair around the GEMM kernel on every 5th
    # step, recorded on the stream the kernels are launched on (torch's current stream).  An event record stops the
    # next dispatch from overlapping the previous kernel's tail (about 6 us per record), hence not on every step.
    gemm_events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] if s % 5 == 0 else None for s in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(gemm_ev=gemm_events[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gemm_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in gemm_events if e is not None]))
    # Per-stage breakdown from a second, fully instrumented pass (not part of `value`: the extra events add ~15 us/step).
    n_prof = min(args.steps, 20)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(n_prof)]
    for s in range(n_prof):
        step(ev=events[s])
    torch.cuda.synchronize()
    stage_ms = {n: float(np.mean([events[s][i].elapsed_time(events[s][i + 1]) for s in range(n_prof)]))
                for i, n in enumerate(stages)}
    if args.no_extras:
        flops = 2.0 * M * N * K
        gemm_tflops_core = flops / (gemm_ms * 1e-3) / 1e12
        line = {
            "metric": "MXFP4+ GEMM TFLOP/s (Llama-8B linear shapes); quantize GB/s; % roofline",
            "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "mxfp4+ (E2M1 elements, E2M3 block max, E8M0 scales), fp32 accumulate", "data": "synthetic",
            "config": {"workload": args.workload, "M": M, "N": N, "K": K, "out_dtype": args.out_dtype,
                       "step": "quantize(A) -> canonical + image in one pass, image(W) -> scaled-MFMA GEMM -> dequantize(A)"},
            "roofline": {"bound": "mfma", "achieved": gemm_tflops_core, "peak": PEAK_FP4_TFLOPS, "unit": "TFLOP/s",
                         "frac": gemm_tflops_core / PEAK_FP4_TFLOPS, "traffic": traffic_from_profiles(args.workload, args.out_dtype),
                         "kernel": "gemm_kernel_dma" if M > 64 else "gemm_skinny_res_kernel", "kernel_ms": gemm_ms},
            "stages_ms": stage_ms,
        }
        if M <= 64:                                          # few rows: bound by reading the weight image once
            wbytes = float(img_w.numel())
            line["roofline"].update({"bound": "hbm", "achieved": wbytes / (gemm_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS,
                                     "unit": "GB/s", "frac": wbytes / (gemm_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS})
        if not args.no_cpu_baseline:
            line["cpu_baseline"] = cpu_baseline(a_bits, w_bits)
        print(json.dumps(line))
        return
    # The paper's main deployment (Sec. 7.1): MXFP4+ activations x plain MXFP4 weights.  The weights stay in 4-bit codes on
    # the B side (E2M1 image).  All products timed the same way: 250 warm-up launches, then 100 back to back, one event pair.
    # The third product is plain MXFP4 x MXFP4 (both images 4-bit): the baseline the paper normalises MX+ to.
    def timed_gemm(a_image, a_kind, b_image, b_kind, n=100, out=None, k=None):
        out = D if out is None else out
        k = K if k is None else k
        for _ in range(250):                                  # the clocks need tens of ms to settle on a new load
            mxp.gemm_prepacked(M, N, k, a_image, b_image, out=out, a_kind=a_kind, b_kind=b_kind)
        torch.cuda.synchronize()
        ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev2[0].record()
        for _ in range(n):
            mxp.gemm_prepacked(M, N, k, a_image, b_image, out=out, a_kind=a_kind, b_kind=b_kind)
        ev2[1].record()
        torch.cuda.synchronize()
        return ev2[0].elapsed_time(ev2[1]) / n

    gemm_pp_ms = timed_gemm(img_a, mxp.IMAGE_E2M3, img_w, w_kind)
    # the same product with the other output type (bf16 = the fp32 result rounded once, half the output bytes)
    other_dt = torch.bfloat16 if out_dt == torch.float32 else torch.float32
    D_other = torch.empty((M, N), dtype=other_dt, device=dev)
    gemm_pp_other_ms = timed_gemm(img_a, mxp.IMAGE_E2M3, img_w, w_kind, out=D_other)
    del D_other
    W4 = to_dev(w_bits)
    img_w4 = mxp.prepack_e2m1(mxp.quantize(W4, mxp.MXFP4))
    del W4
    gemm_w4_ms = timed_gemm(img_a, mxp.IMAGE_E2M3, img_w4, mxp.IMAGE_E2M1)
    img_a4 = mxp.prepack_e2m1(mxp.quantize(A, mxp.MXFP4))
    gemm_a4w4_ms = timed_gemm(img_a4, mxp.IMAGE_E2M1, img_w4, mxp.IMAGE_E2M1)
    del img_w4, img_a4
    # MXFP4++ x MXFP4++ (Sec. 4.3): E4M3 images, FP8 MFMAs at half rate
    W8 = to_dev(w_bits)
    img_w8 = mxp.prepack_e4m3(mxp.quantize(W8, mxp.MXFP4PP), mxp.MXFP4PP)
    del W8
    img_a8 = mxp.prepack_e4m3(mxp.quantize(A, mxp.MXFP4PP), mxp.MXFP4PP)
    gemm_pp8_ms = timed_gemm(img_a8, mxp.IMAGE_E4M3, img_w8, mxp.IMAGE_E4M3)
    # its activation side in one pass: bf16 -> E4M3 image (no canonical bytes), 100 calls back to back
    for _ in range(20):
        mxp.quantize_image(A, mxp.MXFP4PP, out=img_a8)
    torch.cuda.synchronize()
    ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev2[0].record()
    for _ in range(100):
        mxp.quantize_image(A, mxp.MXFP4PP, out=img_a8)
    ev2[1].record()
    torch.cuda.synchronize()
    qimg_pp8_ms = ev2[0].elapsed_time(ev2[1]) / 100
    qimg_pp8_bytes = A.numel() * A.element_size() + img_a8.numel()
    del img_w8, img_a8
    # six-bit operands (Sec. 4.2): MXFP6 x MXFP6 is one E2M3 product; the MXFP6+ BM adds K segments (2 one-sided, 4 two-sided)
    Kp = (K + 127) // 128 * 128
    W6 = to_dev(w_bits)
    qa6 = mxp.quantize(A, mxp.MXFP6P)
    fp6_ms = {}
    for name, fmt_w, n_seg, ma, mb in (("mxfp6p_x_mxfp6", mxp.MXFP6, 2, 0b10, 0), ("mxfp6p_x_mxfp6p", mxp.MXFP6P, 4, 0b1010, 0b1100)):
        ia6 = mxp.prepack_fp6(qa6, mxp.MXFP6P, n_seg, ma)
        iw6 = mxp.prepack_fp6(mxp.quantize(W6, fmt_w), fmt_w, n_seg, mb)
        fp6_ms[name] = timed_gemm(ia6, mxp.IMAGE_E2M3, iw6, mxp.IMAGE_E2M3, k=n_seg * Kp)
        del ia6, iw6
    del qa6, W6
    # the conversion-based product at this shape (Sec. 5; weight-only quantization): bf16 A as it is x canonical MXFP4+ W
    W16 = to_dev(w_bits)
    qw16 = mxp.quantize(W16, mxp.MXFP4P)
    del W16
    for _ in range(20):
        mxp.gemm_w4a16(A, qw16, mxp.MXFP4P, out=D)
    torch.cuda.synchronize()
    ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev2[0].record()
    for _ in range(20):
        mxp.gemm_w4a16(A, qw16, mxp.MXFP4P, out=D)
    ev2[1].record()
    torch.cuda.synchronize()
    w4a16_ms = ev2[0].elapsed_time(ev2[1]) / 20
    del qw16
    # MXFP8+ x MXFP8+ (Sec. 4.2 formats): no block-scaled MFMA element holds an E4M7 BM; de-converted in the kernel, bf16 MFMA
    W8p = to_dev(w_bits)
    qa8p, qw8p = mxp.quantize(A, mxp.MXFP8P), mxp.quantize(W8p, mxp.MXFP8P)
    del W8p
    ws8p = torch.empty(16, dtype=torch.uint8, device=dev)
    for _ in range(5):
        mxp.gemm(qa8p, mxp.MXFP8P, qw8p, mxp.MXFP8P, out=D, workspace=ws8p)
    torch.cuda.synchronize()
    ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev2[0].record()
    for _ in range(10):
        mxp.gemm(qa8p, mxp.MXFP8P, qw8p, mxp.MXFP8P, out=D, workspace=ws8p)
    ev2[1].record()
    torch.cuda.synchronize()
    fp8p_ms = ev2[0].elapsed_time(ev2[1]) / 10
    del qa8p, qw8p

    # Decode configuration (8 x 4096 activations, 4096 x 4096 weights): activations quantized on the fly, prepacked
    # weights, 20 calls back to back.  Bound by reading the weight image once; at this size launch latency dominates.
    def graph_us(call, n=20, reps=3):
        """Per-call time of `call` with n calls captured in one HIP graph: the device-side figure, without the host time
        of a Python call per launch (which is what 'us_per_call' of these few-microsecond products measures)."""
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for _ in range(3):
                    call()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for _ in range(n):
                    call()
            torch.cuda.synchronize()
            best = None
            for _ in range(reps):
                evg = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                evg[0].record()
                for _ in range(10):
                    graph.replay()
                evg[1].record()
                torch.cuda.synchronize()
                t = evg[0].elapsed_time(evg[1]) / (10 * n) * 1e3
                best = t if best is None else min(best, t)
            return best
        except Exception as e:                                # capture is an extra: never fail the benchmark over it
            return "graph capture failed: %s" % type(e).__name__

    def timed_decode():
        a_d, ws_d = synth.make("decode")
        Ad, Wd = to_dev(a_d), to_dev(next(iter(ws_d.values())))
        Md, Kd = Ad.shape
        Nd = Wd.shape[0]
        out = {}
        for name, fmt_w, kind in (("mxfp4p_weights", mxp.MXFP4P, mxp.IMAGE_E2M3), ("mxfp4_weights", mxp.MXFP4, mxp.IMAGE_E2M1),
                                  ("mxfp4p_weights_four_bit_image", mxp.MXFP4P, mxp.IMAGE_E2M1R)):
            qwd = mxp.quantize(Wd, fmt_w)
            img = (mxp.prepack_e2m1(qwd) if kind == mxp.IMAGE_E2M1 else mxp.prepack_e2m1r(qwd) if kind == mxp.IMAGE_E2M1R
                   else mxp.prepack(qwd, fmt_w))
            Dd = torch.empty((Md, Nd), dtype=torch.float32, device=dev)
            wsd = torch.empty(max(mxp.gemm_bf16a_workspace_bytes(Md, Kd), 16), dtype=torch.uint8, device=dev)
            for _ in range(3):
                mxp.gemm_bf16a(Ad, mxp.MXFP4P, img, Nd, out=Dd, workspace=wsd, b_kind=kind)
            torch.cuda.synchronize()
            ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev2[0].record()
            for _ in range(20):
                mxp.gemm_bf16a(Ad, mxp.MXFP4P, img, Nd, out=Dd, workspace=wsd, b_kind=kind)
            ev2[1].record()
            torch.cuda.synchronize()
            us = ev2[0].elapsed_time(ev2[1]) / 20 * 1e3
            ug = graph_us(lambda: mxp.gemm_bf16a(Ad, mxp.MXFP4P, img, Nd, out=Dd, workspace=wsd, b_kind=kind))
            out[name] = {"us_per_call": us, "us_per_call_in_hip_graph": ug, "weight_image_GBps": img.numel() / us / 1e3,
                         "frac_hbm": img.numel() / us / 1e3 / PEAK_HBM_GBPS}
            if isinstance(ug, float):
                out[name].update({"weight_image_GBps": img.numel() / ug / 1e3, "frac_hbm": img.numel() / ug / 1e3 / PEAK_HBM_GBPS})
        # the conversion-based route: bf16 activations as they are, canonical 4-bit weights de-converted in the kernel
        qwd = mxp.quantize(Wd, mxp.MXFP4P)
        Dd = torch.empty((Md, Nd), dtype=torch.float32, device=dev)
        for _ in range(3):
            mxp.gemm_w4a16(Ad, qwd, mxp.MXFP4P, out=Dd)
        torch.cuda.synchronize()
        ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev2[0].record()
        for _ in range(20):
            mxp.gemm_w4a16(Ad, qwd, mxp.MXFP4P, out=Dd)
        ev2[1].record()
        torch.cuda.synchronize()
        us = ev2[0].elapsed_time(ev2[1]) / 20 * 1e3
        wbytes = Nd * Kd * 0.5625
        ug = graph_us(lambda: mxp.gemm_w4a16(Ad, qwd, mxp.MXFP4P, out=Dd))
        out["w4a16_mxfp4p_weights"] = {"us_per_call": us, "us_per_call_in_hip_graph": ug, "weight_GBps": wbytes / us / 1e3,
                                       "frac_hbm": wbytes / us / 1e3 / PEAK_HBM_GBPS}
        if isinstance(ug, float):
            out["w4a16_mxfp4p_weights"].update({"weight_GBps": wbytes / ug / 1e3, "frac_hbm": wbytes / ug / 1e3 / PEAK_HBM_GBPS})
        out["note"] = ("us_per_call: 20 Python calls back to back (host-bound at this size); us_per_call_in_hip_graph: the same "
                       "20 calls captured in one HIP graph and replayed -- the device-side time; GB/s and frac_hbm use the latter")
        out["shape"] = "A bf16 [%d x %d] quantized on the fly (one kernel) + split-K GEMM with W [%d x %d]" % (Md, Kd, Nd, Kd)
        del Wd, qwd
        # the same 8 rows against a 70B-sized layer (28672 x 8192, random codes): the product kernel alone, where the
        # weight image is large enough for the HBM rate to show
        Nl, Kl = 28672, 8192
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        ql = (torch.randint(0, 256, (Nl, Kl // 2), dtype=torch.uint8, device=dev, generator=gen),
              torch.randint(120, 134, (Nl, Kl // 32), dtype=torch.uint8, device=dev, generator=gen),
              torch.randint(0, 32, (Nl, Kl // 32), dtype=torch.uint8, device=dev, generator=gen))
        qal = tuple(t[:Md].contiguous() for t in ql)
        img_al = mxp.prepack(qal, mxp.MXFP4P)
        Dl = torch.empty((Md, Nl), dtype=torch.float32, device=dev)
        for name, kind in (("mxfp4p_weights", mxp.IMAGE_E2M3), ("mxfp4_weights", mxp.IMAGE_E2M1),
                           ("mxfp4p_weights_four_bit_image", mxp.IMAGE_E2M1R)):
            img = (mxp.prepack(ql, mxp.MXFP4P) if kind == mxp.IMAGE_E2M3 else mxp.prepack_e2m1(ql) if kind == mxp.IMAGE_E2M1
                   else mxp.prepack_e2m1r(ql))
            for _ in range(20):
                mxp.gemm_prepacked(Md, Nl, Kl, img_al, img, out=Dl, b_kind=kind)
            torch.cuda.synchronize()
            ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            ev2[0].record()
            for _ in range(50):
                mxp.gemm_prepacked(Md, Nl, Kl, img_al, img, out=Dl, b_kind=kind)
            ev2[1].record()
            torch.cuda.synchronize()
            us = ev2[0].elapsed_time(ev2[1]) / 50 * 1e3
            out["large_layer_" + name] = {"shape": "%d x %d x %d" % (Md, Nl, Kl), "us_per_call": us,
                                          "weight_image_GBps": img.numel() / us / 1e3,
                                          "frac_hbm": img.numel() / us / 1e3 / PEAK_HBM_GBPS}
            del img
        return out

    decode = timed_decode()

    # Measured ceilings: MFMAs alone on register-resident random operands (what the power limit leaves of the nominal
    # rate), and a plain 256 MiB device copy.
    def timed_probe(a_kind, b_kind):
        sink = torch.empty(65536, dtype=torch.float32, device=dev)
        iters = 4000                                           # ~0.1 ms per launch
        for _ in range(300):
            mxp.probe_mfma(iters, a_kind, b_kind, sink=sink)
        torch.cuda.synchronize()
        ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev2[0].record()
        for _ in range(100):
            mxp.probe_mfma(iters, a_kind, b_kind, sink=sink)
        ev2[1].record()
        torch.cuda.synchronize()
        return mxp.PROBE_FLOP_PER_ITER * iters / (ev2[0].elapsed_time(ev2[1]) / 100 * 1e-3) / 1e12

    mfma_peak_e2m3 = timed_probe(mxp.IMAGE_E2M3, mxp.IMAGE_E2M3)
    mfma_peak_e2m1 = timed_probe(mxp.IMAGE_E2M1, mxp.IMAGE_E2M1)
    mfma_peak_e4m3 = timed_probe(mxp.IMAGE_E4M3, mxp.IMAGE_E4M3)   # iterations take twice as long: FP8 runs at half rate
    cp_src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
    cp_dst = torch.empty_like(cp_src)
    for _ in range(3):
        cp_dst.copy_(cp_src)
    torch.cuda.synchronize()
    ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev2[0].record()
    for _ in range(10):
        cp_dst.copy_(cp_src)
    ev2[1].record()
    torch.cuda.synchronize()
    copy_gbps = 2.0 * (256 << 20) * 10 / (ev2[0].elapsed_time(ev2[1]) * 1e-3) / 1e9
    del cp_src, cp_dst

    # Standalone quantize (canonical outputs only), launches queued back to back over rotating source copies whose
    # total exceeds the 256 MB Infinity Cache: the activation tensor (12 copies) and the weight matrix (3 copies).
    def timed_quantize(src_bits, copies, launches):
        srcs = [to_dev(src_bits) for _ in range(copies)]
        q = mxp.quantize(srcs[0], mxp.MXFP4P)
        torch.cuda.synchronize()
        ev2 = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev2[0].record()
        for i in range(launches):
            mxp.quantize_into(srcs[i % copies], mxp.MXFP4P, *q)
        ev2[1].record()
        torch.cuda.synchronize()
        return ev2[0].elapsed_time(ev2[1]) / launches

    q_act_ms = timed_quantize(a_bits, 12, 24)
    q_large_ms = timed_quantize(w_bits, 3, 12)

    flops = 2.0 * M * N * K
    value = flops / (ms_per_step * 1e-3) / 1e12
    gemm_tflops = flops / (gemm_ms * 1e-3) / 1e12
    q_bytes = M * K * 2.5625                                  # bf16 in + nibbles + scale + index
    dq_bytes = M * K * (0.5625 + 2.0)
    pp_bytes = lambda r: r * K * (0.5625 + 0.78125)
    out_line = {
        "metric": "MXFP4+ GEMM TFLOP/s (Llama-8B linear shapes); quantize GB/s; % roofline",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
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
                   "step": "quantize(A) -> canonical + image in one pass, image(W) -> scaled-MFMA GEMM -> dequantize(A)"},
        "roofline": {"bound": "mfma", "achieved": gemm_tflops, "peak": PEAK_FP4_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / PEAK_FP4_TFLOPS, "traffic": traffic_from_profiles(args.workload, args.out_dtype),
                     "kernel": "gemm_kernel_dma" if M > 64 else "gemm_skinny_kernel", "kernel_ms": gemm_ms,
                     "note": "kernel_ms = HIP event pair around the launch on every 5th timed step (includes the dispatch "
                             "gap); traffic = FETCH_SIZE*2.0 + WRITE_SIZE bytes per launch from profiles/"},
        "measured_ceilings": {"mfma_only_e2m3_x_e2m3_TFLOPs": mfma_peak_e2m3, "mfma_only_e2m1_x_e2m1_TFLOPs": mfma_peak_e2m1, "mfma_only_e4m3_x_e4m3_TFLOPs": mfma_peak_e4m3,
                              "device_copy_256MiB_GBps": copy_gbps,
                              "gemm_frac_of_mfma_only": gemm_tflops / mfma_peak_e2m3,
                              "note": "MFMAs alone on register-resident pseudo-random operands, 1024 wavefronts: the rate the "
                                      "chip sustains at its power limit; copy = read + written bytes"},
        "stages_ms": stage_ms,
        # mxp_quantize on the workload's two tensors (bytes = bf16 in + codes + scale + index bytes out).  The weight
        # tensor is the representative one; the activation tensor of this workload is small enough (43 MB of traffic,
        # under 10 us) that launch and tail take a third of the time.
        "quantize_GBps": N * K * 2.5625 / (q_large_ms * 1e-3) / 1e9,
        "quantize_frac_hbm": N * K * 2.5625 / (q_large_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
        "quantize_tensor": "W bf16 [%d x %d], 3 copies in rotation, 12 launches back to back" % (N, K),
        "quantize_small_GBps": q_bytes / (q_act_ms * 1e-3) / 1e9,
        "quantize_small_frac_hbm": q_bytes / (q_act_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS,
        "quantize_small_tensor": "A bf16 [%d x %d], 12 copies in rotation, 24 launches back to back (launch-latency regime)" % (M, K),
        "quantize_a_with_image_GBps": M * K * (2.5625 + 0.78125) / (stage_ms["quantize_a"] * 1e-3) / 1e9,
        "dequantize_GBps": dq_bytes / (stage_ms["dequantize"] * 1e-3) / 1e9,
        "prepack_w_GBps": pp_bytes(N) / (stage_ms["prepack_w"] * 1e-3) / 1e9,
        "decode": decode,
        "gemm_only_TFLOPs": gemm_tflops,
        "gemm_back_to_back_TFLOPs": flops / (gemm_pp_ms * 1e-3) / 1e12,
        "gemm_back_to_back_%s_out_TFLOPs" % ("bf16" if out_dt == torch.float32 else "f32"): flops / (gemm_pp_other_ms * 1e-3) / 1e12,
        "gemm_a_mxfp4p_w_mxfp4_back_to_back_TFLOPs": flops / (gemm_w4_ms * 1e-3) / 1e12,
        "gemm_plain_mxfp4_back_to_back_TFLOPs": flops / (gemm_a4w4_ms * 1e-3) / 1e12,
        "gemm_mxfp4pp_back_to_back_TFLOPs": flops / (gemm_pp8_ms * 1e-3) / 1e12,
        "quantize_image_mxfp4pp_GBps": qimg_pp8_bytes / (qimg_pp8_ms * 1e-3) / 1e9,
        "gemm_w4a16_bf16_x_mxfp4p_TFLOPs": flops / (w4a16_ms * 1e-3) / 1e12,
        "gemm_mxfp8p_x_mxfp8p_TFLOPs": flops / (fp8p_ms * 1e-3) / 1e12,
        "gemm_mxfp6p_x_mxfp6_useful_TFLOPs": flops / (fp6_ms["mxfp6p_x_mxfp6"] * 1e-3) / 1e12,
        "gemm_mxfp6p_x_mxfp6p_useful_TFLOPs": flops / (fp6_ms["mxfp6p_x_mxfp6p"] * 1e-3) / 1e12,
        "gemm_time_vs_plain_mxfp4": {"mxfp4p_x_mxfp4p": gemm_pp_ms / gemm_a4w4_ms, "mxfp4p_x_mxfp4": gemm_w4_ms / gemm_a4w4_ms,
                                     "mxfp4pp_x_mxfp4pp": gemm_pp8_ms / gemm_a4w4_ms,
                                     "note": "same kernel, same shape, back to back; the paper's software MX+ GEMM costs 1.54x "
                                             "its MXFP4 GEMM in prefill on its GPU (Sec. 8)"},
        "gemm_with_prepacked_weights_TFLOPs": flops / ((stage_ms["gemm"] + stage_ms["quantize_a"]) * 1e-3) / 1e12,
    }
    if M <= 64:
        # skinny-M product: bound by reading the weight image once
        wbytes = float(img_w.numel())
        out_line["roofline"].update({"bound": "hbm", "achieved": wbytes / (gemm_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS,
                                     "unit": "GB/s", "frac": wbytes / (gemm_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS})
    if not args.no_cpu_baseline:
        out_line["cpu_baseline"] = cpu_baseline(a_bits, w_bits)
    print(json.dumps(out_line))


if __name__ == "__main__":
    main()
