"""Side measurements of bench.py (`--extras`) and its one-stage profiling modes (`--only`): the other formats and
configurations, the decode shapes and the measured ceilings.  Nothing here feeds `value` or `roofline` of the benchmark
line.  Every figure is per-call time from launches back to back between one event pair, several groups: mean, median, min."""
import numpy as np
import torch

from . import mxp, probe, synth

PEAK_FP4_TFLOPS = 10100.0
PEAK_HBM_GBPS = 8000.0


def _stats(samples):
    s = np.asarray(samples, dtype=np.float64)
    return {"mean": float(s.mean()), "median": float(np.median(s)), "min": float(s.min()), "n": int(s.size)}


def groups(fn, inner=20, n_groups=5, warm=100):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n_groups)]
    for g in range(n_groups):
        evs[g][0].record()
        for _ in range(inner):
            fn()
        evs[g][1].record()
    torch.cuda.synchronize()
    return _stats([e[0].elapsed_time(e[1]) / inner for e in evs])


def graph_us(call, n=20, reps=5):
    """Per-call time (us) of `call` with n calls captured in one HIP graph: the device-side figure, without the host time
    of a Python call per launch.  Every replay is timed; returns mean / median / min over `reps` groups of 10 replays."""
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
        for _ in range(20):
            graph.replay()
        samples = []
        for _ in range(reps):
            evg = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            evg[0].record()
            for _ in range(10):
                graph.replay()
            evg[1].record()
            torch.cuda.synchronize()
            samples.append(evg[0].elapsed_time(evg[1]) / (10 * n) * 1e3)
        return _stats(samples)
    except Exception as e:                                # capture is an extra: never fail the benchmark over it
        return {"error": "graph capture failed: %s" % type(e).__name__}


def _to_dev(x, dev):
    return torch.from_numpy(x.view(np.int16)).view(torch.bfloat16).to(dev)


def only_stage(name, ctx):
    """The callable that `bench.py --only name` runs per step (profiling aid)."""
    A, qa, qw, img_a, img_w, D, back = (ctx[k] for k in ("A", "qa", "qw", "img_a", "img_w", "D", "back"))
    M, N, K, dev, w_bits, w_kind = (ctx[k] for k in ("M", "N", "K", "dev", "w_bits", "w_kind"))
    ctx["convert"]()                                       # the images exist whatever stage is profiled
    torch.cuda.synchronize()
    if name == "quantize":
        return lambda: mxp.quantize_into(A, mxp.MXFP4P, *qa)
    if name == "quantize_w":
        W = _to_dev(w_bits, dev)
        q = mxp.quantize(W, mxp.MXFP4P)
        return lambda: mxp.quantize_into(W, mxp.MXFP4P, *q)
    if name == "quantize_t":
        WT = _to_dev(w_bits, dev).t().contiguous()
        return lambda: mxp.quantize_t(WT, mxp.MXFP4P)
    if name == "quantize_image":
        return lambda: mxp.quantize_image(A, mxp.MXFP4P, out=img_a, q_out=qa)
    if name == "prepack":
        iw = torch.empty(mxp.image_bytes(N, K), dtype=torch.uint8, device=dev)
        return lambda: mxp.prepack(qw, mxp.MXFP4P, out=iw)
    if name == "convert":
        return ctx["convert"]
    if name == "gemm":
        return ctx["product"]
    if name == "gemm_bf16a":
        ws = torch.empty(max(mxp.gemm_bf16a_workspace_bytes(M, K), 16), dtype=torch.uint8, device=dev)
        return lambda: mxp.gemm_bf16a(A, mxp.MXFP4P, img_w, N, out=D, workspace=ws, b_kind=w_kind)
    if name == "gemm_e2m1w":
        iw4 = mxp.prepack_e2m1(mxp.quantize(_to_dev(w_bits, dev), mxp.MXFP4))
        return lambda: mxp.gemm_prepacked(M, N, K, img_a, iw4, out=D, b_kind=mxp.IMAGE_E2M1)
    if name == "gemm_e4m3":
        ia8 = mxp.prepack_e4m3(mxp.quantize(A, mxp.MXFP4PP), mxp.MXFP4PP)
        iw8 = mxp.prepack_e4m3(mxp.quantize(_to_dev(w_bits, dev), mxp.MXFP4PP), mxp.MXFP4PP)
        return lambda: mxp.gemm_prepacked(M, N, K, ia8, iw8, out=D, a_kind=mxp.IMAGE_E4M3, b_kind=mxp.IMAGE_E4M3)
    if name == "gemm_pp_exact":
        qapp = mxp.quantize(A, mxp.MXFP4PP)
        ws = torch.empty(mxp.gemm_workspace_bytes(M, N, K, mxp.MXFP4PP, mxp.MXFP4P), dtype=torch.uint8, device=dev)
        return lambda: mxp.gemm(qapp, mxp.MXFP4PP, qw, mxp.MXFP4P, out=D, workspace=ws)
    if name == "gemm_fp6p":
        qa6, qw6 = mxp.quantize(A, mxp.MXFP6P), mxp.quantize(_to_dev(w_bits, dev), mxp.MXFP6)
        ws6 = torch.empty(mxp.gemm_workspace_bytes(M, N, K, mxp.MXFP6P, mxp.MXFP6), dtype=torch.uint8, device=dev)
        return lambda: mxp.gemm(qa6, mxp.MXFP6P, qw6, mxp.MXFP6, out=D, workspace=ws6)
    if name == "gemm_w4a16":
        return lambda: mxp.gemm_w4a16(A, qw, mxp.MXFP4P, out=D)
    if name in ("gemm_decode_large", "gemm_decode_large_four_bit"):
        ql, img_al, Dl, Nl, Kl = _large_layer(dev)
        img_wl = mxp.prepack(ql, mxp.MXFP4P) if name == "gemm_decode_large" else mxp.prepack_e2m1r(ql)
        kind = mxp.IMAGE_E2M3 if name == "gemm_decode_large" else mxp.IMAGE_E2M1R
        return lambda: mxp.gemm_prepacked(8, Nl, Kl, img_al, img_wl, out=Dl, b_kind=kind)
    if name == "dequantize":
        return lambda: mxp.dequantize(qa, mxp.MXFP4P, out=back)
    if name == "copy":
        # plain device copy of a known size (256 MiB): the reference that scales the FETCH_SIZE / WRITE_SIZE counters
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        return lambda: dst.copy_(src)
    raise ValueError(name)


def _large_layer(dev, rows=8):
    """8 activation rows against a 70B-sized layer (28672 x 8192) of random codes."""
    Nl, Kl = 28672, 8192
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    ql = (torch.randint(0, 256, (Nl, Kl // 2), dtype=torch.uint8, device=dev, generator=gen),
          torch.randint(120, 134, (Nl, Kl // 32), dtype=torch.uint8, device=dev, generator=gen),
          torch.randint(0, 32, (Nl, Kl // 32), dtype=torch.uint8, device=dev, generator=gen))
    img_al = mxp.prepack(tuple(t[:rows].contiguous() for t in ql), mxp.MXFP4P)
    Dl = torch.empty((rows, Nl), dtype=torch.float32, device=dev)
    return ql, img_al, Dl, Nl, Kl


def _decode(dev):
    """Decode configuration (8 x 4096 activations, 4096 x 4096 weights) and its down-projection shape: activations
    quantized on the fly, prepacked weights; bound by reading the weight image once."""
    out = {}
    for label, (Nd, Kd) in (("8x4096x4096", (4096, 4096)), ("8x4096x14336", (4096, 14336)), ("8x14336x4096", (14336, 4096))):
        Ad = _to_dev(synth.activations(8, Kd, config_id=2, tensor_id=0), dev)
        Wd = _to_dev(synth.weights(Nd, Kd, config_id=2, tensor_id=1), dev)
        res = {}
        for name, fmt_w, kind in (("mxfp4p_weights_e2m3_image", mxp.MXFP4P, mxp.IMAGE_E2M3), ("mxfp4_weights", mxp.MXFP4, mxp.IMAGE_E2M1),
                                  ("mxfp4p_weights_four_bit_image", mxp.MXFP4P, mxp.IMAGE_E2M1R)):
            qwd = mxp.quantize(Wd, fmt_w)
            img = (mxp.prepack_e2m1(qwd) if kind == mxp.IMAGE_E2M1 else mxp.prepack_e2m1r(qwd) if kind == mxp.IMAGE_E2M1R
                   else mxp.prepack(qwd, fmt_w))
            Dd = torch.empty((8, Nd), dtype=torch.float32, device=dev)
            wsd = torch.empty(max(mxp.gemm_bf16a_workspace_bytes(8, Kd), 16), dtype=torch.uint8, device=dev)
            call = lambda: mxp.gemm_bf16a(Ad, mxp.MXFP4P, img, Nd, out=Dd, workspace=wsd, b_kind=kind)
            ug = graph_us(call)
            img_a = mxp.quantize_image(Ad, mxp.MXFP4P)
            up = graph_us(lambda: mxp.gemm_prepacked(8, Nd, Kd, img_a, img, out=Dd, b_kind=kind))
            res[name] = {"us_per_call_python": groups(call, 20, 5, warm=10)["mean"] * 1e3, "us_per_call_in_hip_graph": ug,
                         "us_product_kernel_alone_in_hip_graph": up}
            if "mean" in ug:
                res[name].update({"weight_image_GBps": img.numel() / ug["mean"] / 1e3, "frac_hbm": img.numel() / ug["mean"] / 1e3 / PEAK_HBM_GBPS})
        qwd = mxp.quantize(Wd, mxp.MXFP4P)
        Dd = torch.empty((8, Nd), dtype=torch.float32, device=dev)
        res["w4a16_mxfp4p_weights"] = {"us_per_call_in_hip_graph": graph_us(lambda: mxp.gemm_w4a16(Ad, qwd, mxp.MXFP4P, out=Dd))}
        out[label] = res
    out["note"] = ("us_per_call_python: 20 Python calls back to back (host-bound at this size); us_per_call_in_hip_graph: 20 calls "
                   "of mxp_gemm_bf16a (conversion kernel + product kernel) captured in one HIP graph and replayed -- the device-side "
                   "time; GB/s and frac_hbm use its mean")
    ql, img_al, Dl, Nl, Kl = _large_layer(dev)
    for name, kind in (("mxfp4p_weights_e2m3_image", mxp.IMAGE_E2M3), ("mxfp4_weights", mxp.IMAGE_E2M1),
                       ("mxfp4p_weights_four_bit_image", mxp.IMAGE_E2M1R)):
        img = (mxp.prepack(ql, mxp.MXFP4P) if kind == mxp.IMAGE_E2M3 else mxp.prepack_e2m1(ql) if kind == mxp.IMAGE_E2M1
               else mxp.prepack_e2m1r(ql))
        st = groups(lambda: mxp.gemm_prepacked(8, Nl, Kl, img_al, img, out=Dl, b_kind=kind), 25, 4, warm=20)
        out.setdefault("8x28672x8192", {})[name] = {"ms": st, "weight_image_GBps": img.numel() / st["mean"] / 1e6,
                                                      "frac_hbm": img.numel() / st["mean"] / 1e6 / PEAK_HBM_GBPS}
        del img
    return out


def _other_shapes(dev):
    """The product kernel on the other prefill configurations, back to back (images built once)."""
    out = {}
    for label, cfg, wn in (("prefill_attn q/o 2048x4096x4096", "prefill_attn", "wqo"), ("prefill_attn k/v 2048x1024x4096", "prefill_attn", "wkv"),
                           ("prefill_mlp_down 4096x4096x14336", "prefill_mlp_down", "wdown")):
        a, ws = synth.make(cfg)
        Ad, Wd = _to_dev(a, dev), _to_dev(ws[wn], dev)
        Ms, Ks = Ad.shape
        Ns = Wd.shape[0]
        ia = mxp.quantize_image(Ad, mxp.MXFP4P)
        iw = mxp.prepack(mxp.quantize(Wd, mxp.MXFP4P), mxp.MXFP4P)
        Ds = torch.empty((Ms, Ns), dtype=torch.float32, device=dev)
        st = groups(lambda: mxp.gemm_prepacked(Ms, Ns, Ks, ia, iw, out=Ds), 20, 5, warm=200)
        fl = 2.0 * Ms * Ns * Ks
        out[label] = {"ms": st, "TFLOPs": fl / st["mean"] / 1e9, "TFLOPs_best": fl / st["min"] / 1e9, "frac_peak": fl / st["mean"] / 1e9 / PEAK_FP4_TFLOPS}
    return out


def run(ctx):
    """The `--extras` block of the benchmark line."""
    A, qa, qw, img_a, img_w, D = (ctx[k] for k in ("A", "qa", "qw", "img_a", "img_w", "D"))
    M, N, K, dev, w_bits, w_kind, out_dt = (ctx[k] for k in ("M", "N", "K", "dev", "w_bits", "w_kind", "out_dt"))
    flops = 2.0 * M * N * K
    res = {}
    tf = lambda st: {"TFLOPs": flops / st["mean"] / 1e9, "TFLOPs_best": flops / st["min"] / 1e9, "ms": st}

    def timed_gemm(a_image, a_kind, b_image, b_kind, out=None, k=None):
        out = D if out is None else out
        k = K if k is None else k
        return groups(lambda: mxp.gemm_prepacked(M, N, k, a_image, b_image, out=out, a_kind=a_kind, b_kind=b_kind), 20, 5, warm=250)

    fm = {}
    fm["mxfp4p_x_mxfp4p"] = timed_gemm(img_a, mxp.IMAGE_E2M3, img_w, w_kind)
    other_dt = torch.bfloat16 if out_dt == torch.float32 else torch.float32
    D_other = torch.empty((M, N), dtype=other_dt, device=dev)
    fm["mxfp4p_x_mxfp4p_%s_out" % ("bf16" if out_dt == torch.float32 else "f32")] = timed_gemm(img_a, mxp.IMAGE_E2M3, img_w, w_kind, out=D_other)
    del D_other
    if M > 64:
        W = _to_dev(w_bits, dev)
        img_w4 = mxp.prepack_e2m1(mxp.quantize(W, mxp.MXFP4))
        fm["mxfp4p_x_mxfp4"] = timed_gemm(img_a, mxp.IMAGE_E2M3, img_w4, mxp.IMAGE_E2M1)
        img_a4 = mxp.prepack_e2m1(mxp.quantize(A, mxp.MXFP4))
        fm["mxfp4_x_mxfp4"] = timed_gemm(img_a4, mxp.IMAGE_E2M1, img_w4, mxp.IMAGE_E2M1)
        del img_a4
        # MXFP4++ (Sec. 4.3): two-sided through E4M3 images (FP8 MFMAs at half rate); one-sided exactly, over two K segments
        img_w8 = mxp.prepack_e4m3(mxp.quantize(W, mxp.MXFP4PP), mxp.MXFP4PP)
        img_a8 = mxp.prepack_e4m3(mxp.quantize(A, mxp.MXFP4PP), mxp.MXFP4PP)
        fm["mxfp4pp_x_mxfp4pp_fp8_images"] = timed_gemm(img_a8, mxp.IMAGE_E4M3, img_w8, mxp.IMAGE_E4M3)
        st = groups(lambda: mxp.quantize_image(A, mxp.MXFP4PP, out=img_a8), 20, 5, warm=20)
        res["quantize_image_mxfp4pp_GBps"] = (A.numel() * A.element_size() + img_a8.numel()) / st["mean"] / 1e6
        del img_w8, img_a8
        qapp = mxp.quantize(A, mxp.MXFP4PP)
        wspp = torch.empty(mxp.gemm_workspace_bytes(M, N, K, mxp.MXFP4PP, mxp.MXFP4P), dtype=torch.uint8, device=dev)
        fm["mxfp4pp_x_mxfp4p_exact_incl_image_build"] = groups(lambda: mxp.gemm(qapp, mxp.MXFP4PP, qw, mxp.MXFP4P, out=D, workspace=wspp), 10, 4, warm=100)
        del qapp, wspp
        # six-bit operands (Sec. 4.2): MXFP6 x MXFP6 is one E2M3 product; the MXFP6+ BM adds K segments (2 one-sided, 4 two-sided)
        Kp = (K + 127) // 128 * 128
        qa6 = mxp.quantize(A, mxp.MXFP6P)
        for name, fmt_w, n_seg, ma, mb in (("mxfp6p_x_mxfp6", mxp.MXFP6, 2, 0b10, 0), ("mxfp6p_x_mxfp6p", mxp.MXFP6P, 4, 0b1010, 0b1100)):
            ia6 = mxp.prepack_fp6(qa6, mxp.MXFP6P, n_seg, ma)
            iw6 = mxp.prepack_fp6(mxp.quantize(W, fmt_w), fmt_w, n_seg, mb)
            fm[name] = timed_gemm(ia6, mxp.IMAGE_E2M3, iw6, mxp.IMAGE_E2M3, k=n_seg * Kp)
            del ia6, iw6
        del qa6
        # conversion-based product (Sec. 5; weight-only quantization) and MXFP8(+) pairs (bf16 MFMA on de-converted operands)
        fm["bf16_x_mxfp4p_w4a16"] = groups(lambda: mxp.gemm_w4a16(A, qw, mxp.MXFP4P, out=D), 10, 3, warm=20)
        qa8p, qw8p = mxp.quantize(A, mxp.MXFP8P), mxp.quantize(W, mxp.MXFP8P)
        ws0 = torch.empty(16, dtype=torch.uint8, device=dev)
        fm["mxfp8p_x_mxfp8p"] = groups(lambda: mxp.gemm(qa8p, mxp.MXFP8P, qw8p, mxp.MXFP8P, out=D, workspace=ws0), 5, 3, warm=5)
        del qa8p, qw8p, W
        base = fm["mxfp4_x_mxfp4"]["mean"]
        res["gemm_time_vs_plain_mxfp4"] = {k: v["mean"] / base for k, v in fm.items() if k.startswith("mxfp4")}
        res["gemm_time_vs_plain_mxfp4"]["note"] = ("same kernel, same shape, back to back; the paper's software MX+ GEMM costs 1.54x "
                                                   "its MXFP4 GEMM in prefill on its GPU (Sec. 8)")
    res["gemm_formats_useful_TFLOPs"] = {k: tf(v) for k, v in fm.items()}
    res["decode"] = _decode(dev)
    res["other_prefill_shapes"] = _other_shapes(dev)

    # Measured ceilings: MFMAs alone on register-resident operands (what the power limit leaves of the nominal rate), with
    # pseudo-random operand bits and with bits loaded from this run's own images; and a plain 256 MiB device copy.
    sink = torch.empty(65536, dtype=torch.float32, device=dev)
    iters = 4000                                           # ~0.1 ms per launch
    pf = lambda st: probe.FLOP_PER_ITER * iters / st["mean"] / 1e9
    ceil = {}
    for nm, ka, kb in (("e2m3_x_e2m3", mxp.IMAGE_E2M3, mxp.IMAGE_E2M3), ("e2m1_x_e2m1", mxp.IMAGE_E2M1, mxp.IMAGE_E2M1),
                       ("e4m3_x_e4m3", mxp.IMAGE_E4M3, mxp.IMAGE_E4M3)):
        ceil["mfma_only_%s_random_bits_TFLOPs" % nm] = pf(groups(lambda: probe.mfma(iters, ka, kb, sink=sink), 20, 5, warm=300))
    if M > 64:
        st = groups(lambda: probe.mfma_images(iters, img_a, mxp.IMAGE_E2M3, M, img_w, mxp.IMAGE_E2M3, N, K, sink=sink), 20, 5, warm=300)
        ceil["mfma_only_e2m3_x_e2m3_image_bits_TFLOPs"] = pf(st)
        ceil["gemm_back_to_back_frac_of_mfma_only_on_its_own_operand_bits"] = (flops / fm["mxfp4p_x_mxfp4p"]["mean"] / 1e9) / pf(st)
    cp_src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
    cp_dst = torch.empty_like(cp_src)
    st = groups(lambda: cp_dst.copy_(cp_src), 5, 4, warm=3)
    ceil["device_copy_256MiB_GBps"] = 2.0 * (256 << 20) / st["mean"] / 1e6
    # launch floor: the same conversion kernel on one 32 x 32 tile, 20 launches replayed from a HIP graph -- what a launch
    # costs before it moves any bytes (dispatch, ramp-up, drain); a 10 us kernel cannot reach the rate of a 100 us one
    tiny = A[:32, :32].contiguous()
    qt = mxp.quantize(tiny, mxp.MXFP4P)
    ceil["launch_floor_us_quantize_one_tile_in_hip_graph"] = graph_us(lambda: mxp.quantize_into(tiny, mxp.MXFP4P, *qt))
    ceil["note"] = ("MFMAs alone on register-resident operands, 1024 wavefronts: the rate the chip sustains at its power limit; "
                    "image_bits = operand registers loaded once from the benchmark's own images; copy = read + written bytes")
    res["measured_ceilings"] = ceil
    return res
