"""Pins of the CPU oracle for the six- and eight-bit MX / MX+ formats (Sec. 4.2 data layout) against things other than
itself: the element tables of the OCP formats, a library's FP8 conversion, brute-force nearest-value search, numpy's
bit packing, closed forms and the invariants the paper states (the BM keeps e_max as its exponent and spends every
non-sign bit on mantissa).  No GPU."""
import numpy as np
import pytest
import torch

import oracle

W = oracle.wide
FMTS = {"mxfp6": W.MXFP6, "mxfp6p": W.MXFP6P, "mxfp8": W.MXFP8, "mxfp8p": W.MXFP8P}
BITS = {"mxfp6": 6, "mxfp6p": 6, "mxfp8": 8, "mxfp8p": 8}
EMAX = {"mxfp6": 2, "mxfp6p": 2, "mxfp8": 8, "mxfp8p": 8}


def elem_table(name):
    """Values of all non-negative ordinary codes, decoded by the oracle at X = 1."""
    bits = BITS[name]
    n = 1 << (bits - 1)
    vals = np.zeros(n)
    for base in range(0, n, 32):
        codes = np.arange(base, base + 32, dtype=np.uint8)
        vals[base:base + 32] = W.decode_block(codes, 127, 0, FMTS[name.rstrip("p")])
    return vals


def test_e2m3_table_is_the_ocp_one():
    v = elem_table("mxfp6")
    # subnormals k/8, then three binades 1.m, 2*1.m, 4*1.m with 3 fraction bits; largest 7.5, no special codes
    want = np.concatenate([np.arange(8) / 8.0] + [(1 + np.arange(8) / 8.0) * s for s in (1.0, 2.0, 4.0)])
    assert (v == want).all()
    assert v.max() == 7.5 and v[1] == 0.125


def test_e4m3_table_matches_the_library_type():
    v = elem_table("mxfp8")
    lib = torch.arange(0, 128, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    assert np.isnan(lib[127])                                  # S.1111.111 is the NaN code; the oracle never writes it
    assert (v[:127] == lib[:127]).all()
    assert v[126] == 448.0 and v[1] == 2.0 ** -9 and v[8] == 2.0 ** -6


def block_with_bm(bm_value, others, pos=0):
    x = np.zeros(32, np.float32)
    rest = [i for i in range(32) if i != pos]
    x[rest[: len(others)]] = others
    x[pos] = bm_value
    return x


def test_e4m3_encoding_matches_the_library_cast():
    """With the BM at 256 the scale is 1, so ordinary elements must be the library's float -> e4m3fn cast (RNE,
    subnormals included) for every in-range value."""
    rng = np.random.default_rng(3)
    for rep in range(200):
        mag = np.exp2(rng.uniform(-11, 7.99, 31)) * rng.choice([1, -1], 31)
        if rep == 0:   # exact midpoints between neighbours and tiny values around the first subnormal
            mag[:8] = [2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -9 * 1.5, 0.0703125 + 2.0 ** -8 * 0.5, 17.0, 19.0, 208.0 + 8, 2.0 ** -11]
        x = block_with_bm(256.0, mag.astype(np.float32))
        codes, s, i = W.encode_block(x, W.MXFP8)
        assert s == 127 and i == 0
        lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert (codes == lib).all(), (x[codes != lib], codes[codes != lib], lib[codes != lib])


@pytest.mark.parametrize("name", ["mxfp6", "mxfp8"])
def test_ordinary_elements_are_the_nearest_value_ties_to_even(name):
    """Brute force over the table: no other code is closer; on exact midpoints the even code wins; above the largest
    value the result saturates."""
    tab = elem_table(name)
    if name == "mxfp8":
        tab = tab[:127]
    top = tab.max()
    bm = 2.0 ** EMAX[name]                                      # BM at 2^e_max -> X = 1
    rng = np.random.default_rng(11)
    mids = (tab[:-1] + tab[1:]) / 2
    cases = np.concatenate([mids, tab, rng.uniform(0, top, 400), np.exp2(rng.uniform(-12, np.log2(top), 400))])
    cases = cases[cases <= bm]                                  # ordinary elements never exceed the BM
    for lo in range(0, len(cases), 31):
        vals = cases[lo:lo + 31].astype(np.float32)
        x = block_with_bm(bm, vals)
        codes, s, _ = W.encode_block(x, FMTS[name])
        assert s == 127
        for a, c in zip(vals.astype(np.float64), codes[1:]):
            d = np.abs(tab - a)
            best = np.flatnonzero(d == d.min())
            if len(best) == 2:                                  # a midpoint: the even code
                want = best[0] if best[0] % 2 == 0 else best[1]
            else:
                want = best[0]
            assert c == want, (name, a, c, want)
    # saturation: scaled elements above the largest value
    sat = {"mxfp6": [7.6, 7.75, 7.99], "mxfp8": [449.0, 464.0, 480.0, 511.0]}[name]
    x = block_with_bm(np.float32(sat[-1] * 1.0001), np.array(sat, np.float32))
    codes, s, _ = W.encode_block(x, FMTS[name])
    assert s == 127 and (tab[codes[1:1 + len(sat)]] == top).all() and tab[codes[0]] == top


@pytest.mark.parametrize("name", ["mxfp6p", "mxfp8p"])
def test_bm_keeps_emax_and_all_mantissa_bits(name):
    fb = BITS[name] - 1
    emax = EMAX[name]
    rng = np.random.default_rng(5)
    # every BM code round-trips: 2^e_max * (1 + m / 2^fb), at several scales and both signs
    for m in range(1 << fb):
        for sh, sg in ((0, 1), (-20, -1), (37, 1)):
            val = np.float32(sg * 2.0 ** (emax + sh) * (1 + m / 2.0 ** fb))
            x = block_with_bm(val, rng.uniform(-1, 1, 31).astype(np.float32) * np.float32(2.0 ** (emax + sh - 1)), pos=m % 32)
            codes, s, i = W.encode_block(x, FMTS[name])
            assert s == 127 + sh and i == m % 32
            assert codes[i] == (m | ((1 << fb) if sg < 0 else 0))
            assert W.decode_block(codes, s, i, FMTS[name])[i] == float(val)
    # in between: nearest, ties to even, a carry saturates instead of touching the scale
    unit = 2.0 ** (emax - fb)
    for frac, want in ((0.25, 0), (0.5, 0), (0.75, 1), (1.5, 2), (2.5, 2), ((1 << fb) - 0.5, (1 << fb) - 1),
                       ((1 << fb) - 0.25, (1 << fb) - 1)):
        x = block_with_bm(np.float32(2.0 ** emax + frac * unit), np.zeros(0, np.float32), pos=7)
        codes, s, i = W.encode_block(x, FMTS[name])
        assert (s, i, codes[7]) == (127, 7, want), (frac, codes[7], want)


def test_mxfp8p_holds_any_bf16_bm_exactly():
    """An E4M7 number has bf16's seven fraction bits, so the BM of a bf16 block survives the format unchanged."""
    rng = np.random.default_rng(9)
    bits = rng.integers(0x3000, 0x4F00, size=(64, 32), dtype=np.uint16) | (rng.integers(0, 2, size=(64, 32), dtype=np.uint16) << 15)
    q = W.quantize(bits, W.MXFP8P)
    back = W.dequantize(q, W.MXFP8P)
    x = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    idx = q[2]
    assert (np.abs(x).argmax(axis=1) == idx[:, 0]).all()
    r = np.arange(64)
    assert (back[r, idx[:, 0]] == x[r, idx[:, 0]]).all()


@pytest.mark.parametrize("name", list(FMTS))
def test_scale_flush_nan_and_error_bounds(name):
    fmt, emax, bits = FMTS[name], EMAX[name], BITS[name]
    plus = name.endswith("p")
    rng = np.random.default_rng(21)
    x = (rng.standard_normal((50, 64)) * np.exp2(rng.integers(-30, 30, size=(50, 1)))).astype(np.float32)
    x[3, 5] = 0.0
    e, s, i = W.quantize(x, fmt)
    back = W.dequantize((e, s, i), fmt)
    xb = x.reshape(50, 2, 32).astype(np.float64)
    amax = np.abs(xb).max(axis=2)
    # Eq. 1: scale byte = floor(log2 BM) - e_max + 127
    assert (s == np.floor(np.log2(amax)) - emax + 127).all()
    if plus:
        assert (i == np.abs(xb).argmax(axis=2)).all()
    else:
        assert (i == 0).all()
    X = np.exp2(s.astype(np.float64) - 127)[:, :, None]
    err = np.abs(back.reshape(50, 2, 32) - xb) / X
    # ordinary elements: half a step of their binade (3 fraction bits; subnormal spacing below the first binade)
    emin = 0 if bits == 6 else -6
    ex = np.maximum(np.floor(np.log2(np.maximum(np.abs(xb) / X, 1e-300))), emin)
    bound = np.exp2(ex - 3 - 1)
    is_bm = np.zeros_like(err, bool)
    if plus:
        np.put_along_axis(is_bm, i[:, :, None].astype(np.int64), True, axis=2)
    top = 7.5 if bits == 6 else 448.0
    sat = (np.abs(xb) / X > top) & ~is_bm
    assert (err[~is_bm & ~sat] <= bound[~is_bm & ~sat]).all()
    assert (np.abs(back.reshape(50, 2, 32))[sat] == (top * X * np.ones_like(err))[sat]).all()
    if plus:   # BM: half a unit of its last fraction bit, except where the carry saturates
        fb = bits - 1
        bm_err = err[is_bm]
        assert (bm_err <= 2.0 ** (emax - fb) * (1.0 + 1e-12)).all()
        assert (bm_err <= 2.0 ** (emax - fb - 1)).mean() > 0.9
    # flush: BM exponent <= -127 + e_max; zero block; NaN / Inf block
    tiny = np.full((1, 32), np.float32(2.0 ** (-127 + emax) * 1.5), np.float32)
    tiny[0, 4] = np.float32(2.0 ** (-127 + emax) * 1.99)
    assert W.quantize(tiny, fmt)[1][0, 0] == 0 and not W.quantize(tiny, fmt)[0].any()
    just = tiny.copy()
    just[0, 4] = np.float32(2.0 ** (-126 + emax))
    assert W.quantize(just, fmt)[1][0, 0] == 1
    assert W.quantize(np.zeros((1, 32), np.float32), fmt)[1][0, 0] == 0
    for bad in (np.nan, np.inf, -np.inf):
        y = x[:1, :32].copy()
        y[0, 9] = bad
        e1, s1, i1 = W.quantize(y, fmt)
        assert s1[0, 0] == 255 and not e1.any() and i1[0, 0] == 0
        assert np.isnan(W.dequantize((e1, s1, i1), fmt)).all()


@pytest.mark.parametrize("name", list(FMTS))
def test_packing_is_a_little_endian_bit_string(name):
    fmt, bits = FMTS[name], BITS[name]
    rng = np.random.default_rng(2)
    x = rng.standard_normal((7, 96)).astype(np.float32)
    e, s, i = W.quantize(x, fmt)
    assert e.shape == (7, 96 * bits // 8)
    for r in range(7):
        for b in range(3):
            codes, sb, ib = W.encode_block(x[r, 32 * b:32 * b + 32], fmt)
            assert (sb, ib) == (s[r, b], i[r, b])
            bit = ((codes[:, None] >> np.arange(bits)) & 1).astype(np.uint8).reshape(-1)   # element-major, LSB first
            want = np.packbits(bit, bitorder="little")
            assert (e[r, b * 4 * bits:(b + 1) * 4 * bits] == want).all()


def test_plus_differs_from_plain_only_at_the_bm():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((20, 64)).astype(np.float32)
    for plain, plus in ((W.MXFP6, W.MXFP6P), (W.MXFP8, W.MXFP8P)):
        a = W.dequantize(W.quantize(x, plain), plain)
        qp = W.quantize(x, plus)
        b = W.dequantize(qp, plus)
        diff = (a != b).reshape(20, 2, 32)
        assert (qp[1] == W.quantize(x, plain)[1]).all()                  # the scale is never altered (Sec. 4.1)
        for r in range(20):
            for k in range(2):
                where = np.flatnonzero(diff[r, k])
                assert len(where) <= 1 and (len(where) == 0 or where[0] == qp[2][r, k])
        # and the BM never gets worse
        assert (np.abs(b - x) <= np.abs(a - x) + 1e-300).all()


@pytest.mark.parametrize("name", ["mxfp6p", "mxfp8p"])
def test_ties_take_the_lowest_index_and_signs_survive_zero_codes(name):
    fmt, bits, emax = FMTS[name], BITS[name], EMAX[name]
    sign = 1 << (bits - 1)
    x = np.zeros(32, np.float32)
    x[3], x[17], x[20] = -5.0, 5.0, 5.0                          # equal magnitudes: the first one is the BM
    x[1] = -0.0
    x[2] = np.float32(-2.0 ** -40)                              # rounds to a zero magnitude, keeps its sign
    codes, s, i = W.encode_block(x, fmt)
    assert i == 3 and s == 127 + 2 - emax
    assert codes[3] & sign and codes[1] == sign and codes[2] == sign and codes[0] == 0
    d = W.decode_block(codes, s, i, fmt)
    assert d[3] == -5.0 and d[17] == 5.0 and d[20] == 5.0        # 5.0 is exact both as a BM and as an ordinary element
    assert codes[17] == codes[20] and codes[17] != (codes[3] & (sign - 1))
    assert np.signbit(d[1]) and d[1] == 0.0 and np.signbit(d[2])


@pytest.mark.parametrize("fa,fb", [("mxfp6p", "mxfp6p"), ("mxfp6p", "mxfp6"), ("mxfp6", "mxfp6"), ("mxfp8", "mxfp8"),
                                   ("mxfp8p", "mxfp8")])
def test_product_is_the_exact_sum_of_decoded_products(fa, fb):
    """Brute force on a tiny case: every decoded element is a dyadic rational, so the sum over K can be formed without
    any rounding in Python's fractions; the oracle's float64 result and its bound S must equal it."""
    from fractions import Fraction
    rng = np.random.default_rng(11)
    M, N, K = 3, 4, 96
    a = (rng.standard_normal((M, K)) * np.exp2(rng.integers(-3, 4, (M, K)))).astype(np.float32)
    b = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    a[1, 5] = 77.0                                              # an outlier: its block's other elements become tiny codes
    qa, qb = W.quantize(a, FMTS[fa]), W.quantize(b, FMTS[fb])
    D, S = W.gemm(qa, FMTS[fa], qb, FMTS[fb])
    bpb_a, bpb_b = W.block_bytes(FMTS[fa]), W.block_bytes(FMTS[fb])

    def rows_of(q, fmt, bpb, bits):
        e, s, i = q
        out = []
        for r in range(e.shape[0]):
            vals = []
            for kb in range(K // 32):
                blk = e[r, kb * bpb:(kb + 1) * bpb]
                if bits == 6:
                    codes = np.packbits(np.unpackbits(blk, bitorder="little").reshape(32, 6)[:, ::-1], axis=1,
                                        bitorder="big")[:, 0] >> 2
                else:
                    codes = blk
                vals += [Fraction(float(v)) for v in W.decode_block(codes, s[r, kb], i[r, kb], fmt)]
            out.append(vals)
        return out

    ra, rb = rows_of(qa, FMTS[fa], bpb_a, BITS[fa]), rows_of(qb, FMTS[fb], bpb_b, BITS[fb])
    for m in range(M):
        for n in range(N):
            exact = sum(x * y for x, y in zip(ra[m], rb[n]))
            bound = sum(abs(x * y) for x, y in zip(ra[m], rb[n]))
            assert Fraction(float(D[m, n])) == exact or abs(Fraction(float(D[m, n])) - exact) <= abs(exact) * Fraction(1, 2 ** 50)
            assert abs(Fraction(float(S[m, n])) - bound) <= bound * Fraction(1, 2 ** 50)


def test_product_hand_case_with_a_split_bm():
    """One block per operand.  The MXFP6+ BM 4 + 13/8 = 5.625 is not an E2M3 number (it is 5.5 + 0.125); the product
    must use all five mantissa bits."""
    a = np.zeros((1, 32), np.float32)
    b = np.zeros((1, 32), np.float32)
    a[0, 7], a[0, 8] = 5.625, 1.25
    b[0, 7], b[0, 8], b[0, 9] = -4.375, 3.0, 0.875
    qa, qb = W.quantize(a, W.MXFP6P), W.quantize(b, W.MXFP6P)
    assert (W.dequantize(qa, W.MXFP6P) == a).all() and (W.dequantize(qb, W.MXFP6P) == b).all()
    D, S = W.gemm(qa, W.MXFP6P, qb, W.MXFP6P)
    assert D[0, 0] == 5.625 * -4.375 + 1.25 * 3.0 and S[0, 0] == 5.625 * 4.375 + 3.75
    # the plain format keeps only three mantissa bits of each BM (5.625 -> 5.5, 4.375 -> 4.5)
    D6, _ = W.gemm(W.quantize(a, W.MXFP6), W.MXFP6, W.quantize(b, W.MXFP6), W.MXFP6)
    assert D6[0, 0] == 5.5 * -4.5 + 3.75
