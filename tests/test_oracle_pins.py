"""Pins for the CPU oracle: everything here checks oracle/ against something that is NOT the oracle --
values the paper prints, closed forms over the 16 nibbles, the definition of "nearest grid point"
searched by brute force, invariants of the format, and numpy's float64 matmul.  CPU only.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import MXFP4, MXFP4P
from paper_2510_14557_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_values.txt")

E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])          # code 0..7 (Sec. 2: E2M1, bias 1)
BM_GRID = 4.0 + 0.5 * np.arange(8)                                      # code 0..7 (Sec. 4.2: E2M3 at e_max)


def golden():
    d = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            d[k.strip()] = float(v)
    return d


def nibbles(elems):
    e = np.asarray(elems, np.uint8)
    out = np.empty(e.shape[:-1] + (e.shape[-1] * 2,), np.uint8)
    out[..., 0::2] = e & 15
    out[..., 1::2] = e >> 4
    return out


def block(vals, fill=0.0):
    x = np.full(32, fill, np.float32)
    for i, v in vals.items():
        x[i] = v
    return x


def nearest_code(a, grid):
    """Definition of round-to-nearest on a grid, ties to the even code, by exhaustive search."""
    d = np.abs(grid - a)
    best = np.flatnonzero(d == d.min())
    if len(best) == 1:
        return int(best[0])
    assert len(best) == 2
    return int(best[0] if best[0] % 2 == 0 else best[1])


# ------------------------------------------------------------------ values the paper prints
def test_paper_constants_and_layout_sizes():
    g = golden()
    # e_max = 2: a block whose BM is exactly 2^e has shared_exp = e - 2  (Eq. 1)
    for e in (-3, 0, 2, 5):
        _, s, _ = oracle.encode_block(block({7: 2.0 ** e}))
        assert s - 127 == e - int(g["e_max"])
    q = oracle.quantize(np.ones((4, 256), np.float32), MXFP4P)
    bits = 8 * sum(a.size for a in q) / (4 * 256)
    assert bits == g["bits_per_element_mxfp4p"]
    bits4 = 8 * (q[0].size + q[1].size) / (4 * 256)
    assert bits4 == g["bits_per_element_mxfp4"]
    assert 2 ** int(g["bm_index_bits"]) == 32


def test_paper_saturation_example():
    g = golden()
    # 0.99 as the block maximum: exponent -1, shared_exp -3, scaled 7.92 -> 6.0 in plain MXFP4
    e, s, _ = oracle.encode_block(block({0: 0.99}), MXFP4)
    assert s - 127 == g["shared_exp_for_bm_0p99"]
    assert abs(0.99 / 2.0 ** (s - 127) - g["scaled_0p99"]) < 1e-6
    d = oracle.decode_block(e, s, 0, MXFP4)
    assert d[0] / 2.0 ** (s - 127) == g["saturated_to"]
    # the same scaled value as an ordinary element next to a slightly larger BM also saturates to 6
    e, s, i = oracle.encode_block(block({0: 0.995, 1: 0.99}), MXFP4P)
    assert i == 0 and oracle.decode_block(e, s, i)[1] / 2.0 ** (s - 127) == g["saturated_to"]
    # with one more exponent step of head-room 0.99 scales to 3.96 and is not saturated: nearest is 4
    e, s, i = oracle.encode_block(block({0: 1.5, 1: 0.99}), MXFP4P)
    assert abs(0.99 / 2.0 ** (s - 127) - g["scaled_0p99_with_offset"]) < 1e-6
    assert oracle.decode_block(e, s, i)[1] / 2.0 ** (s - 127) == 4.0


def test_paper_nbm_example():
    g = golden()
    # shared_exp = 1  <=>  BM in [8,16):  -0.39 / 2 = -0.195 -> 0
    e, s, i = oracle.encode_block(block({5: 9.0, 6: g["nbm_example"]}))
    assert s - 127 == g["nbm_example_shared_exp"]
    assert oracle.decode_block(e, s, i)[6] == g["nbm_example_decoded"]
    # shared_exp = -2  <=>  BM in [1,2):  -0.39 / 0.25 = -1.56 -> -1.5
    e, s, i = oracle.encode_block(block({5: 1.25, 6: g["nbm_example"]}))
    assert s - 127 == g["nbm_example_shared_exp_new"]
    assert abs(g["nbm_example"] / 2.0 ** (s - 127) - g["nbm_example_scaled_new"]) < 1e-6
    assert oracle.decode_block(e, s, i)[6] / 2.0 ** (s - 127) == g["nbm_example_code_value_new"]


def test_flush_boundary():
    g = golden()
    lim = int(g["flush_max_exponent"])
    for fmt in (MXFP4, MXFP4P):
        for mant in (1.0, 1.5):
            e, s, i = oracle.encode_block(block({9: -mant * 2.0 ** lim, 3: 2.0 ** (lim - 3)}), fmt)
            assert s == 0 and i == 0 and not e.any()
            assert not oracle.decode_block(e, s, i, fmt).any()
            e, s, i = oracle.encode_block(block({9: -mant * 2.0 ** (lim + 1)}), fmt)
            assert s == 1 and (i == 9 or fmt == MXFP4)
            d = oracle.decode_block(e, s, i, fmt)
            assert d[9] == -mant * 2.0 ** (lim + 1)        # scaled 4 and 6 are on both grids
    # fp32 subnormals and an all-zero block are flushed as well
    assert oracle.encode_block(block({0: 1e-40}))[1] == 0
    assert oracle.encode_block(np.zeros(32, np.float32))[1] == 0
    # decoding tests the zero code before the BM branch: index 0 of a flushed block must not become 4*X
    assert oracle.decode_block(np.zeros(16, np.uint8), 0, 0, MXFP4P)[0] == 0.0
    # largest finite input: e = 127 -> scale byte 252
    assert oracle.encode_block(block({0: 3.0e38}))[1] == 252


# ------------------------------------------------------------------ decoder closed forms
def test_decoder_value_sets_all_nibbles():
    for scale in (1, 100, 127, 130, 252):
        X = 2.0 ** (scale - 127)
        for nib in range(16):
            e = np.zeros(16, np.uint8)
            e[2] = nib << 4                       # element 5 = high nibble of byte 2
            sign = -1.0 if nib & 8 else 1.0
            d = oracle.decode_block(e, scale, 9, MXFP4P)      # BM elsewhere -> element 5 is an E2M1 element
            assert d[5] == sign * X * E2M1_GRID[nib & 7]
            assert not d[:5].any() and not d[6:9].any() and not d[10:].any() and d[9] == 4.0 * X
            d = oracle.decode_block(e, scale, 5, MXFP4P)      # element 5 is the BM
            assert d[5] == sign * X * BM_GRID[nib & 7]
            d = oracle.decode_block(e, scale, 5, MXFP4)       # plain MXFP4 ignores the index
            assert d[5] == sign * X * E2M1_GRID[nib & 7]
            e[2] = nib                            # element 4 = low nibble of byte 2
            assert oracle.decode_block(e, scale, 4, MXFP4P)[4] == sign * X * BM_GRID[nib & 7]
    assert np.isnan(oracle.decode_block(np.zeros(16, np.uint8), 255, 0)).all()


def test_bm_split_identity_eq3():
    # BM = BM_H + BM_L with BM_H = 2^e_max * um[3:2], BM_L = 2^(e_max-2) * um[1:0]; both plain E2M1 numbers.
    for nib in range(16):
        s, m = nib & 8, nib & 7
        h_nib = s | 0b110 | (m >> 2)              # exponent field 11b, mantissa bit = m2
        l_nib = s | (m & 3)                       # exponent field 0 m1, mantissa bit m0
        e = np.zeros(16, np.uint8)
        e[0] = nib
        bm = oracle.decode_block(e, 127, 0, MXFP4P)[0]
        e[0] = h_nib
        hi = oracle.decode_block(e, 127, 0, MXFP4)[0]
        e[0] = l_nib
        lo = oracle.decode_block(e, 127, 0, MXFP4)[0]
        assert bm == hi + lo
        assert abs(hi) in (4.0, 6.0) and abs(lo) in (0.0, 0.5, 1.0, 1.5)


# ------------------------------------------------------------------ encoder vs. brute-force nearest
def brute_force_block(x, fmt):
    x = np.asarray(x, np.float64)
    a = np.abs(x)
    idx = int(np.argmax(a))                       # numpy argmax returns the first maximum
    if a[idx] == 0 or np.floor(np.log2(a[idx])) <= -125:
        return np.zeros(32, np.uint8), 0, 0
    se = int(np.floor(np.log2(a[idx]))) - 2
    nib = np.zeros(32, np.uint8)
    for i in range(32):
        v = a[i] / 2.0 ** se
        code = nearest_code(v, BM_GRID if (fmt == MXFP4P and i == idx) else E2M1_GRID)
        nib[i] = (8 if np.signbit(x[i]) else 0) | code
    return nib, se + 127, idx if fmt == MXFP4P else 0


@pytest.mark.parametrize("fmt", [MXFP4, MXFP4P])
def test_encoder_matches_brute_force_random(fmt):
    rng = np.random.default_rng(1234)
    for trial in range(400):
        kind = trial % 4
        x = rng.standard_normal(32).astype(np.float32)
        if kind == 1:
            x[rng.integers(32)] *= 40
        elif kind == 2:                            # many exact ties: small dyadic numbers
            x = (rng.integers(-32, 33, 32) / 8.0).astype(np.float32)
        elif kind == 3:
            x = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x * np.float32(2.0 ** rng.integers(-60, 60))))
        e, s, i = oracle.encode_block(x, fmt)
        nb, sb, ib = brute_force_block(x, fmt)
        assert s == sb and i == ib, (trial, x)
        assert (nibbles(e) == nb).all(), (trial, x, nibbles(e), nb)


def test_every_tie_point_rounds_to_even_code():
    # midpoints of the E2M1 grid with the BM fixed at 4*X; expected code is the even neighbour
    mids = {0.25: 0, 0.75: 2, 1.25: 2, 1.75: 4, 2.5: 4, 3.5: 6, 5.0: 6}
    for k in (-20, 0, 7):
        X = 2.0 ** k
        for mid, code in mids.items():
            for sgn in (1.0, -1.0):
                x = block({0: 4.0 * X * 1.9, 1: sgn * mid * X})
                e, s, i = oracle.encode_block(x)
                assert i == 0 and nibbles(e)[1] == (8 if sgn < 0 else 0) | code
                # one bf16 ulp either side goes to the nearer neighbour
                up = np.nextafter(np.float32(mid * X), np.float32(np.inf))
                dn = np.nextafter(np.float32(mid * X), np.float32(0))
                lo_code = int(np.flatnonzero(E2M1_GRID < mid)[-1])
                assert nibbles(oracle.encode_block(block({0: 7.6 * X, 1: up}))[0])[1] == lo_code + 1
                assert nibbles(oracle.encode_block(block({0: 7.6 * X, 1: dn}))[0])[1] == lo_code
    # BM grid midpoints 4.25, 4.75, ... and the carry region
    for m in range(8):
        v = 4.25 + 0.5 * m
        want = m if m % 2 == 0 else m + 1
        want = min(want, 7)
        assert nibbles(oracle.encode_block(block({3: v}))[0])[3] == want
    for v in (7.75, 7.8, 7.999):                  # would carry to 8.0: saturates at 7.5, scale untouched
        e, s, i = oracle.encode_block(block({3: -v}))
        assert s == 127 and nibbles(e)[3] == 8 | 7


def test_exhaustive_bf16_patterns_as_nbm_and_bm():
    pats = np.arange(1 << 16, dtype=np.uint16)
    vals = synth.bf16_bits_to_f32(pats)
    finite = np.isfinite(vals)
    for k in (-100, -1, 0, 3, 90):
        X = np.float32(2.0 ** k)
        bmval = np.float32(7.96875) * X           # every |v| < 7.97*X may sit next to it as an ordinary element
        sel = finite & (np.abs(vals) < bmval)
        v = vals[sel]
        n = (len(v) + 30) // 31
        pad = np.zeros(n * 31, np.float32)
        pad[: len(v)] = v
        blocks = np.concatenate([np.full((n, 1), bmval, np.float32), pad.reshape(n, 31)], axis=1)
        e, s, i = oracle.quantize(blocks, MXFP4P)
        assert (s == k + 127).all() and (i == 0).all()
        got = nibbles(e)[:, 1:].reshape(-1)[: len(v)]
        a = np.abs(v.astype(np.float64)) / float(X)
        # vectorised definition of nearest-with-ties-to-even on the 8-point grid
        d = np.abs(a[:, None] - E2M1_GRID[None, :])
        dmin = d.min(axis=1, keepdims=True)
        cand = d == dmin
        first = cand.argmax(axis=1)
        last = 7 - cand[:, ::-1].argmax(axis=1)
        code = np.where(first % 2 == 0, first, last)
        want = code | np.where(np.signbit(v), 8, 0)
        assert (got == want).all()
    # every finite bf16 pattern above the flush limit as the BM of its own block
    ok = finite & (np.abs(vals) >= 2.0 ** -124)
    v = vals[ok]
    blocks = np.zeros((len(v), 32), np.float32)
    blocks[:, 17] = v
    e, s, i = oracle.quantize(blocks, MXFP4P)
    ex = np.floor(np.log2(np.abs(v.astype(np.float64)))).astype(int)
    assert (s[:, 0] == ex - 2 + 127).all() and (i == 17).all()
    a = np.abs(v.astype(np.float64)) / 2.0 ** (ex - 2)
    d = np.abs(a[:, None] - BM_GRID[None, :])
    cand = d == d.min(axis=1, keepdims=True)
    first = cand.argmax(axis=1)
    last = 7 - cand[:, ::-1].argmax(axis=1)
    code = np.where(first % 2 == 0, first, last)
    assert (nibbles(e)[:, 17] == (code | np.where(np.signbit(v), 8, 0))).all()
    # the flushed ones
    v = vals[finite & (np.abs(vals) < 2.0 ** -124)]
    blocks = np.zeros((len(v), 32), np.float32)
    blocks[:, 17] = v
    e, s, i = oracle.quantize(blocks, MXFP4P)
    assert not e.any() and not s.any() and not i.any()


# ------------------------------------------------------------------ invariants of the format
def _mixed_tensor(seed, rows=64, K=256):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, K)).astype(np.float32)
    x[rng.random((rows, K)) < 0.02] *= 30
    x[:, 5] *= 50
    x[3, 32:64] = 0                                # an all-zero block
    x[4, 64:96] = 1e-39                            # a flushed block
    x[5, 96] = x[5, 100] = 7.0                     # equal maxima: lowest index wins
    return x


def test_mxfp4p_differs_from_mxfp4_only_in_the_bm_nibble():
    x = _mixed_tensor(7)
    e4, s4, _ = oracle.quantize(x, MXFP4)
    ep, sp, ip = oracle.quantize(x, MXFP4P)
    assert (s4 == sp).all()                                       # MX+ does not alter the shared scale (Sec. 4.1)
    n4, np_ = nibbles(e4).reshape(64, 8, 32), nibbles(ep).reshape(64, 8, 32)
    diff = n4 != np_
    rows, blks, pos = np.nonzero(diff)
    assert (pos == ip[rows, blks]).all()                          # only the BM position may differ
    live = sp > 0
    bm4 = np.take_along_axis(n4, ip[..., None].astype(np.int64), axis=2)[..., 0]
    assert ((bm4[live] & 0b110) == 0b110).all()                   # MXFP4 BM exponent field is always 11b (Sec. 4.1)
    assert (ip[~live] == 0).all() and ip.max() < 32
    assert ip[5, 3] == 0                                          # 96 % 32 == 0 wins over index 4


def test_block_error_never_worse_than_mxfp4_and_bounds():
    x = _mixed_tensor(11)
    q4, qp = oracle.quantize(x, MXFP4), oracle.quantize(x, MXFP4P)
    d4, dp = oracle.dequantize(q4, MXFP4), oracle.dequantize(qp, MXFP4P)
    err4 = ((d4 - x) ** 2).reshape(64, 8, 32)
    errp = ((dp - x) ** 2).reshape(64, 8, 32)
    assert (errp.sum(-1) <= err4.sum(-1)).all()                   # BM grid contains {4,6}
    assert errp.sum() < 0.9 * err4.sum()
    live = qp[1] > 0
    X = 2.0 ** (qp[1].astype(np.float64) - 127)
    ae = np.abs(dp - x).reshape(64, 8, 32) / X[..., None]
    v = np.abs(x).reshape(64, 8, 32) / X[..., None]
    bm = np.zeros_like(ae, bool)
    np.put_along_axis(bm, qp[2][..., None].astype(np.int64), True, axis=2)
    bm &= live[..., None]
    nbm = ~bm & live[..., None]
    assert (ae[bm & (v < 7.75)] <= 0.25).all() and (ae[bm] <= 0.5).all()
    assert (ae[nbm & (v <= 2)] <= 0.25).all() and (ae[nbm & (v <= 4)] <= 0.5).all()
    assert (ae[nbm & (v <= 6)] <= 1.0).all() and (ae[nbm] < 2.0).all()
    # outlier blocks: the BM dominates the MXFP4 block error, the motivating observation of Sec. 3.2
    big = (v.max(-1) > 40 * np.median(v, axis=-1)) & live
    assert big.sum() > 10
    bm_share = (err4 * bm).sum(-1)[big] / err4.sum(-1)[big]
    assert np.median(bm_share) > 8 / 32.0                          # one element of 32 carries far more than 1/32


def test_scale_equivariance_sign_symmetry_fixed_points():
    x = _mixed_tensor(13)
    x[4, 64:96] = 0
    e, s, i = oracle.quantize(x, MXFP4P)
    for k in (-30, 11):
        e2, s2, i2 = oracle.quantize(x * np.float32(2.0 ** k), MXFP4P)
        live = s > 0
        assert (e2 == e).all() and (i2 == i).all() and (s2[live].astype(int) == s[live].astype(int) + k).all() and not s2[~live].any()
    e3, s3, i3 = oracle.quantize(-x, MXFP4P)
    live = np.repeat(s > 0, 16, axis=1)
    assert (s3 == s).all() and (i3 == i).all() and ((e3 ^ e)[live] == 0x88).all()
    # quantize(dequantize(q)) == q : representable values are fixed points.  Plain MXFP4: always.
    q4 = oracle.quantize(x, MXFP4)
    d4 = oracle.dequantize(q4, MXFP4).astype(np.float32)
    r4 = oracle.quantize(d4, MXFP4)
    assert all((a == b).all() for a, b in zip(q4, r4))
    # MXFP4+: whenever the decoded BM is still the largest magnitude of its block (an ordinary element just below
    # a BM of 5.x can round up to 6 and overtake it; then the block maximum itself changes)
    d = oracle.dequantize((e, s, i), MXFP4P).astype(np.float32)
    e4, s4, i4 = oracle.quantize(d, MXFP4P)
    assert (s4 == s).all()
    db = np.abs(d).reshape(64, 8, 32)
    dbm = np.take_along_axis(db, i[..., None].astype(np.int64), axis=2)[..., 0]
    keeps = dbm >= db.max(-1)
    assert keeps.mean() > 0.8
    again = oracle.dequantize((e4, s4, i4), MXFP4P).reshape(64, 8, 32)
    assert (again[keeps] == d.reshape(64, 8, 32)[keeps]).all()
    same = (i4 == i) & keeps
    assert (e4.reshape(64, 8, 16)[same] == e.reshape(64, 8, 16)[same]).all()


def test_nan_inf_blocks_and_negative_zero():
    x = np.ones((1, 64), np.float32)
    x[0, 40] = np.inf
    e, s, i = oracle.quantize(x, MXFP4P)
    assert s[0, 0] == 127 + 0 - 2 and s[0, 1] == 255 and not e[0, 16:].any() and i[0, 1] == 0
    x[0, 40] = np.nan
    assert oracle.quantize(x, MXFP4)[1][0, 1] == 255
    xb = block({0: 4.0, 1: -0.0, 2: -0.1})
    n = nibbles(oracle.encode_block(xb)[0])
    assert n[1] == 8 and n[2] == 8 and n[3] == 0                  # sign kept on zero codes


def test_bf16_and_strided_and_transposed_entry_points_agree():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((24, 160)).astype(np.float32) * 3
    h = synth.f32_to_bf16_bits(x)
    xf = synth.bf16_bits_to_f32(h)
    qa = oracle.quantize(h, MXFP4P)
    qb = oracle.quantize(xf, MXFP4P)
    assert all((a == b).all() for a, b in zip(qa, qb))
    big = np.zeros((24, 200), np.float32)
    big[:, :160] = xf
    qc = oracle.quantize(big[:, :160], MXFP4P)                    # ld = 200
    assert all((a == b).all() for a, b in zip(qa, qc))
    qt = oracle.quantize_t(np.ascontiguousarray(xf.T), MXFP4P)
    assert all((a == b).all() for a, b in zip(qa, qt))
    qt = oracle.quantize_t(np.ascontiguousarray(h.T), MXFP4)
    assert all((a == b).all() for a, b in zip(oracle.quantize(h, MXFP4), qt))
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((2, 48), np.float32))


# ------------------------------------------------------------------ GEMM
def test_gemm_hand_cases_one_block():
    # A block: BM 7.0 at index 2 (exact on the BM grid), ordinary 1.5 at index 9.
    # B block: BM -5.0 at index 2 or 9 (exact: 4*(1+2/8)), ordinary 3 at the other position... by hand:
    a = block({2: 7.0, 9: 1.5})
    for b_bm, b_other, want in ((2, 9, 7.0 * -5.0 + 1.5 * 3.0), (9, 2, 7.0 * 3.0 + 1.5 * -5.0)):
        b = block({b_bm: -5.0, b_other: 3.0})
        qa, qb = oracle.quantize(a[None], MXFP4P), oracle.quantize(b[None], MXFP4P)
        D, S = oracle.gemm(qa, MXFP4P, qb, MXFP4P)
        assert D[0, 0] == want and S[0, 0] == 35.0 + 4.5 if b_bm == 2 else S[0, 0] == 21.0 + 7.5
    # A-only MX+: B quantized as plain MXFP4 sees -5 -> -4 (5 is a tie between 4 and 6, even code is 4)
    b = block({2: -5.0, 9: 3.0})
    D, _ = oracle.gemm(oracle.quantize(a[None], MXFP4P), MXFP4P, oracle.quantize(b[None], MXFP4), MXFP4)
    assert D[0, 0] == 7.0 * -4.0 + 1.5 * 3.0
    # scales multiply: two blocks with different shared exponents
    a2 = np.concatenate([a, a * 2.0 ** -9])[None]
    b2 = np.concatenate([b, b * 2.0 ** 5])[None]
    D, _ = oracle.gemm(oracle.quantize(a2, MXFP4P), MXFP4P, oracle.quantize(b2, MXFP4P), MXFP4P)
    assert D[0, 0] == (-35.0 + 4.5) * (1 + 2.0 ** -4)


def test_gemm_equals_float64_matmul_of_decoded_operands():
    a, b = synth.tiny()
    qa, qb = oracle.quantize(a, MXFP4P), oracle.quantize(b, MXFP4P)
    D, S = oracle.gemm(qa, MXFP4P, qb, MXFP4P)
    da, db = oracle.dequantize(qa), oracle.dequantize(qb)
    assert D.shape == (16, 256)
    ref = da @ db.T
    assert np.abs(D - ref).max() <= 1e-12 * np.abs(ref).max()
    assert np.allclose(S, np.abs(da) @ np.abs(db).T, rtol=1e-13)
    # and with exact integer arithmetic: all decoded values are multiples of 2^-k, so scale to integers
    kmin = min(int(qa[1][qa[1] > 0].min()), int(qb[1][qb[1] > 0].min())) - 127 - 1
    ia = np.round(da[:4] * 2.0 ** -kmin).astype(object)
    ib = np.round(db[:8] * 2.0 ** -kmin).astype(object)
    exact = np.array([[sum(int(p) * int(q) for p, q in zip(ra, rb)) for rb in ib] for ra in ia], dtype=object)
    got = D[:4, :8]
    for m, n in itertools.product(range(4), range(8)):
        assert float(exact[m, n]) * 2.0 ** (2 * kmin) == got[m, n]
    # sampled entry point agrees with the full one
    rm, rn = np.array([0, 3, 15, 7]), np.array([255, 0, 17, 128])
    Ds, Ss = oracle.gemm_sampled(qa, MXFP4P, qb, MXFP4P, rm, rn)
    assert (Ds == D[rm, rn]).all() and (Ss == S[rm, rn]).all()
    # quantization helps: MXFP4+ product is closer to the unquantized product than MXFP4's (sanity, Sec. 3.2)
    full = a.astype(np.float64) @ b.astype(np.float64).T
    D4, _ = oracle.gemm(oracle.quantize(a, MXFP4), MXFP4, oracle.quantize(b, MXFP4), MXFP4)
    assert np.linalg.norm(D - full) < np.linalg.norm(D4 - full)


def test_gemm_transposed_operand_mistake_would_show():
    # non-square, asymmetric operands: D[m,n] must pair A row m with B row n
    rng = np.random.default_rng(3)
    a = rng.standard_normal((3, 64)).astype(np.float32)
    b = rng.standard_normal((5, 64)).astype(np.float32)
    qa, qb = oracle.quantize(a), oracle.quantize(b)
    D, _ = oracle.gemm(qa, MXFP4P, qb, MXFP4P)
    assert D.shape == (3, 5)
    da, db = oracle.dequantize(qa), oracle.dequantize(qb)
    for m in range(3):
        for n in range(5):
            assert D[m, n] == pytest.approx(float(np.dot(da[m], db[n])), rel=1e-13)


# ------------------------------------------------------------------ MX++ (Sec. 4.3): own shared exponent for the NBMs
from oracle import MXFP4PP  # noqa: E402


def test_mxpp_paper_example():
    """The worked example of Sec. 4.3: BM scale 2^1, largest NBM 0.99 -> e = -2; -0.39 -> -1.56 -> -1.5; 0.99 -> 3.96."""
    g = golden()
    x = block({5: 9.0, 6: g["nbm_example"], 7: 0.99})
    e, s, i = oracle.encode_block(x, MXFP4PP)
    assert s - 127 == g["nbm_example_shared_exp"]                       # the BM's scale is that of MXFP4+
    delta = i >> 5
    assert (i & 31) == 5 and delta < 2 ** g["mxpp_delta_bits"]
    assert (s - 127) - delta == g["mxpp_example_e"] == g["nbm_example_shared_exp_new"]
    d = oracle.decode_block(e, s, i, MXFP4PP)
    xnew = 2.0 ** g["mxpp_example_e"]
    assert d[6] / xnew == g["nbm_example_code_value_new"]               # -1.5
    assert abs(0.99 / xnew - g["scaled_0p99_with_offset"]) < 1e-9 and d[7] / xnew == 4.0   # 3.96 stays in range -> 4
    assert d[5] == 9.0
    # without the +1 offset the scale would be 2^-3 and 0.99 would saturate (7.92 -> 6): the encoder must not do that
    assert d[7] != g["saturated_to"] * 2.0 ** g["shared_exp_for_bm_0p99"]
    # the same block in MXFP4+ loses -0.39 entirely
    e1, s1, i1 = oracle.encode_block(x, MXFP4P)
    assert oracle.decode_block(e1, s1, i1, MXFP4P)[6] == g["nbm_example_decoded"]


def mxpp_delta_by_definition(x):
    """delta from the stated purpose of the rule: the finest NBM scale, at most 7 steps below the BM's, that keeps the
    largest NBM below twice the top binade start (scaled value < 4, so rounding cannot saturate)."""
    a = np.abs(np.asarray(x, np.float64))
    idx = int(np.argmax(a))
    se = int(np.floor(np.log2(a[idx]))) - 2
    a2 = np.delete(a, idx).max()
    best = 0
    for d in range(0, 8):
        if a2 * 2.0 ** (d - se) < 4.0 and se + 127 - d >= 1 and a2 >= 2.0 ** -126:
            best = d
    if a2 < 2.0 ** -126:                                # nothing to scale: the lower clip bound (limited by the E8M0 range)
        best = min(7, se + 127 - 1)
    return idx, se, best


def test_mxpp_matches_definition_by_search_and_keeps_the_bm_of_mxfp4p():
    rng = np.random.default_rng(77)
    for trial in range(600):
        kind = trial % 5
        x = rng.standard_normal(32).astype(np.float32)
        if kind == 1:
            x[rng.integers(32)] *= np.float32(2.0 ** rng.integers(1, 12))          # one outlier of any size
        elif kind == 2:
            x = (rng.integers(-32, 33, 32) / 8.0).astype(np.float32)               # ties everywhere
        elif kind == 3:
            x = np.zeros(32, np.float32)
            x[rng.integers(32)] = rng.standard_normal() * 100                      # lone BM, NBMs all zero
        elif kind == 4:
            x *= np.float32(2.0 ** rng.integers(-125, -110))                       # near the bottom of the E8M0 range
        if np.abs(x).max() == 0 or np.floor(np.log2(np.abs(x).max())) <= -125:
            continue
        e, s, i = oracle.encode_block(x, MXFP4PP)
        e1, s1, i1 = oracle.encode_block(x, MXFP4P)
        idx, se, delta = mxpp_delta_by_definition(x)
        assert s == s1 == se + 127 and (i & 31) == i1 == idx
        assert (i >> 5) == delta, (trial, x, i >> 5, delta)
        nb, nb1 = nibbles(e), nibbles(e1)
        assert nb[idx] == nb1[idx]                                                 # BM code untouched (Sec. 4.3)
        for k in range(32):                                                        # NBMs: nearest point of the finer grid
            if k == idx:
                continue
            want = nearest_code(abs(float(x[k])) / 2.0 ** (se - delta), E2M1_GRID)
            assert (nb[k] & 7) == want and (nb[k] >> 3) == int(np.signbit(x[k])), (trial, k)
        if delta > 0:
            assert (np.delete(nb, idx) & 7).max() <= 6                             # no NBM saturates (code 6 = 4.0)
        if delta == 0:
            assert (nb == nb1).all()                                               # then it IS the MXFP4+ block
        # every element at least as close as in MXFP4+
        d2, d1 = oracle.decode_block(e, s, i, MXFP4PP), oracle.decode_block(e1, s1, i1, MXFP4P)
        assert (np.abs(d2 - x.astype(np.float64)) <= np.abs(d1 - x.astype(np.float64)) + 0.0).all(), (trial, x)


def test_mxpp_clip_bounds_equivariance_and_decode():
    # second-largest element in the BM's binade: e exceeds shared_exp, clipped to it (delta = 0)
    e, s, i = oracle.encode_block(block({0: 7.0, 1: 4.5, 2: 0.3}), MXFP4PP)
    assert i >> 5 == 0
    # NBMs 2^9 or more below the BM: clipped at shared_exp - 7
    e, s, i = oracle.encode_block(block({3: 1024.0, 9: 0.75}), MXFP4PP)
    assert i >> 5 == 7 and (i & 31) == 3
    assert oracle.decode_block(e, s, i, MXFP4PP)[9] == 1.0                        # 0.75 / 2^(8-7) = 0.375 -> code 0.5 -> 1.0
    e1, s1, i1 = oracle.encode_block(block({3: 1024.0, 9: 0.75}), MXFP4P)
    assert oracle.decode_block(e1, s1, i1, MXFP4P)[9] == 0.0                      # 0.75 / 2^8 is lost without MX++
    # scale byte 1 leaves no room below: delta limited by the E8M0 range
    e, s, i = oracle.encode_block(block({0: 1.5 * 2.0 ** -124, 1: 2.0 ** -126}), MXFP4PP)
    assert s == 1 and i >> 5 == 0
    # power-of-two equivariance and sign symmetry carry over
    rng = np.random.default_rng(5)
    x = rng.standard_normal(32).astype(np.float32)
    x[11] *= 300
    e, s, i = oracle.encode_block(x, MXFP4PP)
    e2, s2, i2 = oracle.encode_block(x * np.float32(2.0 ** 9), MXFP4PP)
    assert (e == e2).all() and s2 == s + 9 and i2 == i
    e3, s3, i3 = oracle.encode_block(-x, MXFP4PP)
    assert (nibbles(e3) == (nibbles(e) ^ 8)).all() and s3 == s and i3 == i
    # decoded values are fixed points of the encoder
    d = oracle.decode_block(e, s, i, MXFP4PP).astype(np.float32)
    e4, s4, i4 = oracle.encode_block(d, MXFP4PP)
    assert (oracle.decode_block(e4, s4, i4, MXFP4PP) == d).all()
    # MXFP4+ ignores the reserved bits, MXFP4++ applies them to the NBMs only
    d_plus = oracle.decode_block(e, s, i, MXFP4P)
    k = i & 31
    assert d_plus[k] == d[k] and np.allclose(np.delete(d_plus, k), np.delete(d, k) * 2.0 ** (i >> 5))


def test_mxpp_tensor_entry_points_and_mse():
    a = synth.activations(64, 512, config_id=2, tensor_id=0, dtype="f32")
    q1, q2 = oracle.quantize(a, MXFP4P), oracle.quantize(a, MXFP4PP)
    assert (q1[1] == q2[1]).all() and ((q2[2] & 31) == q1[2]).all()
    d1, d2 = oracle.dequantize(q1, MXFP4P), oracle.dequantize(q2, MXFP4PP)
    err1, err2 = ((d1 - a) ** 2).mean(), ((d2 - a) ** 2).mean()
    assert err2 < err1                                                          # Sec. 4.3 / Sec. 8: finer NBM grid
    qb = oracle.quantize(synth.f32_to_bf16_bits(a), MXFP4PP)
    a_b = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(a))
    assert all((x == y).all() for x, y in zip(qb, oracle.quantize(a_b, MXFP4PP)))


def test_gemm_w4a16_agrees_with_the_quantized_product_when_the_activations_are_representable():
    """If the activations happen to be exactly MXFP4+ values, the conversion-based product and the W4A4 product are the
    same sums; and a hand case in closed form."""
    rng = np.random.default_rng(8)
    a = rng.standard_normal((5, 128)).astype(np.float32)
    a[:, 7] *= 40
    w = (rng.standard_normal((9, 128)) * 0.02).astype(np.float32)
    qa, qw = oracle.quantize(a, MXFP4P), oracle.quantize(w, MXFP4P)
    a_rep = oracle.dequantize(qa, MXFP4P).astype(np.float32)            # exact: at most 4 significant bits each
    D1, S1 = oracle.gemm(qa, MXFP4P, qw, MXFP4P)
    D2, S2 = oracle.gemm_w4a16(a_rep, qw, MXFP4P)
    assert np.allclose(D1, D2, rtol=1e-13, atol=0) and np.allclose(S1, S2, rtol=1e-13, atol=0)
    # bf16 bit patterns and float32 inputs are the same numbers
    D3, _ = oracle.gemm_w4a16(synth.f32_to_bf16_bits(a_rep), qw, MXFP4P)
    assert (D3 == D2).all()
    # one block by hand: a = (3, -2.5) at positions 4 and 20, W row = 7 (BM, exact as 1.75 * 4) and 0.5
    x = block({4: 7.0, 20: 0.5})
    qw1 = oracle.quantize(x[None, :], MXFP4P)
    arow = np.zeros((1, 32), np.float32)
    arow[0, 4], arow[0, 20] = 3.0, -2.5
    D, S = oracle.gemm_w4a16(arow, qw1, MXFP4P)
    assert D[0, 0] == 3.0 * 7.0 - 2.5 * 0.5 and S[0, 0] == 3.0 * 7.0 + 2.5 * 0.5
    # plain MXFP4 loses the BM's extra bits: 7 -> 6
    D4, _ = oracle.gemm_w4a16(arow, oracle.quantize(x[None, :], MXFP4), MXFP4)
    assert D4[0, 0] == 3.0 * 6.0 - 2.5 * 0.5
