"""Seeded synthetic inputs shaped like LLM linear-layer operands.

This module holds NO arithmetic of the MXFP4+ method: it only draws numbers and rounds fp32 to the
bf16 storage type.  Both the HIP path and the CPU oracle are fed the bits produced here; neither
shares anything else.  It imports numpy only (no torch, no HIP library).

Stand-ins: the paper measures on Llama/OPT/... activations and weights (WikiText-2, C4); those are not
available, so tensors follow its description instead -- activation outliers concentrated in a few
channels (Sec. 3.2, Sec. 8 "Scattering Outliers"), Gaussian weights with rare heavy-tailed entries.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 25101455700  # + 10 * config_id + tensor_id


def rng_for(config_id: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(SEED_BASE + 10 * config_id + tensor_id))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + r) >> 16).astype(np.uint16)
    out[nan] = ((u[nan] >> 16) | 0x0040).astype(np.uint16)
    return out


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def outlier_channels(K: int, rng: np.random.Generator) -> np.ndarray:
    """8 outlier channels per 4096 of K; two of them are forced to share one 32-wide block."""
    n = max(2, int(round(8 * K / 4096)))
    ch = rng.choice(K, size=n - 1, replace=False)
    blk = int(ch[0]) // 32
    cand = [c for c in range(blk * 32, blk * 32 + 32) if c not in set(int(v) for v in ch)]
    extra = cand[int(rng.integers(len(cand)))]
    return np.sort(np.append(ch, extra)).astype(np.int64)


def activations(rows: int, K: int, config_id: int, tensor_id: int = 0, outlier_scale: float = 50.0,
                dtype: str = "bf16") -> np.ndarray:
    """N(0,1) with channel-concentrated outliers (fixed channels multiplied by outlier_scale)."""
    rng = rng_for(config_id, tensor_id)
    ch = outlier_channels(K, rng)
    x = rng.standard_normal((rows, K), dtype=np.float32)
    x[:, ch] *= np.float32(outlier_scale)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def weights(N: int, K: int, config_id: int, tensor_id: int = 1, std: float = 0.02, t3_frac: float = 0.0,
            t3_factor: float = 10.0, dtype: str = "bf16") -> np.ndarray:
    """W[N][K] (K-contiguous, the way a linear layer stores it): N(0, std^2); optionally a fraction
    t3_frac of entries replaced by std * t3_factor * Student-t(3) samples."""
    rng = rng_for(config_id, tensor_id)
    w = rng.standard_normal((N, K), dtype=np.float32) * np.float32(std)
    if t3_frac > 0.0:
        n_out = int(round(t3_frac * N * K))
        pos = rng.choice(N * K, size=n_out, replace=False)
        w.reshape(-1)[pos] = (rng.standard_t(3, size=n_out) * std * t3_factor).astype(np.float32)
    return f32_to_bf16_bits(w) if dtype == "bf16" else w


def tiny(config_id: int = 0):
    """Config 'Tiny': A[16x256], B[256x256] fp32 N(0,1), 1% of entries x30.  B is returned as Bt[N][K]."""
    out = []
    for tid, shape in ((0, (16, 256)), (1, (256, 256))):
        rng = rng_for(config_id, tid)
        x = rng.standard_normal(shape, dtype=np.float32)
        mask = rng.random(shape) < 0.01
        x[mask] *= np.float32(30.0)
        out.append(x)
    return out[0], out[1]


# name -> (config_id, M, K, [(weight name, N, std, t3_frac)], number of activation tensors)
CONFIGS = {
    "tiny": dict(config_id=0),
    "decode": dict(config_id=1, M=8, K=4096, weights=[("w", 4096, 0.02, 0.0)]),
    "prefill_attn": dict(config_id=2, M=2048, K=4096, weights=[("wqo", 4096, 0.02, 0.0), ("wkv", 1024, 0.02, 0.0)]),
    "prefill_mlp": dict(config_id=3, M=4096, K=4096, weights=[("wgate", 14336, 0.02, 0.001)]),
    "prefill_mlp_down": dict(config_id=3, M=4096, K=14336, weights=[("wdown", 4096, 0.02, 0.001)], tensor_base=4),
    "large70b": dict(config_id=4, M=8192, K=8192, weights=[("w", 28672, 0.015, 0.0)]),
}


def make(name: str, M: int | None = None, N: int | None = None, dtype: str = "bf16"):
    """Returns (A, {wname: W}) for a named workload; M / N override the row counts (same distributions),
    which is how reduced-size parity cases are produced."""
    c = CONFIGS[name]
    if name == "tiny":
        a, b = tiny(c["config_id"])
        return a, {"b": b}
    base = c.get("tensor_base", 0)
    a = activations(M or c["M"], c["K"], c["config_id"], base + 0, dtype=dtype)
    ws = {}
    for j, (wn, n, std, t3) in enumerate(c["weights"]):
        ws[wn] = weights(N or n, c["K"], c["config_id"], base + 1 + j, std=std, t3_frac=t3, dtype=dtype)
    return a, ws
