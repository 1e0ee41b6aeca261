"""mxp_gemm_static: mxp_gemm with its operand images in the library's built-in device array (for callers that cannot
allocate).  Its output must equal mxp_gemm's on the same operands -- the same kernels run in the same order -- on two
calls in a row, the second smaller than the first (the array then still holds the first call's images)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2510_14557_amd import mxp, synth

pytestmark = pytest.mark.gpu


def _operands(M, N, K, seed):
    a = synth.activations(M, K, config_id=3, tensor_id=seed)
    w = synth.weights(N, K, config_id=3, tensor_id=seed + 1, t3_frac=0.001)
    to_dev = lambda x: torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return a, w, mxp.quantize(to_dev(a), mxp.MXFP4P), mxp.quantize(to_dev(w), mxp.MXFP4P)


def test_gemm_static_matches_gemm_on_two_calls_in_a_row():
    assert mxp.gemm_static_capacity() == 64 << 20
    for (M, N, K), dt in (((300, 1000, 2048), torch.float32), ((200, 520, 1024), torch.float32), ((8, 512, 4096), torch.bfloat16)):
        assert mxp.gemm_workspace_size(M, N, K, mxp.MXFP4P, mxp.MXFP4P) <= mxp.gemm_static_capacity()
        a, w, qa, qw = _operands(M, N, K, seed=10 + M % 7)
        want = mxp.gemm(qa, mxp.MXFP4P, qw, mxp.MXFP4P, out_dtype=dt)
        out = torch.full((M, N), float("nan"), dtype=dt, device="cuda")
        mxp.gemm_static(qa, mxp.MXFP4P, qw, mxp.MXFP4P, out)
        torch.cuda.synchronize()
        assert torch.equal(out, want), (M, N, K)
        # and against the oracle, to the bound of the main path
        qh = tuple(t.cpu().numpy() for t in qa), tuple(t.cpu().numpy() for t in qw)
        ref, S = oracle.gemm(qh[0], oracle.MXFP4P, qh[1], oracle.MXFP4P)
        got = out.double().cpu().numpy()
        if dt == torch.float32:
            assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 1e-5
            assert (np.abs(got - ref) <= 2.0 ** -16 * S).all()
    # mixed formats take the same route (plain MXFP4 weights stay 4-bit)
    a, w, qa, qw = _operands(130, 300, 512, seed=3)
    to_dev = lambda x: torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).cuda()
    qw4 = mxp.quantize(to_dev(w), mxp.MXFP4)
    out = torch.empty((130, 300), dtype=torch.float32, device="cuda")
    mxp.gemm_static(qa, mxp.MXFP4P, qw4, mxp.MXFP4, out)
    assert torch.equal(out, mxp.gemm(qa, mxp.MXFP4P, qw4, mxp.MXFP4))


def test_gemm_static_rejects_products_beyond_its_array():
    M, N, K = 8192, 28672, 8192
    assert mxp.gemm_workspace_size(M, N, K, mxp.MXFP4P, mxp.MXFP4P) > mxp.gemm_static_capacity()
    e = torch.zeros(16, dtype=torch.uint8, device="cuda")
    rc = mxp.lib().mxp_gemm_static(M, N, K, e.data_ptr(), e.data_ptr(), e.data_ptr(), mxp.MXFP4P, e.data_ptr(), e.data_ptr(), e.data_ptr(),
                                   mxp.MXFP4P, e.data_ptr(), 0, N, None)
    assert rc == -9 and "scratch" in mxp.status_string(rc)
