"""The allocation-free variant of ssv_qsgd_norms (scratch space inside the library) against the entry point that
takes a caller's workspace: same norms, to the bit, on two calls in a row, the second on a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import oracle as ora
import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def test_norms_with_built_in_scratch_equal_norms_with_caller_workspace():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    import paper_1810_05291_amd as sv
    lib = sv.load_library()
    stream = torch.cuda.current_stream(DEV).cuda_stream
    # first a large input (15 rows of the resnet50 size), then a smaller one (3 ragged rows): the second call
    # finds the scratch array full of the first call's partial results
    for (M, d, pad, dtype) in ((15, wl.RESNET50_D, 24, torch.float32), (3, 100_003, 1, torch.bfloat16), (256, 4097, 0, torch.float32)):
        buf = torch.empty((M, d + pad), dtype=dtype, device=DEV)
        g = buf[:, :d]
        for m in range(M):
            g[m] = wl.gaussian((d,), 1e-2 * (m + 1), seed=31 * m + d % 1000, device=DEV).to(dtype)
        g_dt = sv.SSV_F32 if dtype == torch.float32 else sv.SSV_BF16
        for kind in (sv.SSV_QSGD_L2, sv.SSV_QSGD_MAX):
            ref = sv.qsgd_norms(g, kind)                                        # caller-provided workspace
            out = torch.full((M,), -1.0, device=DEV)
            rc = lib.ssv_qsgd_norms_static(g.data_ptr(), g_dt, M, d, g.stride(0), kind, out.data_ptr(), stream)   # raw C ABI
            assert rc == 0
            torch.cuda.synchronize()
            assert torch.equal(out, ref), f"M={M} d={d} kind={kind}"
            # and both agree with the oracle (max: exactly; Euclidean: to 1e-6 relative, expected equal)
            want = ora.qsgd_norms(np.ascontiguousarray(wl.to_numpy(g.contiguous())), kind)
            got = wl.to_numpy(out)
            assert (np.abs(got.astype(np.float64) - want) <= 1e-6 * want).all()
    # beyond the stated limit: a clear error, nothing launched
    big = torch.zeros((257, 64), device=DEV)
    out = torch.full((257,), -1.0, device=DEV)
    assert lib.ssv_qsgd_norms_static(big.data_ptr(), sv.SSV_F32, 257, 64, 64, sv.SSV_QSGD_L2, out.data_ptr(), stream) == -2
    with pytest.raises(sv.SignvoteError):
        sv.qsgd_norms_static(big, sv.SSV_QSGD_L2, out)
    torch.cuda.synchronize()
    assert (out == -1.0).all()
