"""ms_variant_launch_static: the launch that allocates nothing (its workspace is an array inside the library's own
device image) must give exactly what ms_variant_launch gives with a caller-provided workspace, on two calls in a
row that share the built-in array, the second with a smaller input."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2205_13603_amd import binding as B, devmem, inputs as I

pytestmark = pytest.mark.gpu


def _variant():
    M, N, K = 256, 192, 512
    op = B.gemm_op(M, N, K, "f16")
    sp = op.space(B.SPACE_DEFAULT | B.SPACE_RFACTOR)
    t = B.make_trace(sp, [[161632], [4, 2, 2, 1], [3, 2, 2, 1], [8, 1, 1, 2], [0], [2], [8], [8], [1], [0], [0], [4]])
    return op, sp, t, (M, N, K)


def test_launch_static_matches_launch_on_two_calls_in_a_row():
    op, sp, t, (M, N, K) = _variant()
    v = B.Variant(op, sp, t)
    if not devmem.gpu_available():
        import gpu_util
        gpu_util.PRECOMPILED_ONLY = True
        return
    import torch
    per_instance = v.workspace_bytes()
    assert per_instance == 4 * M * N * 4
    stream = devmem.current_stream()
    g = I.rng(123)
    with pytest.raises(B.MsError, match="ms_variant_prepare"):
        v.launch_static([8, 8], 8)                      # set-up has not run: refused, nothing launched
    v.prepare()
    for R in (5, 2):                                    # the second call is smaller and finds the first call's partial sums
        A = np.stack([I.normal(g, (M, K), 0.5, "f16") for _ in range(R)])
        Bm = np.stack([I.normal(g, (K, N), 0.5, "f16") for _ in range(R)])
        dA, dB = devmem.to_device(A), devmem.to_device(Bm)
        ws = torch.empty(per_instance * R, dtype=torch.uint8, device="cuda")
        ws.fill_(0xFF)
        want = devmem.empty_output((M, N), "f16", R, poison=True)
        v.launch([dA.data_ptr(), dB.data_ptr()], want.data_ptr(), instances=R, stream=stream, workspace=ws.data_ptr())
        got = devmem.empty_output((M, N), "f16", R, poison=True)
        v.launch_static([dA.data_ptr(), dB.data_ptr()], got.data_ptr(), instances=R, stream=stream)
        w, h = devmem.to_host(want, "f16"), devmem.to_host(got, "f16")
        assert np.all(np.isfinite(h)) and np.array_equal(w, h), "R = %d" % R
        from oracle import compare
        for r in range(R):
            compare.assert_float_close(h[r], O.gemm(A[r], Bm[r]), compare.RTOL_HALF, "static launch R %d instance %d" % (R, r))
    # a request beyond the built-in workspace is refused with the sizes in the message, before anything is launched
    too_many = B.STATIC_WORKSPACE_BYTES // per_instance + 1
    with pytest.raises(B.MsError, match="built-in one holds"):
        v.launch_static([dA.data_ptr(), dB.data_ptr()], got.data_ptr(), instances=too_many, stream=stream)
    # a variant without a split reduction needs no workspace and takes the same entry point
    sp1 = op.space()
    t1 = B.make_trace(sp1, [[161632], [4, 2, 2, 1], [3, 2, 2, 1], [8, 1, 1, 2], [0], [2], [8], [8], [1], [0], [0]])
    v1 = B.Variant(op, sp1, t1)
    v1.prepare()
    got1 = devmem.empty_output((M, N), "f16", 2, poison=True)
    v1.launch_static([dA.data_ptr(), dB.data_ptr()], got1.data_ptr(), instances=2, stream=stream)
    compare.assert_float_close(devmem.to_host(got1, "f16")[1], O.gemm(A[1], Bm[1]), compare.RTOL_HALF, "static launch, rfactor 1")
