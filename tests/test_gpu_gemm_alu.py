"""GPU parity of the ALU GEMM kernel family against the CPU oracle (config C1 and friends)."""
import numpy as np
import pytest

from oracle import compare, oracle as O
from paper_2205_13603_amd import binding as B, inputs as I

pytestmark = pytest.mark.gpu


def run_gemm(op, space, trace, A, Bm, out_dtype, shape, instances=1):
    from gpu_util import run_variant
    return run_variant(op, space, trace, [A, Bm], out_dtype, shape, instances)


def test_c1_sixteen_traces():
    """Config C1: fp32 GEMM 128^3, U[-1,1] from seed 0, 16 traces from seed 0 (tiles + unroll only)."""
    A, Bm = I.c1(seed=0)
    ref = O.gemm(A, Bm)
    op = B.gemm_op(128, 128, 128, "f32")
    space = op.space(B.SPACE_UNROLL)
    for idx in range(16):
        t = B.trace_sample_valid(op, space, 0, idx)
        print("trace", idx, t.decisions(), flush=True)
        got = run_gemm(op, space, t, A, Bm, "f32", (128, 128))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_F32, "C1 trace %d" % idx)


def test_c1_full_space_traces():
    A, Bm = I.c1(seed=0)
    ref = O.gemm(A, Bm)
    op = B.gemm_op(128, 128, 128, "f32")
    space = op.space()
    for idx in range(24):
        t = B.trace_sample_valid(op, space, 1, idx)
        print("trace", idx, t.decisions(), flush=True)
        got = run_gemm(op, space, t, A, Bm, "f32", (128, 128))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_F32, "C1 full-space trace %d" % idx)


def test_ragged_shape_exact_small_ints_with_instances():
    """Non power-of-two extents (120 = 2^3*3*5, 84, 90), 3 instances; small-integer inputs make every
    summation order exact, so the result must equal the oracle bit for bit."""
    M, N, K = 120, 84, 90
    A, Bm = I.gemm_inputs(M, N, K, "f32", 3, "ints")
    ref = O.gemm(A, Bm)
    op = B.gemm_op(M, N, K, "f32")
    space = op.space()
    for idx in range(12):
        t = B.trace_sample_valid(op, space, 2, idx)
        print("trace", idx, t.decisions(), flush=True)
        got = run_gemm(op, space, t, A, Bm, "f32", (M, N), instances=3)
        if got is None:
            continue
        for r in range(3):
            assert np.array_equal(got[r], ref), "instance %d trace %d" % (r, idx)


@pytest.mark.parametrize("dtype,out", [("f16", "f16"), ("bf16", "bf16"), ("f16", "f32"), ("i8", "i32")])
def test_alu_other_dtypes(dtype, out):
    M, N, K = 64, 48, 96
    A, Bm = I.gemm_inputs(M, N, K, dtype, 4, "normal", 1.0)
    ref = O.gemm(A, Bm, bf16=(dtype == "bf16"))
    op = B.gemm_op(M, N, K, dtype, out)
    space = op.space(B.SPACE_DEFAULT & ~B.SPACE_TENSORIZE)
    assert space.family == B.FAM_GEMM_ALU
    for idx in range(6):
        t = B.trace_sample_valid(op, space, 5, idx)
        print("trace", idx, t.decisions(), flush=True)
        got = run_gemm(op, space, t, A, Bm, out, (M, N))
        if got is None:
            continue
        if dtype == "i8":
            compare.assert_int_equal(got, ref, "i8 trace %d" % idx)
        else:
            compare.assert_float_close(got, ref, compare.RTOL_HALF if out != "f32" else 1e-4, "%s trace %d" % (dtype, idx))


def test_bmm_nt_and_nn_alu_fp32():
    nb, M, N, K = 3, 40, 24, 36
    g = I.rng(6)
    Q = I.uniform(g, (nb, M, K), -1, 1, "f32")
    Kt = I.uniform(g, (nb, N, K), -1, 1, "f32")
    V = I.uniform(g, (nb, K, N), -1, 1, "f32")
    from paper_2205_13603_amd import devmem
    for trans_b, Bm in [(True, Kt), (False, V)]:
        ref = O.bmm(Q, Bm, trans_b=trans_b)
        op = B.bmm_op(nb, M, N, K, trans_b, "f32")
        space = op.space()
        for idx in range(8):
            t = B.trace_sample_valid(op, space, 7, idx)
            print("trans_b", trans_b, "trace", idx, t.decisions(), flush=True)
            got = run_gemm(op, space, t, Q, Bm, "f32", (nb, M, N))
            if got is None:
                continue
            compare.assert_float_close(got, ref, compare.RTOL_F32, "bmm trans_b=%s trace %d" % (trans_b, idx))


@pytest.mark.parametrize("target_us", [100.0, 1000.0, 5000.0])
def test_event_timing_recovers_a_known_duration(target_us):
    """A kernel that waits for `target_us` of the device's constant-rate wall clock, timed with the routine
    that ms_measure uses: every repeat must report the target plus at most the launch overhead."""
    from paper_2205_13603_amd import devmem
    if not devmem.gpu_available():
        pytest.skip("no GPU in this process")
    import torch
    scratch = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    res = B.calibrate_timer(target_us, scratch.data_ptr(), warmup=2, repeats=7, launches_per_repeat=1, stream=devmem.current_stream())
    print("target", target_us, "min", res.min_us, "median", res.median_us, "mean", res.mean_us, flush=True)
    assert res.n == 7
    assert target_us - 1.0 <= res.min_us <= res.median_us
    assert res.median_us <= target_us * 1.01 + 40.0
    # several launches per repeat: the per-launch figure is the total divided by the count
    res4 = B.calibrate_timer(target_us, scratch.data_ptr(), warmup=1, repeats=3, launches_per_repeat=4, stream=devmem.current_stream())
    assert target_us - 1.0 <= res4.min_us <= target_us * 1.01 + 40.0
