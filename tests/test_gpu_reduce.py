"""GPU parity of the row-reduction kernels (softmax over the last axis, 2-norm per batch entry; Appendix A.2: SFM, NRM)
against the CPU oracle.  fp32 arithmetic on the GPU, float64 in the oracle: fp32 tolerance for fp32 outputs, the
half-precision tolerance where the output is rounded to fp16 / bf16."""
import numpy as np
import pytest

from oracle import compare, oracle as O
from paper_2205_13603_amd import binding as B, inputs as I
from gpu_util import run_variant

pytestmark = pytest.mark.gpu


def test_sfm_config_softmax_256x256():
    g = I.rng(50)
    X = I.normal(g, (1, 256, 256), 2.0, "f32")
    ref = O.softmax(X)
    op = B.softmax_op(1, 256, 256)
    space = op.space()
    assert space.family == B.FAM_REDUCE
    seen = set()
    for n in range(24):
        t = B.trace_sample_valid(op, space, 50, n)
        p = B.trace_validate(op, space, t)
        seen.add((p.cache_read, p.tk[2] > 64))
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X], "f32", ref.shape, instances=2)
        if got is None:
            continue
        compare.assert_float_close(got[0], ref, compare.RTOL_F32, "softmax trace %d" % n)
        assert np.array_equal(got[0], got[1])
        assert np.max(np.abs(got[0].sum(-1) - 1.0)) < 1e-5
    assert {c for c, _ in seen} == {0, 1}


def test_nrm_config_norm_256x256():
    g = I.rng(51)
    X = I.normal(g, (1, 256, 256), 1.0, "f32")
    ref = O.norm(X)
    op = B.norm_op(1, 256, 256)
    space = op.space()
    for n in range(20):
        t = B.trace_sample_valid(op, space, 51, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X], "f32", ref.shape, instances=3)
        if got is None:
            continue
        for r in range(3):
            compare.assert_float_close(got[r], ref, compare.RTOL_F32, "norm trace %d" % n)


def test_groups_wider_than_a_wavefront_and_exact_cases():
    """Rows reduced by 128 and 256 lanes (partial results of the wavefronts meet in LDS), several rows per group in
    flight, both register modes.  Uniform rows of 256 elements give exactly 1/256; sums of squares of small integers
    are exact in fp32."""
    op = B.softmax_op(2, 64, 256)
    space = op.space()
    g = I.rng(52)
    X = I.normal(g, (2, 64, 256), 3.0, "f32")
    X[1, 5, :] = 1.25                  # a uniform row
    X[0, 7, :] = -100.0
    X[0, 7, 100] = 100.0               # one dominant element: no overflow, exp(-200) underflows to 0 in fp32
    ref = O.softmax(X)
    for n, vals in enumerate([[[32, 1, 4, 1], [1, 1, 256, 1], [0]], [[16, 2, 2, 2], [1, 1, 128, 2], [1]],
                              [[8, 4, 4, 1], [1, 2, 128, 1], [1]], [[4, 2, 8, 2], [2, 1, 128, 1], [0]],
                              [[2, 1, 16, 4], [1, 1, 64, 4], [1]], [[1, 2, 64, 1], [4, 4, 16, 1], [0]]]):
        t = B.make_trace(space, vals)
        print("softmax trace", n, vals, flush=True)
        got = run_variant(op, space, t, [X], "f32", ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_F32, "softmax wide trace %d" % n)
        assert np.all(got[1, 5] == 1.0 / 256)
        assert got[0, 7, 100] == 1.0 and np.all(np.delete(got[0, 7], 100) == 0.0)
    op = B.norm_op(4, 96, 128)
    space = op.space()
    Xi = I.small_ints(g, (4, 96, 128), -3, 3, "f32")
    ref = O.norm(Xi)
    for n, vals in enumerate([[[4, 1, 1, 1], [3, 4, 256, 4]], [[2, 1, 2, 1], [6, 4, 128, 4]], [[1, 1, 4, 1], [48, 1, 256, 1]],
                              [[1, 2, 1, 2], [12, 1, 1024, 1]], [[1, 1, 1, 4], [6, 8, 64, 4]]]):
        t = B.make_trace(space, vals)
        print("norm trace", n, vals, flush=True)
        got = run_variant(op, space, t, [Xi], "f32", ref.shape, instances=2)
        if got is None:
            continue
        compare.assert_float_close(got[0], ref, 2e-7, "norm ints trace %d" % n)  # exact sum, one rounding in the root
        assert np.array_equal(got[0], got[1])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_softmax_and_norm_half_inputs_odd_shapes(dtype):
    """Extents with factors 3 and 5; the softmax output is rounded once to the input type."""
    g = I.rng(53)
    X = I.normal(g, (3, 20, 96), 2.0, dtype)
    ref = O.softmax(X, bf16=dtype == "bf16")
    op = B.softmax_op(3, 20, 96, dtype)
    space = op.space()
    for n in range(8):
        t = B.trace_sample_valid(op, space, 53, n)
        print("softmax", dtype, "trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X], dtype, ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "softmax %s trace %d" % (dtype, n))
    op = B.softmax_op(3, 20, 96, dtype, "f32")
    space = op.space()
    for n in range(4):
        t = B.trace_sample_valid(op, space, 54, n)
        got = run_variant(op, space, t, [X], "f32", ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_F32, "softmax %s -> f32 trace %d" % (dtype, n))
    ref = O.norm(X, bf16=dtype == "bf16")
    op = B.norm_op(3, 20, 96, dtype)
    space = op.space()
    for n in range(8):
        t = B.trace_sample_valid(op, space, 55, n)
        print("norm", dtype, "trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X], "f32", ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_F32, "norm %s trace %d" % (dtype, n))
