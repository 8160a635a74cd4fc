"""GPU parity of depthwise conv2d (configs C5a, C5b) against the CPU oracle."""
import numpy as np
import pytest

from oracle import compare, oracle as O
from paper_2205_13603_amd import binding as B, inputs as I
from gpu_util import run_variant, run_variant_distinct

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,shape,stride", [("c5a", (1, 112, 112, 32), 1), ("c5b", (1, 56, 56, 144), 2)])
def test_c5_depthwise(name, shape, stride):
    X, W = I.dw_inputs(*shape, seed=0)
    ref = O.dwconv2d_nhwc(X, W, stride=stride, pad=1)
    op = B.dwconv2d_op(*shape, stride=stride, pad=1)
    space = op.space()
    for n in range(20):
        t = B.trace_sample_valid(op, space, 0, n)
        print(name, "trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, W], "f32", ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_F32, "%s trace %d" % (name, n))


@pytest.mark.parametrize("stride,pad,k", [(1, 1, 3), (2, 1, 3), (1, 2, 5), (2, 0, 2)])
def test_depthwise_other_geometries_exact(stride, pad, k):
    """Batch 2, 2 instances, odd sizes with factors 3, 5, 7; integer-valued inputs -> exact."""
    N, H, W_, Cc = 2, 21, 15, 12
    g = I.rng(3)
    X = I.small_ints(g, (N, H, W_, Cc), -3, 3, "f32")
    Wt = I.small_ints(g, (k, k, Cc), -3, 3, "f32")
    ref = O.dwconv2d_nhwc(X, Wt, stride=stride, pad=pad)
    op = B.dwconv2d_op(N, H, W_, Cc, k, k, stride=stride, pad=pad)
    space = op.space()
    for n in range(10):
        t = B.trace_sample_valid(op, space, 4, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt], "f32", ref.shape, instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % n


def test_depthwise_instances_with_distinct_inputs():
    ins = [list(I.dw_inputs(1, 12, 10, 8, seed=s)) for s in (5, 6, 7)]
    refs = [O.dwconv2d_nhwc(x, w, stride=1, pad=1) for x, w in ins]
    op = B.dwconv2d_op(1, 12, 10, 8)
    space = op.space()
    for n in range(5):
        t = B.trace_sample_valid(op, space, 14, n)
        got = run_variant_distinct(op, space, t, ins, "f32", (1, 12, 10, 8))
        if got is None:
            continue
        for r in range(3):
            compare.assert_float_close(got[r], refs[r], compare.RTOL_F32, "instance %d trace %d" % (r, n))
