"""GPU parity of composed search spaces (Section 3.2): spaces built with Compose from growing module lists and with
Stochastic-Compose from seeds are sampled and every sampled variant is compared with the oracle: whichever modules
a space is made of, its programs compute e0."""
import numpy as np
import pytest

from oracle import compare, oracle as O
from paper_2205_13603_amd import binding as B, inputs as I
from gpu_util import run_variant

pytestmark = pytest.mark.gpu

LADDER = ["multi-level-tiling", "use-mfma", "cache-read", "vectorize", "unroll", "storage-align", "reorder-grid", "cache-write",
          "compute-location", "rfactor"]


def _check(op, space, seed, n, ins, ref, odt, shape, rtol, what):
    for idx in range(n):
        t = B.trace_sample_valid(op, space, seed, idx)
        print(what, "trace", idx, t.decisions(), flush=True)
        got = run_variant(op, space, t, ins, odt, shape)
        if got is None:
            continue
        if odt == "i32":
            compare.assert_int_equal(got, ref, "%s trace %d" % (what, idx))
        elif rtol is None:
            assert np.array_equal(got, ref), "%s trace %d" % (what, idx)
        else:
            compare.assert_float_close(got, ref, rtol, "%s trace %d" % (what, idx))


def test_every_prefix_of_the_module_ladder_gemm():
    """fp16 GEMM with integer-valued inputs (every sum exact, fp32 output): the space of each prefix of the module
    list, from plain tiling on the vector ALUs to the full matrix-core space with rfactor; bit-exact."""
    M, N, K = 256, 192, 512
    A, Bm = I.gemm_inputs(M, N, K, "f16", 9, "ints")
    ref = O.gemm(A, Bm)
    op = B.gemm_op(M, N, K, "f16", "f32")
    for n in range(1, len(LADDER) + 1):
        space, mask = B.space_compose(op, LADDER[:n])
        _check(op, space, 60 + n, 3, [A, Bm], ref, "f32", (M, N), None, "ladder %d (0x%x)" % (n, mask))


def test_stochastically_composed_spaces():
    """Spaces drawn by Stochastic-Compose (6 seeds) for a conv2d + bias + ReLU and for the int8 GEMM."""
    X, W, bias = I.c3(seed=4, H=28, W=28, Cin=32, Cout=32)
    ref = O.conv2d_nhwc(X, W, bias=bias, relu=True, stride=1, pad=1)
    op = B.conv2d_op(1, 28, 28, 32, 32, 3, 3, stride=1, pad=1)
    every = [m["name"] for m in B.modules()]
    masks = set()
    for seed in range(6):
        space, applied = B.space_stochastic_compose(op, every, seed)
        masks.add(space.flags)
        _check(op, space, 70 + seed, 3, [X, W, bias], ref, "f16", (1, 28, 28, 32), compare.RTOL_HALF, "conv %s" % "+".join(applied))
    assert len(masks) >= 3
    A8, B8 = I.gemm_inputs(256, 256, 256, "i8", 5)
    ref8 = O.gemm(A8, B8)
    op8 = B.gemm_op(256, 256, 256, "i8")
    for seed in range(6):
        space, applied = B.space_stochastic_compose(op8, every, 100 + seed)
        _check(op8, space, 80 + seed, 3, [A8, B8], ref8, "i32", (256, 256), None, "int8 %s" % "+".join(applied))
