"""GPU parity of the rfactor decision (Table 2: factorising the reduction across a loop): the k0 loop of one output
tile is shared by S workgroups that write partial sums to a workspace, and a second kernel adds them in run order.
Every staging mode of the matrix-core kernels, GEMM / batched / int8 / conv2d with bias and ReLU, several
instances with distinct data; the workspace is filled with NaN patterns first, so a partial sum that is read
before it is written shows."""
import numpy as np
import pytest

from oracle import compare, oracle as O
from paper_2205_13603_amd import binding as B, inputs as I
from gpu_util import run_variant, run_variant_distinct

pytestmark = pytest.mark.gpu

FLAGS = B.SPACE_DEFAULT | B.SPACE_RFACTOR


def test_gemm_exact_for_every_staging_mode():
    """Integer-valued fp16 inputs, fp32 output: every partial sum and their sum are exact, so the result must
    equal the oracle bit for bit for rfactor 2, 4 and 8 in every cache-read mode."""
    M, N, K = 192, 160, 1024
    g = I.rng(5)
    ins = [[I.small_ints(g, (M, K), -2, 2, "f16"), I.small_ints(g, (K, N), -2, 2, "f16")] for _ in range(3)]
    refs = [O.gemm(a, b) for a, b in ins]
    op = B.gemm_op(M, N, K, "f16", "f32")
    sp = op.space(FLAGS)

    def mk(mfma, i, j, k, unroll=0, cache=2, vec=8, vec_b=8, pad=0, reorder=0, rf=2):
        return B.make_trace(sp, [[mfma], i, j, k, [unroll], [cache], [vec], [vec_b], [pad], [reorder], [0], [rf]])

    traces = [
        mk(161632, [6, 1, 2, 1], [5, 2, 1, 1], [8, 2, 1, 2], cache=1, rf=2),
        mk(161632, [6, 1, 2, 1], [5, 2, 1, 1], [16, 1, 2, 1], cache=2, unroll=64, pad=1, rf=8),
        mk(323216, [3, 2, 1, 1], [5, 1, 1, 1], [16, 1, 1, 4], cache=3, pad=2, reorder=2, rf=4),     # two register sets
        mk(323216, [3, 2, 1, 1], [5, 1, 1, 1], [32, 1, 2, 1], cache=3, unroll=64, reorder=1, rf=8),  # pipelined steps, runs of 4
        mk(161632, [3, 2, 2, 1], [5, 1, 2, 1], [16, 1, 1, 2], cache=4, pad=1, rf=4),                  # ping-pong groups
        mk(161632, [6, 1, 2, 1], [5, 1, 2, 1], [16, 1, 2, 1], cache=5, rf=2),                         # direct-to-LDS rings
        mk(323216, [3, 2, 1, 1], [5, 1, 1, 1], [16, 1, 1, 4], cache=6, unroll=16, reorder=2, rf=8),
        mk(161632, [6, 1, 2, 1], [5, 1, 2, 1], [8, 1, 2, 2], cache=7, unroll=64, rf=4),
        mk(161616, [12, 1, 1, 1], [10, 1, 1, 1], [64, 1, 1, 1], cache=1, vec=4, vec_b=4, rf=8),
        mk(323208, [6, 1, 1, 1], [5, 1, 1, 1], [32, 2, 2, 1], cache=2, vec=4, vec_b=2, rf=4),
    ]
    for n, t in enumerate(traces):
        p = B.trace_validate(op, sp, t)
        print("trace", n, t.decisions(), "grid", p.grid[0], flush=True)
        got = run_variant_distinct(op, sp, t, ins, "f32", (M, N))
        if got is None:
            continue
        for r in range(3):
            assert np.array_equal(got[r], refs[r]), "trace %d instance %d" % (n, r)


def test_c2_shape_and_batched_and_int8():
    """Config 2's shape with fp16 output (one rounding, after the partial sums are added), attention-score batches,
    and int8 -> int32 bit for bit."""
    A, Bm = I.c2(seed=3)
    op = B.gemm_op(1024, 1024, 1024, "f16")
    sp = op.space(FLAGS)
    ref = None
    for n, (i, j, k, cache, rf) in enumerate([([8, 2, 2, 1], [8, 2, 2, 1], [16, 1, 1, 4], 5, 4),
                                              ([16, 1, 2, 1], [8, 2, 2, 1], [32, 1, 2, 1], 3, 8),
                                              ([8, 2, 2, 1], [16, 1, 2, 1], [16, 1, 2, 2], 2, 2)]):
        t = B.make_trace(sp, [[323216], i, j, k, [64], [cache], [8], [8], [0 if cache >= 5 else 1], [2], [0], [rf]])
        print("c2 trace", n, t.decisions(), flush=True)
        got = run_variant(op, sp, t, [A, Bm], "f16", (1024, 1024), instances=2)
        if got is None:
            continue
        ref = O.gemm(A, Bm) if ref is None else ref
        compare.assert_float_close(got[0], ref, compare.RTOL_HALF, "C2 rfactor trace %d" % n)
        assert np.array_equal(got[0], got[1])
    Q, Kk = I.c4a(seed=2)
    op = B.bmm_op(12, 128, 128, 64, True, "f16")
    sp = op.space(FLAGS)
    ref = O.bmm(Q, Kk, trans_b=True)
    for idx in range(12):
        t = B.trace_sample_valid(op, sp, 41, idx)
        print("c4a trace", idx, t.decisions(), flush=True)
        got = run_variant(op, sp, t, [Q, Kk], "f16", (12, 128, 128))
        if got is not None:
            compare.assert_float_close(got, ref, compare.RTOL_HALF, "C4a rfactor trace %d" % idx)
    A8, B8 = I.c4c(seed=4)
    op = B.gemm_op(512, 512, 512, "i8")
    sp = op.space(FLAGS)
    ref = O.gemm(A8, B8)
    pos = sp.n_slots - 1
    n_split = 0
    for idx in range(16):
        t = B.trace_sample_valid(op, sp, 42, idx)
        n_split += sp.slots[pos].candidates[t.d[pos].v[0]] > 1
        print("c4c trace", idx, t.decisions(), flush=True)
        got = run_variant(op, sp, t, [A8, B8], "i32", (512, 512))
        if got is not None:
            compare.assert_int_equal(got, ref, "C4c rfactor trace %d" % idx)
    assert n_split >= 4, "the sampler should draw rfactor > 1 often enough for this test to mean something"


def test_conv_bias_relu_with_split_reduction():
    """conv2d + bias + ReLU: the epilogue moves into the adding kernel (bias and ReLU after the last partial sum);
    im2col staging and the resident input patch; grouped convolution (a group is a batch entry); exact on
    small-integer inputs, then config 3's shape within the fp16 tolerance."""
    g = I.rng(8)
    X = I.small_ints(g, (1, 14, 16, 32), 0, 2, "f16")
    W = I.small_ints(g, (3, 3, 32, 32), -1, 1, "f16")
    bias = g.integers(-40, 40, size=(32,)).astype(np.float32)
    ref = O.conv2d_nhwc(X, W, bias=bias, relu=True, stride=1, pad=1)
    assert (ref == 0).mean() > 0.05 and (ref > 0).mean() > 0.3  # the ReLU is active on some outputs only
    op = B.conv2d_op(1, 14, 16, 32, 32, 3, 3, stride=1, pad=1, out_dtype="f32")
    sp = op.space(FLAGS)
    # K = 3 * 3 * 32 = 288: 18 steps of the 16-deep intrinsic, 36 of the 8-deep one
    for n, (mfma, i, k, cache, cat, rf) in enumerate([(161616, [7, 1, 2, 1], [18, 1, 1, 1], 1, 0, 2), (161616, [7, 1, 2, 1], [6, 1, 3, 1], 3, 1, 2),
                                                      (323208, [7, 1, 1, 1], [36, 1, 1, 1], 2, 1, 4), (323208, [7, 1, 1, 1], [12, 3, 1, 1], 2, 0, 4),
                                                      (161616, [14, 1, 1, 1], [18, 1, 1, 1], 4, 0, 2), (323208, [1, 7, 1, 1], [8, 1, 1, 1] + [], 1, 0, 8)][:5]):
        t = B.make_trace(sp, [[mfma], i, [1, 1, 2, 1] if mfma != 323208 else [1, 1, 1, 1], k, [0], [cache], [8], [8], [1], [0], [0], [cat], [rf]])
        print("conv trace", n, t.decisions(), flush=True)
        got = run_variant(op, sp, t, [X, W, bias], "f32", (1, 14, 16, 32), instances=3)
        if got is None:
            continue
        for r in range(3):
            assert np.array_equal(got[r], ref), "conv trace %d instance %d" % (n, r)
    Xc, Wc, bc = I.c3(seed=6)
    op = B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1)
    sp = op.space(FLAGS)
    ref = None
    for n, (i, k, cache, cat, rf) in enumerate([([49, 1, 2, 1], [12, 1, 1, 3], 2, 1, 4), ([98, 1, 1, 1], [36, 1, 1, 1], 3, 0, 2),
                                                ([14, 1, 7, 1], [18, 1, 2, 1], 1, 1, 2)]):
        t = B.make_trace(sp, [[323216], i, [1, 1, 2, 1], k, [0], [cache], [8], [8], [1], [2], [0], [cat], [rf]])
        print("c3 trace", n, t.decisions(), flush=True)
        got = run_variant(op, sp, t, [Xc, Wc, bc], "f16", (1, 56, 56, 64), instances=2)
        if got is None:
            continue
        ref = O.conv2d_nhwc(Xc, Wc, bias=bc, relu=True, stride=1, pad=1) if ref is None else ref
        compare.assert_float_close(got[1], ref, compare.RTOL_HALF, "C3 rfactor trace %d" % n)
    Xg, Wg, bg = I.grp(seed=7)
    op = B.conv2d_op(1, 56, 56, 64, 128, 3, 3, stride=2, pad=1, groups=4)
    sp = op.space(FLAGS)
    ref = O.conv2d_nhwc(Xg, Wg, bias=bg, relu=True, stride=2, pad=1, groups=4)
    for idx in range(8):
        t = B.trace_sample_valid(op, sp, 43, idx)
        print("grouped trace", idx, t.decisions(), flush=True)
        got = run_variant(op, sp, t, [Xg, Wg, bg], "f16", (1, 28, 28, 128))
        if got is not None:
            compare.assert_float_close(got, ref, compare.RTOL_HALF, "grouped rfactor trace %d" % idx)
