"""GPU parity of the matrix-core GEMM/BMM kernel family against the CPU oracle (configs C2, C4a, C4b, C4c)."""
import numpy as np
import pytest

from oracle import compare, oracle as O
from paper_2205_13603_amd import binding as B, inputs as I
from gpu_util import run_variant, run_variant_distinct

pytestmark = pytest.mark.gpu

F16_INTRINS = [161616, 323208, 161632, 323216]
I8_INTRINS = [161632, 323216, 161664, 323232]


def traces_covering_intrinsics(op, space, seed, per_intrin, intrins):
    """Valid traces from the seeded sampler, `per_intrin` for each tensorize candidate."""
    want = {c: per_intrin for c in intrins}
    out, idx = [], 0
    while any(want.values()) and idx < 5000:
        t = B.trace_sample_valid(op, space, seed, idx)
        idx += 1
        code = space.slots[0].candidates[t.d[0].v[0]]
        if want.get(code, 0) > 0:
            want[code] -= 1
            out.append(t)
    assert not any(want.values()), want
    return out


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_small_gemm_all_intrinsics(dtype):
    M, N, K = 192, 160, 224  # several tiles, factors of 3, 5, 7 in the tile counts
    A, Bm = I.gemm_inputs(M, N, K, dtype, 1, "normal", 1.0)
    ref = O.gemm(A, Bm, bf16=(dtype == "bf16"))
    op = B.gemm_op(M, N, K, dtype)
    space = op.space()
    assert space.family == B.FAM_GEMM_MFMA
    for n, t in enumerate(traces_covering_intrinsics(op, space, 3, 4, F16_INTRINS)):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], dtype, (M, N))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "%s trace %d" % (dtype, n))


def test_small_gemm_exact_on_small_ints_fp32_out_instances():
    """Integer-valued fp16 inputs: every partial sum is exact in fp32, so any trace must equal the oracle
    bit for bit; 2 instances; fp32 output."""
    M, N, K = 128, 96, 160
    A, Bm = I.gemm_inputs(M, N, K, "f16", 2, "ints")
    ref = O.gemm(A, Bm)
    op = B.gemm_op(M, N, K, "f16", "f32")
    space = op.space()
    for n, t in enumerate(traces_covering_intrinsics(op, space, 4, 3, F16_INTRINS)):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "f32", (M, N), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % n


def test_c2_fp16_gemm_1024():
    """Config C2: fp16 GEMM 1024^3, fp32 accumulate, inputs 0.1*N(0,1)."""
    A, Bm = I.c2(seed=0)
    op = B.gemm_op(1024, 1024, 1024, "f16")
    space = op.space()
    traces = traces_covering_intrinsics(op, space, 0, 3, F16_INTRINS)

    def mk(mfma, i, j, k, unroll=0, cache=2, vec=8, vec_b=8, pad=0, reorder=0, cw=0):
        return B.make_trace(space, [[mfma], i, j, k, [unroll], [cache], [vec], [vec_b], [pad], [reorder], [cw]])

    traces.append(mk(323216, [4, 2, 2, 2], [4, 2, 2, 2], [16, 1, 2, 2], unroll=16, pad=1, reorder=2))
    traces.append(mk(323216, [4, 2, 2, 2], [4, 2, 2, 2], [16, 1, 4, 1], unroll=64, pad=2, reorder=2))  # software pipelined, swizzled
    traces.append(mk(161632, [8, 2, 2, 2], [8, 1, 2, 4], [8, 2, 2, 1], unroll=64, cache=1, vec=4, vec_b=2))
    traces.append(mk(161632, [4, 4, 4, 1], [8, 4, 2, 1], [16, 2, 1, 1], unroll=16, cache=1, vec=8, vec_b=2, pad=2, reorder=1))
    traces.append(mk(323216, [4, 1, 2, 4], [4, 1, 8, 1], [16, 1, 1, 4], vec=8, vec_b=1, pad=1, reorder=2, cw=1))
    traces.append(mk(323216, [4, 1, 2, 4], [4, 1, 8, 1], [16, 1, 1, 4], cache=3, vec=8, vec_b=2, pad=1, reorder=2, cw=1))
    traces.append(mk(161632, [8, 2, 2, 2], [8, 1, 2, 4], [32, 1, 1, 1], cache=3, vec=8, vec_b=4, pad=2))
    traces.append(mk(323216, [4, 1, 4, 2], [4, 2, 2, 2], [16, 1, 1, 4], cache=4, vec=8, vec_b=4, pad=1, reorder=2, cw=1))  # ping-pong
    traces.append(mk(161632, [8, 2, 2, 2], [8, 1, 2, 4], [16, 1, 1, 2], cache=4, vec=8, vec_b=2, pad=2))
    # direct-to-LDS ring, 2 / 3 / 4 stages, both intrinsics with 8-element fragments
    traces.append(mk(323216, [4, 2, 2, 2], [4, 2, 2, 2], [16, 1, 4, 1], unroll=64, cache=5, pad=0, reorder=2, cw=1))
    traces.append(mk(161632, [8, 2, 2, 2], [8, 2, 2, 2], [16, 1, 2, 1], unroll=0, cache=6, pad=0, reorder=0))
    traces.append(mk(323216, [8, 1, 4, 1], [4, 2, 2, 2], [32, 1, 1, 2], unroll=16, cache=7, pad=0, reorder=1, cw=1))
    traces.append(mk(161632, [8, 2, 4, 1], [8, 4, 2, 1], [8, 2, 2, 1], unroll=64, cache=5, pad=0, reorder=2))  # BK = 128
    # persistent workgroups on the direct-to-LDS ring
    traces.append(mk(323216, [4, 1, 4, 2], [4, 2, 2, 2], [16, 1, 4, 1], unroll=64, cache=5, pad=0, reorder=3, cw=0))
    traces.append(mk(161632, [8, 2, 4, 1], [8, 4, 2, 1], [16, 1, 2, 1], unroll=64, cache=6, pad=0, reorder=3, cw=1))
    ref = None
    for n, t in enumerate(traces):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "f16", (1024, 1024))
        if got is None:
            continue
        if ref is None:
            ref = O.gemm(A, Bm)
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "C2 trace %d" % n)


def test_c4a_c4b_attention_bmm():
    """Config C4a/b: 12 heads, S = Q.K^T (reduction index contiguous in both) and O = P.V."""
    Q, Kk = I.c4a(seed=0)
    P, V = I.c4b(seed=0)
    for name, trans_b, X, Y, shape in [("c4a", True, Q, Kk, (12, 128, 128)), ("c4b", False, P, V, (12, 128, 64))]:
        ref = O.bmm(X, Y, trans_b=trans_b)
        op = B.bmm_op(12, shape[1], shape[2], X.shape[2], trans_b, "f16")
        space = op.space()
        for n, t in enumerate(traces_covering_intrinsics(op, space, 5, 3, F16_INTRINS)):
            print(name, "trace", n, t.decisions(), flush=True)
            got = run_variant(op, space, t, [X, Y], "f16", shape)
            if got is None:
                continue
            compare.assert_float_close(got, ref, compare.RTOL_HALF, "%s trace %d" % (name, n))


def test_c4a_fused_transpose_layout():
    """TBG (Appendix A.2): Q stored [seq][head][dim]; the transpose is folded into the strides of A."""
    heads, seq, dim = 12, 128, 64
    Q, Kk = I.c4a(seed=1)
    Qs = np.ascontiguousarray(Q.transpose(1, 0, 2))  # [seq][head][dim]
    ref = O.bmm(Qs.transpose(1, 0, 2), Kk, trans_b=True)
    op = B.bmm_op(heads, seq, seq, dim, True, "f16", a_strides=[dim, heads * dim, 1])
    space = op.space()
    for n in range(4):
        t = B.trace_sample_valid(op, space, 6, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [Qs, Kk], "f16", (heads, seq, seq))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "TBG layout trace %d" % n)


def test_c4c_int8_gemm_512_bit_exact():
    """Config C4c: int8 x int8 -> int32, 512^3, values uniform in [-128,127]; bit exact."""
    A, Bm = I.c4c(seed=0)
    ref = O.gemm(A, Bm)
    op = B.gemm_op(512, 512, 512, "i8")
    space = op.space()
    for n, t in enumerate(traces_covering_intrinsics(op, space, 7, 3, I8_INTRINS)):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "i32", (512, 512))
        if got is None:
            continue
        compare.assert_int_equal(got, ref, "C4c trace %d" % n)


def test_int8_direct_to_lds_bit_exact():
    """int8 GEMM (NN) and BMM-NT through the direct-to-LDS ring: A row-major with swizzled chunks, B of the NN form
    read with the 8-bit LDS transpose load; both 16-k-per-lane intrinsics, 2 / 3 / 4 stages, persistent workgroups,
    odd tile counts, 3 instances with distinct inputs; int32 results must equal the oracle bit for bit."""
    M, N, K = 192, 160, 384
    g = I.rng(31)
    ins = [[I.int8_uniform(g, (M, K)), I.int8_uniform(g, (K, N))] for _ in range(3)]
    refs = [O.gemm(a, b) for a, b in ins]
    op = B.gemm_op(M, N, K, "i8")
    space = op.space()

    def mk(mfma, i, j, k, unroll=0, cache=5, reorder=0, cw=0):
        return B.make_trace(space, [[mfma], i, j, k, [unroll], [cache], [16], [16], [0], [reorder], [cw]])

    traces = [mk(161664, [12, 1, 1, 1], [10, 1, 1, 1], [6, 1, 1, 1]),                          # 16x16 tile, 1 wave, BK = 64
              mk(161664, [3, 2, 2, 1], [5, 1, 2, 1], [3, 1, 2, 1], unroll=64, cache=6, cw=1),  # BK = 128
              mk(323232, [3, 1, 2, 1], [5, 1, 1, 1], [6, 1, 1, 2], cache=7, reorder=2),          # BK = 64, 4 stages
              mk(323232, [2, 1, 3, 1], [5, 1, 1, 1], [3, 2, 2, 1], unroll=16, cache=5, reorder=1, cw=1),  # BK = 128
              mk(323232, [3, 2, 1, 1], [5, 1, 1, 1], [6, 1, 1, 2], cache=6, reorder=3),          # persistent workgroups
              mk(161664, [6, 1, 2, 1], [5, 2, 1, 1], [3, 1, 1, 2], unroll=64, cache=5, reorder=3, cw=1)]
    ran = 0
    for n, t in enumerate(traces):
        try:
            B.trace_validate(op, space, t)
        except B.MsError as e:
            print("trace", n, "rejected:", str(e)[:120], flush=True)
            continue
        print("trace", n, t.decisions(), flush=True)
        ran += 1
        got = run_variant_distinct(op, space, t, ins, "i32", (M, N))
        if got is None:
            continue
        for r in range(3):
            compare.assert_int_equal(got[r], refs[r], "int8 direct-to-LDS, instance %d trace %d" % (r, n))
    assert ran == 6
    # NT form (both operands k-contiguous): no transpose load involved
    Bn, Mh, Nh, Kh = 3, 64, 96, 128
    Q = I.int8_uniform(g, (Bn, Mh, Kh))
    Kt = I.int8_uniform(g, (Bn, Nh, Kh))
    ref = O.bmm(Q, Kt, trans_b=True)
    op2 = B.bmm_op(Bn, Mh, Nh, Kh, True, "i8")
    sp2 = op2.space()
    for n, t in enumerate([B.make_trace(sp2, [[323232], [2, 1, 1, 1], [1, 3, 1, 1], [2, 1, 1, 2], [0], [5], [16], [16], [0], [0], [0]]),
                           B.make_trace(sp2, [[161664], [2, 1, 2, 1], [3, 1, 2, 1], [1, 1, 2, 1], [64], [6], [16], [16], [0], [2], [1]])]):
        print("NT trace", n, t.decisions(), flush=True)
        got = run_variant(op2, sp2, t, [Q, Kt], "i32", (Bn, Mh, Nh))
        if got is None:
            continue
        compare.assert_int_equal(got, ref, "int8 NT direct-to-LDS trace %d" % n)


def test_int8_extremes():
    A = np.full((64, 512), -128, np.int8)
    Bm = np.full((512, 64), -128, np.int8)
    op = B.gemm_op(64, 64, 512, "i8")
    space = op.space()
    for n in range(4):
        t = B.trace_sample_valid(op, space, 8, n)
        got = run_variant(op, space, t, [A, Bm], "i32", (64, 64))
        if got is None:
            continue
        assert np.all(got == 8388608)


def test_bmm_instances_with_distinct_inputs():
    ins = [list(I.c4b(seed=s, heads=2, seq=32, dim=16)) for s in (1, 2, 3)]
    refs = [O.bmm(p, v) for p, v in ins]
    op = B.bmm_op(2, 32, 16, 32, False, "f16")
    space = op.space()
    for n in range(5):
        t = B.trace_sample_valid(op, space, 15, n)
        got = run_variant_distinct(op, space, t, ins, "f16", (2, 32, 16))
        if got is None:
            continue
        for r in range(3):
            compare.assert_float_close(got[r], refs[r], compare.RTOL_HALF, "instance %d trace %d" % (r, n))


def test_persistent_workgroups_many_tiles_per_workgroup():
    """reorder = 3: 3 instances x 256 tiles = 768 tiles for at most 256 workgroups, so every workgroup walks
    through several tiles, crossing instance boundaries; distinct inputs per instance; fp32 output."""
    M, N, K = 256, 256, 192
    ins = [list(I.gemm_inputs(M, N, K, "f16", s, "normal", 1.0)) for s in (1, 2, 3)]
    refs = [O.gemm(a, b) for a, b in ins]
    op = B.gemm_op(M, N, K, "f16", "f32")
    space = op.space()

    def mk(mfma, i, j, k, unroll=0, cache=5, pad=0, reorder=3, cw=0):
        return B.make_trace(space, [[mfma], i, j, k, [unroll], [cache], [8], [8], [pad], [reorder], [cw]])

    traces = [mk(161632, [16, 1, 1, 1], [16, 1, 1, 1], [3, 1, 1, 2]),           # 16x16 tiles, 1 wave, K0 = 3
              mk(161632, [16, 1, 1, 1], [8, 1, 2, 1], [6, 1, 1, 1], cache=7),   # 4-stage ring, BK = 32, K0 = 6
              mk(323216, [8, 1, 1, 1], [8, 1, 1, 1], [3, 1, 2, 2], unroll=64, cache=6, cw=1),
              mk(161632, [8, 1, 2, 1], [16, 1, 1, 1], [3, 2, 1, 1], unroll=16, cache=5, cw=1)]
    for n, t in enumerate(traces):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant_distinct(op, space, t, ins, "f32", (M, N))
        if got is None:
            continue
        for r in range(3):
            compare.assert_float_close(got[r], refs[r], 1e-4, "instance %d trace %d" % (r, n))


F32_INTRINS = [161604, 323202]


def test_c1_fp32_on_matrix_cores():
    """Config C1 (fp32 GEMM 128^3) with the opt-in fp32 tensorize module: both fp32 intrinsics, the fp32
    tolerance, 3 instances with distinct inputs."""
    ins = [list(I.c1(seed=s)) for s in (0, 1, 2)]
    refs = [O.gemm(a, b) for a, b in ins]
    op = B.gemm_op(128, 128, 128, "f32")
    space = op.space(B.SPACE_DEFAULT | B.SPACE_TENSORIZE_F32)
    assert space.family == B.FAM_GEMM_MFMA
    for n, t in enumerate(traces_covering_intrinsics(op, space, 6, 4, F32_INTRINS)):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant_distinct(op, space, t, ins, "f32", (128, 128))
        if got is None:
            continue
        for r in range(3):
            compare.assert_float_close(got[r], refs[r], compare.RTOL_F32, "C1 on MFMA, instance %d trace %d" % (r, n))


def test_fp32_matrix_cores_exact_on_small_ints_odd_tiles():
    """fp32 intrinsics on a shape with factors 3, 5, 7 in the tile counts and a batch; integer-valued inputs:
    every product and partial sum is exact, so the result must equal the oracle bit for bit."""
    Bn, M, N, K = 2, 96, 160, 56
    A, Bm = I.gemm_inputs(M, N, K, "f32", 5, "ints", batch=Bn)
    ref = O.bmm(A, Bm, trans_b=False)
    op = B.bmm_op(Bn, M, N, K, False, "f32")
    space = op.space(B.SPACE_DEFAULT | B.SPACE_TENSORIZE_F32)
    assert space.family == B.FAM_GEMM_MFMA
    for n, t in enumerate(traces_covering_intrinsics(op, space, 8, 3, F32_INTRINS)):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "f32", (Bn, M, N), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % n


F8_INTRINS = [161632, 323216]


def test_fp8_gemm_exact_on_small_ints_then_random():
    """8-bit float inputs (4 exponent, 3 mantissa bits) on the fp8 matrix-core intrinsics.  Small integers are exact
    in this format and all partial sums exact in fp32, so the fp32 output must equal the oracle bit for bit (this also
    pins the hardware's reading of the bit patterns: exponent bias 7); then normal values with fp16 output within the
    half-precision tolerance and with fp32 output within the fp8 tolerance (the hardware sums the 32 products of one
    instruction in less than fp32 precision).  NN and NT forms, 2 instances."""
    M, N, K = 192, 160, 224
    A, Bm = I.gemm_inputs(M, N, K, "f8", 3, "ints")
    ref = O.gemm(A, Bm)
    op = B.gemm_op(M, N, K, "f8", "f32")
    space = op.space()
    assert space.family == B.FAM_GEMM_MFMA
    for n, t in enumerate(traces_covering_intrinsics(op, space, 12, 3, F8_INTRINS)):
        print("ints trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "f32", (M, N), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % n
    A, Bm = I.gemm_inputs(M, N, K, "f8", 4, "normal", 1.0)
    ref = O.gemm(A, Bm)
    op = B.gemm_op(M, N, K, "f8", "f16")
    space = op.space()
    for n, t in enumerate(traces_covering_intrinsics(op, space, 13, 2, F8_INTRINS)):
        print("normal trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "f16", (M, N))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "fp8 trace %d" % n)
    # NT form with a batch (both operands contiguous along k)
    Bn, Mh, Nh, Kh = 3, 64, 96, 128
    g = I.rng(41)
    Q = I.normal(g, (Bn, Mh, Kh), 1.0, "f8")
    Kt = I.normal(g, (Bn, Nh, Kh), 1.0, "f8")
    ref = O.bmm(Q, Kt, trans_b=True)
    op = B.bmm_op(Bn, Mh, Nh, Kh, True, "f8", "f32")
    space = op.space()
    for n, t in enumerate(traces_covering_intrinsics(op, space, 14, 2, F8_INTRINS)):
        print("NT trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [Q, Kt], "f32", (Bn, Mh, Nh))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_F8, "fp8 NT trace %d" % n)


F8_DEEP_INTRINS = [1616128, 323264]


def test_fp8_deep_intrinsics_exact_then_random():
    """The 128-deep (16x16) and 64-deep (32x32) 8-bit float intrinsics: a lane feeds 32 bytes per operand, which lie
    in LDS as two 16-byte halves.  Small integers: bit-equal to the oracle (any mismatch between the k positions of
    the two operands, or between the halves, would show); then normal values, NN and NT forms."""
    M, N, K = 192, 160, 384
    A, Bm = I.gemm_inputs(M, N, K, "f8", 5, "ints")
    ref = O.gemm(A, Bm)
    op = B.gemm_op(M, N, K, "f8", "f32")
    space = op.space()
    seen = set()
    for n, t in enumerate(traces_covering_intrinsics(op, space, 15, 4, F8_DEEP_INTRINS)):
        print("ints trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "f32", (M, N), instances=2)
        seen.add(B.trace_validate(op, space, t).mfma)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % n
    assert seen == set(F8_DEEP_INTRINS)
    A, Bm = I.gemm_inputs(M, N, K, "f8", 6, "normal", 1.0)
    ref = O.gemm(A, Bm)
    for n, t in enumerate(traces_covering_intrinsics(op, space, 16, 2, F8_DEEP_INTRINS)):
        print("normal trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "f32", (M, N))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_F8, "fp8 deep trace %d" % n)
    Bn, Mh, Nh, Kh = 3, 64, 96, 256
    g = I.rng(43)
    Q = I.normal(g, (Bn, Mh, Kh), 1.0, "f8")
    Kt = I.normal(g, (Bn, Nh, Kh), 1.0, "f8")
    ref = O.bmm(Q, Kt, trans_b=True)
    op = B.bmm_op(Bn, Mh, Nh, Kh, True, "f8", "f32")
    space = op.space()
    for n, t in enumerate(traces_covering_intrinsics(op, space, 17, 2, F8_DEEP_INTRINS)):
        print("NT trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [Q, Kt], "f32", (Bn, Mh, Nh))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_F8, "fp8 deep NT trace %d" % n)


def test_ping_pong_on_the_ring_exact():
    """cache_read 8, 9, 10: persistent workgroups on the direct-to-LDS ring whose wavefronts form two groups one
    phase apart.  Integer-valued inputs (every sum exact): fp16 NN and NT, int8, both 16-byte-fragment intrinsics,
    1 to 4 slots per k0 step, 2 / 3 / 4 stages, results staged per wavefront or stored from registers, odd tile counts,
    fewer tiles than compute units (3 instances) and runs of several tiles per workgroup (40 instances)."""
    M, N, K = 192, 320, 512
    g = I.rng(77)

    def run(op, space, traces, ins_of, refs_of, odt, what):
        for R in (3, 40):
            ins = [ins_of(r) for r in range(R)]
            refs = [refs_of(x) for x in ins[:3]] + [None] * (R - 3)
            for n, t in enumerate(traces):
                try:
                    p = B.trace_validate(op, space, t)
                except B.MsError as e:
                    raise AssertionError("%s trace %d rejected: %s" % (what, n, e))
                print(what, "R", R, "trace", n, t.decisions(), "lds", p.lds_bytes, flush=True)
                got = run_variant_distinct(op, space, t, ins, odt, (M, N))
                if got is None:
                    continue
                for r in (0, 1, 2, R - 1):
                    ref = refs[r] if refs[r] is not None else refs_of(ins[r])
                    assert np.array_equal(got[r], ref), "%s R %d trace %d instance %d" % (what, R, n, r)

    # fp16, B stored [K][N] (read with the LDS transpose load)
    op = B.gemm_op(M, N, K, "f16", "f32")
    sp = op.space()

    def mk(sp, mfma, i, j, k, cache=8, cw=0, vec=8):
        return B.make_trace(sp, [[mfma], i, j, k, [0], [cache], [vec], [vec], [0], [3], [cw]])

    pool = [(I.small_ints(g, (M, K), -2, 2, "f16"), I.small_ints(g, (K, N), -2, 2, "f16")) for _ in range(5)]
    traces = [mk(sp, 323216, [3, 1, 2, 1], [5, 1, 1, 2], [8, 1, 2, 2], cache=8, cw=1),     # BK = 64, two slots, staged per wavefront
              mk(sp, 323216, [3, 2, 1, 1], [5, 1, 2, 1], [16, 1, 1, 2], cache=10, cw=0),   # BK = 32, 4 stages
              mk(sp, 161632, [3, 2, 2, 1], [5, 2, 1, 2], [4, 1, 4, 1], cache=9, cw=1),     # BK = 128, four slots of one step
              mk(sp, 161632, [6, 1, 2, 1], [10, 1, 2, 1], [16, 1, 1, 1], cache=9, cw=1),   # one intrinsic step per slot
              mk(sp, 161632, [3, 1, 4, 1], [5, 2, 2, 1], [8, 1, 1, 2], cache=8, cw=0)]     # 8 wavefronts, 4 x 2
    run(op, sp, traces, lambda r: list(pool[r % 5]), lambda x: O.gemm(x[0], x[1]), "f32", "f16 NN")
    # fp16, B stored [N][K] (both operands contiguous along k), fp16 output
    opt = B.bmm_op(1, M, N, K, True, "f16")
    spt = opt.space()
    poolt = [(I.small_ints(g, (1, M, K), -1, 1, "f16"), I.small_ints(g, (1, N, K), -1, 1, "f16")) for _ in range(5)]
    tr_t = [mk(spt, 323216, [3, 1, 2, 1], [5, 1, 1, 2], [8, 1, 2, 2], cache=8, cw=1),
            mk(spt, 161632, [3, 2, 2, 1], [10, 1, 2, 1], [8, 1, 2, 1], cache=10, cw=0)]
    run(opt, spt, tr_t, lambda r: list(poolt[r % 5]), lambda x: O.bmm(x[0], x[1], trans_b=True)[0], "f16", "f16 NT")
    # int8 -> int32 (8-bit transpose load for B)
    op8 = B.gemm_op(M, N, K, "i8")
    sp8 = op8.space()
    pool8 = [(I.int8_uniform(g, (M, K)), I.int8_uniform(g, (K, N))) for _ in range(5)]
    tr_8 = [mk(sp8, 323232, [3, 1, 2, 1], [5, 1, 1, 2], [4, 1, 2, 2], cache=8, cw=1, vec=16),
            mk(sp8, 161664, [3, 2, 2, 1], [5, 2, 1, 2], [4, 1, 1, 2], cache=9, cw=0, vec=16)]
    run(op8, sp8, tr_8, lambda r: list(pool8[r % 5]), lambda x: O.gemm(x[0], x[1]), "i32", "int8")


def test_ping_pong_on_the_ring_c2_shape():
    """Config 2's shape in the launch configuration bench.py times (64 instances): sampled instances against the oracle."""
    op = B.gemm_op(1024, 1024, 1024, "f16")
    sp = op.space()
    ins = [I.c2(seed=50 + r) for r in range(4)]
    R = 64
    per_instance = [list(ins[r % 4]) for r in range(R)]
    refs = None
    for n, (i, j, k, cache, cw) in enumerate([([4, 4, 2, 1], [4, 1, 4, 2], [16, 1, 2, 2], 8, 1), ([4, 4, 2, 1], [4, 1, 4, 2], [32, 1, 1, 2], 10, 1),
                                              ([4, 2, 2, 2], [4, 1, 4, 2], [32, 1, 1, 2], 9, 0)]):
        t = B.make_trace(sp, [[323216], i, j, k, [0], [cache], [8], [8], [0], [3], [cw]])
        print("c2 ping-pong trace", n, t.decisions(), flush=True)
        got = run_variant_distinct(op, sp, t, per_instance, "f16", (1024, 1024))
        if got is None:
            continue
        if refs is None:
            refs = [O.gemm(a, b) for a, b in ins]
        for r in (0, 1, 2, 3, 31, 63):
            compare.assert_float_close(got[r], refs[r % 4], compare.RTOL_HALF, "C2 ping-pong trace %d instance %d" % (n, r))


@pytest.mark.parametrize("layout", [3, 4])
def test_row_major_b_in_lds_exact(layout):
    """storage_align 3 (XOR-swizzled granules) and 4 (rows padded by 32 bytes, no swizzle anywhere): the j-contiguous B goes global memory -> registers -> LDS in 16-byte vectors without a register
    transposition and the fragments come out of the transposing LDS loads.  int8 (both 16-k-per-lane intrinsics) and
    integer-valued fp16 / bf16 (both 8-k-per-lane intrinsics) with fp32 output must equal the oracle bit for bit; every
    register-staging mode (single stage, double buffer, prefetch distance 2, software-pipelined k loop, ping-pong wave
    groups), odd tile counts, column counts whose granule count is not a power of two (no swizzle), 3 instances with
    distinct inputs."""
    M, N, K = 192, 160, 384
    g = I.rng(47)
    ins = [[I.int8_uniform(g, (M, K)), I.int8_uniform(g, (K, N))] for _ in range(3)]
    refs = [O.gemm(a, b) for a, b in ins]
    op = B.gemm_op(M, N, K, "i8")
    space = op.space()

    def mk(sp, mfma, i, j, k, vecs, unroll=0, cache=1, reorder=0, cw=0):
        return B.make_trace(sp, [[mfma], i, j, k, [unroll], [cache], [vecs[0]], [vecs[1]], [layout], [reorder], [cw]])

    traces = [mk(space, 161664, [12, 1, 1, 1], [10, 1, 1, 1], [6, 1, 1, 1], (16, 16)),                      # one wave, 16 columns
              mk(space, 161664, [3, 2, 2, 1], [5, 1, 2, 1], [3, 1, 2, 1], (16, 16), unroll=64, cache=2, cw=1),  # pipelined, BN = 32
              mk(space, 323232, [3, 1, 2, 1], [1, 1, 5, 1], [6, 1, 1, 2], (4, 16), cache=3, reorder=2),        # BN = 160: 10 granules
              mk(space, 323232, [2, 1, 3, 1], [5, 1, 1, 1], [3, 2, 2, 1], (8, 16), unroll=16, reorder=1, cw=1),
              mk(space, 161664, [6, 1, 2, 1], [5, 2, 1, 1], [6, 1, 1, 1], (16, 16), cache=4, reorder=2),       # ping-pong wave groups
              mk(space, 161664, [3, 2, 2, 1], [5, 1, 1, 2], [3, 2, 1, 1], (16, 16), unroll=64, cache=2)]
    ran = 0
    for n, t in enumerate(traces):
        p = B.trace_validate(op, space, t)
        assert p.lds_pad == layout
        print("int8 trace", n, t.decisions(), flush=True)
        ran += 1
        got = run_variant_distinct(op, space, t, ins, "i32", (M, N))
        if got is None:
            continue
        for r in range(3):
            compare.assert_int_equal(got[r], refs[r], "row-major B, int8, instance %d trace %d" % (r, n))
    assert ran == 6
    for dtype in ("f16", "bf16"):
        M2, N2, K2 = 192, 160, 224
        A, Bm = I.gemm_inputs(M2, N2, K2, dtype, 2, "ints")
        ref = O.gemm(A, Bm, bf16=(dtype == "bf16"))
        op2 = B.gemm_op(M2, N2, K2, dtype, "f32")
        sp2 = op2.space()
        traces = [mk(sp2, 161632, [12, 1, 1, 1], [10, 1, 1, 1], [7, 1, 1, 1], (8, 8)),
                  mk(sp2, 323216, [3, 1, 2, 1], [5, 1, 1, 1], [7, 1, 1, 2], (8, 8), cache=2, reorder=2, cw=1),
                  mk(sp2, 161632, [3, 2, 2, 1], [1, 1, 5, 2], [7, 1, 1, 1], (4, 8), cache=3, reorder=1),
                  mk(sp2, 323216, [1, 3, 2, 1], [5, 1, 1, 1], [7, 1, 2, 1], (8, 8), unroll=64, cache=2),
                  mk(sp2, 161632, [6, 1, 2, 1], [5, 1, 2, 1], [7, 1, 1, 1], (8, 8), cache=4)]
        for n, t in enumerate(traces):
            B.trace_validate(op2, sp2, t)
            print(dtype, "trace", n, t.decisions(), flush=True)
            got = run_variant(op2, sp2, t, [A, Bm], "f32", (M2, N2), instances=2)
            if got is None:
                continue
            assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "row-major B, %s trace %d" % (dtype, n)
    # batched NN form (the attention product P x V of config C4b's kind)
    Bn, Mh, Nh, Kh = 3, 64, 96, 128
    P = I.gemm_inputs(Bn * Mh, 8, Kh, "f16", 1, "ints")[0].reshape(Bn, Mh, Kh)
    V = I.gemm_inputs(Bn * Kh, 8, Nh, "f16", 1, "ints")[0].reshape(Bn, Kh, Nh)
    ref = O.bmm(P, V, trans_b=False)
    op3 = B.bmm_op(Bn, Mh, Nh, Kh, False, "f16", "f32")
    sp3 = op3.space()
    for n, t in enumerate([mk(sp3, 161632, [2, 1, 2, 1], [3, 1, 2, 1], [2, 1, 2, 1], (8, 8), cache=2, reorder=2),
                           mk(sp3, 323216, [1, 1, 2, 1], [3, 1, 1, 1], [4, 1, 1, 2], (8, 8), cw=1)]):
        B.trace_validate(op3, sp3, t)
        print("bmm NN trace", n, t.decisions(), flush=True)
        got = run_variant(op3, sp3, t, [P, V], "f32", (Bn, Mh, Nh))
        if got is None:
            continue
        assert np.array_equal(got, ref), "row-major B, BMM-NN trace %d" % n


def test_row_major_b_in_lds_c4c_and_c2_shapes():
    """The same layout at the full shapes of config C4c (bit exact) and config C2 (tolerance of the fp16 configs)."""
    A, Bm = I.c4c(seed=2)
    ref = O.gemm(A, Bm)
    op = B.gemm_op(512, 512, 512, "i8")
    space = op.space()
    for n, vals in enumerate([[[161664], [4, 8, 1, 1], [4, 2, 4, 1], [4, 1, 2, 1], [0], [1], [16], [16], [3], [2], [0]],
                              [[323232], [4, 2, 2, 1], [4, 1, 2, 2], [4, 1, 4, 1], [0], [1], [16], [16], [3], [2], [0]],
                              [[161664], [2, 4, 4, 1], [4, 8, 1, 1], [4, 1, 2, 1], [64], [2], [16], [16], [3], [2], [1]],
                              [[161664], [4, 8, 1, 1], [4, 2, 4, 1], [4, 1, 2, 1], [0], [1], [16], [16], [4], [2], [0]],
                              [[323232], [4, 2, 2, 1], [4, 1, 2, 2], [4, 1, 4, 1], [64], [2], [16], [16], [4], [2], [1]]]):
        t = B.make_trace(space, vals)
        B.trace_validate(op, space, t)
        print("C4c trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "i32", (512, 512))
        if got is None:
            continue
        compare.assert_int_equal(got, ref, "row-major B, C4c trace %d" % n)
    A, Bm = I.c2(seed=1)
    ref = O.gemm(A, Bm)
    op = B.gemm_op(1024, 1024, 1024, "f16")
    space = op.space()
    for n, vals in enumerate([[[323216], [4, 2, 2, 2], [4, 2, 2, 2], [16, 1, 4, 1], [64], [2], [8], [8], [3], [2], [0]],
                              [[323216], [4, 1, 4, 2], [4, 2, 2, 2], [16, 1, 1, 4], [0], [4], [8], [8], [3], [2], [1]],
                              [[161632], [8, 2, 2, 2], [8, 1, 2, 4], [32, 1, 1, 1], [0], [3], [8], [8], [3], [0], [0]],
                              [[323216], [4, 4, 2, 1], [4, 4, 2, 1], [16, 1, 2, 2], [0], [1], [8], [8], [4], [2], [1]],   # 128 x 128 wave tiles
                              [[323216], [4, 2, 2, 2], [4, 2, 2, 2], [16, 1, 4, 1], [64], [2], [8], [8], [4], [2], [0]]]):
        t = B.make_trace(space, vals)
        B.trace_validate(op, space, t)
        print("C2 trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [A, Bm], "f16", (1024, 1024))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "row-major B, C2 trace %d" % n)


@pytest.mark.parametrize("layout", [3, 4])
def test_row_major_b_in_lds_every_fragment_size(layout):
    """storage_align 3 and 4 with the other fragment sizes: 4 k per lane of 2-byte inputs (one transposing load), 8 k per
    lane of 1-byte inputs (one load: the shallow int8 and 8-bit float intrinsics) and 32 k per lane (four loads: the
    128-deep and 64-deep 8-bit float intrinsics).  Integer-valued inputs, fp32 / int32 outputs: bit-equal to the oracle."""
    def mk(sp, mfma, i, j, k, vec_b, unroll=0, cache=1, reorder=0, cw=0, vec=0):
        return B.make_trace(sp, [[mfma], i, j, k, [unroll], [cache], [vec or vec_b], [vec_b], [layout], [reorder], [cw]])

    M, N, K = 192, 160, 256
    cases = [("f16", "f32", 8, [(161616, [12, 1, 1, 1], [5, 2, 1, 1], [8, 1, 2, 1], 1), (323208, [3, 1, 2, 1], [5, 1, 1, 1], [8, 2, 1, 2], 2),
                                (161616, [3, 2, 2, 1], [1, 1, 5, 2], [4, 1, 4, 1], 3)]),
             ("i8", "i32", 16, [(161632, [12, 1, 1, 1], [5, 2, 1, 1], [4, 1, 2, 1], 1), (323216, [3, 1, 2, 1], [5, 1, 1, 1], [4, 2, 1, 2], 2),
                                (161632, [3, 2, 2, 1], [1, 1, 5, 2], [8, 1, 1, 1], 4)]),
             ("f8", "f32", 16, [(161632, [12, 1, 1, 1], [5, 2, 1, 1], [4, 1, 2, 1], 1), (323216, [3, 1, 2, 1], [5, 1, 1, 1], [4, 2, 1, 2], 2),
                                (1616128, [6, 1, 2, 1], [5, 1, 2, 1], [2, 1, 1, 1], 1), (323264, [3, 1, 2, 1], [5, 1, 1, 1], [2, 1, 2, 1], 2),
                                (1616128, [3, 2, 2, 1], [1, 1, 5, 2], [1, 1, 2, 1], 3), (323264, [1, 3, 2, 1], [5, 1, 1, 1], [4, 1, 1, 1], 1)])]
    for dtype, odt, vb, traces in cases:
        A, Bm = I.gemm_inputs(M, N, K, dtype, 7, "ints") if dtype != "i8" else (I.int8_uniform(I.rng(9), (M, K)), I.int8_uniform(I.rng(10), (K, N)))
        ref = O.gemm(A, Bm)
        op = B.gemm_op(M, N, K, dtype, odt)
        sp = op.space()
        for n, (mfma, i, j, k, cache) in enumerate(traces):
            t = mk(sp, mfma, i, j, k, vb, cache=cache, reorder=2 * (n % 2), cw=n % 2)
            p = B.trace_validate(op, sp, t)
            assert p.lds_pad == layout and p.mfma == mfma
            print(dtype, "trace", n, t.decisions(), flush=True)
            got = run_variant(op, sp, t, [A, Bm], odt, (M, N), instances=2)
            if got is None:
                continue
            assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "row-major B, %s trace %d" % (dtype, n)


def test_one_wavefront_per_simd_tiles_exact():
    """Workgroups of 4 wavefronts with 128 x 128 wave tiles (256 accumulators per lane, one wavefront per SIMD): these
    kernels fetch their operands through buffer loads (descriptor and tile offset in scalar registers, one lane offset
    per operand).  Integer-valued fp16 with fp32 output and int8: bit-equal to the oracle in every register-staged mode,
    rolled and software-pipelined k loops, all B layouts, two tiles per instance in each direction, 2 instances (the
    staged epilogue of such tiles is covered at the config-2 shape, where the fp16 output fits LDS)."""
    M, N, K = 512, 512, 192
    A, Bm = I.gemm_inputs(M, N, K, "f16", 11, "ints")
    ref = O.gemm(A, Bm)
    op = B.gemm_op(M, N, K, "f16", "f32")
    sp = op.space()

    def mk(space, mfma, k, unroll, cache, vec_b, layout, reorder=2, cw=0, ij=([2, 4, 2, 1], [2, 4, 2, 1]), vec=8):
        return B.make_trace(space, [[mfma], ij[0], ij[1], k, [unroll], [cache], [vec], [vec_b], [layout], [reorder], [cw]])

    traces = [mk(sp, 323216, [6, 1, 2, 1], 0, 3, 8, 4), mk(sp, 323216, [3, 1, 4, 1], 64, 2, 8, 4),
              mk(sp, 323216, [3, 1, 2, 2], 0, 1, 8, 3, reorder=0), mk(sp, 323216, [3, 1, 4, 1], 0, 2, 4, 2),
              mk(sp, 323216, [6, 1, 2, 1], 64, 2, 2, 1, reorder=1, ij=([2, 1, 2, 4], [2, 1, 2, 4])),
              mk(sp, 161632, [6, 1, 1, 1], 0, 1, 8, 4, ij=([2, 8, 2, 1], [2, 8, 2, 1]))]
    for n, t in enumerate(traces):
        p = B.trace_validate(op, sp, t)
        assert p.waves == 4 and p.acc_per_thread == 256
        print("f16 trace", n, t.decisions(), flush=True)
        got = run_variant(op, sp, t, [A, Bm], "f32", (M, N), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "128 x 128 wave tiles, f16 trace %d" % n
    g = I.rng(53)
    A8, B8 = I.int8_uniform(g, (M, 256)), I.int8_uniform(g, (256, N))
    ref8 = O.gemm(A8, B8)
    op8 = B.gemm_op(M, N, 256, "i8")
    sp8 = op8.space()
    for n, t in enumerate([mk(sp8, 323232, [4, 1, 2, 1], 0, 2, 16, 4, vec=16), mk(sp8, 323232, [2, 1, 4, 1], 64, 2, 16, 3, vec=16),
                           mk(sp8, 323232, [4, 1, 1, 2], 0, 1, 4, 2, vec=16)]):
        p = B.trace_validate(op8, sp8, t)
        assert p.waves == 4 and p.acc_per_thread == 256
        print("int8 trace", n, t.decisions(), flush=True)
        got = run_variant(op8, sp8, t, [A8, B8], "i32", (M, N), instances=2)
        if got is None:
            continue
        compare.assert_int_equal(got[0], ref8, "128 x 128 wave tiles, int8 trace %d" % n)
        compare.assert_int_equal(got[1], ref8, "128 x 128 wave tiles, int8 trace %d, instance 1" % n)
