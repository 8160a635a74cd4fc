"""GPU parity of implicit-GEMM conv2d + bias + ReLU (config C3) against the CPU oracle."""
import numpy as np
import pytest

from oracle import compare, oracle as O
from paper_2205_13603_amd import binding as B, inputs as I
from gpu_util import run_variant, run_variant_distinct
from test_gpu_gemm_mfma import traces_covering_intrinsics, F16_INTRINS

pytestmark = pytest.mark.gpu


def test_c3_conv_bias_relu():
    """Config C3: 1x56x56x64 -> 64, 3x3 s1 p1, bias + ReLU, fp16 in/out, fp32 accumulate."""
    X, W, bias = I.c3(seed=0)
    ref = O.conv2d_nhwc(X, W, bias=bias, relu=True, stride=1, pad=1)
    assert (ref == 0).mean() > 0.05, "ReLU must be active on part of the output"
    op = B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1)
    space = op.space()
    for n, t in enumerate(traces_covering_intrinsics(op, space, 0, 4, F16_INTRINS)):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, W, bias], "f16", (1, 56, 56, 64))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "C3 trace %d" % n)


@pytest.mark.parametrize("stride,pad,k,relu,has_bias", [(2, 1, 3, True, True), (1, 0, 1, False, False), (2, 3, 7, True, True),
                                                       (1, 2, 5, False, True)])
def test_conv_other_geometries_exact(stride, pad, k, relu, has_bias):
    """Strides, paddings and kernel sizes beyond C3; batch 2; 2 instances; integer-valued inputs make
    the fp32 accumulation exact, so the fp32 output must equal the oracle exactly."""
    N, H, W_, Cin, Cout = 2, 17, 16, 16, 32
    g = I.rng(11)
    X = I.small_ints(g, (N, H, W_, Cin), -2, 2, "f16")
    Wt = I.small_ints(g, (k, k, Cin, Cout), -2, 2, "f16")
    bias = g.integers(-3, 4, size=Cout).astype(np.float32) if has_bias else None
    ref = O.conv2d_nhwc(X, Wt, bias=bias, relu=relu, stride=stride, pad=pad)
    OH, OW = ref.shape[1], ref.shape[2]
    if (N * OH * OW) % 16:
        pytest.skip("M = %d output pixels is not a multiple of the 16-row intrinsic" % (N * OH * OW))
    op = B.conv2d_op(N, H, W_, Cin, Cout, k, k, stride=stride, pad=pad, has_bias=has_bias, relu=relu, out_dtype="f32")
    space = op.space()
    ins = [X, Wt] + ([bias] if has_bias else [])
    for n in range(6):
        t = B.trace_sample_valid(op, space, 12, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, ins, "f32", (N, OH, OW, Cout), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % n


def test_conv_instances_with_distinct_inputs():
    """Three instances, each with its own activations, weights and bias (every input is per instance)."""
    ins = [list(I.c3(seed=s, H=14, W=16, Cin=16, Cout=32)) for s in (1, 2, 3)]
    refs = [O.conv2d_nhwc(x, w, bias=b, relu=True, stride=1, pad=1) for x, w, b in ins]
    op = B.conv2d_op(1, 14, 16, 16, 32, 3, 3, stride=1, pad=1)
    space = op.space()
    for n in range(5):
        t = B.trace_sample_valid(op, space, 13, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant_distinct(op, space, t, ins, "f16", (1, 14, 16, 32))
        if got is None:
            continue
        for r in range(3):
            compare.assert_float_close(got[r], refs[r], compare.RTOL_HALF, "instance %d trace %d" % (r, n))


def _traces_with_resident_patch(op, space, seed, count, compute_at=1, max_index=1500):
    """Sampled valid traces with the given compute-location decision: 1 = the input patch of a tile is resident
    in LDS, 2 = also the weights, under persistent workgroups."""
    out = []
    for idx in range(max_index):
        if len(out) == count:
            break
        t = B.trace_sample_valid(op, space, seed, idx)
        if B.trace_validate(op, space, t).compute_at == compute_at:
            out.append(t)
    return out


@pytest.mark.parametrize("compute_at", [1, 2, 3, 4])
def test_c3_conv_resident_patch(compute_at):
    """C3 with the cache-read of X under the workgroup tile loop (sample-compute-location = tile), with the
    weights resident as well (2), with helper wavefronts (3), and with the weights in registers (4): row-aligned tiles and tiles that start in the
    middle of an output row."""
    X, W, bias = I.c3(seed=3)
    ref = O.conv2d_nhwc(X, W, bias=bias, relu=True, stride=1, pad=1)
    op = B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1)
    space = op.space()
    traces = _traces_with_resident_patch(op, space, 21, 6, compute_at)
    assert len(traces) == 6
    aligned = [B.trace_validate(op, space, t).block_m % 56 == 0 for t in traces]
    print("row-aligned tiles:", aligned, flush=True)
    for n, t in enumerate(traces):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, W, bias], "f16", (1, 56, 56, 64))
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "C3 compute_at %d, trace %d" % (compute_at, n))


@pytest.mark.parametrize("compute_at", [1, 2, 3, 4])
@pytest.mark.parametrize("stride,pad,k,H,W_", [(1, 1, 3, 16, 16), (2, 1, 3, 16, 32), (1, 0, 1, 8, 16), (2, 3, 7, 32, 16), (1, 2, 5, 12, 16)])
def test_conv_resident_patch_geometries_exact(stride, pad, k, H, W_, compute_at):
    """Resident input patch with other strides, paddings and filter sizes, batch 2, 2 instances with distinct
    data; integer-valued inputs make fp32 accumulation exact: the fp32 output must equal the oracle."""
    N, Cin, Cout = 2, 32, 32
    g = I.rng(17)
    ins, refs = [], []
    for r in range(2):
        X = I.small_ints(g, (N, H, W_, Cin), -2, 2, "f16")
        Wt = I.small_ints(g, (k, k, Cin, Cout), -2, 2, "f16")
        bias = g.integers(-3, 4, size=Cout).astype(np.float32)
        ins.append([X, Wt, bias])
        refs.append(O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=stride, pad=pad))
    OH, OW = refs[0].shape[1], refs[0].shape[2]
    assert (OH * OW) % 16 == 0
    op = B.conv2d_op(N, H, W_, Cin, Cout, k, k, stride=stride, pad=pad, out_dtype="f32")
    space = op.space()
    traces = _traces_with_resident_patch(op, space, 5, 4, compute_at)
    assert traces, "no valid trace with compute_at %d" % compute_at
    for n, t in enumerate(traces):
        print("trace", n, t.decisions(), flush=True)
        got = run_variant_distinct(op, space, t, ins, "f32", (N, OH, OW, Cout))
        if got is None:
            continue
        for r in range(2):
            assert np.array_equal(got[r], refs[r]), "instance %d trace %d" % (r, n)


def test_conv_persistent_runs_cross_instances():
    """Resident weights under persistent workgroups, with more tiles than workgroups: every workgroup walks a
    run of consecutive tiles that crosses image and instance boundaries (weights reloaded, patch prefetched).
    600 instances of 5 distinct data sets in rotation; integer-valued inputs, fp32 output: exact equality."""
    N, H, W_, Cin, Cout, R = 2, 16, 16, 32, 32, 600
    g = I.rng(23)
    sets, refs = [], []
    for r in range(5):
        X = I.small_ints(g, (N, H, W_, Cin), -2, 2, "f16")
        Wt = I.small_ints(g, (3, 3, Cin, Cout), -2, 2, "f16")
        bias = g.integers(-3, 4, size=Cout).astype(np.float32)
        sets.append([X, Wt, bias])
        refs.append(O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=1, pad=1))
    ins = [sets[r % 5] for r in range(R)]
    op = B.conv2d_op(N, H, W_, Cin, Cout, 3, 3, stride=1, pad=1, out_dtype="f32")
    space = op.space()
    for compute_at, cache_read in ((2, 1), (2, 2), (3, 2), (4, 1), (4, 2)):
        traces = [t for t in _traces_with_resident_patch(op, space, 9, 40, compute_at)
                  if B.trace_validate(op, space, t).cache_read == cache_read][:2]
        assert traces, "no valid trace with compute_at %d and cache_read %d" % (compute_at, cache_read)
        for n, t in enumerate(traces):
            p = B.trace_validate(op, space, t)
            tiles = p.grid[0] * R
            print("compute_at", compute_at, "cache_read", cache_read, "trace", n, t.decisions(), "tiles", tiles, flush=True)
            assert tiles > 4 * 256, "the launch must have several tiles per workgroup"
            got = run_variant_distinct(op, space, t, ins, "f32", (N, H, W_, Cout))
            if got is None:
                continue
            for r in range(R):
                assert np.array_equal(got[r], refs[r % 5]), "instance %d trace %d" % (r, n)


@pytest.mark.parametrize("stride,pad,k,dil,H,W_", [(1, 2, 3, 2, 16, 16), (2, 2, 3, 2, 16, 32), (1, 3, 2, 3, 13, 16), (1, 4, 3, 4, 16, 16)])
def test_dilated_conv_exact_for_every_compute_location(stride, pad, k, dil, H, W_):
    """Dilated conv2d (taps `dil` input elements apart; the paper's DIL workload in small): the im2col loader and
    all resident-patch modes, batch 2, 2 instances with distinct data, integer-valued inputs, fp32 output: exact."""
    N, Cin, Cout = 2, 32, 32
    g = I.rng(29)
    ins, refs = [], []
    for r in range(2):
        X = I.small_ints(g, (N, H, W_, Cin), -2, 2, "f16")
        Wt = I.small_ints(g, (k, k, Cin, Cout), -2, 2, "f16")
        bias = g.integers(-3, 4, size=Cout).astype(np.float32)
        ins.append([X, Wt, bias])
        refs.append(O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=stride, pad=pad, dilation=dil))
    OH, OW = refs[0].shape[1], refs[0].shape[2]
    if (N * OH * OW) % 16:
        pytest.skip("M = %d output pixels is not a multiple of the 16-row intrinsic" % (N * OH * OW))
    op = B.conv2d_op(N, H, W_, Cin, Cout, k, k, stride=stride, pad=pad, out_dtype="f32", dilation=dil)
    space = op.space()
    assert op.loops()[0][1] == N * OH * OW
    ran = set()
    for compute_at in (0, 1, 2, 3, 4):
        for n, t in enumerate(_traces_with_resident_patch(op, space, 4, 2, compute_at)):
            print("compute_at", compute_at, "trace", n, t.decisions(), flush=True)
            ran.add(compute_at)
            got = run_variant_distinct(op, space, t, ins, "f32", (N, OH, OW, Cout))
            if got is None:
                continue
            for r in range(2):
                assert np.array_equal(got[r], refs[r]), "compute_at %d instance %d trace %d" % (compute_at, r, n)
    assert {0, 1, 2} <= ran


def test_conv_bf16_every_compute_location():
    """bf16 activations and weights (uint16 bit patterns on the host), fp32 accumulate, bf16 output: the same conv
    kernels with the bf16 intrinsics; 2 instances."""
    X, W, bias = I.c3(seed=5, H=28, W=28, Cin=32, Cout=64, dtype="bf16")
    ref = O.conv2d_nhwc(X, W, bias=bias, relu=True, stride=1, pad=1, bf16=True)
    op = B.conv2d_op(1, 28, 28, 32, 64, 3, 3, stride=1, pad=1, in_dtype="bf16")
    space = op.space()
    ran = set()
    for compute_at in (0, 1, 2, 3, 4):
        for n, t in enumerate(_traces_with_resident_patch(op, space, 6, 2, compute_at)):
            print("compute_at", compute_at, "trace", n, t.decisions(), flush=True)
            ran.add(compute_at)
            got = run_variant(op, space, t, [X, W, bias], "bf16", (1, 28, 28, 64), instances=2)
            if got is None:
                continue
            for r in range(2):
                compare.assert_float_close(got[r], ref, compare.RTOL_HALF, "bf16 conv, compute_at %d trace %d" % (compute_at, n))
    assert {0, 1, 2} <= ran


@pytest.mark.parametrize("Cin,k,stride,pad,H,W_", [(3, 7, 2, 3, 32, 32), (5, 3, 1, 1, 16, 16), (12, 3, 1, 1, 8, 16), (3, 1, 1, 0, 16, 16)])
def test_conv_reduction_extent_not_a_multiple_of_the_intrinsic(Cin, k, stride, pad, H, W_):
    """KH*KW*Cin = 147, 45, 108 and 3: the k split covers the extent rounded up to the intrinsic's k and both loaders
    deliver zeros beyond it (a first layer with 3 input channels is such an operator).  Integer-valued inputs: bit-equal
    to the oracle for every intrinsic that the space offers."""
    N, Cout = 1, 32
    g = I.rng(61)
    X = I.small_ints(g, (N, H, W_, Cin), -2, 2, "f16")
    Wt = I.small_ints(g, (k, k, Cin, Cout), -2, 2, "f16")
    bias = g.integers(-3, 4, size=Cout).astype(np.float32)
    ref = O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=stride, pad=pad)
    OH, OW = ref.shape[1], ref.shape[2]
    op = B.conv2d_op(N, H, W_, Cin, Cout, k, k, stride=stride, pad=pad, out_dtype="f32")
    space = op.space()
    cands = [space.slots[0].candidates[i] for i in range(space.slots[0].n_candidates)]
    assert any((k * k * Cin) % (c % 100) for c in cands)
    want = {c: 2 for c in cands}
    idx = 0
    while any(want.values()) and idx < 400:
        t = B.trace_sample_valid(op, space, 62, idx)
        idx += 1
        p = B.trace_validate(op, space, t)
        if want.get(p.mfma, 0) == 0:
            continue
        want[p.mfma] -= 1
        assert p.compute_at == 0 or (k * k * Cin) % p.tile_unit[2] == 0
        print("trace", idx, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f32", (N, OH, OW, Cout), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % idx
    assert not any(want.values()), want


def test_cbr_first_layer_224x224x3_7x7_stride_2():
    """The paper's CBR shape (Appendix A.2: 224 x 224 x 3 -> 64, 7 x 7, stride 2, padding 3), batch normalisation folded
    into weights and bias: U[0,1] input, N(0, 0.05) weights, fp16 output within the half-precision tolerance."""
    g = I.rng(63)
    X = I.uniform(g, (1, 224, 224, 3), 0.0, 1.0, "f16")
    Wt = I.normal(g, (7, 7, 3, 64), 0.05, "f16")
    bias = I.normal(g, (64,), 0.05, "f32")
    ref = O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=2, pad=3)
    op = B.conv2d_op(1, 224, 224, 3, 64, 7, 7, stride=2, pad=3)
    space = op.space()
    for n in range(6):
        t = B.trace_sample_valid(op, space, 64, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f16", ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "CBR trace %d" % n)


@pytest.mark.parametrize("stride,pad,k,H,W_", [(2, 1, 4, 8, 8), (1, 0, 3, 6, 6), (2, 0, 2, 8, 4), (3, 2, 5, 6, 6), (1, 1, 3, 8, 16)])
def test_transposed_conv_exact(stride, pad, k, H, W_):
    """Transposed convolution (Appendix A.2: T2D): the kernels gather (output pixel <- the input pixels whose scattered
    filter reaches it), the oracle scatters.  Integer-valued inputs, batch 2, 2 instances: bit-equal fp32 outputs."""
    N, Cin, Cout = 2, 16, 32
    g = I.rng(71)
    X = I.small_ints(g, (N, H, W_, Cin), -2, 2, "f16")
    Wt = I.small_ints(g, (k, k, Cin, Cout), -2, 2, "f16")
    bias = g.integers(-3, 4, size=Cout).astype(np.float32)
    ref = O.conv2d_transposed_nhwc(X, Wt, bias=bias, relu=True, stride=stride, pad=pad)
    OH, OW = ref.shape[1], ref.shape[2]
    assert (OH, OW) == ((H - 1) * stride - 2 * pad + k, (W_ - 1) * stride - 2 * pad + k) and (N * OH * OW) % 16 == 0
    op = B.conv2d_transposed_op(N, H, W_, Cin, Cout, k, k, stride=stride, pad=pad, out_dtype="f32")
    space = op.space()
    for n in range(6):
        t = B.trace_sample_valid(op, space, 72, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f32", (N, OH, OW, Cout), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % n


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_t2d_config_transposed_conv_4x4x512(dtype):
    """The paper's T2D shape: 4 x 4 x 512 -> 8 x 8 x 256, 4 x 4 filter, stride 2, padding 1 (K = 8192)."""
    g = I.rng(73)
    X = I.normal(g, (1, 4, 4, 512), 1.0, dtype)
    Wt = I.normal(g, (4, 4, 512, 256), 0.05, dtype)
    bias = I.normal(g, (256,), 0.05, "f32")
    ref = O.conv2d_transposed_nhwc(X, Wt, bias=bias, relu=True, stride=2, pad=1, bf16=dtype == "bf16")
    assert ref.shape == (1, 8, 8, 256)
    op = B.conv2d_transposed_op(1, 4, 4, 512, 256, 4, 4, stride=2, pad=1, in_dtype=dtype)
    space = op.space()
    for n in range(6):
        t = B.trace_sample_valid(op, space, 74, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], dtype, ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "T2D %s trace %d" % (dtype, n))


@pytest.mark.parametrize("groups,Cin,Cout,k,stride,pad", [(4, 64, 128, 3, 2, 1), (2, 16, 64, 3, 1, 1), (8, 64, 128, 1, 1, 0), (3, 48, 96, 3, 1, 1)])
def test_grouped_conv_exact(groups, Cin, Cout, k, stride, pad):
    """Grouped convolution (Appendix A.2: GRP): a group is a batch entry of the implicit GEMM, reading its slice of the
    channels of X, its columns of W and the bias, and writing its slice of the channels of Y.  Integer-valued inputs,
    batch 2, 2 instances: bit-equal fp32 outputs."""
    N, H, W_ = 2, 16, 8
    g = I.rng(81)
    X = I.small_ints(g, (N, H, W_, Cin), -2, 2, "f16")
    Wt = I.small_ints(g, (k, k, Cin // groups, Cout), -2, 2, "f16")
    bias = g.integers(-3, 4, size=Cout).astype(np.float32)
    ref = O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=stride, pad=pad, groups=groups)
    OH, OW = ref.shape[1], ref.shape[2]
    op = B.conv2d_op(N, H, W_, Cin, Cout, k, k, stride=stride, pad=pad, out_dtype="f32", groups=groups)
    space = op.space()
    seen = set()
    for n in range(16):
        t = B.trace_sample_valid(op, space, 82, n)
        seen.add(B.trace_validate(op, space, t).compute_at)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f32", (N, OH, OW, Cout), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % n


def test_grouped_conv_persistent_runs_cross_groups_and_instances():
    """Grouped convolution under the persistent compute locations: the tile list runs over instance x group, so a
    workgroup's run of tiles crosses group and instance boundaries (weights and bias slice change, the patch of the
    next group is prefetched).  200 instances of 5 distinct data sets in rotation, integer-valued inputs, fp32
    output: exact equality."""
    N, H, W_, Cin, Cout, G, R = 2, 16, 8, 64, 128, 4, 200
    g = I.rng(85)
    sets, refs = [], []
    for r in range(5):
        X = I.small_ints(g, (N, H, W_, Cin), -2, 2, "f16")
        Wt = I.small_ints(g, (3, 3, Cin // G, Cout), -2, 2, "f16")
        bias = g.integers(-3, 4, size=Cout).astype(np.float32)
        sets.append([X, Wt, bias])
        refs.append(O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=1, pad=1, groups=G))
    ins = [sets[r % 5] for r in range(R)]
    op = B.conv2d_op(N, H, W_, Cin, Cout, 3, 3, stride=1, pad=1, out_dtype="f32", groups=G)
    space = op.space()
    for compute_at in (2, 3, 4):
        traces = _traces_with_resident_patch(op, space, 86, 2, compute_at)
        assert traces, "no valid trace with compute_at %d" % compute_at
        for n, t in enumerate(traces):
            p = B.trace_validate(op, space, t)
            tiles = p.grid[0] * p.grid[2] * R
            print("compute_at", compute_at, "trace", n, t.decisions(), "tiles", tiles, flush=True)
            assert p.grid[2] == G and tiles > 1024, "the launch must have more tiles than workgroups"
            got = run_variant_distinct(op, space, t, ins, "f32", (N, H, W_, Cout))
            if got is None:
                continue
            for r in range(R):
                assert np.array_equal(got[r], refs[r % 5]), "instance %d trace %d" % (r, n)


@pytest.mark.parametrize("stride,pad,k,L_", [(1, 1, 3, 32), (2, 2, 5, 64)])
def test_grouped_conv1d_exact(stride, pad, k, L_):
    """Grouped 1-D convolution: the group count of the conv1d descriptor on the conv2d kernels, every compute location
    the space offers.  Reference: the oracle's grouped conv2d on an image of height 1 with a 1 x K filter, whose output
    row that reads the image row (row pad / stride) is the 1-D result.  Integer-valued inputs, batch 2, 2 instances:
    bit-equal fp32 outputs."""
    N, Cin, Cout, G = 2, 64, 64, 4
    g = I.rng(93)
    X = I.small_ints(g, (N, L_, Cin), -2, 2, "f16")
    Wt = I.small_ints(g, (k, Cin // G, Cout), -2, 2, "f16")
    bias = g.integers(-3, 4, size=Cout).astype(np.float32)
    assert pad % stride == 0
    ref = O.conv2d_nhwc(X[:, None], Wt[None], bias=bias, relu=True, stride=stride, pad=pad, groups=G)[:, pad // stride]
    OL = ref.shape[1]
    op = B.conv1d_op(N, L_, Cin, Cout, k, stride=stride, pad=pad, out_dtype="f32", groups=G)
    assert op.loops()[0] == ("g", G, False)
    space = op.space()
    want = {0: 2, 1: 2, 2: 1, 3: 1, 4: 1}
    idx = 0
    while any(want.values()) and idx < 800:
        t = B.trace_sample_valid(op, space, 94, idx)
        idx += 1
        ca = B.trace_validate(op, space, t).compute_at
        if want[ca] == 0:
            continue
        want[ca] -= 1
        print("trace", idx, "compute_at", ca, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f32", (N, OL, Cout), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % idx
    assert want[0] == 0 and want[1] == 0, want


def test_grp_config_grouped_conv_56x56x64_to_128():
    """The paper's GRP shape: 56 x 56 x 64 -> 28 x 28 x 128, 3 x 3, stride 2, padding 1, 4 groups; fp16."""
    g = I.rng(83)
    X = I.uniform(g, (1, 56, 56, 64), 0.0, 1.0, "f16")
    Wt = I.normal(g, (3, 3, 16, 128), 0.05, "f16")
    bias = I.normal(g, (128,), 0.05, "f32")
    ref = O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=2, pad=1, groups=4)
    op = B.conv2d_op(1, 56, 56, 64, 128, 3, 3, stride=2, pad=1, groups=4)
    space = op.space()
    for n in range(8):
        t = B.trace_sample_valid(op, space, 84, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f16", ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "GRP trace %d" % n)


@pytest.mark.parametrize("stride,pad,k,dil,L_", [(2, 1, 3, 1, 64), (1, 0, 1, 1, 32), (1, 2, 5, 1, 48), (1, 2, 3, 2, 32), (1, 1, 3, 1, 16)])
def test_conv1d_exact_for_every_compute_location(stride, pad, k, dil, L_):
    """1-D convolution (Appendix A.2: C1D) on the conv2d kernels: an image of height 1, a 1 x K filter, padding at the
    two ends of the row only.  Integer-valued inputs, batch 2, 2 instances: bit-equal fp32 outputs; every cache-read
    location that the space offers is exercised."""
    N, Cin, Cout = 2, 32, 32
    g = I.rng(91)
    X = I.small_ints(g, (N, L_, Cin), -2, 2, "f16")
    Wt = I.small_ints(g, (k, Cin, Cout), -2, 2, "f16")
    bias = g.integers(-3, 4, size=Cout).astype(np.float32)
    ref = O.conv1d_nwc(X, Wt, bias=bias, relu=True, stride=stride, pad=pad, dilation=dil)
    OL = ref.shape[1]
    assert (N * OL) % 16 == 0
    op = B.conv1d_op(N, L_, Cin, Cout, k, stride=stride, pad=pad, out_dtype="f32", dilation=dil)
    space = op.space()
    want = {0: 2, 1: 2, 2: 1, 3: 1, 4: 1}
    idx = 0
    while any(want.values()) and idx < 600:
        t = B.trace_sample_valid(op, space, 92, idx)
        idx += 1
        ca = B.trace_validate(op, space, t).compute_at
        if want[ca] == 0:
            continue
        want[ca] -= 1
        print("trace", idx, "compute_at", ca, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f32", (N, OL, Cout), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % idx
    assert want[0] == 0 and want[1] == 0, want


def test_c1d_config_conv1d_256x64_to_128():
    """The paper's C1D shape: length 256, 64 -> 128 channels, kernel 3, stride 2, padding 1; fp16."""
    g = I.rng(93)
    X = I.uniform(g, (1, 256, 64), 0.0, 1.0, "f16")
    Wt = I.normal(g, (3, 64, 128), 0.05, "f16")
    bias = I.normal(g, (128,), 0.05, "f32")
    ref = O.conv1d_nwc(X, Wt, bias=bias, relu=True, stride=2, pad=1)
    op = B.conv1d_op(1, 256, 64, 128, 3, stride=2, pad=1)
    space = op.space()
    for n in range(8):
        t = B.trace_sample_valid(op, space, 94, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f16", ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "C1D trace %d" % n)


@pytest.mark.parametrize("Cin,k,stride,pad,dil,D,H,W_", [(16, 3, 1, 1, 1, 4, 8, 8), (16, 3, 2, 1, 1, 6, 8, 16), (3, 7, 2, 3, 1, 6, 16, 16),
                                                         (32, 1, 1, 0, 1, 2, 8, 8), (16, 3, 1, 2, 2, 4, 8, 8), (8, 2, 2, 0, 1, 4, 8, 8)])
def test_conv3d_exact(Cin, k, stride, pad, dil, D, H, W_):
    """3-D convolution (Appendix A.2: C3D): the depth is folded into the rows (n, od, oh, ow) and the reduction
    (kd, kh, kw, ci) of the implicit GEMM by the im2col loader.  Integer-valued inputs, batch 2, 2 instances: bit-equal
    fp32 outputs, also where KD*KH*KW*Cin is padded to the intrinsic's k."""
    N, Cout = 2, 32
    g = I.rng(96)
    X = I.small_ints(g, (N, D, H, W_, Cin), -2, 2, "f16")
    Wt = I.small_ints(g, (k, k, k, Cin, Cout), -2, 2, "f16")
    bias = g.integers(-3, 4, size=Cout).astype(np.float32)
    ref = O.conv3d_ndhwc(X, Wt, bias=bias, relu=True, stride=stride, pad=pad, dilation=dil)
    assert ref[0].size // Cout * N % 16 == 0
    op = B.conv3d_op(N, D, H, W_, Cin, Cout, k, stride=stride, pad=pad, out_dtype="f32", dilation=dil)
    space = op.space()
    for n in range(6):
        t = B.trace_sample_valid(op, space, 97, n)
        assert B.trace_validate(op, space, t).compute_at == 0
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f32", ref.shape, instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % n


def test_c3d_config_conv3d_16x224x224x3():
    """The paper's C3D shape: 16 x 224 x 224 x 3 -> 8 x 112 x 112 x 64, 7 x 7 x 7, stride 2, padding 3; fp16 (K = 1029)."""
    g = I.rng(98)
    X = I.uniform(g, (1, 16, 224, 224, 3), 0.0, 1.0, "f16")
    Wt = I.normal(g, (7, 7, 7, 3, 64), 0.02, "f16")
    bias = I.normal(g, (64,), 0.05, "f32")
    ref = O.conv3d_ndhwc(X, Wt, bias=bias, relu=True, stride=2, pad=3)
    assert ref.shape == (1, 8, 112, 112, 64)
    op = B.conv3d_op(1, 16, 224, 224, 3, 64, 7, stride=2, pad=3)
    space = op.space()
    for n in range(3):
        t = B.trace_sample_valid(op, space, 99, n)
        print("trace", n, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f16", ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "C3D trace %d" % n)


@pytest.mark.parametrize("Cin,k,stride,pad,H,W_", [(3, 7, 2, 3, 32, 32), (4, 3, 1, 1, 16, 16), (3, 3, 1, 1, 16, 16), (2, 5, 2, 2, 16, 32), (8, 3, 1, 1, 8, 16),
                                                   (4, 7, 2, 3, 32, 16)])
def test_conv_filter_row_layout_exact(Cin, k, stride, pad, H, W_):
    """The opt-in filter-row layout of the reduction (k = filter row, then the KW * Cin contiguous elements of that row,
    rounded up to the intrinsic's k): im2col staging and, where pixels start at multiples of 4 bytes, the resident patch,
    whose fragments are pieces of image rows.  Integer-valued inputs, batch 2, 2 instances: bit-equal fp32 outputs."""
    N, Cout = 2, 32
    g = I.rng(101)
    X = I.small_ints(g, (N, H, W_, Cin), -2, 2, "f16")
    Wt = I.small_ints(g, (k, k, Cin, Cout), -2, 2, "f16")
    bias = g.integers(-3, 4, size=Cout).astype(np.float32)
    ref = O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=stride, pad=pad)
    OH, OW = ref.shape[1], ref.shape[2]
    op = B.conv2d_op(N, H, W_, Cin, Cout, k, k, stride=stride, pad=pad, out_dtype="f32")
    space = op.space(B.SPACE_DEFAULT | B.SPACE_TAP_ROWS)
    assert space.flags & B.SPACE_TAP_ROWS
    patch_ok = (stride * Cin * 2) % 4 == 0
    want = {0: 3, 1: 3 if patch_ok else 0, 2: 2 if patch_ok else 0, 3: 1 if patch_ok else 0, 4: 2 if patch_ok else 0}
    idx = 0
    while any(want.values()) and idx < 800:
        t = B.trace_sample_valid(op, space, 102, idx)
        idx += 1
        p = B.trace_validate(op, space, t)
        assert p.tap_rows == 1 and (patch_ok or p.compute_at == 0)
        if want[p.compute_at] == 0:
            continue
        want[p.compute_at] -= 1
        print("trace", idx, "compute_at", p.compute_at, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f32", (N, OH, OW, Cout), instances=2)
        if got is None:
            continue
        assert np.array_equal(got[0], ref) and np.array_equal(got[1], ref), "trace %d" % idx
    assert want[0] == 0 and want[1] == 0 and want[2] == 0, want


def test_cbr_first_layer_filter_row_layout():
    """The paper's CBR shape in the filter-row layout (K = 7 rows of 21 -> 32 elements), fp16, both cache-read locations."""
    g = I.rng(63)
    X = I.uniform(g, (1, 224, 224, 3), 0.0, 1.0, "f16")
    Wt = I.normal(g, (7, 7, 3, 64), 0.05, "f16")
    bias = I.normal(g, (64,), 0.05, "f32")
    ref = O.conv2d_nhwc(X, Wt, bias=bias, relu=True, stride=2, pad=3)
    op = B.conv2d_op(1, 224, 224, 3, 64, 7, 7, stride=2, pad=3)
    space = op.space(B.SPACE_DEFAULT | B.SPACE_TAP_ROWS)
    want = {0: 2, 1: 2, 2: 2, 3: 1, 4: 1}
    idx = 0
    while any(want.values()) and idx < 400:
        t = B.trace_sample_valid(op, space, 104, idx)
        idx += 1
        ca = B.trace_validate(op, space, t).compute_at
        if want[ca] == 0:
            continue
        want[ca] -= 1
        print("trace", idx, "compute_at", ca, t.decisions(), flush=True)
        got = run_variant(op, space, t, [X, Wt, bias], "f16", ref.shape)
        if got is None:
            continue
        compare.assert_float_close(got, ref, compare.RTOL_HALF, "CBR filter rows trace %d" % idx)
    assert want[0] == 0 and want[1] == 0 and want[2] == 0, want
