"""Pins of the CPU oracle against facts it does not compute itself:
the paper's worked example, closed forms, invariants, brute force in pure
Python, and independent library routines (numpy float64 matmul, torch CPU
conv2d, scipy's softmax, numpy's norm).  All CPU-only.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import oracle as O
from paper_2205_13603_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- widening
def test_fp16_widening_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    h = bits.view(np.float16)
    want = h.astype(np.float64)
    got = O.widen(h)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bf16_widening():
    g = I.rng(3)
    x = g.normal(0, 10, size=4096).astype(np.float32)
    b = I.f32_to_bf16_bits(x)
    got = O.widen(b, bf16=True)
    assert np.array_equal(got, I.bf16_bits_to_f32(b).astype(np.float64))
    # bf16 keeps 8 significand bits: relative rounding error <= 2^-9
    assert np.all(np.abs(got - x) <= np.abs(x) * 2.0 ** -8)


# ---------------------------------------------------------------- split
def _read_split_example():
    f, e = None, None
    for line in open(os.path.join(GOLD, "split_example.txt")):
        t = line.split("#")[0].split()
        if not t:
            continue
        if t[0] == "factors":
            f = [int(v) for v in t[1:]]
        if t[0] == "extent":
            e = int(t[1])
    return f, e


def test_split_worked_example():
    f, e = _read_split_example()
    assert f == [32, 8, 4] and e == 1024
    walk = O.split_walk(f)
    assert walk.size == e
    # every original iteration exactly once, and consecutive loops keep order
    assert np.array_equal(walk, np.arange(e))


def test_split_index_formula_python():
    f = [3, 5, 2, 7]
    walk = O.split_walk(f)
    want = [((a * 5 + b) * 2 + c) * 7 + d for a in range(3) for b in range(5) for c in range(2) for d in range(7)]
    assert walk.tolist() == want


# ---------------------------------------------------------------- perfect tiles
def _golden_counts():
    rows = []
    for line in open(os.path.join(GOLD, "perfect_tile_counts.txt")):
        t = line.split("#")[0].split()
        if len(t) == 3:
            rows.append(tuple(int(v) for v in t))
    return rows


def _closed_form(extent, n):
    cnt, e, p = 1, extent, 2
    while e > 1:
        a = 0
        while e % p == 0:
            e //= p
            a += 1
        if a:
            cnt *= math.comb(a + n - 1, n - 1)
        p += 1
    return cnt


@pytest.mark.parametrize("extent,n,count", _golden_counts())
def test_perfect_tile_counts(extent, n, count):
    tiles = O.perfect_tiles(extent, n)
    assert tiles.shape == (count, n)
    assert _closed_form(extent, n) == count
    assert np.all(tiles >= 1)
    assert np.all(np.prod(tiles, axis=1) == extent)
    assert len({tuple(t) for t in tiles.tolist()}) == count


def test_perfect_tiles_bruteforce_python():
    for extent, n in [(12, 3), (30, 2), (16, 4), (7, 3)]:
        want = sorted(t for t in itertools.product(range(1, extent + 1), repeat=n) if math.prod(t) == extent)
        got = sorted(tuple(t) for t in O.perfect_tiles(extent, n).tolist())
        assert got == want


# ---------------------------------------------------------------- GEMM / BMM
def _py_matmul(A, B):
    M, K = len(A), len(A[0])
    N = len(B[0])
    return [[sum(A[i][k] * B[k][j] for k in range(K)) for j in range(N)] for i in range(M)]


def test_gemm_tiny_pure_python():
    g = I.rng(1)
    for (M, N, K) in [(1, 1, 1), (2, 3, 4), (5, 2, 7), (8, 8, 8)]:
        A = g.integers(-4, 5, size=(M, K)).astype(np.float32)
        B = g.integers(-4, 5, size=(K, N)).astype(np.float32)
        want = np.array(_py_matmul(A.astype(int).tolist(), B.astype(int).tolist()), np.float64)
        assert np.array_equal(O.gemm(A, B), want)


def test_gemm_identity_zero_ones():
    g = I.rng(2)
    A = g.uniform(-1, 1, size=(17, 9)).astype(np.float32)
    assert np.array_equal(O.gemm(A, np.eye(9, dtype=np.float32)), A.astype(np.float64))
    assert np.array_equal(O.gemm(np.eye(17, dtype=np.float32), A), A.astype(np.float64))
    assert np.all(O.gemm(A, np.zeros((9, 5), np.float32)) == 0)
    assert np.all(O.gemm(np.ones((6, 128), np.float16), np.ones((128, 4), np.float16)) == 128.0)


def test_gemm_linearity_exact_on_small_ints():
    A1, B = I.gemm_inputs(13, 11, 29, "f32", 5, "ints")
    A2, _ = I.gemm_inputs(13, 11, 29, "f32", 6, "ints")
    assert np.array_equal(O.gemm(A1 + A2, B), O.gemm(A1, B) + O.gemm(A2, B))
    assert np.array_equal(O.gemm(3 * A1, B), 3 * O.gemm(A1, B))


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_gemm_vs_numpy_float64(dtype):
    # non-square so that a transposed operand or swapped extent cannot pass
    A, B = I.gemm_inputs(37, 21, 53, dtype, 7, "normal", 1.0)
    if dtype == "bf16":
        Ad, Bd = I.bf16_bits_to_f32(A).astype(np.float64), I.bf16_bits_to_f32(B).astype(np.float64)
        got = O.gemm(A, B, bf16=True)
    else:
        Ad, Bd = A.astype(np.float64), B.astype(np.float64)
        got = O.gemm(A, B)
    want = Ad @ Bd
    # both accumulate in double; only the summation order may differ
    bound = 53 * 2.0 ** -52 * (np.abs(Ad) @ np.abs(Bd))
    assert np.all(np.abs(got - want) <= bound)


def test_bmm_nt_equals_per_head_gemm_with_materialised_transpose():
    Q, Kk = I.c4a(seed=4, heads=3, seq=10, dim=6)
    got = O.bmm(Q, Kk, trans_b=True)
    for h in range(3):
        KT = np.ascontiguousarray(Kk[h].T)
        assert np.array_equal(got[h], O.gemm(Q[h], KT))
    # strided view of a [seq][head][dim] layout gives the same result (fused transpose)
    Qs = np.ascontiguousarray(Q.transpose(1, 0, 2))
    assert np.array_equal(O.bmm(Qs.transpose(1, 0, 2), Kk, trans_b=True), got)


def test_bmm_nn_heads_independent():
    P, V = I.c4b(seed=5, heads=4, seq=8, dim=5)
    got = O.bmm(P, V)
    perm = [2, 0, 3, 1]
    assert np.array_equal(O.bmm(P[perm], V[perm]), got[perm])
    for h in range(4):
        assert np.array_equal(got[h], O.gemm(P[h], V[h]))


def test_int8_gemm_extremes_and_bigint():
    A = np.full((4, 512), -128, np.int8)
    B = np.full((512, 3), -128, np.int8)
    assert np.all(O.gemm(A, B) == 8388608)
    B2 = np.full((512, 3), 127, np.int8)
    assert np.all(O.gemm(A, B2) == -128 * 127 * 512)
    a, b = I.gemm_inputs(5, 4, 9, "i8", 8)
    want = np.array(_py_matmul(a.astype(int).tolist(), b.astype(int).tolist()), np.int64)
    got = O.gemm(a, b)
    assert got.dtype == np.int32 and np.array_equal(got.astype(np.int64), want)


def test_int8_gemm_vs_numpy_int64():
    a, b = I.gemm_inputs(33, 18, 47, "i8", 9)
    assert np.array_equal(O.gemm(a, b).astype(np.int64), a.astype(np.int64) @ b.astype(np.int64))


# ---------------------------------------------------------------- conv2d
def test_conv_out_size():
    assert O.conv_out_size(56, 3, 1, 1) == 56
    assert O.conv_out_size(56, 3, 2, 1) == 28
    assert O.conv_out_size(224, 7, 2, 3) == 112
    assert O.conv_out_size(112, 3, 1, 1) == 112


def test_conv_1x1_is_gemm():
    g = I.rng(10)
    X = g.integers(-3, 4, size=(2, 5, 4, 7)).astype(np.float32)
    W = g.integers(-3, 4, size=(1, 1, 7, 6)).astype(np.float32)
    got = O.conv2d_nhwc(X, W)
    want = O.gemm(X.reshape(-1, 7), W.reshape(7, 6)).reshape(2, 5, 4, 6)
    assert np.array_equal(got, want)


def test_conv_centre_tap_identity_and_shift():
    X, _, _ = I.c3(seed=11, H=9, W=7, Cin=5, Cout=5)
    W = np.zeros((3, 3, 5, 5), np.float16)
    for c in range(5):
        W[1, 1, c, c] = 1
    Y = O.conv2d_nhwc(X, W, bias=np.zeros(5, np.float32), relu=True, stride=1, pad=1)
    assert np.array_equal(Y, X.astype(np.float64))  # ReLU inactive: X in [0,1]
    # one-hot tap at (kh,kw) = (0,0): Y[oh][ow] = Xpad[oh-1][ow-1] -> shifted by (+1,+1)
    W0 = np.zeros((3, 3, 5, 5), np.float16)
    for c in range(5):
        W0[0, 0, c, c] = 1
    Y0 = O.conv2d_nhwc(X, W0, stride=1, pad=1)
    assert np.all(Y0[:, 0, :, :] == 0) and np.all(Y0[:, :, 0, :] == 0)
    assert np.array_equal(Y0[:, 1:, 1:, :], X.astype(np.float64)[:, :-1, :-1, :])
    # tap at (2,1): Y[oh][ow] = Xpad[oh+1][ow]
    W1 = np.zeros((3, 3, 5, 5), np.float16)
    for c in range(5):
        W1[2, 1, c, c] = 1
    Y1 = O.conv2d_nhwc(X, W1, stride=1, pad=1)
    assert np.all(Y1[:, -1, :, :] == 0)
    assert np.array_equal(Y1[:, :-1, :, :], X.astype(np.float64)[:, 1:, :, :])


def test_conv_all_ones_border_pattern():
    Cin = 64
    X = np.ones((1, 6, 8, Cin), np.float16)
    W = np.ones((3, 3, Cin, 3), np.float16)
    Y = O.conv2d_nhwc(X, W, stride=1, pad=1)
    assert np.all(Y[0, 1:-1, 1:-1] == 9 * Cin)
    assert np.all(Y[0, 0, 1:-1] == 6 * Cin) and np.all(Y[0, 1:-1, 0] == 6 * Cin)
    assert np.all(Y[0, -1, 1:-1] == 6 * Cin) and np.all(Y[0, 1:-1, -1] == 6 * Cin)
    for (a, b) in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(Y[0, a, b] == 4 * Cin)


def test_conv_bias_and_relu():
    X, W, bias = I.c3(seed=12, H=6, W=6, Cin=4, Cout=5)
    big_neg = np.full(5, -1e4, np.float32)
    assert np.all(O.conv2d_nhwc(X, W, bias=big_neg, relu=True, stride=1, pad=1) == 0)
    Y = O.conv2d_nhwc(X, np.zeros_like(W), bias=bias, relu=True, stride=1, pad=1)
    assert np.array_equal(Y, np.broadcast_to(np.maximum(0, bias.astype(np.float64)), Y.shape))
    # bias enters before ReLU, once per output element
    Yn = O.conv2d_nhwc(X, W, bias=None, relu=False, stride=1, pad=1)
    Yb = O.conv2d_nhwc(X, W, bias=bias, relu=False, stride=1, pad=1)
    assert np.allclose(Yb - Yn, bias.astype(np.float64), rtol=0, atol=1e-12)
    Yr = O.conv2d_nhwc(X, W, bias=bias, relu=True, stride=1, pad=1)
    assert np.array_equal(Yr, np.maximum(Yb, 0))


@pytest.mark.parametrize("stride,pad,k", [(1, 1, 3), (2, 1, 3), (2, 3, 7), (1, 0, 2)])
def test_conv_vs_torch_cpu(stride, pad, k):
    torch = pytest.importorskip("torch")
    g = I.rng(13)
    X = g.normal(size=(2, 11, 9, 5)).astype(np.float32)
    W = g.normal(size=(k, k, 5, 4)).astype(np.float32)
    b = g.normal(size=4).astype(np.float32)
    got = O.conv2d_nhwc(X, W, bias=b, relu=True, stride=stride, pad=pad)
    xt = torch.from_numpy(X).double().permute(0, 3, 1, 2)
    wt = torch.from_numpy(W).double().permute(3, 2, 0, 1)
    want = torch.relu(torch.nn.functional.conv2d(xt, wt, torch.from_numpy(b).double(), stride=stride, padding=pad))
    want = want.permute(0, 2, 3, 1).numpy()
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("stride,pad,k,dil", [(1, 2, 3, 2), (2, 2, 3, 2), (1, 3, 2, 3), (1, 0, 3, 2)])
def test_dilated_conv_vs_torch_cpu_and_vs_zero_stuffed_filter(stride, pad, k, dil):
    """Dilation: (a) an independent library routine; (b) by definition a dilated k x k filter equals the dense
    (dil*(k-1)+1)-wide filter whose taps sit `dil` apart with zeros between them."""
    torch = pytest.importorskip("torch")
    g = I.rng(19)
    X = g.normal(size=(2, 12, 10, 3)).astype(np.float32)
    W = g.normal(size=(k, k, 3, 4)).astype(np.float32)
    b = g.normal(size=4).astype(np.float32)
    got = O.conv2d_nhwc(X, W, bias=b, relu=True, stride=stride, pad=pad, dilation=dil)
    xt = torch.from_numpy(X).double().permute(0, 3, 1, 2)
    wt = torch.from_numpy(W).double().permute(3, 2, 0, 1)
    want = torch.relu(torch.nn.functional.conv2d(xt, wt, torch.from_numpy(b).double(), stride=stride, padding=pad, dilation=dil))
    want = want.permute(0, 2, 3, 1).numpy()
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    ke = dil * (k - 1) + 1
    Wz = np.zeros((ke, ke, 3, 4), np.float32)
    Wz[::dil, ::dil] = W
    assert np.array_equal(got, O.conv2d_nhwc(X, Wz, bias=b, relu=True, stride=stride, pad=pad))
    # one-hot tap at (k-1, k-1): the image shifted by dil*(k-1) - pad in both directions
    W1 = np.zeros((k, k, 3, 3), np.float32)
    for c in range(3):
        W1[k - 1, k - 1, c, c] = 1
    Y = O.conv2d_nhwc(X, W1, stride=1, pad=pad, dilation=dil)
    sh = dil * (k - 1) - pad
    for oh in range(Y.shape[1]):
        for ow in range(Y.shape[2]):
            ih, iw = oh + sh, ow + sh
            ref = X[:, ih, iw, :] if 0 <= ih < 12 and 0 <= iw < 10 else 0.0
            assert np.array_equal(Y[:, oh, ow, :], np.broadcast_to(ref, (2, 3)).astype(np.float64))


# ---------------------------------------------------------------- depthwise
def test_dw_equals_conv_with_block_diagonal_weights():
    X, W = I.dw_inputs(2, 7, 6, 5, seed=14)
    Wfull = np.zeros((3, 3, 5, 5), np.float32)
    for c in range(5):
        Wfull[:, :, c, c] = W[:, :, c]
    for s in (1, 2):
        assert np.array_equal(O.dwconv2d_nhwc(X, W, stride=s, pad=1), O.conv2d_nhwc(X, Wfull, stride=s, pad=1))


def test_dw_all_ones_patterns():
    X = np.ones((1, 10, 10, 3), np.float32)
    W = np.ones((3, 3, 3), np.float32)
    Y = O.dwconv2d_nhwc(X, W, stride=1, pad=1)
    assert np.all(Y[0, 1:-1, 1:-1] == 9) and np.all(Y[0, 0, 1:-1] == 6) and Y[0, 0, 0, 0] == 4 and Y[0, -1, -1, 0] == 4
    # stride 2, pad 1, even H: only the top/left padding is touched
    X = np.ones((1, 56, 56, 2), np.float32)
    W = np.ones((3, 3, 2), np.float32)
    Y = O.dwconv2d_nhwc(X, W, stride=2, pad=1)
    assert Y.shape == (1, 28, 28, 2)
    assert np.all(Y[0, 0, 0] == 4) and np.all(Y[0, 0, 1:] == 6) and np.all(Y[0, 1:, 0] == 6) and np.all(Y[0, 1:, 1:] == 9)


def test_dw_channel_permutation():
    X, W = I.dw_inputs(1, 9, 8, 6, seed=15)
    perm = np.array([3, 0, 5, 1, 4, 2])
    Y = O.dwconv2d_nhwc(X, W, stride=1, pad=1)
    Yp = O.dwconv2d_nhwc(np.ascontiguousarray(X[..., perm]), np.ascontiguousarray(W[..., perm]), stride=1, pad=1)
    assert np.array_equal(Yp, Y[..., perm])


@pytest.mark.parametrize("stride", [1, 2])
def test_dw_vs_torch_cpu(stride):
    torch = pytest.importorskip("torch")
    X, W = I.dw_inputs(2, 12, 10, 7, seed=16)
    got = O.dwconv2d_nhwc(X, W, stride=stride, pad=1)
    xt = torch.from_numpy(X).double().permute(0, 3, 1, 2)
    wt = torch.from_numpy(W).double().permute(2, 0, 1).unsqueeze(1)
    want = torch.nn.functional.conv2d(xt, wt, None, stride=stride, padding=1, groups=7).permute(0, 2, 3, 1).numpy()
    assert got.shape == want.shape and np.allclose(got, want, rtol=1e-12, atol=1e-12)


def test_full_size_spot_checks():
    """Config-size runs finish in seconds; spot-check single outputs by the definition."""
    A, B = I.c1()
    C = O.gemm(A, B)
    for (i, j) in [(0, 0), (127, 127), (5, 99)]:
        assert abs(C[i, j] - float(np.dot(A[i].astype(np.float64), B[:, j].astype(np.float64)))) < 1e-12
    X, W = I.c5b()
    Y = O.dwconv2d_nhwc(X, W, stride=2, pad=1)
    assert Y.shape == (1, 28, 28, 144)
    oh, ow, c = 27, 27, 143
    acc = 0.0
    for kh in range(3):
        for kw in range(3):
            ih, iw = oh * 2 + kh - 1, ow * 2 + kw - 1
            assert 0 <= ih < 56 and 0 <= iw < 56
            acc += float(X[0, ih, iw, c]) * float(W[kh, kw, c])
    assert abs(Y[0, oh, ow, c] - acc) < 1e-12


# ---------------------------------------------------------------- 8-bit floats
def test_f8e4m3_decoder_all_256_patterns():
    """Every bit pattern of the 8-bit float with 4 exponent and 3 mantissa bits (bias 7, no infinities, 0x7f / 0xff NaN):
    closed forms, and an independent library's decoder."""
    bits = np.arange(256, dtype=np.uint8)
    got = O.widen(bits)
    assert got[0x00] == 0.0 and got[0x80] == 0.0 and np.signbit(got[0x80])
    assert got[0x38] == 1.0 and got[0x40] == 2.0 and got[0x30] == 0.5 and got[0xB8] == -1.0
    assert got[0x01] == 2.0 ** -9 and got[0x07] == 7 * 2.0 ** -9 and got[0x08] == 2.0 ** -6   # subnormals, smallest normal
    assert got[0x7E] == 448.0 and got[0xFE] == -448.0                                          # largest finite
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and np.isfinite(np.delete(got, [0x7F, 0xFF])).all()
    # monotone on the positive half, 8 values per binade
    pos = got[:0x7F]
    assert np.all(np.diff(pos) > 0)
    for e in range(1, 15):
        assert got[8 * e] == 2.0 ** (e - 7) and got[8 * e + 4] == 1.5 * 2.0 ** (e - 7)
    torch = pytest.importorskip("torch")
    if not hasattr(torch, "float8_e4m3fn"):
        pytest.skip("this torch has no 8-bit float type")
    want = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).double().numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(got)
    assert np.array_equal(got[ok], want[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


def test_f8_gemm_against_decoded_float64_matmul():
    g = I.rng(21)
    A = g.integers(0, 256, size=(9, 16), dtype=np.uint8)
    Bm = g.integers(0, 256, size=(16, 7), dtype=np.uint8)
    A[(A & 0x7F) == 0x7F] = 0x38                      # no NaN patterns
    Bm[(Bm & 0x7F) == 0x7F] = 0x38
    got = O.gemm(A, Bm)
    want = O.widen(A) @ O.widen(Bm)
    assert np.allclose(got, want, rtol=1e-13, atol=0)
    # products and sums of these values are exact in double: brute force in index order agrees bit for bit
    a, b = O.widen(A), O.widen(Bm)
    brute = np.zeros((9, 7))
    for i in range(9):
        for j in range(7):
            acc = 0.0
            for k in range(16):
                acc += a[i, k] * b[k, j]
            brute[i, j] = acc
    assert np.array_equal(got, brute)


# ---------------------------------------------------------------- softmax and norm (Appendix A.2: SFM, NRM)

def test_softmax_closed_forms():
    n = 7
    y = O.softmax(np.full((3, n), 2.5, np.float32))
    assert np.array_equal(y, np.full((3, n), 1.0 / n))                      # uniform row
    a, b = 0.75, -1.5
    y = O.softmax(np.array([[a, b]], np.float32))
    assert abs(y[0, 0] - 1.0 / (1.0 + math.exp(b - a))) < 1e-16            # two elements: the logistic function
    assert abs(y[0, 1] - 1.0 / (1.0 + math.exp(a - b))) < 1e-16
    y = O.softmax(np.array([[1000.0, 999.0, -1000.0]], np.float32))         # no overflow, no NaN; the third term vanishes
    assert abs(y[0, 0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15 and y[0, 2] == 0.0


def test_softmax_is_over_the_last_axis_and_rows_are_independent():
    X = np.array([[[0.0, math.log(3.0)], [5.0, 5.0]], [[-2.0, -2.0], [math.log(3.0), 0.0]]], np.float64).astype(np.float32)
    y = O.softmax(X)
    assert y.shape == X.shape
    np.testing.assert_allclose(y[0, 0], [0.25, 0.75], rtol=1e-7)
    np.testing.assert_allclose(y[1, 1], [0.75, 0.25], rtol=1e-7)
    assert np.array_equal(y[0, 1], [0.5, 0.5]) and np.array_equal(y[1, 0], [0.5, 0.5])


def test_softmax_invariants_and_library():
    from scipy.special import softmax as sp_softmax
    g = np.random.default_rng(5)
    X = g.integers(-8, 9, (6, 33)).astype(np.float32)
    y = O.softmax(X)
    assert np.all(y > 0) and np.max(np.abs(y.sum(-1) - 1.0)) < 1e-15
    np.testing.assert_allclose(O.softmax(X + np.float32(3.0)), y, rtol=1e-15)        # shift invariance (integers: exact shift)
    i, j = 4, 17
    np.testing.assert_allclose(y[:, i] / y[:, j], np.exp(X[:, i].astype(np.float64) - X[:, j]), rtol=1e-14)
    for dt in (np.float32, np.float16):
        Xr = (g.standard_normal((5, 256)) * 3).astype(dt)
        np.testing.assert_allclose(O.softmax(Xr), sp_softmax(Xr.astype(np.float64), axis=-1), rtol=1e-13, atol=0)
    perm = g.permutation(33)
    np.testing.assert_allclose(O.softmax(np.ascontiguousarray(X[:, perm])), y[:, perm], rtol=1e-14)


def test_norm_closed_forms_and_library():
    assert np.array_equal(O.norm(np.array([[3.0, 4.0, 0.0, 0.0], [5.0, 0.0, -12.0, 0.0]], np.float32)), [5.0, 13.0])
    assert np.array_equal(O.norm(np.ones((2, 16, 16), np.float16)), [16.0, 16.0])    # sqrt(256 ones)
    g = np.random.default_rng(6)
    X = g.standard_normal((3, 40, 50)).astype(np.float32)
    ref = np.sqrt((X.astype(np.float64) ** 2).reshape(3, -1).sum(-1))
    np.testing.assert_allclose(O.norm(X), ref, rtol=1e-14)
    np.testing.assert_allclose(O.norm(X), np.linalg.norm(X.astype(np.float64).reshape(3, -1), axis=1), rtol=1e-14)
    assert np.array_equal(O.norm(X * np.float32(2.0)), 2.0 * O.norm(X))              # homogeneity (scaling by 2 is exact)
    assert np.array_equal(O.norm(-X), O.norm(X))
    assert np.array_equal(O.norm(X[::-1].copy()), O.norm(X)[::-1])                   # one number per batch entry


# ---------------------------------------------------------------- transposed conv2d (Appendix A.2: T2D)

@pytest.mark.parametrize("stride,pad,k", [(2, 1, 4), (1, 0, 3), (2, 0, 2), (3, 2, 5), (1, 1, 3)])
def test_transposed_conv_vs_torch_cpu_and_adjoint_identity(stride, pad, k):
    import torch
    g = np.random.default_rng(70 + stride + k)
    N, H, W_, Cin, Cout = 2, 5, 4, 3, 6
    X = g.standard_normal((N, H, W_, Cin)).astype(np.float32)
    Wt = g.standard_normal((k, k, Cin, Cout)).astype(np.float32)
    bias = g.standard_normal(Cout).astype(np.float32)
    got = O.conv2d_transposed_nhwc(X, Wt, bias=bias, relu=False, stride=stride, pad=pad)
    # library routine: weight layout (Cin, Cout, KH, KW), activations NCHW
    ref = torch.nn.functional.conv_transpose2d(torch.from_numpy(X).double().permute(0, 3, 1, 2),
                                               torch.from_numpy(Wt).double().permute(2, 3, 0, 1),
                                               torch.from_numpy(bias).double(), stride=stride, padding=pad)
    np.testing.assert_allclose(got, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    assert got.shape == (N, (H - 1) * stride - 2 * pad + k, (W_ - 1) * stride - 2 * pad + k, Cout)
    # adjoint of the (pinned) direct convolution: <conv(Z, W'), X> = <Z, convT(X, W)> with W'[kh][kw][co][ci] = W[kh][kw][ci][co]
    Z = g.standard_normal(got.shape).astype(np.float32)
    fwd = O.conv2d_nhwc(Z, np.ascontiguousarray(Wt.transpose(0, 1, 3, 2)), stride=stride, pad=pad)
    assert fwd.shape == X.shape
    lhs = float((fwd * X).sum())
    rhs = float((Z.astype(np.float64) * O.conv2d_transposed_nhwc(X, Wt, stride=stride, pad=pad)).sum())
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))


def test_transposed_conv_closed_forms():
    # one input pixel, stride 2, no padding: the output is the filter itself, placed at (2*ih, 2*iw)
    Wt = np.arange(1, 10, dtype=np.float32).reshape(3, 3, 1, 1)
    X = np.zeros((1, 2, 2, 1), np.float32)
    X[0, 1, 0, 0] = 2.0
    y = O.conv2d_transposed_nhwc(X, Wt, stride=2, pad=0)
    assert y.shape == (1, 5, 5, 1)
    want = np.zeros((5, 5))
    want[2:5, 0:3] = 2.0 * Wt[:, :, 0, 0]
    assert np.array_equal(y[0, :, :, 0], want)
    # stride 1, 1x1 filter: a plain matrix product over channels; bias then ReLU
    g = np.random.default_rng(9)
    X = g.integers(-3, 4, (1, 3, 3, 4)).astype(np.float32)
    W1 = g.integers(-3, 4, (1, 1, 4, 5)).astype(np.float32)
    b = np.arange(-2, 3, dtype=np.float32)
    y = O.conv2d_transposed_nhwc(X, W1, bias=b, relu=True, stride=1, pad=0)
    assert np.array_equal(y, np.maximum(X.astype(np.float64) @ W1[0, 0].astype(np.float64) + b, 0.0))
    # all ones, 2x2 filter, stride 1: every output counts the inputs that reach it (1, 2 or 4)
    y = O.conv2d_transposed_nhwc(np.ones((1, 3, 3, 1), np.float16), np.ones((2, 2, 1, 1), np.float16), stride=1, pad=0)
    assert np.array_equal(y[0, :, :, 0], [[1, 2, 2, 1], [2, 4, 4, 2], [2, 4, 4, 2], [1, 2, 2, 1]])


# ---------------------------------------------------------------- grouped conv2d (Appendix A.2: GRP)

@pytest.mark.parametrize("groups,stride,pad,k", [(4, 2, 1, 3), (2, 1, 0, 1), (3, 1, 1, 3)])
def test_grouped_conv_vs_torch_cpu_and_vs_block_diagonal_weights(groups, stride, pad, k):
    import torch
    g = np.random.default_rng(80 + groups)
    N, H, W_, Cin, Cout = 2, 7, 6, 12, 24
    Cg, Ng = Cin // groups, Cout // groups
    X = g.standard_normal((N, H, W_, Cin)).astype(np.float32)
    Wt = g.standard_normal((k, k, Cg, Cout)).astype(np.float32)
    bias = g.standard_normal(Cout).astype(np.float32)
    got = O.conv2d_nhwc(X, Wt, bias=bias, relu=False, stride=stride, pad=pad, groups=groups)
    # library routine: weight (Cout, Cin/groups, KH, KW)
    ref = torch.nn.functional.conv2d(torch.from_numpy(X).double().permute(0, 3, 1, 2), torch.from_numpy(Wt).double().permute(3, 2, 0, 1),
                                     torch.from_numpy(bias).double(), stride=stride, padding=pad, groups=groups)
    np.testing.assert_allclose(got, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    # the same operator as a dense convolution whose weights are zero outside the diagonal blocks
    Wd = np.zeros((k, k, Cin, Cout), np.float32)
    for q in range(groups):
        Wd[:, :, q * Cg:(q + 1) * Cg, q * Ng:(q + 1) * Ng] = Wt[:, :, :, q * Ng:(q + 1) * Ng]
    np.testing.assert_allclose(got, O.conv2d_nhwc(X, Wd, bias=bias, stride=stride, pad=pad), rtol=1e-13, atol=1e-13)
    # groups == channels with one output per group is the depthwise operator
    Xd = g.standard_normal((1, 6, 6, 5)).astype(np.float32)
    Wdw = g.standard_normal((3, 3, 5)).astype(np.float32)
    np.testing.assert_allclose(O.conv2d_nhwc(Xd, Wdw.reshape(3, 3, 1, 5), stride=1, pad=1, groups=5),
                               O.dwconv2d_nhwc(Xd, Wdw, stride=1, pad=1), rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- conv1d (Appendix A.2: C1D)

@pytest.mark.parametrize("stride,pad,k,dil", [(2, 1, 3, 1), (1, 0, 1, 1), (1, 2, 5, 1), (1, 2, 3, 2), (3, 0, 4, 1)])
def test_conv1d_vs_torch_cpu_and_closed_forms(stride, pad, k, dil):
    import torch
    g = np.random.default_rng(90 + k)
    N, L_, Cin, Cout = 2, 19, 5, 7
    X = g.standard_normal((N, L_, Cin)).astype(np.float32)
    Wt = g.standard_normal((k, Cin, Cout)).astype(np.float32)
    bias = g.standard_normal(Cout).astype(np.float32)
    got = O.conv1d_nwc(X, Wt, bias=bias, stride=stride, pad=pad, dilation=dil)
    ref = torch.nn.functional.conv1d(torch.from_numpy(X).double().permute(0, 2, 1), torch.from_numpy(Wt).double().permute(2, 1, 0),
                                     torch.from_numpy(bias).double(), stride=stride, padding=pad, dilation=dil)
    np.testing.assert_allclose(got, ref.permute(0, 2, 1).numpy(), rtol=1e-12, atol=1e-12)
    # all ones, no padding: every output = K * Cin; with padding the two ends see fewer taps
    y = O.conv1d_nwc(np.ones((1, 8, 3), np.float32), np.ones((3, 3, 2), np.float32), stride=1, pad=1)
    assert np.array_equal(y[0, :, 0], [6, 9, 9, 9, 9, 9, 9, 6])
    # one-hot tap 0 with padding 1 shifts the signal right by one (pins the padding direction)
    W0 = np.zeros((3, 1, 1), np.float32)
    W0[0, 0, 0] = 1.0
    sig = np.arange(1, 7, dtype=np.float32).reshape(1, 6, 1)
    assert np.array_equal(O.conv1d_nwc(sig, W0, stride=1, pad=1)[0, :, 0], [0, 1, 2, 3, 4, 5])
    # a 1 x K conv2d over an image of height 1 is the same operator when it is not padded
    if pad == 0:
        y2 = O.conv2d_nhwc(X[:, None], Wt[None], bias=bias, stride=stride, pad=0, dilation=dil)
        np.testing.assert_allclose(got, y2[:, 0], rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- conv3d (Appendix A.2: C3D)

@pytest.mark.parametrize("stride,pad,k,dil", [(2, 3, 7, 1), (1, 0, 1, 1), (1, 1, 3, 1), (2, 1, 3, 1), (1, 2, 3, 2)])
def test_conv3d_vs_torch_cpu_and_reductions_to_conv2d(stride, pad, k, dil):
    import torch
    g = np.random.default_rng(95 + k + stride)
    N, D, H, W_, Cin, Cout = 2, 6, 7, 5, 3, 4
    X = g.standard_normal((N, D, H, W_, Cin)).astype(np.float32)
    Wt = g.standard_normal((k, k, k, Cin, Cout)).astype(np.float32)
    bias = g.standard_normal(Cout).astype(np.float32)
    got = O.conv3d_ndhwc(X, Wt, bias=bias, stride=stride, pad=pad, dilation=dil)
    ref = torch.nn.functional.conv3d(torch.from_numpy(X).double().permute(0, 4, 1, 2, 3), torch.from_numpy(Wt).double().permute(4, 3, 0, 1, 2),
                                     torch.from_numpy(bias).double(), stride=stride, padding=pad, dilation=dil)
    np.testing.assert_allclose(got, ref.permute(0, 2, 3, 4, 1).numpy(), rtol=1e-12, atol=1e-12)
    # depth 1 and a filter of depth 1, unpadded: the (pinned) conv2d
    if pad == 0:
        X2 = X[:, :1]
        W2 = g.standard_normal((1, k, k, Cin, Cout)).astype(np.float32)
        np.testing.assert_allclose(O.conv3d_ndhwc(X2, W2, bias=bias, stride=stride, pad=0, dilation=dil)[:, 0],
                                   O.conv2d_nhwc(X2[:, 0], W2[0], bias=bias, stride=stride, pad=0, dilation=dil), rtol=1e-13, atol=1e-13)


def test_conv3d_closed_forms():
    # all ones, 3x3x3, padding 1: an output counts the taps inside the volume: 27 inside, 18 on a face, 12 on an edge, 8 at a corner
    y = O.conv3d_ndhwc(np.ones((1, 4, 4, 4, 1), np.float32), np.ones((3, 3, 3, 1, 1), np.float32), stride=1, pad=1)[0, :, :, :, 0]
    assert y[1, 1, 1] == 27 and y[0, 1, 1] == 18 and y[0, 0, 1] == 12 and y[0, 0, 0] == 8 and y[3, 3, 3] == 8
    # one-hot tap (0, 0, 0) with padding 1 shifts the volume by (+1, +1, +1)
    W0 = np.zeros((3, 3, 3, 1, 1), np.float32)
    W0[0, 0, 0, 0, 0] = 1.0
    vol = np.arange(1, 28, dtype=np.float32).reshape(1, 3, 3, 3, 1)
    y = O.conv3d_ndhwc(vol, W0, stride=1, pad=1)[0, :, :, :, 0]
    assert np.array_equal(y[1:, 1:, 1:], vol[0, :2, :2, :2, 0]) and not y[0].any() and not y[:, 0].any() and not y[:, :, 0].any()
    # the three axes are distinguished: a filter that is 1 only at kd = 2 (kh = kw = 1) shifts along depth only
    W1 = np.zeros((3, 3, 3, 1, 1), np.float32)
    W1[2, 1, 1, 0, 0] = 1.0
    y = O.conv3d_ndhwc(vol, W1, stride=1, pad=1)[0, :, :, :, 0]
    assert np.array_equal(y[:2], vol[0, 1:, :, :, 0]) and not y[2].any()
