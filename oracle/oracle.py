"""ctypes front for oracle/libms_oracle.so (test infrastructure).

Every function takes numpy arrays holding the exact bits the GPU path is
given (fp16 as float16, bf16 as uint16 bit patterns, int8, fp32) and returns
float64 (int32 for the int8 operator).  Definitions: Appendix A.2 workloads
GMM, TBG, C2D/CBR, DEP, SFM, NRM of arXiv 2205.13603, written out in ms_oracle.c.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, F16, BF16, I8, F8E4M3 = 0, 1, 2, 3, 5

_lib = None
_libs = {}
_kind = "f64"


def use_build(kind):
    """Select which build of ms_oracle.c the following calls run: "f64" = the oracle (double accumulation; the only one
    tests ever use), "f32acc" = the same loops accumulating in float, which bench.py times as a second CPU baseline."""
    global _lib, _kind
    assert kind in ("f64", "f32acc")
    _kind = kind
    _lib = _libs.get(kind)


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        if _kind == "f32acc":
            path = _build.LIB_F32ACC
        L = C.CDLL(path)
        i64, vp, dp = C.c_int64, C.c_void_p, C.POINTER(C.c_double)
        L.ms_oracle_threads.restype = C.c_int
        L.ms_oracle_widen.restype = C.c_double
        L.ms_oracle_widen.argtypes = [C.c_int, vp, i64]
        L.ms_oracle_bmm.restype = C.c_int
        L.ms_oracle_bmm.argtypes = [C.c_int, i64, i64, i64, i64, vp, i64, i64, i64, vp, i64, i64, i64, vp]
        L.ms_oracle_bmm_i8.restype = C.c_int
        L.ms_oracle_bmm_i8.argtypes = [i64, i64, i64, i64, vp, i64, i64, i64, vp, i64, i64, i64, vp]
        L.ms_oracle_conv_out_size.restype = i64
        L.ms_oracle_conv_out_size.argtypes = [i64, i64, i64, i64]
        L.ms_oracle_conv2d_nhwc.restype = C.c_int
        L.ms_oracle_conv2d_nhwc.argtypes = [C.c_int] + [i64] * 11 + [vp, vp, vp, C.c_int, vp]
        L.ms_oracle_conv3d_ndhwc.restype = C.c_int
        L.ms_oracle_conv3d_ndhwc.argtypes = [C.c_int] + [i64] * 12 + [vp, vp, vp, C.c_int, vp]
        L.ms_oracle_conv1d_nwc.restype = C.c_int
        L.ms_oracle_conv1d_nwc.argtypes = [C.c_int] + [i64] * 8 + [vp, vp, vp, C.c_int, vp]
        L.ms_oracle_conv2d_transposed_nhwc.restype = C.c_int
        L.ms_oracle_conv2d_transposed_nhwc.argtypes = [C.c_int] + [i64] * 9 + [vp, vp, vp, C.c_int, vp]
        L.ms_oracle_dwconv2d_nhwc.restype = C.c_int
        L.ms_oracle_dwconv2d_nhwc.argtypes = [C.c_int] + [i64] * 8 + [vp, vp, vp]
        L.ms_oracle_softmax.restype = C.c_int
        L.ms_oracle_softmax.argtypes = [C.c_int, i64, i64, vp, vp]
        L.ms_oracle_norm.restype = C.c_int
        L.ms_oracle_norm.argtypes = [C.c_int, i64, i64, vp, vp]
        L.ms_oracle_split_walk.restype = i64
        L.ms_oracle_split_walk.argtypes = [C.c_int, vp, vp, i64]
        L.ms_oracle_perfect_tiles.restype = i64
        L.ms_oracle_perfect_tiles.argtypes = [i64, C.c_int, vp, i64]
        L.ms_oracle_set_threads.restype = None
        L.ms_oracle_set_threads.argtypes = [C.c_int]
        _lib = L
        _libs[_kind] = L
    return _lib


def threads():
    return int(lib().ms_oracle_threads())


def set_threads(n):
    """OpenMP threads of the following oracle calls (0 = the default); for the benchmark's single-thread baseline."""
    lib().ms_oracle_set_threads(int(n))


def _dtype_code(a, bf16=False):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    if a.dtype == np.uint16 and bf16:
        return BF16
    if a.dtype == np.int8:
        return I8
    if a.dtype == np.uint8:
        return F8E4M3  # bit patterns of 8-bit floats (4 exponent bits, 3 mantissa bits)
    raise TypeError("unsupported dtype %s" % a.dtype)


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def widen(a, bf16=False):
    """Element-wise exact widening to float64 through the oracle's own decoder."""
    a = np.ascontiguousarray(a)
    code = _dtype_code(a, bf16)
    flat = a.reshape(-1)
    out = np.empty(flat.size, np.float64)
    L = lib()
    for i in range(flat.size):
        out[i] = L.ms_oracle_widen(code, _ptr(flat), i)
    return out.reshape(a.shape)


def bmm(A, B, trans_b=False, bf16=False):
    """C[b,i,j] = sum_k A[b,i,k] * B[b,k,j].

    A is [nb,M,K] (any strides, they are passed through).  B is [nb,K,N], or
    [nb,N,K] when trans_b (the "NT" form: reduction index contiguous in both).
    """
    assert A.ndim == 3 and B.ndim == 3 and A.dtype == B.dtype
    nb, M, K = A.shape
    if trans_b:
        assert B.shape[0] == nb and B.shape[2] == K
        N = B.shape[1]
        sBb, sBj, sBk = (s // B.itemsize for s in B.strides)
    else:
        assert B.shape[0] == nb and B.shape[1] == K
        N = B.shape[2]
        sBb, sBk, sBj = (s // B.itemsize for s in B.strides)
    sAb, sAi, sAk = (s // A.itemsize for s in A.strides)
    L = lib()
    if A.dtype == np.int8:
        out = np.empty((nb, M, N), np.int32)
        rc = L.ms_oracle_bmm_i8(nb, M, N, K, _ptr(A), sAb, sAi, sAk, _ptr(B), sBb, sBk, sBj, _ptr(out))
    else:
        out = np.empty((nb, M, N), np.float64)
        rc = L.ms_oracle_bmm(_dtype_code(A, bf16), nb, M, N, K, _ptr(A), sAb, sAi, sAk,
                             _ptr(B), sBb, sBk, sBj, _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle bmm failed")
    return out


def gemm(A, B, bf16=False):
    """C = A.B for 2-D A [M,K], B [K,N]."""
    return bmm(A[None], B[None], bf16=bf16)[0]


def conv_out_size(n, k, s, p):
    return int(lib().ms_oracle_conv_out_size(n, k, s, p))


def conv2d_nhwc(X, Wt, bias=None, relu=False, stride=1, pad=0, bf16=False, dilation=1, groups=1):
    """X [N,H,W,Cin], Wt [KH,KW,Cin/groups,Cout], bias fp32 [Cout] or None; taps `dilation` elements apart."""
    X = np.ascontiguousarray(X)
    Wt = np.ascontiguousarray(Wt)
    N, H, W_, Cin = X.shape
    KH, KW, Cin2, Cout = Wt.shape
    assert Cin2 * groups == Cin and Cout % groups == 0 and X.dtype == Wt.dtype
    OH, OW = conv_out_size(H, dilation * (KH - 1) + 1, stride, pad), conv_out_size(W_, dilation * (KW - 1) + 1, stride, pad)
    out = np.empty((N, OH, OW, Cout), np.float64)
    bptr = None
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.shape == (Cout,)
        bptr = _ptr(bias)
    rc = lib().ms_oracle_conv2d_nhwc(_dtype_code(X, bf16), N, H, W_, Cin, Cout, KH, KW, stride, pad, dilation, groups,
                                     _ptr(X), _ptr(Wt), bptr, int(bool(relu)), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle conv2d failed")
    return out


def conv3d_ndhwc(X, Wt, bias=None, relu=False, stride=1, pad=0, bf16=False, dilation=1):
    """X [N,D,H,W,Cin], Wt [KD,KH,KW,Cin,Cout], bias fp32 [Cout] or None."""
    X = np.ascontiguousarray(X)
    Wt = np.ascontiguousarray(Wt)
    N, D, H, W_, Cin = X.shape
    KD, KH, KW, Cin2, Cout = Wt.shape
    assert Cin2 == Cin and X.dtype == Wt.dtype
    OD, OH, OW = (conv_out_size(e, dilation * (k - 1) + 1, stride, pad) for e, k in ((D, KD), (H, KH), (W_, KW)))
    out = np.empty((N, OD, OH, OW, Cout), np.float64)
    bptr = None
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.shape == (Cout,)
        bptr = _ptr(bias)
    rc = lib().ms_oracle_conv3d_ndhwc(_dtype_code(X, bf16), N, D, H, W_, Cin, Cout, KD, KH, KW, stride, pad, dilation,
                                      _ptr(X), _ptr(Wt), bptr, int(bool(relu)), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle conv3d failed")
    return out


def conv1d_nwc(X, Wt, bias=None, relu=False, stride=1, pad=0, bf16=False, dilation=1):
    """X [N,L,Cin], Wt [K,Cin,Cout], bias fp32 [Cout] or None."""
    X = np.ascontiguousarray(X)
    Wt = np.ascontiguousarray(Wt)
    N, L_, Cin = X.shape
    K, Cin2, Cout = Wt.shape
    assert Cin2 == Cin and X.dtype == Wt.dtype
    OL = conv_out_size(L_, dilation * (K - 1) + 1, stride, pad)
    out = np.empty((N, OL, Cout), np.float64)
    bptr = None
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.shape == (Cout,)
        bptr = _ptr(bias)
    rc = lib().ms_oracle_conv1d_nwc(_dtype_code(X, bf16), N, L_, Cin, Cout, K, stride, pad, dilation, _ptr(X), _ptr(Wt), bptr,
                                    int(bool(relu)), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle conv1d failed")
    return out


def conv2d_transposed_nhwc(X, Wt, bias=None, relu=False, stride=1, pad=0, bf16=False):
    """X [N,H,W,Cin], Wt [KH,KW,Cin,Cout]; output [N, (H-1)*stride - 2*pad + KH, (W-1)*stride - 2*pad + KW, Cout]."""
    X = np.ascontiguousarray(X)
    Wt = np.ascontiguousarray(Wt)
    N, H, W_, Cin = X.shape
    KH, KW, Cin2, Cout = Wt.shape
    assert Cin2 == Cin and X.dtype == Wt.dtype
    OH, OW = (H - 1) * stride - 2 * pad + KH, (W_ - 1) * stride - 2 * pad + KW
    out = np.empty((N, OH, OW, Cout), np.float64)
    bptr = None
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        assert bias.shape == (Cout,)
        bptr = _ptr(bias)
    rc = lib().ms_oracle_conv2d_transposed_nhwc(_dtype_code(X, bf16), N, H, W_, Cin, Cout, KH, KW, stride, pad,
                                                _ptr(X), _ptr(Wt), bptr, int(bool(relu)), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle transposed conv2d failed")
    return out


def dwconv2d_nhwc(X, Wt, stride=1, pad=0, bf16=False):
    """X [N,H,W,C], Wt [KH,KW,C]."""
    X = np.ascontiguousarray(X)
    Wt = np.ascontiguousarray(Wt)
    N, H, W_, Cc = X.shape
    KH, KW, C2 = Wt.shape
    assert C2 == Cc and X.dtype == Wt.dtype
    OH, OW = conv_out_size(H, KH, stride, pad), conv_out_size(W_, KW, stride, pad)
    out = np.empty((N, OH, OW, Cc), np.float64)
    rc = lib().ms_oracle_dwconv2d_nhwc(_dtype_code(X, bf16), N, H, W_, Cc, KH, KW, stride, pad,
                                       _ptr(X), _ptr(Wt), _ptr(out))
    if rc != 0:
        raise RuntimeError("oracle dwconv2d failed")
    return out


def softmax(X, bf16=False):
    """Softmax over the last axis of X (Appendix A.2: SFM); float64, same shape."""
    X = np.ascontiguousarray(X)
    n = X.shape[-1]
    rows = X.size // n
    out = np.empty(X.shape, np.float64)
    if lib().ms_oracle_softmax(_dtype_code(X, bf16), rows, n, _ptr(X), _ptr(out)) != 0:
        raise RuntimeError("oracle softmax failed")
    return out


def norm(X, bf16=False):
    """2-norm over all but the first axis of X [B, ...] (Appendix A.2: NRM); float64 [B]."""
    X = np.ascontiguousarray(X)
    nb = X.shape[0]
    out = np.empty((nb,), np.float64)
    if lib().ms_oracle_norm(_dtype_code(X, bf16), nb, X.size // nb, _ptr(X), _ptr(out)) != 0:
        raise RuntimeError("oracle norm failed")
    return out


def split_walk(factors):
    """Original-loop index of each iteration of the split nest, in nest order."""
    f = np.asarray(factors, np.int64)
    total = int(np.prod(f))
    out = np.empty(total, np.int64)
    n = lib().ms_oracle_split_walk(len(f), _ptr(f), _ptr(out), total)
    if n != total:
        raise RuntimeError("split walk failed")
    return out


def perfect_tiles(extent, n):
    """All ordered n-tuples of positive integers with product == extent."""
    L = lib()
    cnt = L.ms_oracle_perfect_tiles(extent, n, None, 0)
    out = np.empty((cnt, n), np.int64)
    L.ms_oracle_perfect_tiles(extent, n, _ptr(out), cnt)
    return out
