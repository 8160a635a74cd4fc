"""Seeded synthetic inputs for the five workload configurations.

This module holds no operator arithmetic: it only draws random tensors with
numpy and rounds them once to the operator's storage dtype on the host.  The
same host arrays feed the GPU path and the CPU oracle.

Recipe (numpy.random.default_rng(seed); one draw per tensor, in the order the
tensors are listed):
  C1  fp32 GEMM 128^3            A, B ~ U[-1, 1]                 (GMM, Appendix A.2)
  C2  fp16 GEMM 1024^3           A, B ~ 0.1 * N(0, 1) -> fp16    (fused-dense, Section 5.3)
  C3  conv2d NHWC fp16 56x56x64 -> 64, 3x3 s1 p1, bias + ReLU
                                 X ~ U[0, 1], W ~ N(0, 0.05), bias ~ N(0, 0.05) fp32
  C4a BMM-NT fp16 12 x [128x64].[128x64]^T     Q, K ~ N(0, 1)   (TBG, Appendix A.2)
  C4b BMM-NN fp16 12 x [128x128].[128x64]      P, V ~ N(0, 1)
  C4c int8 GEMM 512^3 -> int32   integers U{-128..127}
  C5a depthwise fp32 112x112x32 3x3 s1 p1      X, W ~ U[-1, 1]  (DEP, Appendix A.2)
  C5b depthwise fp32 56x56x144 3x3 s2 p1       X, W ~ U[-1, 1]
"""
import numpy as np


def rng(seed):
    return np.random.default_rng(seed)


def f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def f32_to_f8e4m3_bits(x):
    """float32 -> bit patterns (uint8) of the 8-bit float with 4 exponent and 3 mantissa bits, round to nearest even,
    values clipped to the largest finite magnitude 448 first (the conversion routine of torch does the rounding)."""
    import torch
    t = torch.from_numpy(np.clip(np.ascontiguousarray(x, np.float32), -448.0, 448.0))
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy().copy()


def _cast(x, dtype):
    if dtype == "f32":
        return x.astype(np.float32)
    if dtype == "f16":
        return x.astype(np.float32).astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x.astype(np.float32))
    if dtype == "f8":
        return f32_to_f8e4m3_bits(x.astype(np.float32))
    raise ValueError(dtype)


def uniform(g, shape, lo, hi, dtype):
    return _cast(g.uniform(lo, hi, size=shape), dtype)


def normal(g, shape, sigma, dtype):
    return _cast(g.normal(0.0, sigma, size=shape), dtype)


def small_ints(g, shape, lo, hi, dtype):
    """Integer-valued floats: every partial sum is exact in fp32."""
    return _cast(g.integers(lo, hi + 1, size=shape).astype(np.float64), dtype)


def int8_uniform(g, shape):
    return g.integers(-128, 128, size=shape, dtype=np.int64).astype(np.int8)


def gemm_inputs(M, N, K, dtype, seed=0, dist="uniform", scale=1.0, batch=None):
    g = rng(seed)
    sa = (M, K) if batch is None else (batch, M, K)
    sb = (K, N) if batch is None else (batch, K, N)
    if dtype == "i8":
        return int8_uniform(g, sa), int8_uniform(g, sb)
    if dist == "uniform":
        return uniform(g, sa, -scale, scale, dtype), uniform(g, sb, -scale, scale, dtype)
    if dist == "normal":
        return normal(g, sa, scale, dtype), normal(g, sb, scale, dtype)
    if dist == "ints":
        return small_ints(g, sa, -2, 2, dtype), small_ints(g, sb, -2, 2, dtype)
    raise ValueError(dist)


def c1(seed=0):
    return gemm_inputs(128, 128, 128, "f32", seed, "uniform", 1.0)


def c2(seed=0, M=1024, N=1024, K=1024, dtype="f16"):
    return gemm_inputs(M, N, K, dtype, seed, "normal", 0.1)


def c3(seed=0, N=1, H=56, W=56, Cin=64, Cout=64, KH=3, KW=3, dtype="f16"):
    g = rng(seed)
    X = uniform(g, (N, H, W, Cin), 0.0, 1.0, dtype)
    Wt = normal(g, (KH, KW, Cin, Cout), 0.05, dtype)
    bias = g.normal(0.0, 0.05, size=(Cout,)).astype(np.float32)
    return X, Wt, bias


def c4a(seed=0, heads=12, seq=128, dim=64, dtype="f16"):
    g = rng(seed)
    return normal(g, (heads, seq, dim), 1.0, dtype), normal(g, (heads, seq, dim), 1.0, dtype)


def c4b(seed=0, heads=12, seq=128, dim=64, dtype="f16"):
    g = rng(seed)
    return normal(g, (heads, seq, seq), 1.0, dtype), normal(g, (heads, seq, dim), 1.0, dtype)


def c4c(seed=0, M=512, N=512, K=512):
    return gemm_inputs(M, N, K, "i8", seed)


def dw_inputs(N, H, W, C, KH=3, KW=3, seed=0, dtype="f32"):
    g = rng(seed)
    return uniform(g, (N, H, W, C), -1.0, 1.0, dtype), uniform(g, (KH, KW, C), -1.0, 1.0, dtype)


def c5a(seed=0):
    return dw_inputs(1, 112, 112, 32, seed=seed)


def c5b(seed=0):
    return dw_inputs(1, 56, 56, 144, seed=seed)


def sfm(seed=0, B=1, M=256, N=256, dtype="f32"):
    """Softmax workload (batch 1, 256 x 256): logits with standard deviation 2."""
    return (normal(rng(seed), (B, M, N), 2.0, dtype),)


def nrm(seed=0, B=1, M=256, N=256, dtype="f32"):
    """Norm workload (batch 1, 256 x 256): standard normal values."""
    return (normal(rng(seed), (B, M, N), 1.0, dtype),)


def cbr(seed=0, dtype="f16"):
    """First layer of a residual network (224 x 224 x 3 -> 64, 7 x 7, stride 2, padding 3), batch normalisation folded
    into weights and bias: X ~ U[0, 1], W ~ N(0, 0.05), bias ~ N(0, 0.05) fp32."""
    g = rng(seed)
    return (uniform(g, (1, 224, 224, 3), 0.0, 1.0, dtype), normal(g, (7, 7, 3, 64), 0.05, dtype), normal(g, (64,), 0.05, "f32"))


def cbr4(seed=0, dtype="f16"):
    """The same layer with the input stored with 4 channels per pixel (the fourth is zero, and so are its weights):
    one 8-byte load per pixel instead of three 2-byte loads."""
    import numpy as np
    X, W, b = cbr(seed, dtype)
    X4 = np.zeros(X.shape[:3] + (4,), X.dtype)
    X4[..., :3] = X
    W4 = np.zeros(W.shape[:2] + (4,) + W.shape[3:], W.dtype)
    W4[:, :, :3, :] = W
    return (X4, W4, b)


def t2d(seed=0, dtype="f16"):
    """Transposed convolution workload (4 x 4 x 512 -> 8 x 8 x 256, 4 x 4 filter, stride 2, padding 1):
    X ~ N(0, 1), W ~ N(0, 0.05), bias ~ N(0, 0.05) fp32."""
    g = rng(seed)
    return (normal(g, (1, 4, 4, 512), 1.0, dtype), normal(g, (4, 4, 512, 256), 0.05, dtype), normal(g, (256,), 0.05, "f32"))


def grp(seed=0, dtype="f16"):
    """Grouped convolution workload (56 x 56 x 64 -> 28 x 28 x 128, 3 x 3, stride 2, padding 1, 4 groups):
    X ~ U[0, 1], W ~ N(0, 0.05) as [3][3][16][128], bias ~ N(0, 0.05) fp32."""
    g = rng(seed)
    return (uniform(g, (1, 56, 56, 64), 0.0, 1.0, dtype), normal(g, (3, 3, 16, 128), 0.05, dtype), normal(g, (128,), 0.05, "f32"))


def c2nt(seed=0, dtype="f16"):
    """Config 2 with the second operand stored transposed: A [1][1024][1024], B [1][N][K], 0.1 * N(0, 1)."""
    g = rng(seed)
    return (normal(g, (1, 1024, 1024), 0.1, dtype), normal(g, (1, 1024, 1024), 0.1, dtype))


def c1d(seed=0, dtype="f16"):
    """1-D convolution workload (length 256, 64 -> 128 channels, kernel 3, stride 2, padding 1): X ~ U[0, 1],
    W ~ N(0, 0.05) as [3][64][128], bias ~ N(0, 0.05) fp32."""
    g = rng(seed)
    return (uniform(g, (1, 256, 64), 0.0, 1.0, dtype), normal(g, (3, 64, 128), 0.05, dtype), normal(g, (128,), 0.05, "f32"))


def c3d(seed=0, dtype="f16"):
    """3-D convolution workload (16 x 224 x 224 x 3 -> 8 x 112 x 112 x 64, 7 x 7 x 7, stride 2, padding 3):
    X ~ U[0, 1], W ~ N(0, 0.02), bias ~ N(0, 0.05) fp32."""
    g = rng(seed)
    return (uniform(g, (1, 16, 224, 224, 3), 0.0, 1.0, dtype), normal(g, (7, 7, 7, 3, 64), 0.02, dtype), normal(g, (64,), 0.05, "f32"))


def c3d4(seed=0, dtype="f16"):
    """The same 3-D convolution with the input stored with 4 channels per voxel (the fourth is zero, and so are its
    weights): one 8-byte load per voxel and tap instead of three 2-byte loads."""
    import numpy as np
    X, W, b = c3d(seed, dtype)
    X4 = np.zeros(X.shape[:4] + (4,), X.dtype)
    X4[..., :3] = X
    W4 = np.zeros(W.shape[:3] + (4,) + W.shape[4:], W.dtype)
    W4[:, :, :, :3, :] = W
    return (X4, W4, b)
