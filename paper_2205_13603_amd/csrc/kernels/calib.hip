// Calibration kernels: what the device attains on a register-resident MFMA issue loop and on a
// streaming copy.  These ground the roofline percentages; they are not part of any operator.
//   MODE 0: each wave issues ITERS x 8 independent MFMAs on register operands
//   MODE 1: copy `n16` 16-byte words src -> dst, one contiguous range per workgroup
//   MODE 2: read `n16` 16-byte words (sum folded into a value that is stored only if it hits a sentinel)
//   MODE 6: write `n16` 16-byte words to dst
//   MODE 7: copy `n16` 16-byte words, 1 KiB per workgroup of 64 lanes (the launch shape of the bandwidth-bound operator
//           kernels: many small workgroups, all loads of a lane issued first)
//   MODE 5: one wavefront waits until the constant-rate wall clock has advanced by `ticks` (a kernel of known
//           duration: checks the event timing that every measurement here relies on)
#define IN_DT CAL_DT
#define OUT_DT 0
#define I0 1
#define J0 1
#define REORDER 0
#include "common.h"

#if MODE == 0
#define LANE_GROUPS (64 / MI_M)
#define KP (MI_K / LANE_GROUPS)
typedef vec_t<in_t, KP> frag_t;
#if MI_M == 16
typedef acc_t accv_t __attribute__((ext_vector_type(4)));
#else
typedef acc_t accv_t __attribute__((ext_vector_type(16)));
#endif
typedef _Float16 h4_t __attribute__((ext_vector_type(4)));
typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef short s4_t __attribute__((ext_vector_type(4)));
typedef __bf16 b8_t __attribute__((ext_vector_type(8)));
typedef int i4_t __attribute__((ext_vector_type(4)));
typedef int i8_t __attribute__((ext_vector_type(8)));

__device__ __forceinline__ accv_t mfma(const frag_t &a, const frag_t &b, accv_t c)
{
#if IN_DT == DT_F16
#if MI_M == 16 && MI_K == 16
    return __builtin_amdgcn_mfma_f32_16x16x16f16(*(const h4_t *)&a, *(const h4_t *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 8
    return __builtin_amdgcn_mfma_f32_32x32x8f16(*(const h4_t *)&a, *(const h4_t *)&b, c, 0, 0, 0);
#elif MI_M == 16 && MI_K == 32
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(*(const h8_t *)&a, *(const h8_t *)&b, c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const h8_t *)&a, *(const h8_t *)&b, c, 0, 0, 0);
#endif
#elif IN_DT == DT_BF16
#if MI_M == 16 && MI_K == 16
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(*(const s4_t *)&a, *(const s4_t *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 8
    return __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(*(const s4_t *)&a, *(const s4_t *)&b, c, 0, 0, 0);
#elif MI_M == 16 && MI_K == 32
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const b8_t *)&a, *(const b8_t *)&b, c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const b8_t *)&a, *(const b8_t *)&b, c, 0, 0, 0);
#endif
#elif IN_DT == DT_F8E4M3
#if MI_M == 16 && MI_K == 32
    return __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(*(const long *)&a, *(const long *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 16
    return __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(*(const long *)&a, *(const long *)&b, c, 0, 0, 0);
#elif MI_M == 16 && MI_K == 128
    // 32 bytes per lane; format selectors 0 = this 8-bit float for both operands, zero scale operands = unscaled form
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(*(const i8_t *)&a, *(const i8_t *)&b, c, 0, 0, 0, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(*(const i8_t *)&a, *(const i8_t *)&b, c, 0, 0, 0, 0, 0, 0);
#endif
#elif IN_DT == DT_F32
#if MI_M == 16
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[0], b.v[0], c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[0], b.v[0], c, 0, 0, 0);
#endif
#else
#if MI_M == 16 && MI_K == 32
    return __builtin_amdgcn_mfma_i32_16x16x32_i8(*(const long *)&a, *(const long *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 16
    return __builtin_amdgcn_mfma_i32_32x32x16_i8(*(const long *)&a, *(const long *)&b, c, 0, 0, 0);
#elif MI_M == 16 && MI_K == 64
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(*(const i4_t *)&a, *(const i4_t *)&b, c, 0, 0, 0);
#else
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(*(const i4_t *)&a, *(const i4_t *)&b, c, 0, 0, 0);
#endif
#endif
}

extern "C" __global__ void __launch_bounds__(256) ms_calib_kernel(const void *src, const void *, const void *, void *dst, int iters)
{
    // operands: taken from `src` when given (2 fragments per lane; realistic values make the matrix
    // cores draw realistic power, which the clock governor reacts to), else small integers
    frag_t a, b;
    if (src != nullptr) {
        a = ((const frag_t *)src)[threadIdx.x];
        b = ((const frag_t *)src)[256 + threadIdx.x];
    } else {
#pragma unroll
        for (int q = 0; q < KP; ++q) {
#if IN_DT == DT_F8E4M3
            a.v[q] = (in_t)(((threadIdx.x + q) & 3) ? 0x38 + 8 * ((threadIdx.x + q) & 1) : 0); // 0, 1.0 or 2.0
            b.v[q] = (in_t)(((threadIdx.x * 3 + q) & 1) ? 0x38 : 0);
#else
            a.v[q] = (in_t)((threadIdx.x + q) & 3);
            b.v[q] = (in_t)((threadIdx.x * 3 + q) & 1);
#endif
        }
    }
    accv_t acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int e = 0; e < (MI_M == 16 ? 4 : 16); ++e) acc[t][e] = 0;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t) acc[t] = mfma(a, b, acc[t]);
    }
    acc_t s = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) s += acc[t][0];
    if (s == (acc_t)-12345) ((acc_t *)dst)[threadIdx.x] = s; // never true: keeps the loop alive
}
#elif MODE == 5
extern "C" __global__ void __launch_bounds__(64) ms_calib_kernel(const void *, const void *, const void *, void *dst, int ticks)
{
    const long long t0 = wall_clock64();
    long long t = t0;
    int guard = 0;
    // the iteration cap ends the wait even if the clock did not advance
    while (t - t0 < (long long)ticks && guard < (1 << 22)) {
        t = wall_clock64();
        ++guard;
    }
    if (guard < 0) ((long long *)dst)[threadIdx.x] = t; // never true
}
#elif MODE == 3
// LDS read rate: every wave reads 16 bytes per lane, lanes at consecutive addresses (no bank conflict),
// 8 independent reads per iteration
typedef unsigned u4_t __attribute__((ext_vector_type(4)));
extern "C" __global__ void __launch_bounds__(256) ms_calib_kernel(const void *src, const void *, const void *, void *dst, int iters)
{
    __shared__ u4_t buf[4096]; // 64 KiB
    for (int i = threadIdx.x; i < 4096; i += 256) buf[i] = u4_t{(unsigned)i, 1u, 2u, 3u};
    __syncthreads();
    u4_t acc = {0, 0, 0, 0};
    const int base = threadIdx.x;
#pragma unroll 1
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            u4_t x = buf[(base + t * 256 + (it & 7) * 64) & 4095];
            acc ^= x;
        }
    }
    if (acc[0] == 0xdeadbeefu && src != nullptr) ((u4_t *)dst)[threadIdx.x] = acc;
}
#elif MODE == 4
// L2 read rate: every workgroup reads the same 2 MiB window `reps` times (16 bytes per lane, coalesced);
// the window stays resident in each XCD's L2, so this is the rate at which the L2s feed the compute units
typedef vec_t<float, 4> w16_t;
extern "C" __global__ void __launch_bounds__(256) ms_calib_kernel(const void *src, const void *, const void *, void *dst, int reps)
{
    const w16_t *s = (const w16_t *)src;
    constexpr int WORDS = (2 << 20) / 16;
    float acc = 0.f;
    int i = (blockIdx.x * 256 + threadIdx.x) % WORDS;
#pragma unroll 1
    for (int r = 0; r < reps; ++r) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            w16_t x = s[i];
            acc += (x.v[0] + x.v[1]) + (x.v[2] + x.v[3]); // every word is used: a load whose middle words are dead gets split into narrower loads
            i = (i + 256 * 61) % WORDS;
        }
    }
    if (acc == -12345.678f) ((float *)dst)[threadIdx.x] = acc;
}
#elif MODE == 7
// 1 KiB per workgroup of 64 lanes, two 8-byte words per lane, all loads before the stores: the fastest of the shapes
// tried (workgroups of 64-1024 lanes, 1-64 KiB per workgroup, 8- and 16-byte words)
typedef vec_t<float, 2> w8_t;
extern "C" __global__ void __launch_bounds__(64) ms_calib_kernel(const void *src, const void *, const void *, void *dst, int n16_lo)
{
    const long n8 = (long)(unsigned)n16_lo * 512; // the host passes the number of 16-byte words / 256
    const w8_t *s = (const w8_t *)src;
    w8_t *d = (w8_t *)dst;
    const long base = (long)blockIdx.x * 128 + threadIdx.x;
    w8_t x[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if (base + u * 64 < n8) x[u] = s[base + u * 64];
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if (base + u * 64 < n8) d[base + u * 64] = x[u];
}
#else
typedef vec_t<float, 4> w16_t;
extern "C" __global__ void __launch_bounds__(256) ms_calib_kernel(const void *src, const void *, const void *, void *dst, int n16_lo)
{
    const long n16 = (long)(unsigned)n16_lo * 256; // the host passes the word count / 256
    const long stride = (long)gridDim.x * blockDim.x;
    const w16_t *s = (const w16_t *)src;
    w16_t *d = (w16_t *)dst;
#if MODE == 1
    // every workgroup copies one contiguous range (about 10 % faster here than a grid-stride loop, whose
    // workgroups touch addresses 16 MiB apart in every iteration)
    const long per = (n16 + gridDim.x - 1) / gridDim.x;
    const long lo = (long)blockIdx.x * per, hi = lo + per < n16 ? lo + per : n16;
    for (long i = lo + threadIdx.x; i < hi; i += 256) d[i] = s[i];
    (void)stride;
#elif MODE == 6
    // write only: one contiguous range per workgroup
    const long per = (n16 + gridDim.x - 1) / gridDim.x;
    const long lo = (long)blockIdx.x * per, hi = lo + per < n16 ? lo + per : n16;
    w16_t x;
    x.v[0] = x.v[1] = x.v[2] = x.v[3] = (float)blockIdx.x;
    for (long i = lo + threadIdx.x; i < hi; i += 256) d[i] = x;
    (void)stride;
    (void)s;
#else
    float acc = 0.f;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        w16_t x = s[i];
        acc += x.v[0] + x.v[1] + x.v[2] + x.v[3];
    }
    if (acc == -12345.678f) d[threadIdx.x].v[0] = acc;
#endif
}
#endif
