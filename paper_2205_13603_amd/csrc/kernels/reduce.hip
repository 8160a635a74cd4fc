// Row reductions on the vector ALUs: softmax over the last axis and the 2-norm of a batch entry
// (Appendix A.2 of arXiv 2205.13603: SFM, NRM).  Bandwidth-bound kernels, one per decision trace.
//
// Schedule (Table 2 primitives):
//   split   rows i -> I0..I3, reduction k -> K0..K3 (index ((x0*F1+x1)*F2+x2)*F3+x3)
//   bind    i0 -> blockIdx.x; fuse(i2, k2) -> threadIdx.x (k2 fastest): a row is reduced by a group of K2
//           lanes - the cross-thread reduction.  Inside a wavefront the partial results meet through
//           xor-shuffles (no memory); groups wider than a wavefront finish through K2/64 words of LDS
//   i1      rows a group handles one after the other; i3: rows it handles together (independent chains)
//   k0      serial loop of a lane; k1: unrolled, that many loads in flight; k3: one vector load (coalesced:
//           neighbouring lanes read neighbouring vectors)
//   cache-read (CACHE_READ 1, softmax): the lane's share of the row stays in registers between the three
//           passes (maximum, sum of exponentials, scaling), so global memory is read once; 0: every pass
//           reads the row again (from L2)
// All arithmetic is fp32: m = max x; e = exp(x - m); y = e / sum e (one reciprocal per row); norm = sqrt(sum x^2)
// with one accumulator per (k1, k3) position of a lane.
#include "common.h"

#define RD_SOFTMAX 0
#define RD_NORM 1

constexpr int TPR = K2;                         // lanes per row
constexpr int WPG = TPR > 64 ? TPR / 64 : 1;    // wavefronts per row group
constexpr int NW = NTHREADS / 64;
static_assert(NTHREADS == I2 * K2 && NTHREADS % 64 == 0, "fuse(i2, k2) fills whole wavefronts");
static_assert((K2 & (K2 - 1)) == 0, "lanes per row: a power of two");
static_assert((long)I0 * I1 * I2 * I3 == RD_ROWS && (long)K0 * K1 * K2 * K3 == RD_LEN, "perfect tiles");

typedef vec_t<in_t, K3> vin_t;
typedef vec_t<out_t, K3> vout_t;

template <bool IS_MAX> __device__ __forceinline__ float combine(float a, float b) { return IS_MAX ? fmaxf(a, b) : a + b; }

// Reduce v[r] over the TPR lanes of the row group; every lane of the group ends with the result.
template <bool IS_MAX> __device__ __forceinline__ void group_reduce(float (&v)[I3], float *__restrict__ red, int tid)
{
#pragma unroll
    for (int r = 0; r < I3; ++r)
#pragma unroll
        for (int off = (TPR < 64 ? TPR : 64) / 2; off > 0; off >>= 1) v[r] = combine<IS_MAX>(v[r], __shfl_xor(v[r], off));
    if constexpr (TPR > 64) {
        const int wave = tid / 64, lane = tid % 64;
        __syncthreads(); // the previous reduction's words have been read
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < I3; ++r) red[wave * I3 + r] = v[r];
        }
        __syncthreads();
        const int w0 = (tid / TPR) * WPG;
#pragma unroll
        for (int r = 0; r < I3; ++r) {
            float a = red[w0 * I3 + r];
#pragma unroll
            for (int w = 1; w < WPG; ++w) a = combine<IS_MAX>(a, red[(w0 + w) * I3 + r]);
            v[r] = a;
        }
    }
}

// element offset inside a row of the vector (q0, q1) of lane t
__device__ __forceinline__ int vec_off(int q0, int q1, int t) { return ((q0 * K1 + q1) * K2 + t) * K3; }

extern "C" __global__ void __launch_bounds__(NTHREADS)
ms_kernel(const void *__restrict__ x_, const void *__restrict__ unused1_, const void *__restrict__ unused2_, void *__restrict__ y_, int instances)
{
    (void)unused1_;
    (void)unused2_;
    const int z = blockIdx.z * gridDim.y + blockIdx.y; // instance
    if (z >= instances) return;                        // the whole workgroup leaves together
    const in_t *__restrict__ X = (const in_t *)x_ + (long)z * RD_ROWS * RD_LEN;
    const int tid = threadIdx.x, g = tid / TPR, t = tid % TPR;
    __shared__ float red[TPR > 64 ? NW * I3 : 1];

#pragma unroll 1
    for (int i1 = 0; i1 < I1; ++i1) {
        const long row0 = (((long)blockIdx.x * I1 + i1) * I2 + g) * I3;
        const in_t *__restrict__ xr = X + row0 * RD_LEN;
#if RD_OP == RD_NORM
        out_t *__restrict__ Y = (out_t *)y_ + (long)z * RD_ROWS;
        float acc[I3][K1][K3];
#pragma unroll
        for (int r = 0; r < I3; ++r)
#pragma unroll
            for (int q1 = 0; q1 < K1; ++q1)
#pragma unroll
                for (int q3 = 0; q3 < K3; ++q3) acc[r][q1][q3] = 0.f;
#pragma unroll 1
        for (int q0 = 0; q0 < K0; ++q0) {
            vin_t x[I3][K1];
#pragma unroll
            for (int r = 0; r < I3; ++r)
#pragma unroll
                for (int q1 = 0; q1 < K1; ++q1) x[r][q1] = *reinterpret_cast<const vin_t *>(xr + (long)r * RD_LEN + vec_off(q0, q1, t));
#pragma unroll
            for (int r = 0; r < I3; ++r)
#pragma unroll
                for (int q1 = 0; q1 < K1; ++q1)
#pragma unroll
                    for (int q3 = 0; q3 < K3; ++q3) {
                        const float f = to_acc(x[r][q1].v[q3]);
                        acc[r][q1][q3] = fmaf(f, f, acc[r][q1][q3]);
                    }
        }
        float s[I3];
#pragma unroll
        for (int r = 0; r < I3; ++r) {
            s[r] = 0.f;
#pragma unroll
            for (int q1 = 0; q1 < K1; ++q1)
#pragma unroll
                for (int q3 = 0; q3 < K3; ++q3) s[r] += acc[r][q1][q3];
        }
        group_reduce<false>(s, red, tid);
        if (t == 0) {
#pragma unroll
            for (int r = 0; r < I3; ++r) Y[row0 + r] = from_acc(sqrtf(s[r]));
        }
#else
        out_t *__restrict__ yr = (out_t *)y_ + (long)z * RD_ROWS * RD_LEN + row0 * RD_LEN;
        float m[I3], s[I3];
#if CACHE_READ == 1
        // one pass over global memory: the lane's K0*K1 vectors of each row stay in registers
        float e[I3][K0 * K1][K3];
#pragma unroll
        for (int r = 0; r < I3; ++r)
#pragma unroll
            for (int q = 0; q < K0 * K1; ++q) {
                const vin_t x = *reinterpret_cast<const vin_t *>(xr + (long)r * RD_LEN + vec_off(q / K1, q % K1, t));
#pragma unroll
                for (int q3 = 0; q3 < K3; ++q3) e[r][q][q3] = to_acc(x.v[q3]);
            }
#pragma unroll
        for (int r = 0; r < I3; ++r) {
            m[r] = e[r][0][0];
#pragma unroll
            for (int q = 0; q < K0 * K1; ++q)
#pragma unroll
                for (int q3 = 0; q3 < K3; ++q3) m[r] = fmaxf(m[r], e[r][q][q3]);
        }
        group_reduce<true>(m, red, tid);
#pragma unroll
        for (int r = 0; r < I3; ++r) {
            s[r] = 0.f;
#pragma unroll
            for (int q = 0; q < K0 * K1; ++q)
#pragma unroll
                for (int q3 = 0; q3 < K3; ++q3) {
                    e[r][q][q3] = expf(e[r][q][q3] - m[r]);
                    s[r] += e[r][q][q3];
                }
        }
        group_reduce<false>(s, red, tid);
#pragma unroll
        for (int r = 0; r < I3; ++r) {
            const float inv = 1.0f / s[r];
#pragma unroll
            for (int q = 0; q < K0 * K1; ++q) {
                vout_t y;
#pragma unroll
                for (int q3 = 0; q3 < K3; ++q3) y.v[q3] = from_acc(e[r][q][q3] * inv);
                *reinterpret_cast<vout_t *>(yr + (long)r * RD_LEN + vec_off(q / K1, q % K1, t)) = y;
            }
        }
#else
        // three passes, K1 loads in flight per row in each
#pragma unroll
        for (int r = 0; r < I3; ++r) m[r] = to_acc(xr[(long)r * RD_LEN + vec_off(0, 0, t)]);
#pragma unroll 1
        for (int q0 = 0; q0 < K0; ++q0) {
            vin_t x[I3][K1];
#pragma unroll
            for (int r = 0; r < I3; ++r)
#pragma unroll
                for (int q1 = 0; q1 < K1; ++q1) x[r][q1] = *reinterpret_cast<const vin_t *>(xr + (long)r * RD_LEN + vec_off(q0, q1, t));
#pragma unroll
            for (int r = 0; r < I3; ++r)
#pragma unroll
                for (int q1 = 0; q1 < K1; ++q1)
#pragma unroll
                    for (int q3 = 0; q3 < K3; ++q3) m[r] = fmaxf(m[r], to_acc(x[r][q1].v[q3]));
        }
        group_reduce<true>(m, red, tid);
#pragma unroll
        for (int r = 0; r < I3; ++r) s[r] = 0.f;
#pragma unroll 1
        for (int q0 = 0; q0 < K0; ++q0) {
            vin_t x[I3][K1];
#pragma unroll
            for (int r = 0; r < I3; ++r)
#pragma unroll
                for (int q1 = 0; q1 < K1; ++q1) x[r][q1] = *reinterpret_cast<const vin_t *>(xr + (long)r * RD_LEN + vec_off(q0, q1, t));
#pragma unroll
            for (int r = 0; r < I3; ++r)
#pragma unroll
                for (int q1 = 0; q1 < K1; ++q1)
#pragma unroll
                    for (int q3 = 0; q3 < K3; ++q3) s[r] += expf(to_acc(x[r][q1].v[q3]) - m[r]);
        }
        group_reduce<false>(s, red, tid);
        float inv[I3];
#pragma unroll
        for (int r = 0; r < I3; ++r) inv[r] = 1.0f / s[r];
#pragma unroll 1
        for (int q0 = 0; q0 < K0; ++q0) {
            vin_t x[I3][K1];
#pragma unroll
            for (int r = 0; r < I3; ++r)
#pragma unroll
                for (int q1 = 0; q1 < K1; ++q1) x[r][q1] = *reinterpret_cast<const vin_t *>(xr + (long)r * RD_LEN + vec_off(q0, q1, t));
#pragma unroll
            for (int r = 0; r < I3; ++r)
#pragma unroll
                for (int q1 = 0; q1 < K1; ++q1) {
                    vout_t y;
#pragma unroll
                    for (int q3 = 0; q3 < K3; ++q3) y.v[q3] = from_acc(expf(to_acc(x[r][q1].v[q3]) - m[r]) * inv[r]);
                    *reinterpret_cast<vout_t *>(yr + (long)r * RD_LEN + vec_off(q0, q1, t)) = y;
                }
        }
#endif
#endif
    }
}
