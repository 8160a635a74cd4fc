// GEMM / batched matmul on the vector ALUs, one kernel per decision trace.
//
// Schedule (Table 2 primitives of arXiv 2205.13603, applied in this order):
//   split   i -> I0,I1,I2,I3   j -> J0,J1,J2,J3   k -> K0,K1,K2,K3
//   reorder i0 j0 | k0 | i2 j2 | k1 k2 k3 | i1 j1 i3 j3
//   bind    fuse(i0,j0) -> blockIdx.x, fuse(i2,j2) -> threadIdx.x
//   cache-read A,B into LDS at k0 (CACHE_READ 1: one buffer, 2: two buffers,
//           0: operands come straight from global memory)
//   storage-align: LDS rows padded by 16 bytes when LDS_PAD != 0
//   vectorize: global loads of VEC (A) and VEC_B (B) elements; stores of J3 elements
//   unroll  k1 by UNROLL_K1, k2 by UNROLL_K2; k3 and the register tile fully
// Index of a split loop: ((x0*F1 + x1)*F2 + x2)*F3 + x3.
#include "common.h"

constexpr int BM = I1 * I2 * I3;
constexpr int BN = J1 * J2 * J3;
constexpr int BK = K1 * K2 * K3;
constexpr int RM = I1 * I3;
constexpr int RN = J1 * J3;
constexpr int PAD = LDS_PAD ? 4 : 0; // elements of 4 bytes
constexpr int LDA = BK + PAD;
constexpr int LDB = BN + PAD;
constexpr int STAGES = CACHE_READ == 2 ? 2 : 1;

#if CACHE_READ
__device__ __forceinline__ void load_tiles(const in_t *__restrict__ A, const in_t *__restrict__ B, acc_t *__restrict__ As,
                                           acc_t *__restrict__ Bs, int i0, int j0, int k0, int tid)
{
    const long arow0 = (long)i0 * BM, bcol0 = (long)j0 * BN, kbase = (long)k0 * BK;
    // A tile: BM x BK, vectors along k when k is contiguous
    {
        constexpr int VA = (SA_K == 1) ? VEC : 1;
        constexpr int KV = BK / VA;
        constexpr int TOTAL = BM * KV;
        for (int idx = tid; idx < TOTAL; idx += NTHREADS) {
            const int m = idx / KV, kv = idx % KV;
            const in_t *src = A + (arow0 + m) * SA_I + (kbase + kv * VA) * SA_K;
            vec_t<in_t, VA> x = *reinterpret_cast<const vec_t<in_t, VA> *>(src);
#pragma unroll
            for (int q = 0; q < VA; ++q) As[m * LDA + kv * VA + q] = to_acc(x.v[q]);
        }
    }
    // B tile: BK x BN
    if (SB_K == 1 && SB_J != 1) { // reduction index contiguous ("NT"): vectors along k
        constexpr int VB = VEC_B;
        constexpr int KV = BK / VB;
        constexpr int TOTAL = BN * KV;
        for (int idx = tid; idx < TOTAL; idx += NTHREADS) {
            const int j = idx / KV, kv = idx % KV;
            const in_t *src = B + (kbase + kv * VB) * SB_K + (bcol0 + j) * SB_J;
            vec_t<in_t, VB> x = *reinterpret_cast<const vec_t<in_t, VB> *>(src);
#pragma unroll
            for (int q = 0; q < VB; ++q) Bs[(kv * VB + q) * LDB + j] = to_acc(x.v[q]);
        }
    } else {
        constexpr int VB = (SB_J == 1) ? VEC_B : 1;
        constexpr int JV = BN / VB;
        constexpr int TOTAL = BK * JV;
        for (int idx = tid; idx < TOTAL; idx += NTHREADS) {
            const int k = idx / JV, jv = idx % JV;
            const in_t *src = B + (kbase + k) * SB_K + (bcol0 + jv * VB) * SB_J;
            vec_t<in_t, VB> x = *reinterpret_cast<const vec_t<in_t, VB> *>(src);
#pragma unroll
            for (int q = 0; q < VB; ++q) Bs[k * LDB + jv * VB + q] = to_acc(x.v[q]);
        }
    }
}
#endif

extern "C" __global__ void __launch_bounds__(NTHREADS)
ms_kernel(const void *__restrict__ a_, const void *__restrict__ b_, const void *__restrict__ unused_, void *__restrict__ c_, int instances)
{
    (void)unused_;
    int z, i0, j0;
    int ks; // always 0: the vector kernels keep the reduction inside one workgroup
    block_to_tile(z, i0, j0, ks);
    const int inst = z / DIM_B, bb = z % DIM_B;
    if (inst >= instances) return;
    const in_t *__restrict__ A = (const in_t *)a_ + (long)inst * A_INST + (long)bb * SA_B;
    const in_t *__restrict__ B = (const in_t *)b_ + (long)inst * B_INST + (long)bb * SB_B;
    out_t *__restrict__ C = (out_t *)c_ + ((long)inst * DIM_B + bb) * ((long)DIM_M * DIM_N);

    const int tid = threadIdx.x;
    const int ti = tid / J2, tj = tid % J2;

    acc_t acc[RM][RN];
#pragma unroll
    for (int r = 0; r < RM; ++r)
#pragma unroll
        for (int c = 0; c < RN; ++c) acc[r][c] = 0;

#if CACHE_READ
    __shared__ acc_t As[STAGES][BM * LDA];
    __shared__ acc_t Bs[STAGES][BK * LDB];
    int stage = 0;
#if CACHE_READ == 2
    load_tiles(A, B, As[0], Bs[0], i0, j0, 0, tid);
    __syncthreads();
#endif
#endif

#pragma unroll 1
    for (int k0 = 0; k0 < K0; ++k0) {
#if CACHE_READ == 1
        load_tiles(A, B, As[0], Bs[0], i0, j0, k0, tid);
        __syncthreads();
#elif CACHE_READ == 2
        if (k0 + 1 < K0) load_tiles(A, B, As[stage ^ 1], Bs[stage ^ 1], i0, j0, k0 + 1, tid);
#endif
#pragma unroll UNROLL_K1
        for (int k1 = 0; k1 < K1; ++k1) {
#pragma unroll UNROLL_K2
            for (int k2 = 0; k2 < K2; ++k2) {
                const int kk = (k1 * K2 + k2) * K3;
                acc_t a[RM][K3], b[K3][RN];
#pragma unroll
                for (int r1 = 0; r1 < I1; ++r1)
#pragma unroll
                    for (int r3 = 0; r3 < I3; ++r3) {
                        const int ml = (r1 * I2 + ti) * I3 + r3;
#pragma unroll
                        for (int q = 0; q < K3; ++q) {
#if CACHE_READ
                            a[r1 * I3 + r3][q] = As[stage][ml * LDA + kk + q];
#else
                            a[r1 * I3 + r3][q] = to_acc(A[((long)i0 * BM + ml) * SA_I + ((long)k0 * BK + kk + q) * SA_K]);
#endif
                        }
                    }
#pragma unroll
                for (int q = 0; q < K3; ++q)
#pragma unroll
                    for (int c1 = 0; c1 < J1; ++c1)
#pragma unroll
                        for (int c3 = 0; c3 < J3; ++c3) {
                            const int nl = (c1 * J2 + tj) * J3 + c3;
#if CACHE_READ
                            b[q][c1 * J3 + c3] = Bs[stage][(kk + q) * LDB + nl];
#else
                            b[q][c1 * J3 + c3] = to_acc(B[((long)k0 * BK + kk + q) * SB_K + ((long)j0 * BN + nl) * SB_J]);
#endif
                        }
#pragma unroll
                for (int q = 0; q < K3; ++q)
#pragma unroll
                    for (int r = 0; r < RM; ++r)
#pragma unroll
                        for (int c = 0; c < RN; ++c) acc[r][c] += a[r][q] * b[q][c];
            }
        }
#if CACHE_READ
        __syncthreads();
#if CACHE_READ == 2
        stage ^= 1;
#endif
#endif
    }

    // epilogue: one rounding to the output type; J3 contiguous columns per store
#pragma unroll
    for (int r1 = 0; r1 < I1; ++r1)
#pragma unroll
        for (int r3 = 0; r3 < I3; ++r3) {
            const long i = (long)i0 * BM + (r1 * I2 + ti) * I3 + r3;
#pragma unroll
            for (int c1 = 0; c1 < J1; ++c1) {
                const long j = (long)j0 * BN + (c1 * J2 + tj) * J3;
                constexpr bool vst = (J3 == 2 || J3 == 4 || J3 == 8) && (J3 * sizeof(out_t) <= 16) && (DIM_N % J3 == 0);
                if (vst) {
                    constexpr int SV = vst ? J3 : 1;
                    vec_t<out_t, SV> o;
#pragma unroll
                    for (int c3 = 0; c3 < SV; ++c3) o.v[c3] = from_acc(acc[r1 * I3 + r3][c1 * J3 + c3]);
                    *reinterpret_cast<vec_t<out_t, SV> *>(C + i * DIM_N + j) = o;
                } else {
#pragma unroll
                    for (int c3 = 0; c3 < J3; ++c3) C[i * DIM_N + j + c3] = from_acc(acc[r1 * I3 + r3][c1 * J3 + c3]);
                }
            }
        }
}
