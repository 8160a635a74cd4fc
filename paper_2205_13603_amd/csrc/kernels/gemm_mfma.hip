// GEMM / batched matmul / implicit-GEMM conv2d (+bias +ReLU) on the CDNA4
// matrix cores, one kernel per decision trace.
//
// Schedule (Table 2 primitives of arXiv 2205.13603, applied in this order):
//   tensorize the inner MI_M x MI_N x MI_K block of C += A.B onto one MFMA
//           instruction; the loops i, j, k are from here on counted in tiles
//   split   i -> I0,I1,I2,I3   j -> J0,J1,J2,J3   k -> K0,K1,K2,K3
//   reorder i0 j0 | k0 | i2 j2 | k1 k2 k3 | i1 j1 i3 j3
//   bind    fuse(i0,j0) -> blockIdx.x (REORDER 3: -> a loop of persistent workgroups), fuse(i2,j2) -> wavefront
//   cache-read A,B tiles of one k0 step into LDS (CACHE_READ 1: one buffer;
//           2: two buffers, the next tile is fetched into registers while the
//           current one is multiplied; 3: two buffers and two register sets, the
//           tile two steps ahead is in flight, and with k1, k2 fully unrolled the LDS
//           writes of the next tile are spread between the MFMAs as well; 4: two buffers, the wavefronts split
//           into two groups half a step apart so that one group's memory phase
//           runs under the other's MFMA phase; 5, 6, 7: tiles loaded from global memory
//           straight into a ring of 2, 3, 4 LDS buffers (see "Direct-to-LDS path" below); 8, 9: the same ring
//           of 2, 3 buffers under persistent workgroups whose wavefronts form two groups one phase apart:
//           while one group multiplies a k step from registers, the other reads the next step's fragments
//           from LDS (see "Ping-pong on the ring" below))
//   storage-align: LDS_PAD 1, 2: each LDS plane padded by 16 bytes; 2: slots of a plane XOR-swizzled; 3, 4: B row-major
//           in LDS (see B_ROWMAJOR)
//   vectorize: global loads of VEC (A) and VEC_B (B) elements
//   cache-write (CACHE_WRITE 1): the output tile is assembled in LDS and stored as whole rows
//   rfactor (RFACTOR S > 1): the k0 loop is cut into S runs of K0 / S steps, S consecutive workgroups share an
//           output tile and each writes the accumulators of its run to the workspace [S][instance x batch][M][N];
//           ms_rfactor_reduce (second kernel of the launch) adds the S partial results in run order and applies
//           the epilogue.  Nothing is added atomically: the result does not depend on scheduling
//   unroll  k1 by UNROLL_K1, k2 by UNROLL_K2; k3 and the wave's tile loops fully.  When the
//           budget unrolls k1 and k2 completely the k step becomes a software pipeline: each of
//           its K1*K2 slots issues the next slot's LDS reads and a share of the next tile's global
//           loads ahead of its own MFMAs
//
// LDS layout of both operands: [k group][row][KP], KP = the k elements one
// lane feeds to one MFMA.  A lane's fragment is then one 8- or 16-byte LDS
// read (two 16-byte reads from two sub-planes for the 32-byte fragments of
// the deepest 8-bit float intrinsics), and the 16 or 32 lanes of a row group
// read consecutive addresses (no bank conflict).  Operands whose contiguous dimension is not k (B of
// C = A.B, the conv weights) are transposed in registers on the way in.
//
// conv2d with COMPUTE_AT 1 (the cache-read of X computed under the workgroup tile loop instead of
// under k0): the input rows that the tile's BM output pixels need, zero halo included, are staged
// once as [patch row][patch column][Cin] and the A fragments of every k step are read straight
// from that patch (pixel of the lane + tap offset + channel offset); the k0 loop then stages the
// weights only.  No im2col copy exists anywhere, and X is fetched once per tile instead of KH*KW times.
//
// conv2d with COMPUTE_AT 2: additionally the cache-read of W sits above the tile loop.  Workgroups are
// persistent (about one per compute unit) and own a run of consecutive tiles; the weights of the current
// instance stay in LDS in fragment layout (reloaded only when the run crosses into the next instance), the
// k loop is free of barriers and global loads, and with CACHE_READ 2 the next tile's input patch is
// fetched into registers while the current tile is multiplied.
//
// conv2d with COMPUTE_AT 3: as 2, with HELPER_WAVES extra wavefronts that do all global memory traffic of
// the tile loop.  While the I2*J2 matrix-core wavefronts multiply tile t, the helpers write tile t-1 from
// its LDS staging area to global memory and fetch the patch of tile t+1; between two k loops only LDS is
// touched (accumulators -> staging area, patch registers -> patch).
//
// conv2d with COMPUTE_AT 4: as 2, but the cache-read of W ends in registers: every wavefront keeps the
// weight fragments of its own output columns for all k steps (loaded through a one-step LDS staging
// buffer when the run enters a new instance), the k loop is fully unrolled and reads only the A
// fragments from LDS - a third to two thirds less LDS traffic, which is what bounds modes 2 and 3.
#include "common.h"

#ifndef COMPUTE_AT
#define COMPUTE_AT 0
#endif
#define CONV_PATCH (IS_CONV && COMPUTE_AT >= 1)
#define CONV_RESIDENT (IS_CONV && COMPUTE_AT >= 2)
#define CONV_HELPERS (IS_CONV && COMPUTE_AT == 3)
#define CONV_BREG (IS_CONV && COMPUTE_AT == 4)
#ifndef HELPER_WAVES
#define HELPER_WAVES 0
#endif
#ifndef CV_TRANSPOSED
#define CV_TRANSPOSED 0
#endif
// Grouped conv2d: the batch index of the launch is the group.  A group reads CV_CIN of the CV_XC channels of a pixel
// (offset SA_B per group), DIM_N of the LDC output channels (weights, bias and output offset by DIM_N per group).
#ifndef LDC
#define LDC DIM_N                  // elements between two rows of the output = bias values per instance
#endif
#ifndef C_BATCH
#define C_BATCH ((long)DIM_M * DIM_N) // output elements between two batch entries
#endif
#if IS_CONV
#ifndef CV_PAD_H
#define CV_PAD_H CV_PAD            // zero rows above the image (CV_PAD: zero columns left of it)
#endif
#ifndef CV_XC
#define CV_XC CV_CIN               // channels per pixel of X
#endif
// Filter-row layout of the reduction (CV_TAPROWS 1): k = (kh, q) with q running over the KW * Cin contiguous elements of
// one filter row across all its taps, rounded up to CV_KR (a multiple of the intrinsic's k); q >= KW * Cin is padding.
// In the input, the elements of one run are contiguous too (consecutive pixels of a row), so a matrix-core k step reads
// a piece of an image row: what a first layer with 3 or 4 channels per pixel needs.
#ifndef CV_TAPROWS
#define CV_TAPROWS 0
#define CV_KR 0
#endif
#ifndef CV_D
#define CV_D 1                     // 3-D convolution: input depth, filter depth, output depth (padded like the columns)
#define CV_KD 1
#define CV_OD 1
#endif
#endif

#define B_KMAJOR (!IS_CONV && SB_K == 1 && SB_J != 1)
// LDS_PAD 3 (j-contiguous B of a GEMM, register staging): B lies in LDS as in global memory, row-major k-rows of BN
// elements, and the fragments come out of the transposing LDS loads; A as with LDS_PAD 2.  LDS_PAD 4: the same without
// any XOR swizzle - the rows of B are padded by 32 bytes and the planes of A by 16 instead - so that every fragment
// address is one per-lane base plus a compile-time constant (the immediate offset of the LDS instruction): unrolled
// k loops then need two address registers instead of one per fragment
#define B_ROWMAJOR (!IS_CONV && !B_KMAJOR && (LDS_PAD == 3 || LDS_PAD == 4) && CACHE_READ <= 4)
#define NWAVES (I2 * J2)
#define LANE_GROUPS (64 / MI_M)
#define KP (MI_K / LANE_GROUPS)

constexpr int TM = I1 * I3;
constexpr int TN = J1 * J3;
constexpr int BM = I1 * I2 * I3 * MI_M;
constexpr int BN = J1 * J2 * J3 * MI_N;
constexpr int BK = K1 * K2 * K3 * MI_K;
constexpr int KG = BK / KP;                       // k groups per tile
constexpr int ES = sizeof(in_t);
constexpr int FRAG_BYTES = KP * ES;               // a lane's operand of one MFMA: 4, 8, 16 or 32 bytes
// A 32-byte fragment (the 128-deep and 64-deep 8-bit float intrinsics) lies in LDS as two 16-byte halves in
// two consecutive sub-planes, so that every LDS access stays one 16-byte instruction with the bank
// behaviour of the 16-byte layouts.
constexpr int LSPLIT = FRAG_BYTES > 16 ? FRAG_BYTES / 16 : 1;
constexpr int KPL = KP / LSPLIT;                  // k elements of one LDS fragment
constexpr int LFRAG_BYTES = KPL * ES;
constexpr int SUBPLANE_A = BM * LFRAG_BYTES + (LDS_PAD ? 16 : 0); // bytes of one plane of LDS fragments
constexpr int SUBPLANE_B = BN * LFRAG_BYTES + (LDS_PAD ? 16 : 0);
constexpr int PLANE_A = LSPLIT * SUBPLANE_A;      // bytes of one k-group plane (all rows, the KP k elements of one lane group)
constexpr int PLANE_B = LSPLIT * SUBPLANE_B;

// Slot of row `n` inside a plane (a slot = one fragment).  The swizzle XORs the low 3 bits of the slot
// with bits 3..5: a thread that writes 8 consecutive slots (the transposed j-contiguous operand) then
// starts in a different bank group than its 7 neighbours, and 8 consecutive lanes that read 8
// consecutive rows still touch 8 distinct slots of one aligned group.
__device__ __forceinline__ int lds_slot(int n)
{
#if LDS_PAD == 2 || LDS_PAD == 3
    return n ^ ((n >> 3) & 7);
#else
    return n;
#endif
}
constexpr int A_STAGE_BYTES = CONV_PATCH ? 0 : KG * PLANE_A; // the per-k-step stage holds A unless X is resident as a patch
constexpr int RM_ROW = BN * ES + (LDS_PAD == 4 ? 32 : 0); // bytes of one k-row of the row-major B stage
constexpr int B_STAGE_BYTES = B_ROWMAJOR ? BK * RM_ROW : KG * PLANE_B;
constexpr int B_LGRP = B_ROWMAJOR ? 0 : PLANE_B;  // offset of a lane group's fragments inside the B stage
constexpr int STAGE_BYTES = A_STAGE_BYTES + B_STAGE_BYTES;
constexpr int STAGES = CACHE_READ >= 2 ? 2 : 1;
constexpr int KSTEPS = K1 * K2 * K3;              // MFMA k steps per tile

static_assert(MI_M == MI_N, "square intrinsics only");
static_assert(FRAG_BYTES == 4 || FRAG_BYTES == 8 || FRAG_BYTES == 16 || FRAG_BYTES == 32, "fragment is 4 (fp32), 8, 16 or 32 bytes");

// ---- fragment and accumulator types, one MFMA
typedef vec_t<in_t, KP> frag_t;
typedef vec_t<in_t, KPL> lfrag_t;

// a lane's fragment from its LSPLIT LDS fragments, SUB bytes apart
template <int SUB> __device__ __forceinline__ frag_t lds_frag(const char *__restrict__ p)
{
    if constexpr (LSPLIT == 1) {
        return *reinterpret_cast<const frag_t *>(p);
    } else {
        frag_t f;
#pragma unroll
        for (int h = 0; h < LSPLIT; ++h) {
            const lfrag_t part = *reinterpret_cast<const lfrag_t *>(p + h * SUB);
#pragma unroll
            for (int q = 0; q < KPL; ++q) f.v[h * KPL + q] = part.v[q];
        }
        return f;
    }
}
#if MI_M == 16
typedef acc_t accv_t __attribute__((ext_vector_type(4)));
constexpr int ACC_N = 4;
#else
typedef acc_t accv_t __attribute__((ext_vector_type(16)));
constexpr int ACC_N = 16;
#endif

typedef _Float16 h4_t __attribute__((ext_vector_type(4)));
typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef short s4_t __attribute__((ext_vector_type(4)));
typedef __bf16 b8_t __attribute__((ext_vector_type(8)));
typedef int i4_t __attribute__((ext_vector_type(4)));
typedef int i8v_t __attribute__((ext_vector_type(8)));

__device__ __forceinline__ accv_t mfma(const frag_t &a, const frag_t &b, accv_t c)
{
#if IN_DT == DT_F16
#if MI_M == 16 && MI_K == 16
    return __builtin_amdgcn_mfma_f32_16x16x16f16(*(const h4_t *)&a, *(const h4_t *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 8
    return __builtin_amdgcn_mfma_f32_32x32x8f16(*(const h4_t *)&a, *(const h4_t *)&b, c, 0, 0, 0);
#elif MI_M == 16 && MI_K == 32
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(*(const h8_t *)&a, *(const h8_t *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 16
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(*(const h8_t *)&a, *(const h8_t *)&b, c, 0, 0, 0);
#else
#error "no such fp16 intrinsic"
#endif
#elif IN_DT == DT_BF16
#if MI_M == 16 && MI_K == 16
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(*(const s4_t *)&a, *(const s4_t *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 8
    return __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(*(const s4_t *)&a, *(const s4_t *)&b, c, 0, 0, 0);
#elif MI_M == 16 && MI_K == 32
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const b8_t *)&a, *(const b8_t *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 16
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const b8_t *)&a, *(const b8_t *)&b, c, 0, 0, 0);
#else
#error "no such bf16 intrinsic"
#endif
#elif IN_DT == DT_I8
#if MI_M == 16 && MI_K == 32
    return __builtin_amdgcn_mfma_i32_16x16x32_i8(*(const long *)&a, *(const long *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 16
    return __builtin_amdgcn_mfma_i32_32x32x16_i8(*(const long *)&a, *(const long *)&b, c, 0, 0, 0);
#elif MI_M == 16 && MI_K == 64
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(*(const i4_t *)&a, *(const i4_t *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 32
    return __builtin_amdgcn_mfma_i32_32x32x32_i8(*(const i4_t *)&a, *(const i4_t *)&b, c, 0, 0, 0);
#else
#error "no such int8 intrinsic"
#endif
#elif IN_DT == DT_F8E4M3
#if MI_M == 16 && MI_K == 32
    return __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(*(const long *)&a, *(const long *)&b, c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 16
    return __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(*(const long *)&a, *(const long *)&b, c, 0, 0, 0);
#elif MI_M == 16 && MI_K == 128
    // the 8/6/4-bit float family: format selectors 0 = this 8-bit float for both operands; zero scale
    // operands select the unscaled form
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(*(const i8v_t *)&a, *(const i8v_t *)&b, c, 0, 0, 0, 0, 0, 0);
#elif MI_M == 32 && MI_K == 64
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(*(const i8v_t *)&a, *(const i8v_t *)&b, c, 0, 0, 0, 0, 0, 0);
#else
#error "no such 8-bit float intrinsic"
#endif
#elif IN_DT == DT_F32
#if MI_M == 16 && MI_K == 4
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a.v[0], b.v[0], c, 0, 0, 0);
#elif MI_M == 32 && MI_K == 2
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[0], b.v[0], c, 0, 0, 0);
#else
#error "no such fp32 intrinsic"
#endif
#else
#error "matrix-core kernels take fp16, bf16, int8, fp8 or fp32 inputs"
#endif
}

// One-wavefront-per-SIMD tiles (256 accumulators per lane) load their operands through buffer instructions: the
// address of a load is a resource descriptor and a byte offset in scalar registers plus one 32-bit per-lane offset
// shared by all loads of the operand, where flat 64-bit addresses take two vector registers per load once the k loop
// is unrolled.  The descriptor covers 2 GiB from the operand's base and checks nothing: the offsets are those of the
// pointer form.
#define BUFFER_LOADS (!IS_CONV && CACHE_READ <= 4 && (I1) * (I3) * (J1) * (J3) * (MI_M == 16 ? 4 : 16) >= 256)
#if BUFFER_LOADS
typedef int bl4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bl4_t buffer_load16(const void *base, unsigned voff, long uniform_bytes)
{
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, 0x7FFFFFF0, 0x00020000);
    return __builtin_amdgcn_raw_buffer_load_b128(rs, (int)voff, __builtin_amdgcn_readfirstlane((int)uniform_bytes), 0);
}
#endif

// ---- global -> registers -> LDS staging of one operand tile
//
// K-contiguous operand (A; B of the NT form; conv activations): a thread
// moves vectors of V elements along k (V = VEC for A, VEC_B for B); vector idx -> (row, kv), kv fastest.
template <int ROWS, int V> struct kmajor_stage {
    static constexpr int VK = V;                          // elements per vector along k
    static constexpr int KV = BK / V;                     // vectors per tile row
    static constexpr int PARTS = V > KPL ? V / KPL : 1;   // LDS writes per vector
    static constexpr int PART_E = V > KPL ? KPL : V;      // elements per LDS write
    static constexpr int TOTAL = ROWS * KV;
    static constexpr int ITERS = (TOTAL + NTHREADS - 1) / NTHREADS;
    vec_t<in_t, V> r[ITERS];
};

#if IS_CONV
// A reduction extent KH*KW*Cin that is no multiple of the intrinsic's k is rounded up: the loaders of both operands
// deliver zeros for k >= KH*KW*Cin (im2col staging only)
constexpr int CV_KREAL = CV_TAPROWS ? CV_KH * CV_KR : CV_KD * CV_KH * CV_KW * CV_CIN;
constexpr int CV_RUN = CV_KW * CV_CIN; // real elements of a filter row
constexpr bool K_PADDED = K0 * BK != CV_KREAL;
static_assert(K0 * BK >= CV_KREAL && K0 * BK - CV_KREAL < MI_K, "the k split covers the reduction, padded by less than one intrinsic");
static_assert(!CV_TAPROWS || (CV_KR % MI_K == 0 && CV_KR >= CV_RUN && !K_PADDED && CV_DIL == 1 && !CV_TRANSPOSED && CV_D == 1 &&
                              CV_KD == 1 && DIM_B == 1), "filter-row layout: plain conv2d");
static_assert(!K_PADDED || COMPUTE_AT == 0, "a padded reduction needs the im2col loader");
static_assert(!CV_TRANSPOSED || (COMPUTE_AT == 0 && CV_DIL == 1), "the transposed convolution exists in the im2col loader only");
static_assert((CV_D == 1 && CV_KD == 1) || (COMPUTE_AT == 0 && !CV_TRANSPOSED), "3-D convolution exists in the im2col loader only");
// im2col on the fly: row = output pixel, k = (kh, kw, ci)
template <int V> __device__ __forceinline__ vec_t<in_t, V> load_conv_a(const in_t *__restrict__ X, int row, int k)
{
    // row = (n, od, oh, ow), k = (kd, kh, kw, ci); od = kd = 0 for a 2-D convolution (CV_OD = CV_KD = 1)
    const int ow = row % CV_OW, oh = (row / CV_OW) % CV_OH, od = (row / (CV_OW * CV_OH)) % CV_OD, n = row / (CV_OW * CV_OH * CV_OD);
#if CV_TAPROWS
    const int q = k % CV_KR, kh = k / CV_KR, kd = 0;
    const int ci = q % CV_CIN, kw = q / CV_CIN; // kw >= CV_KW: padding of the run
    if (q >= CV_RUN) {
        vec_t<in_t, V> z;
#pragma unroll
        for (int e = 0; e < V; ++e) z.v[e] = 0;
        return z;
    }
#else
    const int ci = k % CV_CIN, kw = (k / CV_CIN) % CV_KW, kh = (k / (CV_CIN * CV_KW)) % CV_KH, kd = k / (CV_CIN * CV_KW * CV_KH);
#endif
    const int id = CV_D > 1 || CV_KD > 1 ? od * CV_STRIDE + kd * CV_DIL - CV_PAD : 0;
#if CV_TRANSPOSED
    // transposed convolution: input element ih reaches outputs ih * stride + kh - pad, so output row oh takes tap kh
    // from input row (oh + pad - kh) / stride when that is a whole number inside the image
    const int ihn = oh + CV_PAD_H - kh, iwn = ow + CV_PAD - kw;
    const bool on_grid = ihn >= 0 && iwn >= 0 && ihn % CV_STRIDE == 0 && iwn % CV_STRIDE == 0;
    const int ih = on_grid ? ihn / CV_STRIDE : -1, iw = on_grid ? iwn / CV_STRIDE : -1;
#else
    const int ih = oh * CV_STRIDE + kh * CV_DIL - CV_PAD_H, iw = ow * CV_STRIDE + kw * CV_DIL - CV_PAD;
#endif
    vec_t<in_t, V> x;
    if (ih >= 0 && ih < CV_H && iw >= 0 && iw < CV_W && id >= 0 && id < CV_D && (!K_PADDED || k < CV_KREAL)) {
        x = *reinterpret_cast<const vec_t<in_t, V> *>(X + ((((long)n * CV_D + id) * CV_H + ih) * CV_W + iw) * CV_XC + ci);
    } else {
#pragma unroll
        for (int q = 0; q < V; ++q) x.v[q] = 0;
    }
    return x;
}
#endif

// Loads are numbered ("units") so that a caller can issue any sub-range [u0, u1) of a tile's loads:
// the software-pipelined main loop spreads them between the MFMAs of a k step.
template <int ROWS, int V, bool CONV_A>
__device__ __forceinline__ void kmajor_load(kmajor_stage<ROWS, V> &st, const in_t *__restrict__ src, long row0, long k0e, long row_stride,
                                            int tid, int u0, int u1)
{
    typedef kmajor_stage<ROWS, V> S;
    constexpr int KV = S::KV;
#pragma unroll
    for (int it = 0; it < S::ITERS; ++it) {
        if (it < u0 || it >= u1) continue;
        const int idx = it * NTHREADS + tid;
        if (S::TOTAL % NTHREADS == 0 || idx < S::TOTAL) {
            const int row = idx / KV, kv = idx % KV;
#if IS_CONV
            if (CONV_A) {
                st.r[it] = load_conv_a<V>(src, (int)row0 + row, (int)k0e + kv * V);
                continue;
            }
#endif
            if (NTHREADS % KV == 0) {
                // address = uniform base (scalar registers) + one 32-bit per-lane offset shared by all iterations
                const unsigned voff = (unsigned)(((tid / KV) * row_stride + (tid % KV) * V) * ES);
#if BUFFER_LOADS
                if constexpr (V * ES == 16) {
                    const bl4_t x = buffer_load16(src, voff, ((row0 + it * (NTHREADS / KV)) * row_stride + k0e) * ES);
                    st.r[it] = *reinterpret_cast<const vec_t<in_t, V> *>(&x);
                    continue;
                }
#endif
                const char *ub = (const char *)(src + (row0 + it * (NTHREADS / KV)) * row_stride + k0e);
                st.r[it] = *reinterpret_cast<const vec_t<in_t, V> *>(ub + voff);
            } else {
                st.r[it] = *reinterpret_cast<const vec_t<in_t, V> *>(src + (row0 + row) * row_stride + k0e + kv * V);
            }
        }
    }
}

template <int ROWS, int V, int PLANE>
__device__ __forceinline__ void kmajor_store(const kmajor_stage<ROWS, V> &st, char *__restrict__ lds, int tid, int u0, int u1)
{
    typedef kmajor_stage<ROWS, V> S;
    constexpr int KV = S::KV, PARTS = S::PARTS, PART_E = S::PART_E;
    // when the thread count is a multiple of the vectors per row, every iteration of a thread differs
    // from the first by a constant number of rows: one address register, constant offsets
    constexpr bool AFFINE = NTHREADS % KV == 0;
    const int row_t = tid / KV, kv_t = tid % KV;
#pragma unroll
    for (int it = 0; it < S::ITERS; ++it) {
        if (it < u0 || it >= u1) continue;
        const int idx = it * NTHREADS + tid;
        if (S::TOTAL % NTHREADS == 0 || idx < S::TOTAL) {
            const int row = AFFINE ? row_t + it * (NTHREADS / KV) : idx / KV;
            const int kv = AFFINE ? kv_t : idx % KV;
            const int k = kv * V;
#pragma unroll
            for (int p = 0; p < PARTS; ++p) {
                const int kk = k + p * PART_E;
                char *dst = lds + (kk / KPL) * PLANE + lds_slot(row) * LFRAG_BYTES + (kk % KPL) * ES;
                vec_t<in_t, PART_E> part;
#pragma unroll
                for (int q = 0; q < PART_E; ++q) part.v[q] = st.r[it].v[p * PART_E + q];
                *reinterpret_cast<vec_t<in_t, PART_E> *>(dst) = part;
            }
        }
    }
}

// J-contiguous operand (B of the NN form, conv weights): a thread moves a
// block of KPL k-rows x VEC_B columns and transposes it in registers, so that it
// lands in LDS as VEC_B consecutive fragments.
constexpr int VJ = VEC_B;
constexpr int JV = BN / VJ;

struct jmajor_stage {
    static constexpr int TOTAL = (BK / KPL) * JV;
    static constexpr int ITERS = (TOTAL + NTHREADS - 1) / NTHREADS;
    vec_t<in_t, VJ> r[ITERS][KPL];
};

__device__ __forceinline__ void jmajor_load(jmajor_stage &st, const in_t *__restrict__ src, long col0, long k0e, long k_stride, int tid,
                                            int u0, int u1)
{
    typedef jmajor_stage S;
#pragma unroll
    for (int it = 0; it < S::ITERS; ++it) {
        const int idx = it * NTHREADS + tid;
        if (S::TOTAL % NTHREADS == 0 || idx < S::TOTAL) {
            const int kg = idx / JV, jv = idx % JV;
#pragma unroll
            for (int q = 0; q < KPL; ++q) {
                const int u = it * KPL + q;
                if (u < u0 || u >= u1) continue;
#if IS_CONV
                if (K_PADDED && k0e + kg * KPL + q >= CV_KREAL) { // rows of the padding: zeros, nothing is read
#pragma unroll
                    for (int c = 0; c < VJ; ++c) st.r[it][q].v[c] = 0;
                    continue;
                }
#if CV_TAPROWS
                {
                    // row (kh, qq) of the filter-row layout is row kh * KW * Cin + qq of W, or padding
                    const int kk = (int)k0e + kg * KPL + q, qq = kk % CV_KR;
                    if (qq >= CV_RUN) {
#pragma unroll
                        for (int c = 0; c < VJ; ++c) st.r[it][q].v[c] = 0;
                    } else {
                        st.r[it][q] = *reinterpret_cast<const vec_t<in_t, VJ> *>(src + (long)((kk / CV_KR) * CV_RUN + qq) * k_stride + col0 + jv * VJ);
                    }
                    continue;
                }
#endif
#endif
                if (NTHREADS % JV == 0) {
                    const char *ub = (const char *)(src + (k0e + (it * (NTHREADS / JV)) * KPL + q) * k_stride + col0);
                    const unsigned voff = (unsigned)(((tid / JV) * KPL * k_stride + (tid % JV) * VJ) * ES);
                    st.r[it][q] = *reinterpret_cast<const vec_t<in_t, VJ> *>(ub + voff);
                } else {
                    st.r[it][q] = *reinterpret_cast<const vec_t<in_t, VJ> *>(src + (k0e + kg * KPL + q) * k_stride + col0 + jv * VJ);
                }
            }
        }
    }
}

__device__ __forceinline__ void jmajor_store(const jmajor_stage &st, char *__restrict__ lds, int tid, int u0, int u1)
{
    typedef jmajor_stage S;
    constexpr bool AFFINE = NTHREADS % JV == 0;
    const int kg_t = tid / JV, jv_t = tid % JV;
#pragma unroll
    for (int it = 0; it < S::ITERS; ++it) {
        if (it < u0 || it >= u1) continue;
        const int idx = it * NTHREADS + tid;
        if (S::TOTAL % NTHREADS == 0 || idx < S::TOTAL) {
            const int kg = AFFINE ? kg_t + it * (NTHREADS / JV) : idx / JV;
            const int jv = AFFINE ? jv_t : idx % JV;
            char *dst = lds + kg * SUBPLANE_B;
#pragma unroll
            for (int c = 0; c < VJ; ++c) {
                lfrag_t f;
#pragma unroll
                for (int q = 0; q < KPL; ++q) f.v[q] = st.r[it][q].v[c];
                *reinterpret_cast<lfrag_t *>(dst + lds_slot(jv * VJ + c) * LFRAG_BYTES) = f;
            }
        }
    }
}

#if CONV_PATCH
// ---- resident input patch (COMPUTE_AT 1)
constexpr int P_ROWS_OUT = BM % CV_OW == 0 ? BM / CV_OW : (CV_OW + BM - 2) / CV_OW + 1; // output rows a tile can touch
constexpr int P_R = (P_ROWS_OUT - 1) * CV_STRIDE + CV_DIL * (CV_KH - 1) + 1; // patch rows (taps CV_DIL apart)
// filter-row layout: dense pixels (a run crosses pixel boundaries), plus the pixels that the padding of a run reaches
// behind the last tap (zeros or the next pixels: finite values that meet zero weights), rows at multiples of 4 bytes
constexpr int P_W0 = (CV_OW - 1) * CV_STRIDE + CV_DIL * (CV_KW - 1) + 1 + (CV_TAPROWS ? (CV_KR - CV_RUN + CV_CIN - 1) / CV_CIN : 0);
constexpr int P_PS = CV_CIN * ES + (LDS_PAD && !CV_TAPROWS ? 16 : 0); // bytes per patch pixel; the pad staggers neighbouring pixels over the banks
constexpr int P_W = P_W0 + (CV_TAPROWS && (P_W0 * P_PS) % 4 ? 1 : 0);  // patch columns (column pc = input column pc - pad)
constexpr int P_RS = P_W * P_PS;                            // bytes per patch row
constexpr int PATCH_BYTES = ((P_R * P_RS + 15) / 16) * 16;
static_assert(CV_TAPROWS || CV_CIN % MI_K == 0, "resident input patch: an MFMA k step must stay inside one filter tap");
static_assert(!CV_TAPROWS || ((CV_STRIDE * CV_CIN * ES) % 4 == 0 && P_RS % 4 == 0 && FRAG_BYTES % 4 == 0), "filter-row layout: fragments start at multiples of 4 bytes");
static_assert((CV_OH * CV_OW) % BM == 0, "resident input patch: tiles must not straddle images");

struct conv_ctx {
    const char *patch; // + this lane's k-group offset
    int pix[TM];       // byte offset of the lane's output pixel (tap 0, 0) per MFMA tile row
};

// The patch goes global memory -> registers -> LDS in two calls (fetch, commit), so that a persistent
// workgroup can fetch the next tile's patch while it multiplies the current one.  A patch row is
// P_CR vectors of VEC channels; threads are laid over rows so that a thread's column, its channel
// vector and the in-image test of the column do not depend on the tile.
constexpr int P_NT = CONV_HELPERS ? HELPER_WAVES * 64 : NTHREADS; // threads that move the patch
constexpr int P_CPP = CV_CIN / VEC;                              // vectors per pixel
constexpr int P_CR = P_W * P_CPP;                                // vectors per patch row
constexpr int P_PPR = (P_CR + P_NT - 1) / P_NT;                  // passes of the movers over one row
constexpr int P_RPP = P_NT >= P_CR ? P_NT / P_CR : 1;            // rows per pass
constexpr int P_PASSES = (P_R + P_RPP - 1) / P_RPP;
constexpr int P_ITERS = P_PASSES * P_PPR;

struct patch_regs {
    vec_t<in_t, VEC> r[P_ITERS];
};

struct patch_map {   // per thread, the same for every tile
    int row_t;       // row inside a pass (0 when a row takes the whole workgroup)
    int goff[P_PPR]; // element offset of the thread's vector from the start of an input row (may be negative: left halo)
    int loff[P_PPR]; // byte offset inside a patch row
    bool ok[P_PPR];  // the vector exists and its column is inside the image
};

__device__ __forceinline__ void patch_map_init(patch_map &pm, int tid)
{
    pm.row_t = P_NT >= P_CR ? tid / P_CR : 0;
#pragma unroll
    for (int s = 0; s < P_PPR; ++s) {
        const int q = P_NT >= P_CR ? tid % P_CR : s * P_NT + tid;
        const int pc = q / P_CPP, c = q % P_CPP;
        const int iw = pc - CV_PAD;
        pm.goff[s] = iw * CV_XC + c * VEC;
        pm.loff[s] = pc * P_PS + c * (VEC * ES);
        pm.ok[s] = q < P_CR && pm.row_t < P_RPP && (unsigned)iw < (unsigned)CV_W;
    }
}

// request input rows [ih_lo, ih_lo + P_R) of the image that holds output tile i0 (X: the instance's activations)
__device__ __forceinline__ void patch_fetch(patch_regs &pr, const patch_map &pm, const in_t *__restrict__ X, int i0)
{
    const int m0 = i0 * BM;
    const int n = m0 / (CV_OH * CV_OW);
    const int ih_lo = ((m0 % (CV_OH * CV_OW)) / CV_OW) * CV_STRIDE - CV_PAD_H;
    const in_t *img = X + (long)n * (CV_H * CV_W * CV_XC);
#pragma unroll
    for (int p = 0; p < P_PASSES; ++p)
#pragma unroll
        for (int s = 0; s < P_PPR; ++s) {
            const int row = p * P_RPP + pm.row_t;
            const int ih = ih_lo + row;
            const bool ok = pm.ok[s] && (unsigned)ih < (unsigned)CV_H && (P_R % P_RPP == 0 || row < P_R);
            // elements outside the image read element 0 (always mapped) and become zero: no divergent loads
            const int off = ok ? ih * (CV_W * CV_XC) + pm.goff[s] : 0;
            vec_t<in_t, VEC> x = *reinterpret_cast<const vec_t<in_t, VEC> *>(img + off);
            if (!ok) {
#pragma unroll
                for (int q = 0; q < VEC; ++q) x.v[q] = 0;
            }
            pr.r[p * P_PPR + s] = x;
        }
}

// write the fetched patch to LDS (halo elements as zeros)
__device__ __forceinline__ void patch_commit(const patch_regs &pr, const patch_map &pm, char *__restrict__ patch, int tid)
{
#pragma unroll
    for (int p = 0; p < P_PASSES; ++p)
#pragma unroll
        for (int s = 0; s < P_PPR; ++s) {
            const int row = p * P_RPP + pm.row_t;
            const int q = P_NT >= P_CR ? tid % P_CR : s * P_NT + tid;
            const bool live = (P_NT >= P_CR ? pm.row_t < P_RPP : q < P_CR) && (P_R % P_RPP == 0 || row < P_R);
            if (live) *reinterpret_cast<vec_t<in_t, VEC> *>(patch + row * P_RS + pm.loff[s]) = pr.r[p * P_PPR + s];
        }
}

__device__ __forceinline__ void conv_ctx_init(conv_ctx &cx, const char *patch, int i0, int wi, int lrow, int lgrp)
{
    const int m0 = i0 * BM;
    const int oh_lo = (m0 % (CV_OH * CV_OW)) / CV_OW;
    cx.patch = patch + lgrp * FRAG_BYTES;
#pragma unroll
    for (int r1 = 0; r1 < I1; ++r1)
#pragma unroll
        for (int r3 = 0; r3 < I3; ++r3) {
            const int trow = (r1 * I2 + wi) * I3 + r3;
            const int mm = (m0 + trow * MI_M + lrow) % (CV_OH * CV_OW);
            const int oh = mm / CV_OW, ow = mm % CV_OW;
            cx.pix[r1 * I3 + r3] = (oh - oh_lo) * CV_STRIDE * P_RS + ow * CV_STRIDE * P_PS;
        }
}

// a lane's A fragment from the patch; in the filter-row layout it starts at a multiple of 4 bytes only
__device__ __forceinline__ frag_t patch_frag(const char *__restrict__ p)
{
#if CV_TAPROWS
    frag_t f;
    const unsigned *w = reinterpret_cast<const unsigned *>(__builtin_assume_aligned(p, 4));
    unsigned *o = reinterpret_cast<unsigned *>(&f);
#pragma unroll
    for (int i = 0; i < FRAG_BYTES / 4; ++i) o[i] = w[i];
    return f;
#else
    return *reinterpret_cast<const frag_t *>(p);
#endif
}

// byte offset inside the patch of MFMA k step `step` of tile k0, relative to a pixel's (tap 0, 0, channel 0)
__device__ __forceinline__ int conv_koff(int k0, int step)
{
    const int kg = k0 * BK + step * MI_K; // wave-uniform
#if CV_TAPROWS
    return (kg / CV_KR) * P_RS + (kg % CV_KR) * ES; // filter row kh, then the position inside the run
#endif
    const int tap = kg / CV_CIN, ci = kg % CV_CIN;
    const int kh = tap / CV_KW, kw = tap % CV_KW;
    return kh * CV_DIL * P_RS + kw * CV_DIL * P_PS + ci * ES;
}
#else
struct conv_ctx {
};
#endif

// ---- j-contiguous B kept row-major in LDS (direct-to-LDS rings and LDS_PAD 3): k-rows of BN elements, the
// 16-column granules (what one transposing LDS load covers: 32 bytes of 2-byte, 16 bytes of 1-byte elements) of a row
// XOR-swizzled with the row number; needs a power-of-two granule count
constexpr int CE = 16 / ES;                               // elements per 16-byte chunk
#if !B_KMAJOR
constexpr int CB = BN / CE;                               // 16-byte chunks per k-row of the j-contiguous B tile
constexpr int BROW_BYTES = BN * ES;
constexpr int NGRAN = BN / 16;
constexpr int GRAN_MASK = (NGRAN & (NGRAN - 1)) ? 0 : (NGRAN > 16 ? 15 : NGRAN - 1);
// chunk-index XOR for k-row `k`: moves whole 16-column granules (ES chunks each)
__device__ __forceinline__ int dl_swz_b(int k) { return (k & GRAN_MASK) * ES; }
#endif
typedef short tr4_t __attribute__((ext_vector_type(4)));
typedef int tr2_t __attribute__((ext_vector_type(2)));

#if B_ROWMAJOR
// chunk-index XOR of k-row `k` in the register-staged row-major stage (none with padded rows)
__device__ __forceinline__ int rm_swz(int k) { return LDS_PAD == 4 ? 0 : dl_swz_b(k); }
static_assert((ES == 2 && (KP == 4 || KP == 8)) || (ES == 1 && (KP == 8 || KP == 16 || KP == 32)),
              "row-major B in LDS: fragments of whole transposing loads (4 k of 2-byte, 8 k of 1-byte elements)");
static_assert(VEC_B == CE, "row-major B in LDS moves 16-byte vectors");
// a thread moves 16-byte chunks; chunk idx -> (k-row, chunk of the row), chunks of a row on consecutive lanes
struct rowmajor_stage {
    static constexpr int TOTAL = BK * CB;
    static constexpr int ITERS = (TOTAL + NTHREADS - 1) / NTHREADS;
    vec_t<in_t, CE> r[ITERS];
};

__device__ __forceinline__ void rowmajor_load(rowmajor_stage &st, const in_t *__restrict__ src, long col0, long k0e, long k_stride, int tid, int u0,
                                              int u1)
{
    typedef rowmajor_stage S;
#pragma unroll
    for (int it = 0; it < S::ITERS; ++it) {
        if (it < u0 || it >= u1) continue;
        const int idx = it * NTHREADS + tid;
        if (S::TOTAL % NTHREADS == 0 || idx < S::TOTAL) {
            if (NTHREADS % CB == 0) {
                // wave-uniform base + 32-bit per-lane offset
                const unsigned voff = (unsigned)(((tid / CB) * k_stride + (tid % CB) * CE) * ES);
#if BUFFER_LOADS
                {
                    const bl4_t x = buffer_load16(src, voff, ((k0e + it * (NTHREADS / CB)) * k_stride + col0) * ES);
                    st.r[it] = *reinterpret_cast<const vec_t<in_t, CE> *>(&x);
                    continue;
                }
#endif
                const char *ub = (const char *)(src + (k0e + it * (NTHREADS / CB)) * k_stride + col0);
                st.r[it] = *reinterpret_cast<const vec_t<in_t, CE> *>(ub + voff);
            } else {
                st.r[it] = *reinterpret_cast<const vec_t<in_t, CE> *>(src + (k0e + idx / CB) * k_stride + col0 + (idx % CB) * CE);
            }
        }
    }
}

__device__ __forceinline__ void rowmajor_store(const rowmajor_stage &st, char *__restrict__ lds, int tid, int u0, int u1)
{
    typedef rowmajor_stage S;
#pragma unroll
    for (int it = 0; it < S::ITERS; ++it) {
        if (it < u0 || it >= u1) continue;
        const int idx = it * NTHREADS + tid;
        if (S::TOTAL % NTHREADS == 0 || idx < S::TOTAL) {
            const int k = idx / CB, c = idx % CB;
            *reinterpret_cast<vec_t<in_t, CE> *>(lds + k * RM_ROW + ((c ^ rm_swz(k)) * 16)) = st.r[it];
        }
    }
}

// the B fragment of MFMA k step `step` for the 16 x 16 or 32 x 32 tile at tile column `tcol`, from the stage's B
// region at `b`.  A lane's KP k values come from KP/4 (2-byte elements) or KP/8 (1-byte elements) transposing loads.
// 2-byte (ds_read_b64_tr_b16): 16 lanes hand in 4 k-rows x 16 columns (lane: k-row li/4, 4 columns from li%4) and every
// lane receives 4 consecutive k of its own column.  1-byte (ds_read_b64_tr_b8): 8 k-rows x 16 columns per 16 lanes
// (lane: k-row li/2, 8 columns from li%2), every lane receives 8 consecutive k of its own column.
__device__ __forceinline__ frag_t rowmajor_frag(const char *__restrict__ b, int step, int tcol, int lane)
{
    const int lrow = lane % MI_M, lgrp = lane / MI_M, li = lane % 16;
    const int pn = (tcol * MI_N + lrow) / 16; // 16-column granule of this lane's column
    frag_t f;
#if IN_DT != DT_I8 && IN_DT != DT_F8E4M3
#pragma unroll
    for (int h = 0; h < KP / 4; ++h) {
        const int krow = step * MI_K + lgrp * KP + h * 4 + li / 4;
        const char *src = b + krow * RM_ROW + (((pn << 1) ^ rm_swz(krow)) * 16) + (li % 4) * 8;
        *reinterpret_cast<tr4_t *>(&f.v[4 * h]) = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) tr4_t *)(src));
    }
#else
#pragma unroll
    for (int h = 0; h < KP / 8; ++h) {
        const int krow = step * MI_K + lgrp * KP + h * 8 + li / 2;
        const char *src = b + krow * RM_ROW + ((pn ^ rm_swz(krow)) * 16) + (li % 2) * 8;
        *reinterpret_cast<tr2_t *>(&f.v[8 * h]) = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) tr2_t *)(src));
    }
#endif
    return f;
}
#endif

struct tile_stage {
#if !CONV_PATCH
    kmajor_stage<BM, VEC> a;
#endif
#if B_KMAJOR
    kmajor_stage<BN, VEC_B> b;
    static constexpr int UNITS_B = kmajor_stage<BN, VEC_B>::ITERS;
#elif B_ROWMAJOR
    rowmajor_stage b;
    static constexpr int UNITS_B = rowmajor_stage::ITERS;
#else
    jmajor_stage b;
    static constexpr int UNITS_B = jmajor_stage::ITERS * KPL;
#endif
    static constexpr int UNITS_A = CONV_PATCH ? 0 : kmajor_stage<BM, VEC>::ITERS;
    static constexpr int UNITS = UNITS_A + UNITS_B; // global load instructions per thread and tile
    static constexpr int SUNITS_A = UNITS_A;
    static constexpr int SUNITS = SUNITS_A + (B_KMAJOR || B_ROWMAJOR ? UNITS_B : UNITS_B / KPL); // store units (one per staged vector / block)
};

// issue load units [u0, u1) of the tile of step k0
__device__ __forceinline__ void stage_load(tile_stage &st, const in_t *__restrict__ A, const in_t *__restrict__ B, int i0, int j0, int k0,
                                           int tid, int u0 = 0, int u1 = tile_stage::UNITS)
{
    const long k0e = (long)k0 * BK;
#if !CONV_PATCH
    kmajor_load<BM, VEC, true>(st.a, A, (long)i0 * BM, k0e, SA_I, tid, u0, u1);
#endif
#if B_KMAJOR
    kmajor_load<BN, VEC_B, false>(st.b, B, (long)j0 * BN, k0e, SB_J, tid, u0 - tile_stage::UNITS_A, u1 - tile_stage::UNITS_A);
#elif B_ROWMAJOR
    rowmajor_load(st.b, B, (long)j0 * BN, k0e, SB_K, tid, u0 - tile_stage::UNITS_A, u1 - tile_stage::UNITS_A);
#else
    jmajor_load(st.b, B, (long)j0 * BN, k0e, SB_K, tid, u0 - tile_stage::UNITS_A, u1 - tile_stage::UNITS_A);
#endif
}

// write store units [u0, u1) of a staged tile to the LDS stage at `lds`
__device__ __forceinline__ void stage_store(const tile_stage &st, char *__restrict__ lds, int tid, int u0 = 0, int u1 = tile_stage::SUNITS)
{
#if !CONV_PATCH
    kmajor_store<BM, VEC, SUBPLANE_A>(st.a, lds, tid, u0, u1);
#endif
#if B_KMAJOR
    kmajor_store<BN, VEC_B, SUBPLANE_B>(st.b, lds + A_STAGE_BYTES, tid, u0 - tile_stage::SUNITS_A, u1 - tile_stage::SUNITS_A);
#elif B_ROWMAJOR
    rowmajor_store(st.b, lds + A_STAGE_BYTES, tid, u0 - tile_stage::SUNITS_A, u1 - tile_stage::SUNITS_A);
#else
    jmajor_store(st.b, lds + A_STAGE_BYTES, tid, u0 - tile_stage::SUNITS_A, u1 - tile_stage::SUNITS_A);
#endif
}

// fragments of slot `slot` (K3 consecutive MFMA k steps) for the wave's TM x TN tiles
// (COMPUTE_AT 1: the A fragments come from the resident input patch; `la` is unused, `kcur` is the tile's k0)
__device__ __forceinline__ void read_frags(frag_t (&fa)[K3][TM], frag_t (&fb)[K3][TN], const char *__restrict__ la,
                                           const char *__restrict__ lb, int slot, int wi, int wj, int lrow, const conv_ctx &cx, int kcur)
{
#pragma unroll
    for (int q = 0; q < K3; ++q) {
        const int step = slot * K3 + q;
#if CONV_PATCH
        const int koff = conv_koff(kcur, step);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) fa[q][tm] = patch_frag(cx.patch + (cx.pix[tm] + koff));
#else
#pragma unroll
        for (int r1 = 0; r1 < I1; ++r1)
#pragma unroll
            for (int r3 = 0; r3 < I3; ++r3) {
                const int trow = (r1 * I2 + wi) * I3 + r3;
                fa[q][r1 * I3 + r3] = lds_frag<SUBPLANE_A>(la + step * LANE_GROUPS * PLANE_A + lds_slot(trow * MI_M + lrow) * LFRAG_BYTES);
            }
#endif
#pragma unroll
        for (int c1 = 0; c1 < J1; ++c1)
#pragma unroll
            for (int c3 = 0; c3 < J3; ++c3) {
                const int tcol = (c1 * J2 + wj) * J3 + c3;
#if B_ROWMAJOR
                fb[q][c1 * J3 + c3] = rowmajor_frag(lb, step, tcol, (int)(threadIdx.x % 64));
#else
                fb[q][c1 * J3 + c3] = lds_frag<SUBPLANE_B>(lb + step * LANE_GROUPS * PLANE_B + lds_slot(tcol * MI_N + lrow) * LFRAG_BYTES);
#endif
            }
    }
}

// operands swapped: the instruction produces the transposed tile, so that a lane ends up with 4
// consecutive columns of one row of C (one vector store in the epilogue)
__device__ __forceinline__ void mfma_slot(accv_t (&acc)[TM][TN], const frag_t (&fa)[K3][TM], const frag_t (&fb)[K3][TN])
{
#pragma unroll
    for (int q = 0; q < K3; ++q)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = mfma(fb[q][tn], fa[q][tm], acc[tm][tn]);
}

// One fully software-pipelined step (k1, k2 unrolled): multiplies the tile staged at `cur` while it
// writes the already arrived tile `ready` to the other LDS stage `nxt` and requests tile `kload`
// into `inflight`.  Each of the NS slots issues, ahead of its own MFMAs, the next slot's LDS reads,
// its share of the LDS writes and its share of the global loads: loads, LDS traffic and matrix
// cores work at the same time instead of taking turns.
#define NS_ (K1 * K2)
__device__ __forceinline__ void pipelined_step(accv_t (&acc)[TM][TN], const char *__restrict__ cur, char *__restrict__ nxt,
                                               const tile_stage &ready, tile_stage &inflight, const in_t *__restrict__ A,
                                               const in_t *__restrict__ B, int i0, int j0, int kload, int tid, int lgrp, int wi, int wj, int lrow,
                                               const conv_ctx &cx, int kcur)
{
    const char *la = cur + lgrp * PLANE_A;
    const char *lb = cur + A_STAGE_BYTES + lgrp * B_LGRP;
    frag_t fa[2][K3][TM], fb[2][K3][TN];
    read_frags(fa[0], fb[0], la, lb, 0, wi, wj, lrow, cx, kcur);
#pragma unroll
    for (int s = 0; s < NS_; ++s) {
        if (s + 1 < NS_) read_frags(fa[(s + 1) & 1], fb[(s + 1) & 1], la, lb, s + 1, wi, wj, lrow, cx, kcur);
        stage_store(ready, nxt, tid, s * tile_stage::SUNITS / NS_, (s + 1) * tile_stage::SUNITS / NS_);
        stage_load(inflight, A, B, i0, j0, kload, tid, s * tile_stage::UNITS / NS_, (s + 1) * tile_stage::UNITS / NS_);
        mfma_slot(acc, fa[s & 1], fb[s & 1]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// multiply the tile staged at `stage_base` (rolled / partly unrolled k1, k2 loops)
__device__ __forceinline__ void multiply_tile(accv_t (&acc)[TM][TN], const char *__restrict__ stage_base, int lgrp, int wi, int wj, int lrow,
                                              const conv_ctx &cx, int kcur)
{
    const char *la = stage_base + lgrp * PLANE_A;
    const char *lb = stage_base + A_STAGE_BYTES + lgrp * B_LGRP;
#pragma unroll UNROLL_K1
    for (int k1 = 0; k1 < K1; ++k1) {
#pragma unroll UNROLL_K2
        for (int k2 = 0; k2 < K2; ++k2) {
            frag_t fa[K3][TM], fb[K3][TN];
            read_frags(fa, fb, la, lb, k1 * K2 + k2, wi, wj, lrow, cx, kcur);
            mfma_slot(acc, fa, fb);
        }
    }
}

// the same with k1, k2 fully unrolled: slot s issues the LDS reads of slot s+1 ahead of its own MFMAs
__device__ __forceinline__ void multiply_tile_unrolled(accv_t (&acc)[TM][TN], const char *__restrict__ stage_base, int lgrp, int wi, int wj,
                                                       int lrow, const conv_ctx &cx, int kcur)
{
    const char *la = stage_base + lgrp * PLANE_A;
    const char *lb = stage_base + A_STAGE_BYTES + lgrp * B_LGRP;
    frag_t fa[2][K3][TM], fb[2][K3][TN];
    read_frags(fa[0], fb[0], la, lb, 0, wi, wj, lrow, cx, kcur);
#pragma unroll
    for (int s = 0; s < K1 * K2; ++s) {
        if (s + 1 < K1 * K2) read_frags(fa[(s + 1) & 1], fb[(s + 1) & 1], la, lb, s + 1, wi, wj, lrow, cx, kcur);
        mfma_slot(acc, fa[s & 1], fb[s & 1]);
        __builtin_amdgcn_sched_barrier(0);
    }
}

#if CONV_BREG
constexpr int NSTEP = K0 * KSTEPS; // all MFMA k steps of the reduction

// weights of output columns j0*BN .. of one instance -> registers of the wavefronts that own the columns
__device__ __forceinline__ void weights_to_regs(frag_t (&bw)[NSTEP][TN], const in_t *__restrict__ Wt, int j0, char *__restrict__ wstage, int tid,
                                                int lgrp, int wj, int lrow)
{
    tile_stage st;
#pragma unroll
    for (int k0 = 0; k0 < K0; ++k0) {
        stage_load(st, nullptr, Wt, 0, j0, k0, tid);
        if (k0 > 0) __syncthreads(); // the previous step's fragments have been read
        stage_store(st, wstage, tid);
        __syncthreads();
        const char *lb = wstage + lgrp * PLANE_B;
#pragma unroll
        for (int q = 0; q < KSTEPS; ++q)
#pragma unroll
            for (int c1 = 0; c1 < J1; ++c1)
#pragma unroll
                for (int c3 = 0; c3 < J3; ++c3) {
                    const int tcol = (c1 * J2 + wj) * J3 + c3;
                    bw[k0 * KSTEPS + q][c1 * J3 + c3] = lds_frag<SUBPLANE_B>(lb + q * LANE_GROUPS * PLANE_B + lds_slot(tcol * MI_N + lrow) * LFRAG_BYTES);
                }
    }
}

// the whole reduction of one tile: A fragments from the patch (read one step ahead), B from registers
__device__ __forceinline__ void multiply_all_k(accv_t (&acc)[TM][TN], const frag_t (&bw)[NSTEP][TN], const conv_ctx &cx)
{
    frag_t fa[2][TM];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) fa[0][tm] = patch_frag(cx.patch + (cx.pix[tm] + conv_koff(0, 0)));
#pragma unroll
    for (int s = 0; s < NSTEP; ++s) {
        if (s + 1 < NSTEP) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                fa[(s + 1) & 1][tm] = patch_frag(cx.patch + (cx.pix[tm] + conv_koff(0, s + 1)));
        }
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = mfma(bw[s][tn], fa[s & 1][tm], acc[tm][tn]);
        __builtin_amdgcn_sched_barrier(0);
    }
}
#endif

constexpr int NS = K1 * K2;
#define PIPELINED (CACHE_READ < 3 && UNROLL_K1 == K1 && UNROLL_K2 == K2 && K1 * K2 > 1)

// ======================================================================================
// Direct-to-LDS path (CACHE_READ 5, 6, 7 = a ring of 2, 3, 4 LDS stages).
//
// Tiles go from global memory straight into LDS (global_load_lds, 16 bytes per lane, the 64
// lanes of a wavefront fill 1 KiB of consecutive LDS): no staging registers, no LDS write
// instructions, and up to 3 tiles in flight while one is multiplied.  Because the LDS side of
// such a load is fixed (lane i -> byte 16*i), the layouts are chosen for the readers and the
// global address of each lane is derived from them:
//   k-contiguous operand (A; B of NT): row-major rows of BK elements, the 16-byte chunks of a
//       row XOR-swizzled with the row number, so that the 8 or 16 lanes that read the same
//       logical chunk of consecutive rows hit different banks; one load instruction covers
//       whole 128-byte lines of 64/CPR rows.
//   j-contiguous operand (B of NN): row-major k-rows of BN elements as in global memory (a load
//       instruction covers whole 128-byte lines), the 32-byte granules (16 columns) of a row
//       XOR-swizzled with the row number, read with the LDS
//       transpose load (ds_read_b64_tr_b16: inside a group of 16 lanes, lane i receives element
//       i%4 of lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4): four lanes hand in one k-row of the panel,
//       every lane gets 4 consecutive k of its own column - the MFMA B fragment.
// 16-byte fragments only: 2-byte inputs with 16x16x32 / 32x32x16, 1-byte inputs with 16x16x64 / 32x32x32 (their B of NN
// is read with the 8-bit transpose load, 8 k-rows x 16 columns per group of 16 lanes).
#if CACHE_READ >= 5
constexpr int DL_STAGES = CACHE_READ >= 8 ? CACHE_READ - 6 : CACHE_READ - 3; // 5, 6, 7 and 8, 9, 10: rings of 2, 3, 4 stages
constexpr int CPR = BK / CE;                              // 16-byte chunks per k-contiguous row
constexpr int ROW_BYTES = BK * ES;
constexpr int SWZ_DIV = CPR >= 8 ? 1 : 8 / CPR;           // rows that share one 128-byte line
constexpr int RPI = 64 / CPR;                             // rows per load instruction
constexpr int DL_A_BYTES = BM * ROW_BYTES;
#if B_KMAJOR
constexpr int DL_B_BYTES = BN * ROW_BYTES;
#else
constexpr int DL_B_BYTES = ((BK * (BN / CE) + 63) / 64) * 1024;
#endif
constexpr int DL_STAGE_BYTES = DL_A_BYTES + DL_B_BYTES;
constexpr int DL_IA = BM / RPI;                           // load instructions per A tile
#if B_KMAJOR
constexpr int DL_IB = BN / RPI;
#else
constexpr int DL_IB = (BK * CB + 63) / 64;
#endif
constexpr int DL_INSTR = DL_IA + DL_IB;
constexpr int DL_LPW_MIN = DL_INSTR / NWAVES;             // loads every wavefront issues per tile, at least
static_assert((ES == 2 && KP == 8) || (ES == 1 && KP == 16), "direct-to-LDS path: 16-byte fragments of 2-byte or 1-byte inputs");
static_assert(CPR == 4 || CPR == 8 || CPR == 16, "direct-to-LDS path: k tile of 64, 128 or 256 bytes");

#define AS1(p) ((const __attribute__((address_space(1))) void *)(p))
#define AS3(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ int dl_swz(int row) { return (row / SWZ_DIV) % CPR; }

// issue this wavefront's share of the loads of tile `k0` into the stage at `stage`
__device__ __forceinline__ void dl_issue(const in_t *__restrict__ A, const in_t *__restrict__ B, char *stage, int i0, int j0, int k0, int wave,
                                         int lane)
{
    const long k0e = (long)k0 * BK;
#pragma unroll
    for (int n = 0; n < (DL_INSTR + NWAVES - 1) / NWAVES; ++n) {
        const int inst = n * NWAVES + wave; // wave-uniform
        // every address = wave-uniform base (scalar registers) + a 32-bit per-lane byte offset
        if (inst < DL_IA) {
            const int row = inst * RPI + lane / CPR;
            const int c = (lane % CPR) ^ dl_swz(row);
            const char *ub = (const char *)(A + ((long)i0 * BM + inst * RPI) * SA_I + k0e);
            const unsigned voff = (unsigned)(((lane / CPR) * SA_I + c * CE) * ES);
            __builtin_amdgcn_global_load_lds(AS1(ub + voff), AS3(stage + inst * 1024), 16, 0, 0);
        } else if (inst < DL_INSTR) {
            const int ib = inst - DL_IA;
#if B_KMAJOR
            const int row = ib * RPI + lane / CPR;
            const int c = (lane % CPR) ^ dl_swz(row);
            const char *ub = (const char *)(B + ((long)j0 * BN + ib * RPI) * SB_J + k0e);
            const unsigned voff = (unsigned)(((lane / CPR) * SB_J + c * CE) * ES);
#else
            // lane-linear over the tile's chunks: whole 128-byte lines of consecutive k-rows per instruction
            const int idx = ib * 64 + lane;
            const int k = (BK * CB) % 64 == 0 ? idx / CB : (idx / CB < BK ? idx / CB : BK - 1);
            const int c = (idx % CB) ^ dl_swz_b(k);
            const char *ub = (const char *)(B + k0e * SB_K + (long)j0 * BN);
            const unsigned voff = (unsigned)((k * SB_K + c * CE) * ES);
#endif
            __builtin_amdgcn_global_load_lds(AS1(ub + voff), AS3(stage + DL_A_BYTES + ib * 1024), 16, 0, 0);
        }
    }
}

// load instruction number n (wave-uniform, at run time; n counts as in dl_issue) of this wavefront's share
__device__ __forceinline__ void dl_issue_one(const in_t *__restrict__ A, const in_t *__restrict__ B, char *stage, int i0, int j0, int k0, int wave,
                                             int lane, int n)
{
    const long k0e = (long)k0 * BK;
    const int inst = n * NWAVES + wave; // wave-uniform
    if (inst < DL_IA) {
        const int row = inst * RPI + lane / CPR;
        const int c = (lane % CPR) ^ dl_swz(row);
        const char *ub = (const char *)(A + ((long)i0 * BM + inst * RPI) * SA_I + k0e);
        const unsigned voff = (unsigned)(((lane / CPR) * SA_I + c * CE) * ES);
        __builtin_amdgcn_global_load_lds(AS1(ub + voff), AS3(stage + inst * 1024), 16, 0, 0);
    } else if (DL_INSTR % NWAVES == 0 || inst < DL_INSTR) {
        const int ib = inst - DL_IA;
#if B_KMAJOR
        const int row = ib * RPI + lane / CPR;
        const int c = (lane % CPR) ^ dl_swz(row);
        const char *ub = (const char *)(B + ((long)j0 * BN + ib * RPI) * SB_J + k0e);
        const unsigned voff = (unsigned)(((lane / CPR) * SB_J + c * CE) * ES);
#else
        const int idx = ib * 64 + lane;
        const int k = (BK * CB) % 64 == 0 ? idx / CB : (idx / CB < BK ? idx / CB : BK - 1);
        const int c = (idx % CB) ^ dl_swz_b(k);
        const char *ub = (const char *)(B + k0e * SB_K + (long)j0 * BN);
        const unsigned voff = (unsigned)((k * SB_K + c * CE) * ES);
#endif
        __builtin_amdgcn_global_load_lds(AS1(ub + voff), AS3(stage + DL_A_BYTES + ib * 1024), 16, 0, 0);
    }
}

__device__ __forceinline__ void dl_read_frags(frag_t (&fa)[K3][TM], frag_t (&fb)[K3][TN], const char *__restrict__ stage, int slot, int wi, int wj,
                                              int lane)
{
    const int lrow = lane % MI_M, lgrp = lane / MI_M;
#pragma unroll
    for (int q = 0; q < K3; ++q) {
        const int step = slot * K3 + q;
        const int chunk = step * LANE_GROUPS + lgrp;
#pragma unroll
        for (int r1 = 0; r1 < I1; ++r1)
#pragma unroll
            for (int r3 = 0; r3 < I3; ++r3) {
                const int row = ((r1 * I2 + wi) * I3 + r3) * MI_M + lrow;
                fa[q][r1 * I3 + r3] = *reinterpret_cast<const frag_t *>(stage + row * ROW_BYTES + ((chunk ^ dl_swz(row)) * 16));
            }
#pragma unroll
        for (int c1 = 0; c1 < J1; ++c1)
#pragma unroll
            for (int c3 = 0; c3 < J3; ++c3) {
                const int tcol = (c1 * J2 + wj) * J3 + c3;
#if B_KMAJOR
                const int row = tcol * MI_N + lrow;
                fb[q][c1 * J3 + c3] = *reinterpret_cast<const frag_t *>(stage + DL_A_BYTES + row * ROW_BYTES + ((chunk ^ dl_swz(row)) * 16));
#else
                const int pn = (tcol * MI_N + lrow) / 16; // 16-column granule of this lane's column
                const int li = lane % 16;
                frag_t f;
#if IN_DT != DT_I8 // 2-byte elements
                // 16 lanes hand in 4 k-rows x 16 columns (lane: k-row li/4, 4 columns from li%4); two loads = 8 k
                const int krow = step * MI_K + lgrp * 8 + li / 4;
                const char *b0 = stage + DL_A_BYTES + krow * BROW_BYTES + (((pn << 1) ^ dl_swz_b(krow)) * 16) + (li % 4) * 8;
                const char *b1 = stage + DL_A_BYTES + (krow + 4) * BROW_BYTES + (((pn << 1) ^ dl_swz_b(krow + 4)) * 16) + (li % 4) * 8;
                const tr4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) tr4_t *)(b0));
                const tr4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) tr4_t *)(b1));
                *reinterpret_cast<tr4_t *>(&f.v[0]) = lo;
                *reinterpret_cast<tr4_t *>(&f.v[4]) = hi;
#else
                // 8-bit transpose load (ds_read_b64_tr_b8: inside a group of 16 lanes, lane i receives byte i%8 of
                // lanes i/8, 2 + i/8, ..., 14 + i/8): 16 lanes hand in 8 k-rows x 16 columns (lane: k-row li/2,
                // 8 columns from li%2), every lane gets 8 consecutive k of its own column; two loads = 16 k
                const int krow = step * MI_K + lgrp * 16 + li / 2;
                const char *b0 = stage + DL_A_BYTES + krow * BROW_BYTES + ((pn ^ dl_swz_b(krow)) * 16) + (li % 2) * 8;
                const char *b1 = stage + DL_A_BYTES + (krow + 8) * BROW_BYTES + ((pn ^ dl_swz_b(krow + 8)) * 16) + (li % 2) * 8;
                const tr2_t lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) tr2_t *)(b0));
                const tr2_t hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) tr2_t *)(b1));
                *reinterpret_cast<tr2_t *>(&f.v[0]) = lo;
                *reinterpret_cast<tr2_t *>(&f.v[8]) = hi;
#endif
                fb[q][c1 * J3 + c3] = f;
#endif
            }
    }
}

// wait until at most `n` of this wavefront's vector-memory operations are outstanding
#define DL_WAIT_VM(n) __builtin_amdgcn_s_waitcnt((((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8)))
#endif // CACHE_READ >= 5


constexpr int CROW = BN * (int)sizeof(out_t) + 16; // bytes of one staged output row (cache-write)

// second half of the CACHE_WRITE epilogue: NT threads (t = 0 .. NT-1) write the staged tile as whole rows
template <int NT>
__device__ __forceinline__ void flush_cstage(out_t *__restrict__ C, int i0, int j0, const char *__restrict__ cstage, int t)
{
    constexpr int CHUNKS_PER_ROW = BN * (int)sizeof(out_t) / 16;
    constexpr int TOTAL = BM * CHUNKS_PER_ROW;
    typedef vec_t<unsigned, 4> chunk_t;
#pragma unroll 4
    for (int idx = t; idx < TOTAL; idx += NT) {
        const int row = idx / CHUNKS_PER_ROW, ch = idx % CHUNKS_PER_ROW;
        const chunk_t v = *reinterpret_cast<const chunk_t *>(cstage + row * CROW + ch * 16);
        char *dst = (char *)(C + ((long)i0 * BM + row) * LDC + (long)j0 * BN) + ch * 16;
        *reinterpret_cast<chunk_t *>(dst) = v;
    }
}

// Epilogue of one workgroup tile.  `cstage`: LDS region of BM * CROW bytes for CACHE_WRITE 1 (must not be
// read or written by anything else between the caller's preceding barrier and the end of this call).
__device__ __forceinline__ void write_tile(accv_t (&acc)[TM][TN], out_t *__restrict__ C, const void *__restrict__ bias_, int inst, int i0, int j0,
                                           char *__restrict__ cstage, int tid, int wi, int wj, int lrow, int lgrp)
{
    // epilogue: (+bias, ReLU,) one rounding to the output type.
    // With the operands swapped a lane holds row `lrow` of the tile and, per group g of 4 accumulator
    // elements, the 4 consecutive columns 4*lgrp (16x16) or 8*g + 4*lgrp (32x32) onwards.
    // CACHE_WRITE 0: those 4 values go to global memory as one vector.  CACHE_WRITE 1: the workgroup's
    // tile is first assembled in LDS (the operand buffers are free: the k loop ended with a barrier) and
    // then written as whole rows, 16 bytes per lane, consecutive lanes at consecutive addresses.
#pragma unroll
    for (int r1 = 0; r1 < I1; ++r1)
#pragma unroll
        for (int r3 = 0; r3 < I3; ++r3)
#pragma unroll
            for (int c1 = 0; c1 < J1; ++c1)
#pragma unroll
                for (int c3 = 0; c3 < J3; ++c3) {
                    const int trow = (r1 * I2 + wi) * I3 + r3, tcol = (c1 * J2 + wj) * J3 + c3;
                    const int lr = trow * MI_M + lrow; // row inside the workgroup tile
#pragma unroll
                    for (int g = 0; g < ACC_N / 4; ++g) {
                        const int lc = tcol * MI_N + (MI_M == 16 ? 4 * lgrp : 8 * g + 4 * lgrp); // column inside the tile
                        const long col = (long)j0 * BN + lc;
                        vec_t<out_t, 4> o;
#if HAS_BIAS
                        const vec_t<float, 4> bias = *reinterpret_cast<const vec_t<float, 4> *>((const float *)bias_ + (long)inst * LDC + col);
#endif
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            acc_t x = acc[r1 * I3 + r3][c1 * J3 + c3][4 * g + e];
#if HAS_BIAS
                            x += bias.v[e];
#endif
#if RELU
                            x = x > 0 ? x : 0;
#endif
                            o.v[e] = from_acc(x);
                        }
#if CACHE_WRITE
                        *reinterpret_cast<vec_t<out_t, 4> *>(cstage + lr * CROW + lc * (int)sizeof(out_t)) = o;
#else
                        *reinterpret_cast<vec_t<out_t, 4> *>(C + ((long)i0 * BM + lr) * LDC + col) = o;
#endif
                    }
                }
#if CACHE_WRITE && !CONV_HELPERS
    __syncthreads();
    flush_cstage<NTHREADS>(C, i0, j0, cstage, tid);
#endif
    (void)bias_;
    (void)inst;
    (void)cstage;
    (void)tid;
}

#if REORDER == 3
// --------------------------------------------------------------------------------------
// Persistent workgroups (REORDER 3, direct-to-LDS staging only): the launch has about one workgroup
// per compute unit, and workgroup w multiplies the tiles w, w + gridDim.x, ... of the launch-wide
// tile list (XCD-grouped order as in REORDER 2).  The LDS ring runs across tile boundaries: while
// a tile's result is written out the first k steps of the next tile are already in flight, so there
// is neither a fill bubble per tile nor a new workgroup to start.
struct tile_id {
    int inst, bb, i0, j0;
};

__device__ __forceinline__ tile_id decode_tile(long f, long total)
{
    constexpr int G = I0 * J0;
    if (total % 8 == 0) f = (f % 8) * (total / 8) + f / 8;
    const int wg = (int)(f % G), z = (int)(f / G);
    tile_id t; // wave-uniform, and in scalar registers: the addresses derived from it are scalar arithmetic
    t.inst = __builtin_amdgcn_readfirstlane(z / DIM_B);
    t.bb = __builtin_amdgcn_readfirstlane(z % DIM_B);
    t.i0 = __builtin_amdgcn_readfirstlane(wg / J0);
    t.j0 = __builtin_amdgcn_readfirstlane(wg % J0);
    return t;
}

#if CACHE_READ >= 8
// --------------------------------------------------------------------------------------
// Ping-pong on the ring (CACHE_READ 8, 9 = 2, 3 stages; persistent workgroups, K1 = K2 = 1).
//
// The wavefronts form two groups (wavefront w and w + NWAVES/2 share a SIMD).  A k0 step (one ring stage) is
// K2 slots of K3 MFMA k steps; a slot of a group is two phases: R = read the slot's fragments from LDS into
// registers, M = the slot's MFMAs from registers.
// Group 1 runs one phase behind group 0 and every phase ends with a workgroup barrier, so in every phase one
// wavefront of each SIMD multiplies while the other moves data: matrix cores and the LDS port work at the
// same time by construction, not by the luck of the scheduler.  The loads of step n + STAGES - 1 are issued
// from the phase on in which group 0 reads the first slot of step n (the stage they refill was last read one
// phase earlier, by group 1), by the group that is multiplying.  A tile ends with one more phase per group in which the group writes its results:
// through a staging area of its own per wavefront (CACHE_WRITE 1: whole 128-byte lines, no workgroup
// barrier) or straight from the registers.
#define WAIT_LGKM0() __builtin_amdgcn_s_waitcnt((15 | (3 << 14) | (7 << 4) | (0 << 8)))
#define PHASE_END()                          \
    do {                                     \
        __builtin_amdgcn_sched_barrier(0);   \
        __builtin_amdgcn_s_barrier();        \
        __builtin_amdgcn_sched_barrier(0);   \
    } while (0)

static_assert(K1 == 1, "ping-pong on the ring: a step is K2 slots of K3 MFMA k steps, each slot one read phase and one multiply phase");
static_assert(NWAVES % 2 == 0, "ping-pong on the ring: two groups of wavefronts");

// staging area of one wavefront: MI_M rows of its J3 adjacent tiles, 16-byte chunks XOR-swizzled by the row
constexpr int WS_COLS = J3 * MI_N;
constexpr int WS_ROW = WS_COLS * (int)sizeof(out_t);
constexpr int WS_CH = WS_ROW / 16;
constexpr int WS_SWZ = (WS_CH & (WS_CH - 1)) == 0 ? (WS_CH > 8 ? 7 : WS_CH - 1) : 0;
constexpr int WS_BYTES = CACHE_WRITE ? MI_M * WS_ROW : 0;
static_assert(!CACHE_WRITE || WS_ROW % 16 == 0, "staged output rows are whole 16-byte chunks");

__device__ __forceinline__ void write_tile_wave(accv_t (&acc)[TM][TN], out_t *__restrict__ C, int i0, int j0, char *__restrict__ wstage, int lane,
                                                int wi, int wj, int lrow, int lgrp)
{
#pragma unroll
    for (int r1 = 0; r1 < I1; ++r1)
#pragma unroll
        for (int r3 = 0; r3 < I3; ++r3)
#pragma unroll
            for (int c1 = 0; c1 < J1; ++c1) {
                const int trow = (r1 * I2 + wi) * I3 + r3;
                const int tcol0 = (c1 * J2 + wj) * J3; // first of the J3 adjacent tiles
#pragma unroll
                for (int c3 = 0; c3 < J3; ++c3)
#pragma unroll
                    for (int g = 0; g < ACC_N / 4; ++g) {
                        const int lc = c3 * MI_N + (MI_M == 16 ? 4 * lgrp : 8 * g + 4 * lgrp); // column inside the staged rows
                        vec_t<out_t, 4> o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o.v[e] = from_acc(acc[r1 * I3 + r3][c1 * J3 + c3][4 * g + e]);
#if CACHE_WRITE
                        const int byte = lc * (int)sizeof(out_t);
                        *reinterpret_cast<vec_t<out_t, 4> *>(wstage + lrow * WS_ROW + (((byte / 16) ^ (lrow & WS_SWZ)) * 16) + byte % 16) = o;
#else
                        *reinterpret_cast<vec_t<out_t, 4> *>(C + ((long)i0 * BM + trow * MI_M + lrow) * LDC + (long)j0 * BN + tcol0 * MI_N + lc) = o;
#endif
                    }
#if CACHE_WRITE
                // the same wavefront reads what it wrote (LDS operations of one wavefront execute in order)
                typedef vec_t<unsigned, 4> chunk_t;
#pragma unroll
                for (int idx = lane; idx < MI_M * WS_CH; idx += 64) {
                    const int row = idx / WS_CH, ch = idx % WS_CH;
                    const chunk_t v = *reinterpret_cast<const chunk_t *>(wstage + row * WS_ROW + ((ch ^ (row & WS_SWZ)) * 16));
                    char *dst = (char *)(C + ((long)i0 * BM + trow * MI_M + row) * LDC + (long)j0 * BN + tcol0 * MI_N) + ch * 16;
                    *reinterpret_cast<chunk_t *>(dst) = v;
                }
#endif
            }
}

// The loads of a step are cut into PP_PARTS parts, one per M phase that may carry them, and inside an M phase they
// are spread evenly between the MFMAs.  A load instruction holds the wavefront that issues it until the memory
// pipeline accepts it (about 30 cycles of the compute unit's time per KiB when the unit streams its tiles): issued
// in a row they lengthen the phase by that much, spread out they find the pipeline free and the matrix cores keep
// working on the MFMAs already issued.  With two stages the last slot of a step carries no loads: they would have to
// land within that same phase.
constexpr int PP_NI = (DL_INSTR + NWAVES - 1) / NWAVES;                          // load instructions per wavefront and step
constexpr int PP_PARTS = DL_STAGES == 2 ? (K2 > 1 ? K2 - 1 : 1) : K2;
constexpr int PP_LOADS = (PP_NI + PP_PARTS - 1) / PP_PARTS;                     // load instructions of one part
constexpr int PP_NM = K3 * TM * TN;                                              // MFMAs of one M phase

extern "C" __global__ void __launch_bounds__(NTHREADS)
ms_kernel(const void *__restrict__ a_, const void *__restrict__ b_, const void *__restrict__ bias_, void *__restrict__ c_, int instances)
{
    (void)bias_;
    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int wi = wave / J2, wj = wave % J2;
    const int lrow = lane % MI_M, lgrp = lane / MI_M;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const bool late = wave_u >= NWAVES / 2; // group 1: one phase behind

    constexpr int OPND_BYTES = DL_STAGES * DL_STAGE_BYTES;
    constexpr int LDS_BYTES = OPND_BYTES + NWAVES * WS_BYTES;
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    char *const wstage = lds + OPND_BYTES + wave_u * WS_BYTES;

    const long total = (long)I0 * J0 * DIM_B * instances;
    const long first = blockIdx.x, stride = gridDim.x;
    if (first >= total) return;
    const long my_tiles = (total - first + stride - 1) / stride;
    const long my_steps = my_tiles * K0;

    // load cursor: the step whose loads are being requested = k step lk of tile lt, into stage wr; past the end the
    // last step is requested again (never read), so that every wavefront keeps issuing the same number of loads
    long ls = 0;
    int lk = 0;
    tile_id lt = decode_tile(first, total);
    long lf = first;
    int wr = 0;
    const in_t *cA = (const in_t *)a_ + (long)lt.inst * A_INST + (long)lt.bb * SA_B;
    const in_t *cB = (const in_t *)b_ + (long)lt.inst * B_INST + (long)lt.bb * SB_B;
    auto advance = [&]() {
        wr = wr + 1 == DL_STAGES ? 0 : wr + 1;
        if (ls + 1 < my_steps) {
            ++ls;
            if (++lk == K0) {
                lk = 0;
                lf += stride;
                lt = decode_tile(lf, total);
                cA = (const in_t *)a_ + (long)lt.inst * A_INST + (long)lt.bb * SA_B;
                cB = (const in_t *)b_ + (long)lt.inst * B_INST + (long)lt.bb * SB_B;
            }
        }
    };
#pragma unroll
    for (int t = 0; t < DL_STAGES - 1; ++t) {
        dl_issue(cA, cB, lds + wr * DL_STAGE_BYTES, lt.i0, lt.j0, lk, wave_u, lane);
        advance();
    }

    accv_t acc[TM][TN];
    frag_t fa[K3][TM], fb[K3][TN];
    auto zero_acc = [&]() {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int e = 0; e < ACC_N; ++e) acc[tm][tn][e] = 0;
    };
    zero_acc();
    int rd = 0;
    bool drain = false; // stores of an epilogue are outstanding: the next wait counts them too, so it waits for everything

    // step 0 has landed for everybody
    DL_WAIT_VM((DL_STAGES - 2) * DL_LPW_MIN);
    PHASE_END();
    if (late) {
        // the phase in which group 0 reads slot 0 of step 0: group 1 only requests part 0 of the step at the cursor
#pragma unroll
        for (int n = 0; n < PP_LOADS; ++n)
            if (n < PP_NI) dl_issue_one(cA, cB, lds + wr * DL_STAGE_BYTES, lt.i0, lt.j0, lk, wave_u, lane, n);
        if (PP_PARTS == 1) advance();
        PHASE_END();
    }
#pragma unroll 1
    for (long ti = 0; ti < my_tiles; ++ti) {
        const tile_id ct = decode_tile(first + ti * stride, total);
#pragma unroll 1
        for (int k0 = 0; k0 < K0; ++k0) {
#pragma unroll
            for (int h = 0; h < K2; ++h) { // the K2 slots of a step: K3 MFMA k steps each, one R and one M phase
                // ---- phase R: fragments of this slot -> registers
                dl_read_frags(fa, fb, lds + rd * DL_STAGE_BYTES, h, wi, wj, lane);
                WAIT_LGKM0(); // after its last slot the stage may be refilled from the next phase on
                if (late && h == K2 - 1) {
                    // group 1: its loads of the next step (requested one or more phases ago) have landed
                    if (drain) DL_WAIT_VM(0);
                    else DL_WAIT_VM((DL_STAGES - 2) * DL_LPW_MIN);
                    drain = false;
                }
                PHASE_END();
                // ---- phase M: request this phase's part of the step at the cursor, multiply from registers
                // (group 0 in slot h: part h; group 1 runs one phase behind, its slot h coincides with group 0's
                // reading of slot h + 1: part h + 1, or part 0 of the following step after the last slot)
                const int part = late ? (h + 1) % K2 : h; // wave-uniform
                const bool loading = part < PP_PARTS;
                const int n0 = part * PP_LOADS;
                char *const wstg = lds + wr * DL_STAGE_BYTES;
                __builtin_amdgcn_s_setprio(1);
                {
                    int m = 0; // a constant after unrolling
#pragma unroll
                    for (int q = 0; q < K3; ++q)
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int tn = 0; tn < TN; ++tn) {
                                acc[tm][tn] = mfma(fb[q][tn], fa[q][tm], acc[tm][tn]);
                                ++m;
                                // after m of the NM MFMAs, floor(m * (LOADS + 1) / NM) of the phase's loads are out (all of
                                // them before the last MFMA): evenly spread, several per gap when there are more loads than MFMAs
                                const int due = (m * (PP_LOADS + 1)) / PP_NM, was = ((m - 1) * (PP_LOADS + 1)) / PP_NM;
#pragma unroll
                                for (int l = was; l < due; ++l)
                                    if (l < PP_LOADS && loading && n0 + l < PP_NI) dl_issue_one(cA, cB, wstg, lt.i0, lt.j0, lk, wave_u, lane, n0 + l);
                            }
                }
                if (loading && part == PP_PARTS - 1) advance();
                __builtin_amdgcn_s_setprio(0);
                if (!late && h == K2 - 1) {
                    if (drain) DL_WAIT_VM(0);
                    else DL_WAIT_VM((DL_STAGES - 2) * DL_LPW_MIN);
                    drain = false;
                }
                PHASE_END();
            }
            rd = rd + 1 == DL_STAGES ? 0 : rd + 1;
        }
        // ---- phase E: results of the tile (the other group multiplies its last slot, or reads its first)
        out_t *C = (out_t *)c_ + ((long)ct.inst * DIM_B + ct.bb) * ((long)DIM_M * DIM_N);
        write_tile_wave(acc, C, ct.i0, ct.j0, wstage, lane, wi, wj, lrow, lgrp);
        zero_acc();
        drain = true;
        PHASE_END();
    }
    if (!late) PHASE_END(); // group 1's last phase
    DL_WAIT_VM(0);          // the re-loads past the end must land before the workgroup's LDS is released
}
#else
extern "C" __global__ void __launch_bounds__(NTHREADS)
ms_kernel(const void *__restrict__ a_, const void *__restrict__ b_, const void *__restrict__ bias_, void *__restrict__ c_, int instances)
{
    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int wi = wave / J2, wj = wave % J2;
    const int lrow = lane % MI_M, lgrp = lane / MI_M;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);

    constexpr int OPND_BYTES = DL_STAGES * DL_STAGE_BYTES;
    constexpr int LDS_BYTES = OPND_BYTES + (CACHE_WRITE ? BM * CROW : 0); // the output staging area sits behind the ring
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];

    const long total = (long)I0 * J0 * DIM_B * instances;
    const long first = blockIdx.x, stride = gridDim.x;
    if (first >= total) return;
    const long my_tiles = (total - first + stride - 1) / stride;
    const long my_steps = my_tiles * K0;

    // load cursor: step `ls` of this workgroup's step list = k step lk of tile lt
    long ls = 0;
    int lk = 0;
    tile_id lt = decode_tile(first, total);
    long lf = first;
    int wr = 0;
    auto issue_next = [&]() {
        // past the end the last step is loaded again (never read): every wavefront keeps issuing the same number of loads
        const in_t *A = (const in_t *)a_ + (long)lt.inst * A_INST + (long)lt.bb * SA_B;
        const in_t *B = (const in_t *)b_ + (long)lt.inst * B_INST + (long)lt.bb * SB_B;
        dl_issue(A, B, lds + wr * DL_STAGE_BYTES, lt.i0, lt.j0, lk, wave_u, lane);
        wr = wr + 1 == DL_STAGES ? 0 : wr + 1;
        if (ls + 1 < my_steps) {
            ++ls;
            if (++lk == K0) {
                lk = 0;
                lf += stride;
                lt = decode_tile(lf, total);
            }
        }
    };
#pragma unroll
    for (int t = 0; t < DL_STAGES - 1; ++t) issue_next();

    int rd = 0;
#pragma unroll 1
    for (long ti = 0; ti < my_tiles; ++ti) {
        const tile_id ct = decode_tile(first + ti * stride, total);
        accv_t acc[TM][TN];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int e = 0; e < ACC_N; ++e) acc[tm][tn][e] = 0;
#pragma unroll 1
        for (int k0 = 0; k0 < K0; ++k0) {
            // right after an epilogue the counter also holds that tile's stores, which need not retire in
            // order with the loads: drain it once, then count loads again
            if (k0 == 0 && ti > 0) DL_WAIT_VM(0);
            else DL_WAIT_VM((DL_STAGES - 2) * DL_LPW_MIN);
            __builtin_amdgcn_s_barrier();
            issue_next();
            const char *stage = lds + rd * DL_STAGE_BYTES;
#if UNROLL_K1 == K1 && UNROLL_K2 == K2 && K1 * K2 > 1
            {
                frag_t fa[2][K3][TM], fb[2][K3][TN];
                dl_read_frags(fa[0], fb[0], stage, 0, wi, wj, lane);
#pragma unroll
                for (int sl = 0; sl < K1 * K2; ++sl) {
                    if (sl + 1 < K1 * K2) dl_read_frags(fa[(sl + 1) & 1], fb[(sl + 1) & 1], stage, sl + 1, wi, wj, lane);
                    mfma_slot(acc, fa[sl & 1], fb[sl & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#else
#pragma unroll UNROLL_K1
            for (int k1 = 0; k1 < K1; ++k1) {
#pragma unroll UNROLL_K2
                for (int k2 = 0; k2 < K2; ++k2) {
                    frag_t fa[K3][TM], fb[K3][TN];
                    dl_read_frags(fa, fb, stage, k1 * K2 + k2, wi, wj, lane);
                    mfma_slot(acc, fa, fb);
                }
            }
#endif
            rd = rd + 1 == DL_STAGES ? 0 : rd + 1;
        }
        out_t *C = (out_t *)c_ + ((long)ct.inst * DIM_B + ct.bb) * ((long)DIM_M * DIM_N);
#if CACHE_WRITE
        // the staging area was last read by the previous tile's row stores, K0 barriers ago
        write_tile(acc, C, bias_, ct.inst, ct.i0, ct.j0, lds + OPND_BYTES, tid, wi, wj, lrow, lgrp);
#else
        write_tile(acc, C, bias_, ct.inst, ct.i0, ct.j0, lds, tid, wi, wj, lrow, lgrp);
#endif
    }
    DL_WAIT_VM(0); // the re-loads past the end must land before the workgroup's LDS is released
}
#endif // CACHE_READ >= 8
#elif CONV_RESIDENT
// --------------------------------------------------------------------------------------
// conv2d, COMPUTE_AT 2: persistent workgroups, resident weights, input patch per tile.
// Tile list of the launch: index f = ((inst * DIM_B + group) * J0 + j0) * I0 + i0; workgroup w owns the run
// [w * run, (w + 1) * run): consecutive tiles share their weights and neighbouring patches.
extern "C" __global__ void __launch_bounds__(NTHREADS)
ms_kernel(const void *__restrict__ a_, const void *__restrict__ b_, const void *__restrict__ bias_, void *__restrict__ c_, int instances)
{
    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int wi = wave / J2, wj = wave % J2;
    const int lrow = lane % MI_M, lgrp = lane / MI_M;

    // all k steps of the weights in fragment layout; with the weights in registers, one step as a staging buffer
    constexpr int W_BYTES = (CONV_BREG ? 1 : K0) * STAGE_BYTES;
    constexpr int LDS_BYTES = W_BYTES + PATCH_BYTES + (CACHE_WRITE ? BM * CROW : 0);
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    char *const patch = lds + W_BYTES;
    char *const cstage = lds + W_BYTES + PATCH_BYTES;

    const long total = (long)I0 * J0 * DIM_B * instances;
    // z = f / (I0 * J0) = instance * DIM_B + group: where that entry's image, weights, bias slice and output start
    auto x_of = [&](long z) { return (const in_t *)a_ + (z / DIM_B) * A_INST + (z % DIM_B) * SA_B; };
    auto w_of = [&](long z) { return (const in_t *)b_ + (z / DIM_B) * B_INST + (z % DIM_B) * SB_B; };
    auto c_of = [&](long z) { return (out_t *)c_ + (z / DIM_B) * ((long)DIM_B * DIM_M * DIM_N) + (z % DIM_B) * C_BATCH; };
#if HAS_BIAS
    auto bias_of = [&](long z) { return (const void *)((const float *)bias_ + (z % DIM_B) * DIM_N); };
#else
    auto bias_of = [&](long) { return bias_; };
#endif
    const long run = (total + gridDim.x - 1) / gridDim.x;
    const long first = (long)blockIdx.x * run;
    const long last = first + run < total ? first + run : total;
    if (first >= last) return;

#if CONV_HELPERS
    static_assert(CACHE_WRITE == 1, "helper wavefronts write the tile from its LDS staging area");
    // wave-uniform role: matrix-core wavefronts 0 .. NWAVES-1, then the helpers
    const bool helper = __builtin_amdgcn_readfirstlane(wave) >= NWAVES;
    const int htid = tid - NWAVES * 64;
    patch_map pm;
    patch_regs pr;
    if (helper) {
        patch_map_init(pm, htid);
        patch_fetch(pr, pm, x_of(first / (I0 * J0)), (int)(first % I0));
        patch_commit(pr, pm, patch, htid);
    }
    long have_w = -1;
#pragma unroll 1
    for (long f = first; f < last; ++f) {
        const int i0 = (int)(f % I0), j0 = (int)((f / I0) % J0);
        const long z = f / (I0 * J0);
        if (f / I0 != have_w) {
            // all wavefronts load the weights; the previous tile's k loop ended with barrier B
            have_w = f / I0;
            const in_t *Wt = w_of(z);
            tile_stage st;
#pragma unroll 1
            for (int k0 = 0; k0 < K0; ++k0) {
                stage_load(st, nullptr, Wt, 0, j0, k0, tid);
                stage_store(st, lds + k0 * STAGE_BYTES, tid);
            }
        }
        __syncthreads(); // barrier A: patch f, weights and the staged result of tile f-1 are in place
        if (helper) {
            // loads before stores: the wait for the patch then does not include the younger stores
            if (f + 1 < last) {
                const long g = f + 1;
                patch_fetch(pr, pm, x_of(g / (I0 * J0)), (int)(g % I0));
            }
            if (f > first) {
                const long g = f - 1;
                out_t *Cp = c_of(g / (I0 * J0));
                flush_cstage<P_NT>(Cp, (int)(g % I0), (int)((g / I0) % J0), cstage, htid);
            }
            __syncthreads(); // barrier B: the matrix-core wavefronts are done with patch f, the helpers with the staging area
            if (f + 1 < last) patch_commit(pr, pm, patch, htid);
        } else {
            conv_ctx cx;
            conv_ctx_init(cx, patch, i0, wi, lrow, lgrp);
            accv_t acc[TM][TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int e = 0; e < ACC_N; ++e) acc[tm][tn][e] = 0;
#pragma unroll 1
            for (int k0 = 0; k0 < K0; ++k0) {
#if UNROLL_K1 == K1 && UNROLL_K2 == K2 && K1 * K2 > 1
                multiply_tile_unrolled(acc, lds + k0 * STAGE_BYTES, lgrp, wi, wj, lrow, cx, k0);
#else
                multiply_tile(acc, lds + k0 * STAGE_BYTES, lgrp, wi, wj, lrow, cx, k0);
#endif
            }
            __syncthreads(); // barrier B
            write_tile(acc, nullptr, bias_of(z), (int)(z / DIM_B), i0, j0, cstage, tid, wi, wj, lrow, lgrp); // accumulators -> staging area only
        }
    }
    __syncthreads();
    if (helper) {
        const long g = last - 1;
        out_t *Cp = c_of(g / (I0 * J0));
        flush_cstage<P_NT>(Cp, (int)(g % I0), (int)((g / I0) % J0), cstage, htid);
    }
}
#else
    patch_map pm;
    patch_regs pr;
    patch_map_init(pm, tid);
    {
        patch_fetch(pr, pm, x_of(first / (I0 * J0)), (int)(first % I0));
        patch_commit(pr, pm, patch, tid);
    }
    long have_w = -1; // (inst, j0) of the weights in LDS (or registers)
#if CONV_BREG
    frag_t bw[NSTEP][TN];
#endif
#pragma unroll 1
    for (long f = first; f < last; ++f) {
        const int i0 = (int)(f % I0), j0 = (int)((f / I0) % J0);
        const long z = f / (I0 * J0);
        if (f / I0 != have_w) {
            // every wavefront has passed the barrier that ended the previous tile's k loop: the old weights are dead
            have_w = f / I0;
            const in_t *Wt = w_of(z);
#if CONV_BREG
            weights_to_regs(bw, Wt, j0, lds, tid, lgrp, wj, lrow);
#else
            tile_stage st;
#pragma unroll 1
            for (int k0 = 0; k0 < K0; ++k0) {
                stage_load(st, nullptr, Wt, 0, j0, k0, tid);
                stage_store(st, lds + k0 * STAGE_BYTES, tid);
            }
#endif
        }
        __syncthreads(); // patch and weights are in place
#if CACHE_READ >= 2
        if (f + 1 < last) {
            const long g = f + 1;
            patch_fetch(pr, pm, x_of(g / (I0 * J0)), (int)(g % I0));
        }
#endif
        conv_ctx cx;
        conv_ctx_init(cx, patch, i0, wi, lrow, lgrp);
        accv_t acc[TM][TN];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int e = 0; e < ACC_N; ++e) acc[tm][tn][e] = 0;
#if CONV_BREG
        multiply_all_k(acc, bw, cx);
#else
#pragma unroll 1
        for (int k0 = 0; k0 < K0; ++k0) {
#if UNROLL_K1 == K1 && UNROLL_K2 == K2 && K1 * K2 > 1
            multiply_tile_unrolled(acc, lds + k0 * STAGE_BYTES, lgrp, wi, wj, lrow, cx, k0);
#else
            multiply_tile(acc, lds + k0 * STAGE_BYTES, lgrp, wi, wj, lrow, cx, k0);
#endif
        }
#endif
        __syncthreads(); // the patch has been read by everyone
        if (f + 1 < last) {
#if CACHE_READ < 2
            const long g = f + 1;
            patch_fetch(pr, pm, x_of(g / (I0 * J0)), (int)(g % I0));
#endif
            patch_commit(pr, pm, patch, tid);
        }
        write_tile(acc, c_of(z), bias_of(z), (int)(z / DIM_B), i0, j0, cstage, tid, wi, wj, lrow, lgrp);
    }
}
#endif // CONV_HELPERS
#else // REORDER != 3
constexpr int K0L = K0 / RFACTOR; // k0 steps of one workgroup
static_assert(K0 % RFACTOR == 0, "rfactor divides the k0 loop");
static_assert(RFACTOR == 1 || (!CACHE_WRITE && !CONV_RESIDENT), "rfactor: partial sums leave straight from the accumulators");

#if RFACTOR > 1
// partial sums of run ks: accumulator values, no epilogue, to ws[ks][z][row][col]
__device__ __forceinline__ void write_partial(accv_t (&acc)[TM][TN], acc_t *__restrict__ W, int i0, int j0, int wi, int wj, int lrow, int lgrp)
{
#pragma unroll
    for (int r1 = 0; r1 < I1; ++r1)
#pragma unroll
        for (int r3 = 0; r3 < I3; ++r3)
#pragma unroll
            for (int c1 = 0; c1 < J1; ++c1)
#pragma unroll
                for (int c3 = 0; c3 < J3; ++c3) {
                    const int trow = (r1 * I2 + wi) * I3 + r3, tcol = (c1 * J2 + wj) * J3 + c3;
                    const long row = (long)i0 * BM + trow * MI_M + lrow;
#pragma unroll
                    for (int g = 0; g < ACC_N / 4; ++g) {
                        const long col = (long)j0 * BN + tcol * MI_N + (MI_M == 16 ? 4 * lgrp : 8 * g + 4 * lgrp);
                        vec_t<acc_t, 4> o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o.v[e] = acc[r1 * I3 + r3][c1 * J3 + c3][4 * g + e];
                        *reinterpret_cast<vec_t<acc_t, 4> *>(W + row * DIM_N + col) = o;
                    }
                }
}

// Second kernel of an rfactor launch: one thread per 4 consecutive output columns adds the RFACTOR partial
// results in run order (a fixed order: the result is reproducible), then bias, ReLU and the single rounding.
extern "C" __global__ void __launch_bounds__(256)
ms_rfactor_reduce(const void *__restrict__ ws_, const void *__restrict__ bias_, void *__restrict__ c_, int instances)
{
    const long nz = (long)instances * DIM_B;
    const long quads = nz * DIM_M * (DIM_N / 4);
    const long q = (long)blockIdx.x * 256 + threadIdx.x;
    if (q >= quads) return;
    const int col = (int)(q % (DIM_N / 4)) * 4;
    const long zr = q / (DIM_N / 4);
    const int row = (int)(zr % DIM_M);
    const long z = zr / DIM_M;
    const int inst = (int)(z / DIM_B), bb = (int)(z % DIM_B);
    const acc_t *W = (const acc_t *)ws_ + (z * DIM_M + row) * DIM_N + col;
    vec_t<acc_t, 4> sum = *reinterpret_cast<const vec_t<acc_t, 4> *>(W);
#pragma unroll
    for (int ks = 1; ks < RFACTOR; ++ks) {
        const vec_t<acc_t, 4> part = *reinterpret_cast<const vec_t<acc_t, 4> *>(W + (long)ks * nz * DIM_M * DIM_N);
#pragma unroll
        for (int e = 0; e < 4; ++e) sum.v[e] += part.v[e];
    }
#if HAS_BIAS
    const vec_t<float, 4> bias = *reinterpret_cast<const vec_t<float, 4> *>((const float *)bias_ + (long)inst * LDC + (long)bb * DIM_N + col);
#endif
    vec_t<out_t, 4> o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        acc_t x = sum.v[e];
#if HAS_BIAS
        x += bias.v[e];
#endif
#if RELU
        x = x > 0 ? x : 0;
#endif
        o.v[e] = from_acc(x);
    }
    out_t *C = (out_t *)c_ + (long)inst * ((long)DIM_B * DIM_M * DIM_N) + (long)bb * C_BATCH;
    *reinterpret_cast<vec_t<out_t, 4> *>(C + (long)row * LDC + col) = o;
    (void)bias_;
}
#endif

extern "C" __global__ void __launch_bounds__(NTHREADS)
ms_kernel(const void *__restrict__ a_, const void *__restrict__ b_, const void *__restrict__ bias_, void *__restrict__ c_, int instances,
          void *__restrict__ ws_)
{
    int z, i0, j0, ks;
    block_to_tile(z, i0, j0, ks);
    const int inst = z / DIM_B, bb = z % DIM_B;
    if (inst >= instances) return;
    const int KB = ks * K0L, KE = KB + K0L; // this workgroup's run of k0 steps
    (void)ws_;
    const in_t *__restrict__ A = (const in_t *)a_ + (long)inst * A_INST + (long)bb * SA_B;
    const in_t *__restrict__ B = (const in_t *)b_ + (long)inst * B_INST + (long)bb * SB_B;
    out_t *__restrict__ C = (out_t *)c_ + (long)inst * ((long)DIM_B * DIM_M * DIM_N) + (long)bb * C_BATCH;
#if IS_CONV && HAS_BIAS
    bias_ = (const float *)bias_ + (long)bb * DIM_N; // the group's slice of the bias
#endif

    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int wi = wave / J2, wj = wave % J2;
    const int lrow = lane % MI_M, lgrp = lane / MI_M;

#if CACHE_READ >= 5
    constexpr int OPND_BYTES = DL_STAGES * DL_STAGE_BYTES;
#else
    constexpr int OPND_BYTES = STAGES * STAGE_BYTES;
#endif
#if CONV_PATCH
    constexpr int RES_BYTES = OPND_BYTES + PATCH_BYTES; // weight stages, then the resident input patch
#else
    constexpr int RES_BYTES = OPND_BYTES;
#endif
    constexpr int LDS_BYTES = (CACHE_WRITE && BM * CROW > RES_BYTES) ? BM * CROW : RES_BYTES;
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];

    conv_ctx cx;
#if CONV_PATCH
    // every staging mode below passes a barrier between its first LDS writes and its first fragment reads
    {
        patch_map pm;
        patch_regs pr;
        patch_map_init(pm, tid);
        patch_fetch(pr, pm, A, i0);
        patch_commit(pr, pm, lds + OPND_BYTES, tid);
    }
    conv_ctx_init(cx, lds + OPND_BYTES, i0, wi, lrow, lgrp);
#endif

    accv_t acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int e = 0; e < ACC_N; ++e) acc[tm][tn][e] = 0;

#if CACHE_READ >= 5
    {
        const int wave_u = __builtin_amdgcn_readfirstlane(wave); // scalar register: load addresses and LDS targets become wave-uniform
        // prologue: DL_STAGES - 1 tiles in flight
#pragma unroll
        for (int t = 0; t < DL_STAGES - 1; ++t) dl_issue(A, B, lds + t * DL_STAGE_BYTES, i0, j0, KB + t < KE ? KB + t : KE - 1, wave_u, lane);
        int rd = 0, wr = DL_STAGES - 1; // stage multiplied in this step / stage refilled in this step
#pragma unroll 1
        for (int k0 = KB; k0 < KE; ++k0) {
            // this wavefront's loads of tile k0 have landed once at most the loads of the DL_STAGES - 2
            // younger tiles are outstanding; the barrier then covers every wavefront's share, and also
            // tells that all of them are done reading the stage that is refilled next
            DL_WAIT_VM((DL_STAGES - 2) * DL_LPW_MIN);
            __builtin_amdgcn_s_barrier();
            dl_issue(A, B, lds + wr * DL_STAGE_BYTES, i0, j0, k0 + DL_STAGES - 1 < KE ? k0 + DL_STAGES - 1 : KE - 1, wave_u, lane);
            const char *stage = lds + rd * DL_STAGE_BYTES;
#if UNROLL_K1 == K1 && UNROLL_K2 == K2 && K1 * K2 > 1
            {
                frag_t fa[2][K3][TM], fb[2][K3][TN];
                dl_read_frags(fa[0], fb[0], stage, 0, wi, wj, lane);
#pragma unroll
                for (int sl = 0; sl < K1 * K2; ++sl) {
                    if (sl + 1 < K1 * K2) dl_read_frags(fa[(sl + 1) & 1], fb[(sl + 1) & 1], stage, sl + 1, wi, wj, lane);
                    mfma_slot(acc, fa[sl & 1], fb[sl & 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#else
#pragma unroll UNROLL_K1
            for (int k1 = 0; k1 < K1; ++k1) {
#pragma unroll UNROLL_K2
                for (int k2 = 0; k2 < K2; ++k2) {
                    frag_t fa[K3][TM], fb[K3][TN];
                    dl_read_frags(fa, fb, stage, k1 * K2 + k2, wi, wj, lane);
                    mfma_slot(acc, fa, fb);
                }
            }
#endif
            rd = rd + 1 == DL_STAGES ? 0 : rd + 1;
            wr = wr + 1 == DL_STAGES ? 0 : wr + 1;
        }
        // the clamped re-loads of the last steps are still in flight and the epilogue may reuse LDS
        DL_WAIT_VM(0);
        __syncthreads();
    }
#elif CACHE_READ == 3
    // Two LDS buffers and two register sets: the tile of step k+2 is requested while step k is
    // multiplied, so a global load has two whole steps to arrive.  The k0 loop advances by two
    // steps per iteration so that each register set has a fixed name; tile indices beyond the
    // last are clamped (a harmless re-load) instead of branching.
    {
        tile_stage st0, st1;
        stage_load(st0, A, B, i0, j0, KB, tid);
        stage_load(st1, A, B, i0, j0, K0L > 1 ? KB + 1 : KB, tid);
        stage_store(st0, lds, tid);
        __syncthreads();
#pragma unroll 1
        for (int k0 = KB; k0 < KE; k0 += 2) {
#if UNROLL_K1 == K1 && UNROLL_K2 == K2
            pipelined_step(acc, lds, lds + STAGE_BYTES, st1, st0, A, B, i0, j0, k0 + 2 < KE ? k0 + 2 : KE - 1, tid, lgrp, wi, wj, lrow, cx, k0);
            __syncthreads();
            if (k0 + 1 < KE) {
                pipelined_step(acc, lds + STAGE_BYTES, lds, st0, st1, A, B, i0, j0, k0 + 3 < KE ? k0 + 3 : KE - 1, tid, lgrp, wi, wj, lrow, cx, k0 + 1);
                __syncthreads();
            }
#else
            stage_load(st0, A, B, i0, j0, k0 + 2 < KE ? k0 + 2 : KE - 1, tid);
            multiply_tile(acc, lds, lgrp, wi, wj, lrow, cx, k0);
            stage_store(st1, lds + STAGE_BYTES, tid);
            __syncthreads();
            if (k0 + 1 < KE) {
                stage_load(st1, A, B, i0, j0, k0 + 3 < KE ? k0 + 3 : KE - 1, tid);
                multiply_tile(acc, lds + STAGE_BYTES, lgrp, wi, wj, lrow, cx, k0 + 1);
                stage_store(st0, lds, tid);
                __syncthreads();
            }
#endif
        }
    }
#elif CACHE_READ == 4
    // Ping-pong: the wavefronts form two groups that run the same code half a step apart.  A step is
    // a memory phase (LDS reads of all fragments of the current tile, LDS writes of the next tile,
    // global loads of the tile after it), a barrier, an MFMA phase, a barrier.  The second group
    // passes one extra barrier before the loop, so while one group multiplies the other moves data;
    // the first group passes the matching extra barrier after the loop.  (K1 = K2 = 1: a tile's
    // fragments are all in registers when its MFMA phase starts.)
    {
        tile_stage st;
        const bool late = wave >= NWAVES / 2;
        stage_load(st, A, B, i0, j0, KB, tid);
        stage_store(st, lds, tid);
        stage_load(st, A, B, i0, j0, K0L > 1 ? KB + 1 : KB, tid);
        __syncthreads();
        if (late) __builtin_amdgcn_s_barrier();
        int stage = 0;
#pragma unroll 1
        for (int k0 = KB; k0 < KE; ++k0) {
            frag_t fa[K3][TM], fb[K3][TN];
            const char *base = lds + stage * STAGE_BYTES;
            read_frags(fa, fb, base + lgrp * PLANE_A, base + A_STAGE_BYTES + lgrp * B_LGRP, 0, wi, wj, lrow, cx, k0);
            stage_store(st, lds + (stage ^ 1) * STAGE_BYTES, tid);
            stage_load(st, A, B, i0, j0, k0 + 2 < KE ? k0 + 2 : KE - 1, tid);
            __syncthreads();
            __builtin_amdgcn_s_setprio(1);
            mfma_slot(acc, fa, fb);
            __builtin_amdgcn_s_setprio(0);
            __syncthreads();
            stage ^= 1;
        }
        if (!late) __builtin_amdgcn_s_barrier();
    }
#else
    tile_stage st;
    int stage = 0;
#if CACHE_READ == 2
    stage_load(st, A, B, i0, j0, KB, tid);
    stage_store(st, lds, tid);
    __syncthreads();
#endif

#pragma unroll 1
    for (int k0 = KB; k0 < KE; ++k0) {
#if CACHE_READ == 1
        stage_load(st, A, B, i0, j0, k0, tid);
        stage_store(st, lds, tid);
        __syncthreads();
#endif
        const char *la = lds + stage * STAGE_BYTES + lgrp * PLANE_A;
        const char *lb = lds + stage * STAGE_BYTES + A_STAGE_BYTES + lgrp * B_LGRP;
#if PIPELINED
        // k1, k2 fully unrolled: software pipeline over the NS = K1*K2 slots of this tile.  Slot s
        // first issues the LDS reads of slot s+1 and its share of the next tile's global loads, then
        // its own MFMAs; nothing is moved across a slot boundary.
        {
            frag_t fa[2][K3][TM], fb[2][K3][TN];
            read_frags(fa[0], fb[0], la, lb, 0, wi, wj, lrow, cx, k0);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                if (s + 1 < NS) read_frags(fa[(s + 1) & 1], fb[(s + 1) & 1], la, lb, s + 1, wi, wj, lrow, cx, k0);
#if CACHE_READ == 2
                // the last step fetches its own tile again instead of branching: the loop body stays one block
                stage_load(st, A, B, i0, j0, k0 + 1 < KE ? k0 + 1 : k0, tid, s * tile_stage::UNITS / NS, (s + 1) * tile_stage::UNITS / NS);
#endif
                mfma_slot(acc, fa[s & 1], fb[s & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#else
#if CACHE_READ == 2
        if (k0 + 1 < KE) stage_load(st, A, B, i0, j0, k0 + 1, tid);
#endif
#pragma unroll UNROLL_K1
        for (int k1 = 0; k1 < K1; ++k1) {
#pragma unroll UNROLL_K2
            for (int k2 = 0; k2 < K2; ++k2) {
                frag_t fa[K3][TM], fb[K3][TN];
                read_frags(fa, fb, la, lb, k1 * K2 + k2, wi, wj, lrow, cx, k0);
                mfma_slot(acc, fa, fb);
            }
        }
#endif
#if CACHE_READ == 1
        __syncthreads();
#else
#if PIPELINED
        // unconditional (the last step re-stores its own tile into the idle buffer): a conditional store
        // would let the compiler sink the prefetch loads down here, behind the MFMAs
        stage_store(st, lds + (stage ^ 1) * STAGE_BYTES, tid);
#else
        if (k0 + 1 < KE) stage_store(st, lds + (stage ^ 1) * STAGE_BYTES, tid);
#endif
        __syncthreads();
        stage ^= 1;
#endif
    }

#endif // CACHE_READ != 3

#if RFACTOR > 1
    write_partial(acc, (acc_t *)ws_ + (((long)ks * instances * DIM_B + z) * DIM_M) * DIM_N, i0, j0, wi, wj, lrow, lgrp);
    (void)C;
    (void)tid;
#else
    write_tile(acc, C, bias_, inst, i0, j0, lds, tid, wi, wj, lrow, lgrp);
#endif
}
#endif // REORDER != 3
