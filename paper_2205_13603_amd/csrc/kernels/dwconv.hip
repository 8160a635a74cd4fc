// Depthwise conv2d, NHWC, fp32, on the vector ALUs: a bandwidth-bound kernel,
// one per decision trace.
//
// Schedule (Table 2 primitives of arXiv 2205.13603):
//   split   oh -> I0..I3, ow -> J0..J3, c -> C0..C3 (index ((x0*F1+x1)*F2+x2)*F3+x3)
//   reorder i0 j0 c0 | i2 j2 c2 | i1 j1 c1 | i3 j3 | kh kw | c3
//   bind    fuse(i0,j0,c0) -> blockIdx.x (c fastest), fuse(i2,j2,c2) -> threadIdx.x (c fastest:
//           neighbouring lanes touch neighbouring channels of one pixel = coalesced)
//   reorder (REORDER 2): workgroup order grouped per XCD
//   vectorize c3 (4 or 2 channels per load/store when 4 or 2 divides C3)
//   cache-read (CACHE_READ 1): the workgroup's input halo tile is staged in LDS, zero padded
//   unroll  the kh,kw tap loops (UNROLL_K1 == 0: fully, with the I3 x J3 output patch sharing one
//           register copy of its input patch; 1: rolled, every tap re-reads its input)
#include "common.h"

constexpr int BOH = I1 * I2 * I3;
constexpr int BOW = J1 * J2 * J3;
constexpr int BC = C1 * C2 * C3;
constexpr int VC = C3 % 4 == 0 ? 4 : (C3 % 2 == 0 ? 2 : 1); // channels per memory instruction
constexpr int NV = C3 / VC;
constexpr int TIH = (BOH - 1) * CV_STRIDE + CV_KH;  // input halo tile of a workgroup
constexpr int TIW = (BOW - 1) * CV_STRIDE + CV_KW;
constexpr int PH = (I3 - 1) * CV_STRIDE + CV_KH;    // input patch of one I3 x J3 output patch
constexpr int PW = (J3 - 1) * CV_STRIDE + CV_KW;

typedef vec_t<float, VC> cv_t;

__device__ __forceinline__ cv_t zero_cv()
{
    cv_t z;
#pragma unroll
    for (int q = 0; q < VC; ++q) z.v[q] = 0.f;
    return z;
}

// input pixel (ih, iw), channels [c, c+VC): zero outside the image
__device__ __forceinline__ cv_t load_x(const float *__restrict__ X, int ih, int iw, int c)
{
    if (ih >= 0 && ih < CV_H && iw >= 0 && iw < CV_W) return *reinterpret_cast<const cv_t *>(X + ((long)ih * CV_W + iw) * CV_C + c);
    return zero_cv();
}

extern "C" __global__ void __launch_bounds__(NTHREADS)
ms_kernel(const void *__restrict__ x_, const void *__restrict__ w_, const void *__restrict__ unused_, void *__restrict__ y_, int instances)
{
    (void)unused_;
    int z = blockIdx.z * gridDim.y + blockIdx.y; // instance * N + n
    int wg = blockIdx.x;
#if REORDER == 2
    // undo the round-robin of workgroups over the 8 XCDs (workgroup f of the launch goes to XCD f mod 8):
    // neighbouring tiles, which share halo rows and columns, then sit behind the same L2
    {
        constexpr int G = I0 * J0 * C0;
        const long total = (long)G * gridDim.y * gridDim.z;
        if (total % 8 == 0) {
            const long f = wg + (long)G * z;
            const long g = (f % 8) * (total / 8) + f / 8;
            wg = (int)(g % G);
            z = (int)(g / G);
        }
    }
#endif
    if (z >= instances * CV_N) return;
    const float *__restrict__ X = (const float *)x_ + (long)z * CV_H * CV_W * CV_C;
    const float *__restrict__ Wt = (const float *)w_ + (long)(z / CV_N) * CV_KH * CV_KW * CV_C;
    float *__restrict__ Y = (float *)y_ + (long)z * CV_OH * CV_OW * CV_C;

    const int c0 = wg % C0, j0 = (wg / C0) % J0, i0 = wg / (C0 * J0);
    const int tid = threadIdx.x;
    const int tc = tid % C2, tj = (tid / C2) % J2, ti = tid / (C2 * J2);

#if CACHE_READ
    __shared__ __attribute__((aligned(16))) float tile[TIH * TIW * BC];
    {
        const int ih0 = i0 * BOH * CV_STRIDE - CV_PAD, iw0 = j0 * BOW * CV_STRIDE - CV_PAD;
        constexpr int CV_PER_PIX = BC / VC;
        constexpr int TOTAL = TIH * TIW * CV_PER_PIX;
        for (int idx = tid; idx < TOTAL; idx += NTHREADS) {
            const int cv = idx % CV_PER_PIX, pix = idx / CV_PER_PIX;
            const int pw = pix % TIW, ph = pix / TIW;
            // channels of the tile are stored in block order: local channel lc <-> global c0*BC + lc
            *reinterpret_cast<cv_t *>(&tile[(ph * TIW + pw) * BC + cv * VC]) = load_x(X, ih0 + ph, iw0 + pw, c0 * BC + cv * VC);
        }
    }
    __syncthreads();
#endif

#pragma unroll 1
    for (int r1 = 0; r1 < I1; ++r1)
#pragma unroll 1
        for (int q1 = 0; q1 < J1; ++q1)
#pragma unroll 1
            for (int s1 = 0; s1 < C1; ++s1) {
                const int ohl = (r1 * I2 + ti) * I3, owl = (q1 * J2 + tj) * J3, cl = (s1 * C2 + tc) * C3; // block-local
                const int oh = i0 * BOH + ohl, ow = j0 * BOW + owl, c = c0 * BC + cl;
#pragma unroll 1
                for (int v = 0; v < NV; ++v) {
                    const int cc = c + v * VC, ccl = cl + v * VC;
                    (void)ccl;
                    cv_t acc[I3][J3];
#pragma unroll
                    for (int a = 0; a < I3; ++a)
#pragma unroll
                        for (int b = 0; b < J3; ++b) acc[a][b] = zero_cv();
#if UNROLL_K1 == 0
                    // taps unrolled: one register copy of the input patch serves the whole output patch
                    cv_t w[CV_KH][CV_KW], x[PH][PW];
#pragma unroll
                    for (int kh = 0; kh < CV_KH; ++kh)
#pragma unroll
                        for (int kw = 0; kw < CV_KW; ++kw) w[kh][kw] = *reinterpret_cast<const cv_t *>(Wt + (kh * CV_KW + kw) * CV_C + cc);
#pragma unroll
                    for (int ph = 0; ph < PH; ++ph)
#pragma unroll
                        for (int pw = 0; pw < PW; ++pw) {
#if CACHE_READ
                            x[ph][pw] = *reinterpret_cast<const cv_t *>(&tile[((ohl * CV_STRIDE + ph) * TIW + owl * CV_STRIDE + pw) * BC + ccl]);
#else
                            x[ph][pw] = load_x(X, oh * CV_STRIDE - CV_PAD + ph, ow * CV_STRIDE - CV_PAD + pw, cc);
#endif
                        }
#pragma unroll
                    for (int a = 0; a < I3; ++a)
#pragma unroll
                        for (int b = 0; b < J3; ++b)
#pragma unroll
                            for (int kh = 0; kh < CV_KH; ++kh)
#pragma unroll
                                for (int kw = 0; kw < CV_KW; ++kw)
#pragma unroll
                                    for (int q = 0; q < VC; ++q)
                                        acc[a][b].v[q] += x[a * CV_STRIDE + kh][b * CV_STRIDE + kw].v[q] * w[kh][kw].v[q];
#else
#pragma unroll 1
                    for (int kh = 0; kh < CV_KH; ++kh)
#pragma unroll 1
                        for (int kw = 0; kw < CV_KW; ++kw) {
                            const cv_t w = *reinterpret_cast<const cv_t *>(Wt + (kh * CV_KW + kw) * CV_C + cc);
#pragma unroll
                            for (int a = 0; a < I3; ++a)
#pragma unroll
                                for (int b = 0; b < J3; ++b) {
#if CACHE_READ
                                    const cv_t x = *reinterpret_cast<const cv_t *>(
                                        &tile[(((ohl + a) * CV_STRIDE + kh) * TIW + (owl + b) * CV_STRIDE + kw) * BC + ccl]);
#else
                                    const cv_t x = load_x(X, (oh + a) * CV_STRIDE - CV_PAD + kh, (ow + b) * CV_STRIDE - CV_PAD + kw, cc);
#endif
#pragma unroll
                                    for (int q = 0; q < VC; ++q) acc[a][b].v[q] += x.v[q] * w.v[q];
                                }
                        }
#endif
#pragma unroll
                    for (int a = 0; a < I3; ++a)
#pragma unroll
                        for (int b = 0; b < J3; ++b)
                            *reinterpret_cast<cv_t *>(Y + ((long)(oh + a) * CV_OW + ow + b) * CV_C + cc) = acc[a][b];
                }
            }
}
