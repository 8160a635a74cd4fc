// Shared by every kernel template (spliced in before run-time compilation).
// Everything that depends on the schedule arrives as a -D constant.

#define DT_F32 0
#define DT_F16 1
#define DT_BF16 2
#define DT_I8 3
#define DT_I32 4
#define DT_F8E4M3 5 // input of the matrix-core kernels only: bit patterns, never converted in software

typedef _Float16 half_t;

template <int DT> struct dt_traits;
template <> struct dt_traits<DT_F32> { typedef float type; };
template <> struct dt_traits<DT_F16> { typedef half_t type; };
template <> struct dt_traits<DT_BF16> { typedef unsigned short type; };
template <> struct dt_traits<DT_I8> { typedef signed char type; };
template <> struct dt_traits<DT_I32> { typedef int type; };
template <> struct dt_traits<DT_F8E4M3> { typedef unsigned char type; };

typedef dt_traits<IN_DT>::type in_t;
typedef dt_traits<OUT_DT>::type out_t;

#if IN_DT == DT_I8
typedef int acc_t;
#else
typedef float acc_t;
#endif

// A naturally aligned group of N elements: loads and stores of it become one
// memory instruction of N*sizeof(T) bytes.
template <typename T, int N> struct __attribute__((aligned(sizeof(T) * N))) vec_t {
    T v[N];
};

__device__ __forceinline__ float bf16_to_float(unsigned short b) { return __uint_as_float((unsigned)b << 16); }

// round to nearest even; NaN stays NaN.  The conversion is the hardware's (one instruction per pair of values):
// spelled out in integer arithmetic with its NaN test it costs a branch per element, and an epilogue of 128
// values per lane then shows in the run time of a tile
__device__ __forceinline__ unsigned short float_to_bf16(float f) { return __builtin_bit_cast(unsigned short, (__bf16)f); }

__device__ __forceinline__ acc_t to_acc(in_t x)
{
#if IN_DT == DT_BF16
    return bf16_to_float(x);
#else
    return (acc_t)x;
#endif
}

// the single rounding from the accumulator to the output type
__device__ __forceinline__ out_t from_acc(acc_t x)
{
#if OUT_DT == DT_BF16
    return float_to_bf16(x);
#else
    return (out_t)x;
#endif
}

// Workgroup -> (z, i0, j0): z = instance * batch + batch index, (i0, j0) = the two outer spatial loops.
// REORDER 0: i outer.  1: j outer.  2: i outer, after a permutation of the launch-wide workgroup
// id that undoes the round-robin of workgroups over the 8 XCDs: the hardware sends workgroup f
// (x fastest, then y, z) to XCD f mod 8, so id (f mod 8) * (total / 8) + f / 8 makes the workgroups
// one XCD receives consecutive in (z, i0, j0) order; tiles that share operand panels, and whole
// instances, then sit behind one L2.
// RFACTOR > 1 (matrix-core kernels): RFACTOR consecutive workgroups share one output tile, workgroup ks
// of them reduces over the ks-th run of k0 steps.
#ifndef RFACTOR
#define RFACTOR 1
#endif
__device__ __forceinline__ void block_to_tile(int &z, int &i0, int &j0, int &ks)
{
    constexpr int G = I0 * J0 * RFACTOR;
    int wg = blockIdx.x;
    z = blockIdx.z * gridDim.y + blockIdx.y;
#if REORDER >= 2
    const int nz = gridDim.y * gridDim.z;
    const long total = (long)G * nz;
    if (total % 8 == 0) {
        const long f = wg + (long)G * z;
        const long g = (f % 8) * (total / 8) + f / 8;
        wg = (int)(g % G);
        z = (int)(g / G);
    }
#endif
    ks = wg % RFACTOR;
    wg /= RFACTOR;
#if REORDER == 1
    j0 = wg / I0;
    i0 = wg % I0;
#else
    i0 = wg / J0;
    j0 = wg % J0;
#endif
}
