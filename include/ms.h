/*
 * ms.h - C ABI of the schedule-parameterised operator kernel library for
 * AMD MI355X (gfx950).
 *
 * What the library is, in the vocabulary of "Tensor Program Optimization with
 * Probabilistic Programs" (arXiv 2205.13603):
 *
 *   e0        an operator definition (ms_op): a loop nest with spatial and
 *             reduction loops (Section 2; workloads of Appendix A.2).
 *   S(e0)     the search space (ms_space): an ordered list of sampling
 *             instructions, sample-perfect-tile and sample-categorical
 *             (Table 2), produced by the transformation modules enabled in
 *             `flags` (Section 3.2: Multi-Level-Tiling, the hardware-specific
 *             tensorize module, cache-read, unroll/vectorize).
 *   tau       a trace (ms_trace): one decision per sampling instruction
 *             (Section 4, "Execution tracing").  A trace is plain data owned
 *             by the caller.
 *   g(e0,tau) a variant (ms_variant): the concrete GPU kernel the trace
 *             selects.  Every valid trace computes the same function as e0.
 *   validator ms_trace_validate: rejects traces that exceed hardware limits
 *             (Section 4, "Trace validation").
 *   f(e)      ms_measure: latency of a variant on the device (Eq. 1).
 *   search    ms_search: evolutionary search over traces by mutating
 *             decisions, accept/reject with the annealed weight exp(-f/T)
 *             (Section 4, "End-to-end search", Eq. 1), on measured latency.
 *
 * Conventions
 *   - Every call returns an ms_status.  On failure ms_last_error() gives a
 *     NUL-terminated reason, valid until the next failing call on the same
 *     thread.  No exception crosses this boundary and nothing aborts.
 *   - "device pointer" = memory of the current HIP device, owned by the
 *     caller; the library never allocates, frees or retains user tensors.
 *     "host pointer" = ordinary process memory.  `stream` is a hipStream_t
 *     passed as void* (NULL = the default stream).
 *   - Handles (ms_op*, ms_variant*) are created and destroyed by the library;
 *     destroy accepts NULL.  ms_space and ms_trace are caller-owned PODs.
 *   - Tensors are row-major with the last index contiguous unless element
 *     strides in the op descriptor say otherwise.  Outputs are always dense.
 *   - An "instance" is one independent copy of the operator's whole problem;
 *     a launch over R instances reads R consecutive dense copies of each
 *     input and writes R consecutive copies of the output.  Per-instance
 *     tiling is exactly what the trace says.
 */
#ifndef MS_H
#define MS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MS_ABI_VERSION 3

typedef enum ms_status {
    MS_OK = 0,
    MS_ERR_BAD_ARG = 1,       /* NULL pointer, bad enum, bad size */
    MS_ERR_INVALID_TRACE = 2, /* the validator rejected the trace */
    MS_ERR_UNSUPPORTED = 3,   /* well-formed request outside what is implemented */
    MS_ERR_COMPILE = 4,       /* run-time compilation of the variant failed */
    MS_ERR_HIP = 5,           /* a HIP runtime call failed */
    MS_ERR_NOMEM = 6
} ms_status;

/* ------------------------------------------------------------------ e0 */

typedef enum ms_op_kind {
    MS_OP_GEMM = 0,          /* C[i][j]    = sum_k A[i][k]    * B[k][j]     (GMM) */
    MS_OP_BMM_NT = 1,        /* C[b][i][j] = sum_k A[b][i][k] * B[b][j][k]  (TBG: Q.K^T) */
    MS_OP_BMM_NN = 2,        /* C[b][i][j] = sum_k A[b][i][k] * B[b][k][j] */
    MS_OP_CONV2D_NHWC = 3,   /* Y = act(bias + conv(X, W)), X NHWC, W HWIO  (C2D / CBR) */
    MS_OP_DWCONV2D_NHWC = 4, /* depthwise, X NHWC, W [KH][KW][C]            (DEP) */
    MS_OP_SOFTMAX = 5,       /* Y[b][i][:] = softmax(X[b][i][:]), last axis  (SFM) */
    MS_OP_NORM = 6,          /* Y[b] = sqrt(sum_{i,j} X[b][i][j]^2)          (NRM) */
    MS_OP_CONV2D_TRANSPOSED_NHWC = 7, /* Y = act(bias + convT(X, W)): the adjoint of CONV2D_NHWC in X; X NHWC,
                                        W [KH][KW][Cin][Cout]                (T2D) */
    MS_OP_CONV1D_NWC = 8,    /* Y = act(bias + conv(X, W)), X [N][L][Cin], W [K][Cin][Cout]  (C1D) */
    MS_OP_CONV3D_NDHWC = 9   /* Y = act(bias + conv(X, W)), X [N][D][H][W][Cin], W [K][K][K][Cin][Cout]  (C3D) */
} ms_op_kind;

typedef enum ms_dtype { MS_F32 = 0, MS_F16 = 1, MS_BF16 = 2, MS_I8 = 3, MS_I32 = 4,
                        MS_F8E4M3 = 5 /* input only, GEMM / BMM on the matrix cores: 8-bit float, 4 exponent bits (bias 7),
                                         3 mantissa bits, no infinities, 0x7f / 0xff NaN; fp32 accumulate, output F16 or F32 */
} ms_dtype;

/*
 * dims:
 *   GEMM            M, N, K
 *   BMM_NT, BMM_NN  B, M, N, K
 *   CONV2D_NHWC     N, H, W, Cin, Cout, KH, KW, groups   (groups 0 or 1: dense.  groups G > 1 (GRP): output channel co
 *                   sums over the Cin/G input channels of group co / (Cout/G) only; W is [KH][KW][Cin/G][Cout])
 *   DWCONV2D_NHWC   N, H, W, C, KH, KW
 *   CONV3D_NDHWC    N, D, H, W, Cin, Cout, K    (a K x K x K filter; one stride, padding and dilation for the three
 *                   axes; runs on the conv2d kernels with im2col staging, the depth folded into rows and reduction)
 *   CONV1D_NWC      N, L, Cin, Cout, K, groups   (zero padding `pad` at both ends of L only; runs on the conv2d
 *                   kernels as an image of height 1 with a 1 x K filter that is not padded vertically)
 *   CONV2D_TRANSPOSED_NHWC  N, H, W, Cin, Cout, KH, KW   (input element (ih, iw) contributes X * W[kh][kw] to output
 *                           (ih*stride + kh - pad, iw*stride + kw - pad); output size (H-1)*stride - 2*pad + KH;
 *                           dense filters only; same inputs, bias and ReLU as CONV2D_NHWC)
 *   SOFTMAX, NORM   B, M, N   (X dense [B][M][N]; F32, F16 or BF16 in; softmax writes the input dtype or F32,
 *                              the norm writes F32 [B]; all arithmetic in fp32: max, exp(x - max), sum, scale)
 * Convolutions: cross-correlation, zero padding `pad` on all four sides,
 * output size floor((H + 2*pad - KH)/stride) + 1.  bias is fp32 [Cout], added
 * to the accumulator before ReLU, before the single rounding to out_dtype.
 * Accumulation is fp32 for F32/F16/BF16 inputs and exact int32 for I8.
 * out_dtype: F32 or the input dtype for float inputs; I32 for I8.
 * a_strides / b_strides (GEMM and BMM only; element units; all zero = the
 * dense default of the op kind): A element (b,i,k) at b*a[0] + i*a[1] + k*a[2];
 * B element (b,k,j) at b*b[0] + k*b[1] + j*b[2].
 * Inputs of a launch: GEMM/BMM {A, B}; CONV {X, W, bias or NULL}; DW {X, W}; SOFTMAX/NORM {X}.
 */
typedef struct ms_op_desc {
    int32_t kind;
    int32_t in_dtype;
    int32_t out_dtype;
    int32_t stride;
    int32_t pad;
    int32_t has_bias;
    int32_t relu;
    int32_t dilation;   /* conv2d: distance between filter taps in input elements; 0 or 1 = dense filter */
    int64_t dims[8];
    int64_t a_strides[3];
    int64_t b_strides[3];
} ms_op_desc;

typedef struct ms_op ms_op;

/* Create an operator from a descriptor (host pointer, copied).  Errors:
 * BAD_ARG for a NULL pointer, non-positive dim or unknown enum; UNSUPPORTED
 * for a dtype combination outside the list above. */
int32_t ms_op_create(const ms_op_desc *desc, ms_op **out);
void ms_op_destroy(ms_op *op);
/* Copy the descriptor back, with default strides filled in. */
int32_t ms_op_get_desc(const ms_op *op, ms_op_desc *out);

/* The loop nest of e0 after the fusions fixed per operator (conv: n,oh,ow are
 * fused into one spatial loop, kh,kw,ci into one reduction loop). */
#define MS_MAX_LOOPS 8
typedef struct ms_loop {
    char name[8];
    int64_t extent;
    int32_t is_reduction; /* 0 = spatial (data parallel), 1 = reduction */
    int32_t reserved;
} ms_loop;
int32_t ms_op_loops(const ms_op *op, ms_loop *loops /* [MS_MAX_LOOPS] */, int32_t *n_loops);
/* Algorithmic work of one instance: flop = 2 * MACs of the definition,
 * bytes = every input and output tensor moved once. */
int32_t ms_op_work(const ms_op *op, double *flop, double *bytes);
/* Byte size of input `idx` / of the output, for one instance. */
int32_t ms_op_tensor_bytes(const ms_op *op, int32_t idx /* -1 = output */, int64_t *bytes);

/* ------------------------------------------------------------------ S(e0) */

#define MS_MAX_SLOTS 16
#define MS_MAX_FACTORS 4
#define MS_MAX_CANDS 12

typedef enum ms_slot_kind { MS_SLOT_PERFECT_TILE = 0, MS_SLOT_CATEGORICAL = 1 } ms_slot_kind;

/* Semantic ids of the sampling instructions. */
typedef enum ms_slot_id {
    MS_SLOT_TENSORIZE = 0, /* categorical: matrix-core intrinsic (candidates = codes below) */
    MS_SLOT_TILE_I = 1,    /* perfect tile of spatial loop 0 (rows / oh) */
    MS_SLOT_TILE_J = 2,    /* perfect tile of spatial loop 1 (cols / ow) */
    MS_SLOT_TILE_C = 3,    /* perfect tile of the channel loop (depthwise) */
    MS_SLOT_TILE_K = 4,    /* perfect tile of the reduction loop */
    MS_SLOT_UNROLL = 5,    /* categorical: unroll budget, candidates {0,16,64} */
    MS_SLOT_CACHE_READ = 6,/* categorical: 0 = operands read from global memory,
                              1 = staged in LDS, 2 = staged in LDS, double buffered,
                              3 (matrix-core kernels) = double buffered, prefetch two tiles ahead,
                              4 (matrix-core kernels) = double buffered, two wavefront groups half a step apart,
                              5, 6, 7 (matrix-core kernels, 2-byte and 1-byte inputs) = global memory -> LDS directly,
                              a ring of 2, 3, 4 buffers,
                              8, 9, 10 = that ring of 2, 3, 4 buffers under persistent workgroups (reorder 3) whose
                              wavefronts form two groups one phase apart: while one group multiplies a slot of
                              k3 intrinsic steps from registers, the other reads its next slot from LDS; a k0 step
                              is k2 such slots (k1 = 1); with cache_write 1 every wavefront stages its results in an
                              LDS area of its own */
    MS_SLOT_VECTORIZE = 7, /* categorical: elements per global load instruction of operand A (conv: X) */
    MS_SLOT_STORAGE_ALIGN = 8, /* categorical: LDS layout: 0 = dense, 1 = each row / plane padded by 16 bytes,
                              2 (matrix-core kernels) = padded, and the 16-byte slots of a plane XOR-swizzled,
                              3 (matrix-core GEMMs whose B is contiguous along j, 1- and 2-byte inputs, register staging,
                              B loaded in 16-byte vectors) = A as with 2, B kept in LDS as in global memory (row-major
                              k-rows, 16-column granules XOR-swizzled with the row) and read with the transposing LDS
                              loads instead of being transposed in registers (Table 2, transform-layout),
                              4 = as 3 without any swizzle: the k-rows of B padded by 32 bytes, the planes of A by 16, so
                              that every fragment address is a per-lane base plus a constant */
    MS_SLOT_REORDER = 9,   /* categorical: order of the grid loops, 0 = i outer, 1 = j outer,
                              2 = i outer with workgroups grouped per XCD, 3 (with cache_read 5..7) = as 2 with
                              persistent workgroups that loop over tiles */
    MS_SLOT_VECTORIZE_B = 10, /* categorical: elements per global load instruction of operand B (conv: W) */
    MS_SLOT_CACHE_WRITE = 11, /* categorical (matrix-core kernels): 0 = results go from registers to global memory,
                                 1 = the workgroup's output tile is staged in LDS and written as whole rows */
    MS_SLOT_COMPUTE_AT = 12   /* categorical (conv2d; Table 2, sample-compute-location): loop under which the
                                 cache-read of the activations X is computed.  0 = under k0: every k step stages its
                                 im2col tile; 1 = under fuse(i0, j0): the input rows the workgroup's output tile needs
                                 are staged once (zero halo included) and every k step reads its operands from that
                                 patch; the cache_read decision then governs the weights only (1, 2 or 3);
                                 2 = as 1, and the cache-read of the weights W moves above the tile loop: persistent
                                 workgroups own runs of consecutive tiles, the weights of the current instance stay in
                                 LDS, the k loop has no barrier and no global load; cache_read 1 = the next patch is
                                 loaded between tiles, 2 = it is prefetched into registers during the k loop;
                                 3 = as 2 with cache_read 2 and cache_write 1, plus four helper wavefronts that do all
                                 global loads and stores of the tile loop while the others multiply;
                                 4 = as 2 (cache_read 1 or 2), but the weights end in registers: each wavefront keeps
                                 the fragments of its own output columns for all k steps, the k loop is fully
                                 unrolled whatever the unroll budget (the k split only sets the size of the staging
                                 steps) and reads only activations from LDS.
                                 Candidates that an operator cannot use are listed with weight 0: 1..4 need Cin (per
                                 group) to be a multiple of 8 unless the space has MS_SPACE_TAP_ROWS (for a grouped
                                 convolution the tile list of 2..4 runs over instance x group, "the weights of the
                                 current instance" being those of the current group), 3-D and transposed
                                 convolutions stop at 0 */
    ,
    MS_SLOT_RFACTOR = 13      /* categorical (matrix-core kernels; Table 2, rfactor: "factorize a reduction across a
                                 loop"): the k0 loop is cut into S = 1, 2, 4 or 8 consecutive runs and the runs of one
                                 output tile go to S workgroups.  Each writes the fp32 (int32) partial sums of its run
                                 to the workspace; a second kernel of the same launch adds the S partial results of
                                 every output element in run order, applies bias and ReLU and rounds once.  The result
                                 does not depend on how the workgroups are scheduled.  S must divide k0; persistent
                                 workgroups (reorder 3, compute_at 2..4) and cache_write 1 own the whole reduction
                                 and the epilogue and need S = 1 */
} ms_slot_id;

/* Tensorize candidates: (m, n, k) of one matrix-core instruction.  The code
 * is m*10000 + n*100 + k, e.g. 161616, 323208, 161632, 323216, 161664, 323232; fp32: 161604, 323202.
 * With k of three digits it is m*100000 + n*1000 + k: 1616128, the 128-deep 8-bit float instruction
 * (its 32x32 sibling is 323264).  Codes of 1000000 and above are of the second form. */
#define MS_MFMA_CODE(m, n, k) ((k) >= 100 ? (m) * 100000 + (n) * 1000 + (k) : (m) * 10000 + (n) * 100 + (k))
#define MS_MFMA_NONE 0

/*
 * One sampling instruction.  Perfect tile: draw n_factors positive integers,
 * outermost first, with product `extent` (Table 2, sample-perfect-tile; the
 * split of Section 3.1 with extents 32, 8, 4 is the tuple [32,8,4]).  If
 * depends_on >= 0 the extent is fixed only once the categorical slot at
 * position depends_on has been decided: extent = extent_by_choice[choice]
 * (the loop counted in units of the chosen intrinsic's tile); `extent` then
 * holds the loop's element extent.  Categorical: draw an index into
 * candidates with probability weight[i] / sum(weight) (Table 2,
 * sample-categorical).
 *
 * Roles of the four factors [f0,f1,f2,f3] of a spatial loop, index
 * ((x0*f1 + x1)*f2 + x2)*f3 + x3:  x0 -> workgroup (bind blockIdx),
 * x1 -> register tile, strided; x2 -> thread (ALU kernels) or wavefront
 * (matrix-core kernels) (bind threadIdx); x3 -> register tile, contiguous.
 * Reduction loop: x0 -> steps of the LDS tile loop, x1 -> rolled loop inside
 * a tile, x2 -> loop inside a tile subject to the unroll budget, x3 ->
 * innermost, always unrolled (vector reads along k / back-to-back intrinsics).
 */
typedef struct ms_slot {
    int32_t slot_id;
    int32_t kind;
    char name[16];
    int64_t extent;
    int32_t n_factors;
    int32_t n_candidates;
    int64_t candidates[MS_MAX_CANDS];
    int32_t weight[MS_MAX_CANDS];
    int32_t depends_on;
    int32_t reserved;
    int64_t extent_by_choice[MS_MAX_CANDS];
} ms_slot;

/* Transformation modules that may be composed into the space (Section 3.2). */
#define MS_SPACE_TENSORIZE 0x1u     /* use the matrix cores (needs F16/BF16/I8 inputs) */
#define MS_SPACE_CACHE_READ 0x2u    /* sample LDS staging; off = always staged, single buffer */
#define MS_SPACE_VECTORIZE 0x4u     /* sample global load width; off = scalar loads */
#define MS_SPACE_UNROLL 0x8u        /* sample the unroll budget; off = 0 */
#define MS_SPACE_STORAGE_ALIGN 0x10u/* sample LDS padding; off = no padding */
#define MS_SPACE_REORDER 0x20u      /* sample the grid loop order; off = i outer */
#define MS_SPACE_CACHE_WRITE 0x40u   /* sample LDS staging of the output tile; off = direct stores */
#define MS_SPACE_COMPUTE_AT 0x80u    /* conv2d: sample the loop that holds the cache-read of X; off = under k0 */
#define MS_SPACE_TENSORIZE_F32 0x100u /* opt-in, not part of the default: fp32 operators on the fp32 matrix-core
                                         intrinsics (16x16x4, 32x32x2) instead of the vector ALUs; the products are
                                         summed in another order than in the vector kernels, within the fp32 tolerance */
#define MS_SPACE_TAP_ROWS 0x200u      /* opt-in, conv2d with dense filters and one group: the reduction is laid out as KH
                                         runs of KW*Cin contiguous elements (one filter row across all its taps), each
                                         rounded up to the intrinsic's k.  With few input channels (first layers) a
                                         matrix-core k step then reads consecutive pixels of an input row instead of
                                         the channels of one pixel (the resident-patch modes then need pixels of an output
                                         row to start at multiples of 4 bytes) */
#define MS_SPACE_RFACTOR 0x400u       /* opt-in, matrix-core kernels: sample the rfactor decision (splits the reduction
                                         across workgroups through a caller-provided workspace): for launches that
                                         would otherwise leave most compute units idle; off = 1 */
#define MS_SPACE_DEFAULT 0xffu       /* every module above except the opt-in one; masks with bit 31 set (the
                                         all-ones default of earlier tuning records) mean the same */

typedef enum ms_family { MS_FAM_GEMM_ALU = 0, MS_FAM_GEMM_MFMA = 1, MS_FAM_DWCONV = 2,
                         MS_FAM_REDUCE = 3 /* softmax, norm: rows reduced by groups of lanes */ } ms_family;

typedef struct ms_space {
    int32_t family;
    uint32_t flags;
    int32_t n_slots;
    int32_t reserved;
    ms_slot slots[MS_MAX_SLOTS];
} ms_space;

/*
 * The modules as data (Section 3.2): every transformation module has a name, the location of e0 it applies to, the
 * Table 2 primitives it emits, its bit in a module mask and the bits that must already be in the space.  Module 0 is
 * Multi-Level-Tiling, the base every kernel family is built on.
 */
#define MS_MAX_MODULES 16
typedef enum ms_location {
    MS_LOC_BLOCK = 0,   /* the compute block C of e0 */
    MS_LOC_READS = 1,   /* the reads of C's operands (exists once the block is tiled) */
    MS_LOC_LDS = 2,     /* the LDS stage of the operands (exists once the block is tiled) */
    MS_LOC_WRITE = 3,   /* the write of C's result (exists once the block is tiled) */
    MS_LOC_LAUNCH = 4   /* the grid loops bound to workgroups (exists once the block is tiled) */
} ms_location;
typedef struct ms_module_info {
    char name[32];        /* e.g. "multi-level-tiling", "use-mfma", "cache-read" */
    char primitives[96];  /* the sampling and transformation primitives of Table 2 the module consists of */
    int32_t location;     /* ms_location */
    uint32_t flag;        /* its bit in a module mask (0 for the base module) */
    uint32_t requires;    /* bits of modules that must have been applied before it */
    int32_t reserved;
} ms_module_info;
int32_t ms_module_count(void);
int32_t ms_module_get(int32_t index, ms_module_info *out);
/*
 * Compose(modules, e0): apply an ordered list of modules (indices of ms_module_get) to the operator and write the
 * resulting space.  The list must start with module 0; a module whose `requires` bits were not applied earlier in the
 * list is an error (BAD_ARG, the message names both); a module that does not apply to this operator (the matrix-core
 * module on an fp32 depthwise convolution, compute-location on a plain matrix product, ...) is the identity, as a
 * module's own program analysis would make it.  *applied_mask (may be NULL) receives the bits that took effect.  The
 * space equals ms_space_describe(op, *applied_mask): slot order is canonical, so traces and stored records of one
 * mask stay valid whatever order the modules were listed in.
 */
int32_t ms_space_compose(const ms_op *op, const int32_t *modules, int32_t n, uint32_t *applied_mask, ms_space *out);
/*
 * Stochastic-Compose (Section 3.2, its composition algorithm): while locations remain, take the next location of the
 * program, draw one module from `module_set` and apply it there.  In this build a draw at a location is uniform over
 * the not yet applied modules of the set that belong to that location, apply to the operator and have their
 * requirements met, plus one "identity" outcome that retires the location; a module that was applied leaves the
 * (changed) location in the list, so it is visited again.  Module 0 is always applied first (it creates the other
 * locations); for an operator that has no vector-ALU kernel family (convolutions, 8-bit float inputs) the matrix-core
 * module follows it at once (UNSUPPORTED if the set lacks it).  Deterministic in `seed`.  applied[MS_MAX_MODULES] / *n_applied: the modules in the order they were
 * applied.  The space is ms_space_compose of that list.
 */
int32_t ms_space_stochastic_compose(const ms_op *op, const int32_t *module_set, int32_t n, uint64_t seed,
                                    int32_t *applied, int32_t *n_applied, ms_space *out);

/* Write the space of `op` under the enabled modules.  MS_SPACE_TENSORIZE is
 * dropped silently for F32 inputs.  UNSUPPORTED if no kernel family covers the
 * op with these flags (conv2d needs the tensorize module). */
int32_t ms_space_describe(const ms_op *op, uint32_t flags, ms_space *out);
/* log10 of the number of distinct traces of the space (support size). */
int32_t ms_space_log10_size(const ms_space *space, double *out);

/* ------------------------------------------------------------------ tau */

typedef struct ms_decision {
    int32_t slot_id;
    int32_t kind;
    int32_t n; /* number of values: n_factors, or 1 for a categorical (v[0] = index) */
    int32_t reserved;
    int64_t v[MS_MAX_FACTORS];
} ms_decision;

typedef struct ms_trace {
    int32_t n;
    int32_t reserved;
    ms_decision d[MS_MAX_SLOTS];
} ms_trace;

/* Draw trace number `index` of the stream `seed`.  Integer-only, reproducible
 * across runs and machines.  Perfect tiles are uniform over all ordered
 * factorisations; the result may be rejected by the validator. */
int32_t ms_trace_sample(const ms_space *space, uint64_t seed, uint64_t index, ms_trace *out);
/* As above, but redraws (index, attempt) until the validator accepts, at most
 * max_tries times; INVALID_TRACE if none was accepted. */
int32_t ms_trace_sample_valid(const ms_op *op, const ms_space *space, uint64_t seed, uint64_t index,
                              int32_t max_tries, ms_trace *out);
/* Propose a neighbour: exactly one decision is redrawn or, for a perfect
 * tile, a prime factor moves between two positions (the product is kept).
 * A tensorize mutation redraws the tiles that depend on it. */
int32_t ms_trace_mutate(const ms_space *space, const ms_trace *in, uint64_t seed, ms_trace *out);

/* Linearised program text (Section 4, "Execution tracing"): one instruction
 * per line, sampling instructions with their decisions followed by the
 * transformation instructions they parameterise.  from_text reads the
 * sampling lines only and reproduces the trace exactly.  to_text writes at
 * most cap bytes including the NUL and reports the needed size in *needed. */
int32_t ms_trace_to_text(const ms_op *op, const ms_space *space, const ms_trace *trace,
                         char *buf, size_t cap, size_t *needed);
int32_t ms_trace_from_text(const ms_space *space, const char *text, ms_trace *out);

/* ------------------------------------------------------------------ g(e0,tau) */

/* What the trace interpreter derives.  Unused fields are zero. */
typedef struct ms_variant_params {
    int32_t family;
    int32_t mfma;           /* MS_MFMA_CODE or MS_MFMA_NONE */
    int32_t ti[4], tj[4], tc[4], tk[4]; /* the tile decisions (tc: depthwise channels) */
    int32_t tile_unit[3];   /* elements per unit of ti, tj, tk (intrinsic m, n, k; 1 for ALU) */
    int32_t block_m, block_n, block_k; /* workgroup tile in elements (depthwise: oh, ow; block_k = channels) */
    int32_t grid[3];        /* workgroups per instance */
    int32_t threads;        /* workgroup size */
    int32_t waves;
    int32_t acc_per_thread; /* accumulator registers per lane */
    int32_t lds_bytes;
    int32_t cache_read;     /* 0 .. 10 as in MS_SLOT_CACHE_READ */
    int32_t vec;            /* elements per global load of A (depthwise: channels per access) */
    int32_t unroll;         /* budget */
    int32_t unroll_k1, unroll_k2; /* unroll factors of the two rolled reduction loops */
    int32_t lds_pad;        /* the storage-align decision: 0, 1 or 2 */
    int32_t reorder;
    int32_t vec_b;          /* elements per global load of B */
    int32_t cache_write;    /* 0, 1 as in MS_SLOT_CACHE_WRITE */
    int32_t compute_at;     /* 0 .. 4 as in MS_SLOT_COMPUTE_AT */
    int32_t tap_rows;       /* 1: the reduction of the MS_SPACE_TAP_ROWS layout (tile_unit[2] * the k split = KH * run) */
    int32_t rfactor;        /* workgroups that share the reduction of one output tile (1 = no workspace) */
    int32_t reserved[3];
    uint64_t key;           /* hash of everything that selects the kernel */
} ms_variant_params;

/* Pure host check (no GPU needed).  Rejects with INVALID_TRACE and a reason:
 * wrong slot order/ids, factor product != extent, non-positive factors,
 * categorical index out of range, workgroup threads outside [1,1024] (matrix
 * core kernels: waves outside [1,16]), LDS bytes above the limit,
 * accumulators per lane above the register budget, vector width that does
 * not divide the contiguous extent or breaks alignment, grid overflow.
 * On success fills *out if it is not NULL. */
int32_t ms_trace_validate(const ms_op *op, const ms_space *space, const ms_trace *trace,
                          ms_variant_params *out);

/* Hardware limits the validator checks against.  Defaults are those of
 * MI355X; ms_set_limits replaces them (tests use it to force rejections). */
typedef struct ms_limits {
    int32_t max_threads;      /* 1024 */
    int32_t max_lds_bytes;    /* 163840: the 160 KiB of a compute unit, which one workgroup may take whole */
    int32_t max_acc_per_thread; /* 256 */
    int32_t wave_size;        /* 64 */
    int32_t max_waves;        /* 16 */
    int32_t reserved[3];
} ms_limits;
int32_t ms_get_limits(ms_limits *out);
int32_t ms_set_limits(const ms_limits *in);

typedef struct ms_variant ms_variant;

/* Validate, then materialise the kernel: the family's HIP template is
 * compiled for gfx950 with the parameters as constants (in memory and on-disk
 * cache keyed by params.key).  Needs no GPU until the first launch.
 * Errors: INVALID_TRACE, COMPILE (compiler log in ms_last_error). */
int32_t ms_variant_build(const ms_op *op, const ms_space *space, const ms_trace *trace, ms_variant **out);
void ms_variant_destroy(ms_variant *v);
/* params and workspace_bytes may be NULL.  *workspace_bytes = bytes of workspace ONE instance needs (0 unless
 * rfactor > 1: rfactor x batch x M x N accumulator values); a launch over R instances needs R times as much. */
int32_t ms_variant_info(const ms_variant *v, ms_variant_params *params, size_t *workspace_bytes);
/* What materialising a variant compiles (Section 4, building a candidate): the kernel template's file name, then the
 * -D options that specialise it, one per line.  Two parameter sets that give the same text are the same kernel and
 * have the same params.key.  Writes at most cap bytes including the NUL; *needed (may be NULL) = size needed. */
int32_t ms_variant_kernel_text(const ms_op *op, const ms_variant_params *params, char *buf, size_t cap, size_t *needed);
/* What the compiled kernel occupies, read from the metadata of its code object (no GPU needed): vector registers per
 * lane (architectural and accumulation registers: a wavefront is granted their sum), scalar registers, bytes of
 * scratch memory per lane (non-zero = the compiler spilled registers), vector registers spilled, bytes of LDS. */
typedef struct ms_variant_resources {
    int32_t vgprs, agprs, sgprs;
    int32_t scratch_bytes;
    int32_t spilled_vgprs;
    int32_t lds_bytes;
    int32_t reserved[2];
} ms_variant_resources;
int32_t ms_variant_resources_get(const ms_variant *v, ms_variant_resources *out);
/* Compile the kernels of n traces ahead of use on `threads` host threads
 * (invalid traces are skipped).  *n_built = kernels now in the cache. */
int32_t ms_prebuild(const ms_op *op, const ms_space *space, const ms_trace *traces, int32_t n,
                    int32_t threads, int32_t *n_built);
/* Directory of the on-disk kernel cache (NULL or "" = in-memory only). */
int32_t ms_set_cache_dir(const char *path);
/* Where this process got its kernels from so far (Section 4: building a candidate is part of the cost of measuring
 * it): kernels compiled now, code objects read from the on-disk cache, requests served from memory; and the
 * version of the run-time compiler the process is bound to.  The version is part of every cache key, so a code
 * object is only reused by the compiler that made it: a stored latency and a later launch then refer to the same
 * machine code.  Any pointer may be NULL. */
int32_t ms_jit_stats(int64_t *compiled, int64_t *from_disk, int64_t *from_memory, int32_t *compiler_major, int32_t *compiler_minor);

/* Enqueue one execution over `instances` instances on `stream`.  inputs /
 * outputs: host arrays of device pointers (see ms_op_desc for the order; one
 * output).  workspace: device pointer, 16-byte aligned, of at least instances x
 * workspace_bytes (ms_variant_info), owned by the caller and not shared with a
 * launch that may run at the same time; NULL if that is 0.  Its contents need no
 * initialisation and are undefined afterwards.  Asynchronous (a variant with
 * rfactor > 1 enqueues two kernels); returns launch errors only.  BAD_ARG if
 * instances < 1, the grid would exceed 2^31-1 workgroups, or a needed workspace is NULL. */
int32_t ms_variant_launch(ms_variant *v, const void *const *inputs, void *const *outputs,
                          void *workspace, int32_t instances, void *stream);

/*
 * For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): ms_variant_launch with the workspace taken from an array inside the library's own device image
 * instead of from the caller.  MS_STATIC_WORKSPACE_BYTES of it exist on every GPU the library runs on, from the first
 * ms_variant_prepare on that GPU until the process ends.
 *   ms_variant_prepare        set-up, may allocate: loads the variant's kernels on the current device and resolves
 *                             that device's copy of the workspace.  Once per variant and device.
 *   ms_variant_launch_static  allocates nothing and frees nothing.  Same inputs / outputs / instances / stream as
 *                             ms_variant_launch.  BAD_ARG if ms_variant_prepare has not run for this variant on the
 *                             current device, or if instances x workspace_bytes exceeds MS_STATIC_WORKSPACE_BYTES
 *                             (a variant with rfactor = 1 needs none and always fits).
 * All calls on one GPU share that GPU's array, which keeps the previous call's partial sums: every value a call
 * reads it has written itself, so nothing needs clearing, but two calls that overlap on one GPU (two streams, two
 * threads) race on it; callers serialise them, e.g. by using one stream.
 */
#define MS_STATIC_WORKSPACE_BYTES (32u << 20)
int32_t ms_variant_prepare(ms_variant *v);
int32_t ms_variant_launch_static(ms_variant *v, const void *const *inputs, void *const *outputs, int32_t instances, void *stream);

/*
 * Host-side coverage check of the interpreted loop nest (no GPU): walks the
 * grid / thread / register loops the parameters describe and counts, for
 * every output element, how often it is produced.  counts: host pointer to
 * out_elems int32 (one instance).  A correct split/bind visits each exactly
 * once.  This executes index arithmetic only, never the operator.
 */
int32_t ms_variant_coverage(const ms_op *op, const ms_variant_params *params, int32_t *counts, int64_t out_elems);
/*
 * The same for the reduction: walks the rfactor / k0 / k1 / k2 / k3 / intrinsic-k loops (depthwise: the filter taps)
 * that produce ONE output element and counts how often each position of the reduction is visited.  counts: host
 * pointer to k_elems int32; *k_elems_needed (may be NULL) receives the length of the interpreted reduction (the
 * operator's K, rounded up where a convolution pads it to the intrinsic's k).  A correct split visits every position
 * exactly once, whatever the decisions.  Index arithmetic only.
 */
int32_t ms_variant_reduction_coverage(const ms_op *op, const ms_variant_params *params, int32_t *counts, int64_t k_elems,
                                      int64_t *k_elems_needed);

/* ------------------------------------------------------------------ f(e) */

typedef struct ms_bufset {
    const void *inputs[4]; /* device pointers */
    void *output;          /* device pointer */
    void *workspace;       /* device pointer or NULL */
} ms_bufset;

/*
 * One repeat = hipEventRecord, launches_per_repeat launches back to back on
 * `stream` (launch l uses buffer set l mod n_sets), hipEventRecord, wait.
 * Per-launch time = elapsed / launches_per_repeat.  `warmup` untimed launches
 * come first.  Three protocols are built from this:
 *   single launch      launches_per_repeat = 1, one buffer set
 *   steady state       launches_per_repeat >= 200 over buffer sets whose
 *                      footprint exceeds the last-level cache
 *   device filling     instances = R so that one launch fills the device
 */
typedef struct ms_measure_cfg {
    int32_t warmup;
    int32_t repeats;
    int32_t launches_per_repeat;
    int32_t instances;
} ms_measure_cfg;

typedef struct ms_measure_result {
    double min_us, median_us, mean_us; /* per launch */
    double flop, bytes;                /* algorithmic, per launch (instances included) */
    int32_t n;                         /* repeats timed */
    int32_t reserved;
} ms_measure_result;

/* Synchronises `stream`.  HIP errors are returned as MS_ERR_HIP and leave the
 * variant destroyable. */
int32_t ms_measure(ms_variant *v, const ms_bufset *sets, int32_t n_sets, const ms_measure_cfg *cfg,
                   void *stream, ms_measure_result *out);

/* ------------------------------------------------------------------ search */

typedef struct ms_search_cfg {
    uint64_t seed;
    int32_t trials;          /* measured candidates (invalid / failed ones are not counted) */
    int32_t init_population; /* random valid traces measured first */
    int32_t population;      /* survivors kept */
    int32_t children;        /* proposals per generation */
    int32_t eps_permille;    /* share of fresh random samples among proposals, in 1/1000 */
    int32_t compile_threads;
    double temperature0;     /* T anneals geometrically from temperature0 to temperature1 */
    double temperature1;
    ms_measure_cfg measure;
    int32_t cost_model;       /* 0 = every proposal is measured; 1 = a learned cost model picks which proposals to measure */
    int32_t model_candidates; /* with the cost model: proposals scored per measured candidate (e.g. 8) */
    int32_t model_min_trials; /* measurements needed before the model is used (earlier generations run as without it);
                               * pre-training rows count as measurements */
    int32_t pretrain_n;       /* rows of pretrain_X / pretrain_y, 0 = none */
    /* Rows the cost model is fitted on before the search starts (Section 4, "End-to-end search", allows a model
     * trained beforehand besides the refits during the search): host arrays, read during the call only, of feature
     * vectors (row-major, pretrain_n x pretrain_d, as ms_variant_features writes them for this operator) and targets (log2 of the latency in
     * microseconds) of earlier measurements of the same operator under the same measurement protocol, e.g. the log
     * of an earlier search.  Every fit sees these rows followed by this search's own measurements.  With enough
     * rows (>= model_min_trials) the model also picks the initial population: model_candidates x init_population
     * valid samples are drawn, half of the slots go to the best predicted ones and half to samples in the order
     * drawn.  Ignored without cost_model. */
    const double *pretrain_X;
    const double *pretrain_y;
    int32_t pretrain_d;
    int32_t reserved;
} ms_search_cfg;
void ms_search_cfg_default(ms_search_cfg *cfg);

typedef struct ms_trial {
    int32_t index;   /* 1-based among measured candidates */
    int32_t status;  /* MS_OK or the error that made the candidate fail */
    double us;       /* measured latency per launch (median) */
    double best_us;  /* best so far, this trial included */
    ms_trace trace;
    uint64_t key;
} ms_trial;
/* Called after every measured or failed candidate; return non-zero to stop. */
typedef int32_t (*ms_trial_cb)(const ms_trial *trial, void *user);
/* Test hook: if not NULL, latency comes from this function (microseconds,
 * <= 0 = failed) and neither compiler nor GPU is touched. */
typedef double (*ms_latency_fn)(const ms_variant_params *params, void *user);

typedef struct ms_search_result {
    ms_trace best_trace;
    double best_us;
    int32_t best_trial;    /* first trial within 1 % of the final best, 1-based */
    int32_t n_measured;
    int32_t n_invalid;     /* proposals the validator rejected */
    int32_t n_failed;      /* compile or launch failures */
    int32_t n_duplicate;   /* proposals that mapped to an already measured kernel */
    int32_t reserved;
    double wall_seconds;
} ms_search_result;

/* ------------------------------------------------------------ cost model */

/* The learned cost model of Section 4 ("End-to-end search"): least-squares gradient boosting of regression trees
 * with exact greedy splits, deterministic, host only.  Rows of X are feature vectors (row-major, n x d doubles),
 * y the targets (the search uses log2 of the measured microseconds).  fit() replaces whatever was fitted before;
 * predict() needs the same d.  A tree splits a node on the (feature, midpoint between two consecutive distinct
 * values) that lowers the squared error most, both sides keeping at least min_leaf rows; depth = number of split
 * levels; every tree's prediction is added with weight learning_rate.  n_trees = 0 predicts the mean of y. */
typedef struct ms_cost_model ms_cost_model;
int32_t ms_cost_model_create(int32_t n_trees, int32_t depth, double learning_rate, int32_t min_leaf, ms_cost_model **out);
void ms_cost_model_destroy(ms_cost_model *m);
int32_t ms_cost_model_fit(ms_cost_model *m, const double *X, const double *y, int32_t n, int32_t d);
int32_t ms_cost_model_predict(const ms_cost_model *m, const double *X, int32_t n, int32_t d, double *out);
/* Feature vector of a variant as the search feeds it to the model (tile factors, workgroup shape, LDS and
 * register footprints, staging decisions, mostly log2).  out may be NULL to query the count (*n). */
int32_t ms_variant_features(const ms_op *op, const ms_variant_params *params, double *out, int32_t cap, int32_t *n);

/* Evolutionary search (Section 4): sample init_population traces; then per
 * generation propose children by mutating parents drawn with probability
 * proportional to exp(-f/(T f_best)) (Eq. 1 with measured f), plus a share of
 * fresh samples; validate; measure; a child enters the population if it
 * beats the worst member or with probability exp(-(f_child - f_parent)/(T f_best)).
 * Deterministic in (seed, latency values). */
int32_t ms_search(const ms_op *op, const ms_space *space, const ms_search_cfg *cfg,
                  const ms_bufset *sets, int32_t n_sets, void *stream,
                  ms_latency_fn fake_latency, void *fake_user,
                  ms_trial_cb cb, void *cb_user, ms_search_result *out);

/* ------------------------------------------------------------------ misc */

typedef struct ms_device_info {
    char name[64];
    char arch[32];
    int32_t compute_units;
    int32_t wave_size;
    int32_t lds_bytes_per_block;
    int32_t max_threads_per_block;
    int32_t clock_khz;
    int32_t mem_clock_khz;
    int32_t mem_bus_bits;
    int32_t l2_bytes;
    int64_t global_mem_bytes;
} ms_device_info;
/* Properties of the current HIP device.  MS_ERR_HIP if there is none. */
int32_t ms_device_info_get(ms_device_info *out);

/*
 * Attainable peaks of the current device, measured: they ground the roofline
 * fractions next to the published ones (Section 5 reports measured latency
 * only; the roofline is this build's yardstick).
 * ms_calibrate_mfma: register-resident issue loop of one matrix-core
 * intrinsic (in_dtype F16/BF16/I8, MS_MFMA_CODE) on every SIMD; *tflops =
 * 2*m*n*k operations per instruction times instructions per second / 1e12.
 * operands: NULL (small-integer operands), or a device pointer to 16 KiB of
 * values of in_dtype from which every lane takes its two fragments (the
 * attainable rate depends on the operand values through power management).
 * scratch: device pointer to at least 4 KiB (never written in practice).
 * ms_calibrate_stream: mode 1 copies `bytes` from src to dst, mode 2 only
 * reads src, mode 3 only writes dst, mode 4 copies like mode 1 but with one 64-lane workgroup per KiB (the launch
 * shape of the bandwidth-bound operator kernels; the fastest copy found on this device); bytes must be a multiple of 4096; device pointers, 16-byte
 * aligned; *gbs = bytes moved (copy: read + written) per second / 1e9.
 * Both synchronise `stream`.
 */
int32_t ms_calibrate_mfma(int32_t in_dtype, int32_t mfma_code, const void *operands, void *scratch, void *stream, double *tflops);
int32_t ms_calibrate_stream(int32_t mode, const void *src, void *dst, size_t bytes, void *stream, double *gbs);
/* LDS read rate with 16-byte conflict-free reads on every CU: aggregate GB/s and bytes per clock per CU
 * at the device's nominal clock. */
int32_t ms_calibrate_lds(void *scratch, void *stream, double *bytes_per_clk_per_cu, double *gbs);
/* Rate at which the L2 caches feed the compute units: every workgroup reads the same 2 MiB window at src
 * (device pointer, at least 2 MiB) over and over; aggregate GB/s. */
int32_t ms_calibrate_l2(const void *src, void *scratch, void *stream, double *gbs);

/* Times a kernel of known duration with the event timing that ms_measure uses: one wavefront waits until the
 * device's constant-rate wall clock has advanced by target_us (1 .. 20000).  `cfg->instances` is ignored;
 * `scratch`: at least 512 bytes of device memory (never written).  On return out->min_us / median_us / mean_us are the
 * measured durations per launch: they exceed target_us by the launch overhead only.  Synchronises `stream`. */
int32_t ms_calibrate_timer(double target_us, const ms_measure_cfg *cfg, void *scratch, void *stream, ms_measure_result *out);

int32_t ms_version(void);
const char *ms_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MS_H */
