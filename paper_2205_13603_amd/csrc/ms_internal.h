// Internal declarations shared by the translation units of libms.
#pragma once
#include "../../include/ms.h"

#include <cstdarg>
#include <cstdint>
#include <string>
#include <vector>

struct ms_op {
    ms_op_desc d;        // the operator in the form the kernels see (a 1-D convolution as a conv2d of height 1)
    ms_op_desc user;     // the descriptor as given, default strides filled in
    int32_t pad_h;       // convolutions: zero rows above and below the image (d.pad: columns left and right)
    int64_t depth, kd, OD; // 3-D convolution: input depth, filter depth, output depth (1 otherwise); padded by d.pad
    // derived
    int64_t nb;          // batch (BMM) or 1
    int64_t M, N, K;     // implicit-GEMM view (conv: M = N*OH*OW, N = Cout, K = KH*KW*Cin)
    int64_t OH, OW;      // convolutions
    int in_size, out_size; // bytes per element
};

namespace ms {

int32_t fail(int32_t code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

// the two operators that share the conv2d kernels (the transposed one differs in the im2col index map only)
inline bool is_conv2d(int32_t kind) { return kind == MS_OP_CONV2D_NHWC || kind == MS_OP_CONV2D_TRANSPOSED_NHWC; }
inline bool is_3d(const ms_op *op) { return op->depth > 1 || op->kd > 1; }

// (m, n, k) of an MS_MFMA_CODE
inline void mfma_dims(int64_t code, int *m, int *n, int *k)
{
    if (code >= 1000000) {
        *m = int(code / 100000);
        *n = int(code / 1000 % 100);
        *k = int(code % 1000);
    } else {
        *m = int(code / 10000);
        *n = int(code / 100 % 100);
        *k = int(code % 100);
    }
}
void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));

// 64-bit counter-based generator: integer only, platform independent.
struct Rng {
    uint64_t s;
    explicit Rng(uint64_t seed) : s(seed) {}
    uint64_t next();
    // uniform in [0, n) by rejection, n >= 1
    uint64_t below(uint64_t n);
};
uint64_t mix64(uint64_t x);

const ms_slot *find_slot(const ms_space *sp, int32_t slot_id, int *pos);
const ms_decision *find_decision(const ms_trace *t, int32_t slot_id);
int64_t slot_extent(const ms_space *sp, const ms_trace *t, int pos); // resolves depends_on, -1 if unresolved

int dtype_size(int32_t dt);
const char *dtype_name(int32_t dt);
const char *op_kind_name(int32_t kind);

extern ms_limits g_limits;

// Kernel source generation: template file + "-D" defines for a variant.
struct KernelSpec {
    std::string template_name; // file in kernels/
    std::vector<std::string> defines;
    std::string entry;         // kernel symbol
    unsigned block[3];
    unsigned grid[3];          // per instance; instances multiply grid[2]
    unsigned lds_dynamic;
};
int32_t make_kernel_spec(const ms_op *op, const ms_variant_params *p, KernelSpec *out);

// JIT (ms_jit.cpp)
struct CodeObject;
int32_t jit_get_code(const KernelSpec &spec, uint64_t key, std::vector<char> **code_out);
std::string kernels_dir();

} // namespace ms
