// Host side of libms: operator definitions, search space description,
// trace sampling / mutation / text form, trace interpreter and validator.
// Nothing in this file touches the GPU.
#include "ms_internal.h"

#include <algorithm>
#include <cinttypes>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

namespace ms {

static thread_local char g_err[4096] = "";

// The message is formatted into a buffer of its own first: callers may pass ms_last_error() (= g_err) as an
// argument, and vsnprintf must not read from the buffer it writes.
static void format_error(const char *fmt, va_list ap)
{
    char tmp[sizeof g_err];
    vsnprintf(tmp, sizeof tmp, fmt, ap);
    memcpy(g_err, tmp, sizeof g_err);
}

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    format_error(fmt, ap);
    va_end(ap);
}

int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    format_error(fmt, ap);
    va_end(ap);
    return code;
}

// MI355X: 1024 threads per workgroup, 160 KiB LDS per compute unit (one
// workgroup may take all of it), 512 vector registers per lane at one wave
// per SIMD of which at most half can sensibly hold accumulators.
ms_limits g_limits = {1024, 160 * 1024, 256, 64, 16, {0, 0, 0}};

uint64_t mix64(uint64_t x)
{
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

uint64_t Rng::next()
{
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t Rng::below(uint64_t n)
{
    if (n <= 1) return 0;
    uint64_t limit = UINT64_MAX - (UINT64_MAX % n + 1) % n; // largest value kept
    for (;;) {
        uint64_t r = next();
        if (r <= limit) return r % n;
    }
}

int dtype_size(int32_t dt)
{
    switch (dt) {
    case MS_F32: return 4;
    case MS_F16: return 2;
    case MS_BF16: return 2;
    case MS_I8: return 1;
    case MS_I32: return 4;
    case MS_F8E4M3: return 1;
    default: return 0;
    }
}

const char *dtype_name(int32_t dt)
{
    switch (dt) {
    case MS_F32: return "f32";
    case MS_F16: return "f16";
    case MS_BF16: return "bf16";
    case MS_I8: return "i8";
    case MS_I32: return "i32";
    case MS_F8E4M3: return "f8e4m3";
    default: return "?";
    }
}

const char *op_kind_name(int32_t kind)
{
    switch (kind) {
    case MS_OP_GEMM: return "gemm";
    case MS_OP_BMM_NT: return "bmm_nt";
    case MS_OP_BMM_NN: return "bmm_nn";
    case MS_OP_CONV2D_NHWC: return "conv2d_nhwc";
    case MS_OP_CONV2D_TRANSPOSED_NHWC: return "conv2d_transposed_nhwc";
    case MS_OP_CONV1D_NWC: return "conv1d_nwc";
    case MS_OP_CONV3D_NDHWC: return "conv3d_ndhwc";
    case MS_OP_DWCONV2D_NHWC: return "dwconv2d_nhwc";
    case MS_OP_SOFTMAX: return "softmax";
    case MS_OP_NORM: return "norm";
    default: return "?";
    }
}

const ms_slot *find_slot(const ms_space *sp, int32_t slot_id, int *pos)
{
    for (int i = 0; i < sp->n_slots; ++i)
        if (sp->slots[i].slot_id == slot_id) {
            if (pos) *pos = i;
            return &sp->slots[i];
        }
    return nullptr;
}

const ms_decision *find_decision(const ms_trace *t, int32_t slot_id)
{
    for (int i = 0; i < t->n; ++i)
        if (t->d[i].slot_id == slot_id) return &t->d[i];
    return nullptr;
}

int64_t slot_extent(const ms_space *sp, const ms_trace *t, int pos)
{
    const ms_slot &s = sp->slots[pos];
    if (s.depends_on < 0) return s.extent;
    if (s.depends_on >= pos || s.depends_on >= t->n) return -1;
    int64_t c = t->d[s.depends_on].v[0];
    const ms_slot &ctl = sp->slots[s.depends_on];
    if (c < 0 || c >= ctl.n_candidates) return -1;
    return s.extent_by_choice[c];
}

static bool space_ok(const ms_space *sp)
{
    if (!sp || sp->n_slots < 1 || sp->n_slots > MS_MAX_SLOTS) return false;
    for (int i = 0; i < sp->n_slots; ++i) {
        const ms_slot &s = sp->slots[i];
        if (s.kind == MS_SLOT_PERFECT_TILE) {
            if (s.n_factors < 1 || s.n_factors > MS_MAX_FACTORS) return false;
            if (s.depends_on >= i) return false;
            if (s.depends_on >= 0 && sp->slots[s.depends_on].kind != MS_SLOT_CATEGORICAL) return false;
        } else if (s.kind == MS_SLOT_CATEGORICAL) {
            if (s.n_candidates < 1 || s.n_candidates > MS_MAX_CANDS) return false;
            int64_t tot = 0;
            for (int c = 0; c < s.n_candidates; ++c) {
                if (s.weight[c] < 0) return false;
                tot += s.weight[c];
            }
            if (tot <= 0) return false;
        } else {
            return false;
        }
    }
    return true;
}

} // namespace ms

using namespace ms;

// ---------------------------------------------------------------- e0

static int64_t conv_out(int64_t in, int64_t k, int64_t s, int64_t p)
{
    int64_t span = in + 2 * p - k;
    return span < 0 ? 0 : span / s + 1;
}

extern "C" int32_t ms_op_create(const ms_op_desc *desc, ms_op **out)
{
    if (!desc || !out) return fail(MS_ERR_BAD_ARG, "ms_op_create: NULL argument");
    *out = nullptr;
    ms_op op;
    memset(&op, 0, sizeof op);
    ms_op_desc conv = *desc;
    const bool is_1d = desc->kind == MS_OP_CONV1D_NWC;
    if (is_1d) {
        // N, L, Cin, Cout, K, groups -> an image of height 1, a 1 x K filter, no vertical padding
        for (int i = 0; i < 5; ++i)
            if (desc->dims[i] < 1 || desc->dims[i] > (int64_t(1) << 30)) return fail(MS_ERR_BAD_ARG, "ms_op_create: dims[%d] = %" PRId64 " out of range", i, desc->dims[i]);
        conv.kind = MS_OP_CONV2D_NHWC;
        const int64_t v[8] = {desc->dims[0], 1, desc->dims[1], desc->dims[2], desc->dims[3], 1, desc->dims[4], desc->dims[5]};
        for (int i = 0; i < 8; ++i) conv.dims[i] = v[i];
    }
    op.depth = op.kd = op.OD = 1;
    const bool is_3d_op = desc->kind == MS_OP_CONV3D_NDHWC;
    if (is_3d_op) {
        // N, D, H, W, Cin, Cout, K -> the conv2d form plus the depth of the input and of the filter
        for (int i = 0; i < 7; ++i)
            if (desc->dims[i] < 1 || desc->dims[i] > (int64_t(1) << 30)) return fail(MS_ERR_BAD_ARG, "ms_op_create: dims[%d] = %" PRId64 " out of range", i, desc->dims[i]);
        conv.kind = MS_OP_CONV2D_NHWC;
        const int64_t v[8] = {desc->dims[0], desc->dims[2], desc->dims[3], desc->dims[4], desc->dims[5], desc->dims[6], desc->dims[6], 0};
        for (int i = 0; i < 8; ++i) conv.dims[i] = v[i];
        op.depth = desc->dims[1];
        op.kd = desc->dims[6];
    }
    op.d = conv;
    const ms_op_desc &d = conv;
    int ndims = 0;
    switch (d.kind) {
    case MS_OP_GEMM: ndims = 3; break;
    case MS_OP_BMM_NT:
    case MS_OP_BMM_NN: ndims = 4; break;
    case MS_OP_CONV2D_NHWC:
    case MS_OP_CONV2D_TRANSPOSED_NHWC: ndims = 7; break;
    case MS_OP_DWCONV2D_NHWC: ndims = 6; break;
    case MS_OP_SOFTMAX:
    case MS_OP_NORM: ndims = 3; break;
    default: return fail(MS_ERR_BAD_ARG, "ms_op_create: unknown op kind %d", d.kind);
    }
    for (int i = 0; i < ndims; ++i)
        if (d.dims[i] < 1 || d.dims[i] > (int64_t(1) << 30))
            return fail(MS_ERR_BAD_ARG, "ms_op_create: dims[%d] = %" PRId64 " out of range", i, d.dims[i]);
    if ((d.in_dtype < MS_F32 || d.in_dtype > MS_I8) && d.in_dtype != MS_F8E4M3)
        return fail(MS_ERR_BAD_ARG, "ms_op_create: bad in_dtype %d", d.in_dtype);
    if (d.in_dtype == MS_F8E4M3 && d.kind != MS_OP_GEMM && d.kind != MS_OP_BMM_NT && d.kind != MS_OP_BMM_NN)
        return fail(MS_ERR_UNSUPPORTED, "ms_op_create: 8-bit float inputs are for matrix products only");
    const bool is_reduce = d.kind == MS_OP_SOFTMAX || d.kind == MS_OP_NORM;
    bool out_ok;
    if (is_reduce)
        out_ok = (d.in_dtype == MS_F32 || d.in_dtype == MS_F16 || d.in_dtype == MS_BF16) &&
                 (d.out_dtype == MS_F32 || (d.kind == MS_OP_SOFTMAX && d.out_dtype == d.in_dtype));
    else if (d.in_dtype == MS_I8)
        out_ok = d.out_dtype == MS_I32;
    else if (d.in_dtype == MS_F8E4M3)
        out_ok = d.out_dtype == MS_F32 || d.out_dtype == MS_F16;
    else
        out_ok = d.out_dtype == MS_F32 || d.out_dtype == d.in_dtype;
    if (!out_ok)
        return fail(MS_ERR_UNSUPPORTED, "ms_op_create: in %s -> out %s is not supported", dtype_name(d.in_dtype),
                    dtype_name(d.out_dtype));
    op.in_size = dtype_size(d.in_dtype);
    op.out_size = dtype_size(d.out_dtype);
    op.nb = 1;
    if (d.kind == MS_OP_GEMM || d.kind == MS_OP_BMM_NT || d.kind == MS_OP_BMM_NN) {
        int o = d.kind == MS_OP_GEMM ? 0 : 1;
        if (o) op.nb = d.dims[0];
        op.M = d.dims[o];
        op.N = d.dims[o + 1];
        op.K = d.dims[o + 2];
        bool a_zero = !d.a_strides[0] && !d.a_strides[1] && !d.a_strides[2];
        bool b_zero = !d.b_strides[0] && !d.b_strides[1] && !d.b_strides[2];
        if (a_zero) {
            op.d.a_strides[0] = op.M * op.K;
            op.d.a_strides[1] = op.K;
            op.d.a_strides[2] = 1;
        }
        if (b_zero) {
            op.d.b_strides[0] = op.K * op.N;
            if (d.kind == MS_OP_BMM_NT) {
                op.d.b_strides[1] = 1;
                op.d.b_strides[2] = op.K;
            } else {
                op.d.b_strides[1] = op.N;
                op.d.b_strides[2] = 1;
            }
        }
        for (int i = 0; i < 3; ++i)
            if (op.d.a_strides[i] < 0 || op.d.b_strides[i] < 0)
                return fail(MS_ERR_BAD_ARG, "ms_op_create: negative stride");
        if (d.stride || d.pad || d.has_bias || d.relu || d.dilation)
            return fail(MS_ERR_BAD_ARG, "ms_op_create: stride/pad/bias/relu/dilation only apply to convolutions");
    } else if (is_reduce) {
        if (d.stride || d.pad || d.has_bias || d.relu || d.dilation)
            return fail(MS_ERR_BAD_ARG, "ms_op_create: stride/pad/bias/relu/dilation only apply to convolutions");
        for (int i = 0; i < 3; ++i)
            if (d.a_strides[i] || d.b_strides[i]) return fail(MS_ERR_BAD_ARG, "ms_op_create: softmax and norm take dense inputs");
        // rows that are reduced independently, and their length
        op.M = d.kind == MS_OP_SOFTMAX ? d.dims[0] * d.dims[1] : d.dims[0];
        op.K = d.kind == MS_OP_SOFTMAX ? d.dims[2] : d.dims[1] * d.dims[2];
        op.N = 1;
        if (op.M > (int64_t(1) << 30) || op.K > (int64_t(1) << 30) || op.M * op.K > (int64_t(1) << 40))
            return fail(MS_ERR_BAD_ARG, "ms_op_create: tensor too large");
    } else {
        if (d.stride < 1 || d.pad < 0) return fail(MS_ERR_BAD_ARG, "ms_op_create: bad stride/pad");
        int64_t H = d.dims[1], W = d.dims[2];
        int64_t KH = is_conv2d(d.kind) ? d.dims[5] : d.dims[4];
        int64_t KW = is_conv2d(d.kind) ? d.dims[6] : d.dims[5];
        if (d.dilation < 0 || d.dilation > 64) return fail(MS_ERR_BAD_ARG, "ms_op_create: bad dilation");
        if (op.d.dilation == 0) op.d.dilation = 1;
        if (op.d.dilation != 1 && !is_conv2d(d.kind)) return fail(MS_ERR_UNSUPPORTED, "ms_op_create: dilation is for conv2d only");
        // a filter whose taps are `dilation` apart spans dilation * (K - 1) + 1 input elements
        op.pad_h = is_1d ? 0 : d.pad;
        op.OH = conv_out(H, op.d.dilation * (KH - 1) + 1, d.stride, op.pad_h);
        op.OW = conv_out(W, op.d.dilation * (KW - 1) + 1, d.stride, d.pad);
        if (d.kind == MS_OP_CONV2D_TRANSPOSED_NHWC) {
            // the adjoint of a stride-s convolution: input element ih reaches outputs ih*s + kh - pad
            if (op.d.dilation != 1) return fail(MS_ERR_UNSUPPORTED, "ms_op_create: the transposed convolution has dense filters");
            op.OH = (H - 1) * d.stride - 2 * (int64_t)d.pad + KH;
            op.OW = (W - 1) * d.stride - 2 * (int64_t)d.pad + KW;
        }
        if (is_3d_op) op.OD = conv_out(op.depth, op.d.dilation * (op.kd - 1) + 1, d.stride, d.pad);
        if (op.OH < 1 || op.OW < 1 || op.OD < 1) return fail(MS_ERR_BAD_ARG, "ms_op_create: empty convolution output");
        if (is_conv2d(d.kind)) {
            if (d.in_dtype == MS_I8) return fail(MS_ERR_UNSUPPORTED, "ms_op_create: int8 conv2d is not supported");
            // dims[7] = groups (0 or 1: a dense convolution); a group is a batch entry of the implicit GEMM
            const int64_t G = d.dims[7] ? d.dims[7] : 1;
            if (G < 1 || d.dims[3] % G || d.dims[4] % G) return fail(MS_ERR_BAD_ARG, "ms_op_create: %" PRId64 " groups do not divide the channel counts", G);
            if (G > 1 && d.kind == MS_OP_CONV2D_TRANSPOSED_NHWC) return fail(MS_ERR_UNSUPPORTED, "ms_op_create: the transposed convolution has no groups");
            op.nb = G;
            op.M = d.dims[0] * op.OD * op.OH * op.OW;
            op.N = d.dims[4] / G;
            op.K = op.kd * KH * KW * (d.dims[3] / G);
            if (op.M > (int64_t(1) << 30) || op.K > (int64_t(1) << 30)) return fail(MS_ERR_BAD_ARG, "ms_op_create: convolution too large");
        } else {
            if (d.in_dtype != MS_F32) return fail(MS_ERR_UNSUPPORTED, "ms_op_create: depthwise conv is fp32 only");
            if (d.has_bias || d.relu) return fail(MS_ERR_UNSUPPORTED, "ms_op_create: depthwise has no epilogue");
            if (KH > 7 || KW > 7) return fail(MS_ERR_UNSUPPORTED, "ms_op_create: depthwise kernel larger than 7x7");
            op.M = op.OH;
            op.N = op.OW;
            op.K = KH * KW;
        }
    }
    op.user = op.d;
    if (is_1d || is_3d_op) op.user = *desc;
    ms_op *p = new (std::nothrow) ms_op(op);
    if (!p) return fail(MS_ERR_NOMEM, "ms_op_create: out of memory");
    *out = p;
    return MS_OK;
}

extern "C" void ms_op_destroy(ms_op *op) { delete op; }

extern "C" int32_t ms_op_get_desc(const ms_op *op, ms_op_desc *out)
{
    if (!op || !out) return fail(MS_ERR_BAD_ARG, "ms_op_get_desc: NULL argument");
    *out = op->user;
    return MS_OK;
}

static void set_loop(ms_loop *l, const char *name, int64_t extent, int red)
{
    memset(l, 0, sizeof *l);
    snprintf(l->name, sizeof l->name, "%s", name);
    l->extent = extent;
    l->is_reduction = red;
}

extern "C" int32_t ms_op_loops(const ms_op *op, ms_loop *loops, int32_t *n_loops)
{
    if (!op || !loops || !n_loops) return fail(MS_ERR_BAD_ARG, "ms_op_loops: NULL argument");
    int n = 0;
    switch (op->d.kind) {
    case MS_OP_BMM_NT:
    case MS_OP_BMM_NN: set_loop(&loops[n++], "b", op->nb, 0); /* fallthrough */
    case MS_OP_GEMM:
        set_loop(&loops[n++], "i", op->M, 0);
        set_loop(&loops[n++], "j", op->N, 0);
        set_loop(&loops[n++], "k", op->K, 1);
        break;
    case MS_OP_CONV2D_NHWC:
    case MS_OP_CONV2D_TRANSPOSED_NHWC:
        if (op->nb > 1) set_loop(&loops[n++], "g", op->nb, 0); // groups
        set_loop(&loops[n++], "i", op->M, 0); // fuse(n, oh, ow)
        set_loop(&loops[n++], "j", op->N, 0); // co
        set_loop(&loops[n++], "k", op->K, 1); // fuse(kh, kw, ci)
        break;
    case MS_OP_DWCONV2D_NHWC:
        set_loop(&loops[n++], "n", op->d.dims[0], 0);
        set_loop(&loops[n++], "i", op->OH, 0);
        set_loop(&loops[n++], "j", op->OW, 0);
        set_loop(&loops[n++], "c", op->d.dims[3], 0);
        set_loop(&loops[n++], "kh", op->d.dims[4], 1);
        set_loop(&loops[n++], "kw", op->d.dims[5], 1);
        break;
    case MS_OP_SOFTMAX:
        set_loop(&loops[n++], "i", op->M, 0); // fuse(b, m)
        set_loop(&loops[n++], "k", op->K, 1); // n: reduced for the maximum and the sum, then revisited for the output
        break;
    case MS_OP_NORM:
        set_loop(&loops[n++], "i", op->M, 0); // b
        set_loop(&loops[n++], "k", op->K, 1); // fuse(m, n)
        break;
    }
    *n_loops = n;
    return MS_OK;
}

extern "C" int32_t ms_op_tensor_bytes(const ms_op *op, int32_t idx, int64_t *bytes)
{
    if (!op || !bytes) return fail(MS_ERR_BAD_ARG, "ms_op_tensor_bytes: NULL argument");
    const ms_op_desc &d = op->d;
    int64_t e = -1;
    int sz = idx < 0 ? op->out_size : op->in_size;
    switch (d.kind) {
    case MS_OP_GEMM:
    case MS_OP_BMM_NT:
    case MS_OP_BMM_NN:
        if (idx < 0) e = op->nb * op->M * op->N;
        // inputs may be strided views: the span they touch
        else if (idx == 0)
            e = (op->nb - 1) * d.a_strides[0] + (op->M - 1) * d.a_strides[1] + (op->K - 1) * d.a_strides[2] + 1;
        else if (idx == 1)
            e = (op->nb - 1) * d.b_strides[0] + (op->K - 1) * d.b_strides[1] + (op->N - 1) * d.b_strides[2] + 1;
        break;
    case MS_OP_CONV2D_NHWC:
    case MS_OP_CONV2D_TRANSPOSED_NHWC:
        if (idx < 0) e = op->M * op->N * op->nb;
        else if (idx == 0) e = d.dims[0] * op->depth * d.dims[1] * d.dims[2] * d.dims[3];
        else if (idx == 1) e = op->K * op->N * op->nb; // [KD][KH][KW][Cin / groups][Cout]
        else if (idx == 2 && d.has_bias) { e = d.dims[4]; sz = 4; }
        break;
    case MS_OP_DWCONV2D_NHWC:
        if (idx < 0) e = d.dims[0] * op->OH * op->OW * d.dims[3];
        else if (idx == 0) e = d.dims[0] * d.dims[1] * d.dims[2] * d.dims[3];
        else if (idx == 1) e = d.dims[4] * d.dims[5] * d.dims[3];
        break;
    case MS_OP_SOFTMAX:
        if (idx < 0 || idx == 0) e = op->M * op->K;
        break;
    case MS_OP_NORM:
        if (idx < 0) e = op->M;
        else if (idx == 0) e = op->M * op->K;
        break;
    }
    if (e < 0) return fail(MS_ERR_BAD_ARG, "ms_op_tensor_bytes: no tensor %d", idx);
    *bytes = e * sz;
    return MS_OK;
}

extern "C" int32_t ms_op_work(const ms_op *op, double *flop, double *bytes)
{
    if (!op || !flop || !bytes) return fail(MS_ERR_BAD_ARG, "ms_op_work: NULL argument");
    const ms_op_desc &d = op->d;
    double f = 0, b = 0;
    switch (d.kind) {
    case MS_OP_GEMM:
    case MS_OP_BMM_NT:
    case MS_OP_BMM_NN:
        f = 2.0 * op->nb * op->M * op->N * op->K;
        b = (double)op->nb * (op->M * op->K + op->K * op->N) * op->in_size + (double)op->nb * op->M * op->N * op->out_size;
        break;
    case MS_OP_CONV2D_TRANSPOSED_NHWC:
        // every input element meets every tap once (contributions that fall outside the output are not discounted)
        f = 2.0 * d.dims[0] * d.dims[1] * d.dims[2] * op->K * op->N;
        b = (double)(d.dims[0] * d.dims[1] * d.dims[2] * d.dims[3] + op->K * op->N) * op->in_size +
            (d.has_bias ? 4.0 * op->N : 0.0) + (double)op->M * op->N * op->out_size;
        break;
    case MS_OP_CONV2D_NHWC:
        f = 2.0 * op->M * op->N * op->K * op->nb;
        b = (double)(d.dims[0] * op->depth * d.dims[1] * d.dims[2] * d.dims[3] + op->K * op->N * op->nb) * op->in_size +
            (d.has_bias ? 4.0 * op->N * op->nb : 0.0) + (double)op->M * op->N * op->nb * op->out_size;
        break;
    case MS_OP_DWCONV2D_NHWC: {
        double outs = (double)d.dims[0] * op->OH * op->OW * d.dims[3];
        f = 2.0 * outs * d.dims[4] * d.dims[5];
        b = ((double)d.dims[0] * d.dims[1] * d.dims[2] * d.dims[3] + (double)d.dims[4] * d.dims[5] * d.dims[3]) * op->in_size +
            outs * op->out_size;
        break;
    }
    case MS_OP_SOFTMAX:
        // per element: compare, subtract, exponential, add, scale
        f = 5.0 * op->M * op->K;
        b = (double)op->M * op->K * (op->in_size + op->out_size);
        break;
    case MS_OP_NORM:
        f = 2.0 * op->M * op->K;
        b = (double)op->M * op->K * op->in_size + (double)op->M * op->out_size;
        break;
    }
    *flop = f;
    *bytes = b;
    return MS_OK;
}

// ---------------------------------------------------------------- S(e0)

static ms_slot *add_slot(ms_space *sp, int32_t id, int32_t kind, const char *name)
{
    ms_slot *s = &sp->slots[sp->n_slots++];
    memset(s, 0, sizeof *s);
    s->slot_id = id;
    s->kind = kind;
    s->depends_on = -1;
    snprintf(s->name, sizeof s->name, "%s", name);
    return s;
}

static void add_tile(ms_space *sp, int32_t id, const char *name, int64_t extent)
{
    ms_slot *s = add_slot(sp, id, MS_SLOT_PERFECT_TILE, name);
    s->extent = extent;
    s->n_factors = 4;
}

static void add_cat(ms_space *sp, int32_t id, const char *name, std::initializer_list<int64_t> cands)
{
    ms_slot *s = add_slot(sp, id, MS_SLOT_CATEGORICAL, name);
    for (int64_t c : cands) {
        s->candidates[s->n_candidates] = c;
        s->weight[s->n_candidates] = 1;
        ++s->n_candidates;
    }
}

extern "C" int32_t ms_space_describe(const ms_op *op, uint32_t flags, ms_space *out)
{
    if (!op || !out) return fail(MS_ERR_BAD_ARG, "ms_space_describe: NULL argument");
    memset(out, 0, sizeof *out);
    const ms_op_desc &d = op->d;
    if (flags & 0x80000000u) flags &= 0xffu; // all-ones masks of earlier records: the default set, opt-in modules off
    if (d.in_dtype == MS_F32 && !((flags & MS_SPACE_TENSORIZE_F32) && d.kind != MS_OP_DWCONV2D_NHWC && !is_conv2d(d.kind)))
        flags &= ~(MS_SPACE_TENSORIZE | MS_SPACE_TENSORIZE_F32);
    if (d.in_dtype != MS_F32) flags &= ~MS_SPACE_TENSORIZE_F32;
    if (flags & MS_SPACE_TENSORIZE_F32) flags |= MS_SPACE_TENSORIZE;
    if (d.kind == MS_OP_DWCONV2D_NHWC) flags &= ~(MS_SPACE_TENSORIZE | MS_SPACE_VECTORIZE | MS_SPACE_STORAGE_ALIGN | MS_SPACE_CACHE_WRITE);
    if (!(flags & MS_SPACE_TENSORIZE)) flags &= ~MS_SPACE_RFACTOR; // the matrix-core kernels implement it
    if (d.kind != MS_OP_CONV2D_NHWC) flags &= ~MS_SPACE_COMPUTE_AT; // the resident-patch modes assume the direct index map
    // the filter-row layout of the reduction: plain conv2d only (dense filter, one group, two dimensions)
    if (!(d.kind == MS_OP_CONV2D_NHWC && op->nb == 1 && !is_3d(op) && d.dilation == 1)) flags &= ~MS_SPACE_TAP_ROWS;
    flags &= 0x7ffu;
    if (d.kind == MS_OP_SOFTMAX || d.kind == MS_OP_NORM) {
        // rows i: [workgroups, serial, thread groups, rows of one group at a time]; reduction k: [serial, loads in
        // flight, lanes of a group (cross-thread reduction), vector]
        flags &= d.kind == MS_OP_SOFTMAX ? MS_SPACE_CACHE_READ : 0u;
        out->flags = flags;
        out->family = MS_FAM_REDUCE;
        add_tile(out, MS_SLOT_TILE_I, "i", op->M);
        add_tile(out, MS_SLOT_TILE_K, "k", op->K);
        if (flags & MS_SPACE_CACHE_READ) add_cat(out, MS_SLOT_CACHE_READ, "cache_read", {0, 1});
        return MS_OK;
    }
    out->flags = flags;
    if (d.kind == MS_OP_DWCONV2D_NHWC) {
        out->family = MS_FAM_DWCONV;
        add_tile(out, MS_SLOT_TILE_I, "i", op->OH);
        add_tile(out, MS_SLOT_TILE_J, "j", op->OW);
        add_tile(out, MS_SLOT_TILE_C, "c", d.dims[3]);
        if (flags & MS_SPACE_UNROLL) add_cat(out, MS_SLOT_UNROLL, "unroll", {0, 16, 64});
        if (flags & MS_SPACE_CACHE_READ) add_cat(out, MS_SLOT_CACHE_READ, "cache_read", {0, 1});
        if (flags & MS_SPACE_REORDER) add_cat(out, MS_SLOT_REORDER, "reorder", {0, 2});
        return MS_OK;
    }
    if (flags & MS_SPACE_TENSORIZE) {
        out->family = MS_FAM_GEMM_MFMA;
        if (d.a_strides[2] != 1 && !is_conv2d(d.kind))
            return fail(MS_ERR_UNSUPPORTED, "ms_space_describe: matrix-core kernels need A contiguous along k");
        if (!is_conv2d(d.kind) && d.b_strides[1] != 1 && d.b_strides[2] != 1)
            return fail(MS_ERR_UNSUPPORTED, "ms_space_describe: matrix-core kernels need B contiguous along k or j");
        ms_slot *t = add_slot(out, MS_SLOT_TENSORIZE, MS_SLOT_CATEGORICAL, "tensorize");
        static const int64_t f16_list[] = {161616, 323208, 161632, 323216};
        static const int64_t i8_list[] = {161632, 323216, 161664, 323232};
        static const int64_t f32_list[] = {161604, 323202};
        static const int64_t f8_list[] = {161632, 323216, 1616128, 323264};
        const int64_t *list = d.in_dtype == MS_I8 ? i8_list : (d.in_dtype == MS_F32 ? f32_list : (d.in_dtype == MS_F8E4M3 ? f8_list : f16_list));
        for (int c = 0; c < (d.in_dtype == MS_F32 ? 2 : 4); ++c) {
            int m, n, k;
            mfma_dims(list[c], &m, &n, &k);
            // conv2d: a reduction extent that k does not divide is rounded up (zero padded by the loaders)
            if (op->M % m || op->N % n || (op->K % k && !is_conv2d(d.kind))) continue;
            t->candidates[t->n_candidates] = list[c];
            t->weight[t->n_candidates] = 1;
            ++t->n_candidates;
        }
        if (t->n_candidates == 0)
            return fail(MS_ERR_UNSUPPORTED, "ms_space_describe: no matrix-core intrinsic divides M=%" PRId64 " N=%" PRId64 " K=%" PRId64,
                        op->M, op->N, op->K);
        const int32_t ids[3] = {MS_SLOT_TILE_I, MS_SLOT_TILE_J, MS_SLOT_TILE_K};
        const char *names[3] = {"i", "j", "k"};
        const int64_t ext[3] = {op->M, op->N, op->K};
        for (int l = 0; l < 3; ++l) {
            add_tile(out, ids[l], names[l], ext[l]);
            ms_slot *s = &out->slots[out->n_slots - 1];
            s->depends_on = 0;
            for (int c = 0; c < t->n_candidates; ++c) {
                int mnk[3];
                mfma_dims(t->candidates[c], &mnk[0], &mnk[1], &mnk[2]);
                s->extent_by_choice[c] = (ext[l] + mnk[l] - 1) / mnk[l];
                if (l == 2 && (flags & MS_SPACE_TAP_ROWS)) {
                    // KH runs of KW * Cin elements, each rounded up to the intrinsic's k
                    const int64_t run = d.dims[6] * d.dims[3];
                    s->extent_by_choice[c] = d.dims[5] * ((run + mnk[2] - 1) / mnk[2]);
                }
            }
        }
        if (flags & MS_SPACE_UNROLL) add_cat(out, MS_SLOT_UNROLL, "unroll", {0, 16, 64});
        if (flags & MS_SPACE_CACHE_READ) {
            // direct-to-LDS staging (5, 6, 7) exists for 2-byte and 1-byte inputs of plain matrix products
            if (d.in_dtype != MS_F32 && d.in_dtype != MS_F8E4M3 && !is_conv2d(d.kind))
                add_cat(out, MS_SLOT_CACHE_READ, "cache_read", {1, 2, 3, 4, 5, 6, 7, 8, 9, 10});
            else add_cat(out, MS_SLOT_CACHE_READ, "cache_read", {1, 2, 3, 4});
        }
        if (flags & MS_SPACE_VECTORIZE) {
            if (d.in_dtype == MS_I8 || d.in_dtype == MS_F8E4M3) {
                add_cat(out, MS_SLOT_VECTORIZE, "vectorize", {1, 4, 8, 16});
                add_cat(out, MS_SLOT_VECTORIZE_B, "vectorize_b", {1, 4, 8, 16});
            } else if (d.in_dtype == MS_F32) {
                add_cat(out, MS_SLOT_VECTORIZE, "vectorize", {1, 2, 4});
                add_cat(out, MS_SLOT_VECTORIZE_B, "vectorize_b", {1, 2, 4});
            } else {
                add_cat(out, MS_SLOT_VECTORIZE, "vectorize", {1, 2, 4, 8});
                add_cat(out, MS_SLOT_VECTORIZE_B, "vectorize_b", {1, 2, 4, 8});
            }
        }
        if (flags & MS_SPACE_STORAGE_ALIGN) {
            // 3 (B row-major in LDS, read with the transposing loads): GEMMs whose B is contiguous along j, 1- and 2-byte inputs
            const bool b_rows = !is_conv2d(d.kind) && d.b_strides[2] == 1 && d.b_strides[1] != 1 &&
                                (d.in_dtype == MS_F16 || d.in_dtype == MS_BF16 || d.in_dtype == MS_I8 || d.in_dtype == MS_F8E4M3);
            if (b_rows) add_cat(out, MS_SLOT_STORAGE_ALIGN, "storage_align", {0, 1, 2, 3, 4});
            else add_cat(out, MS_SLOT_STORAGE_ALIGN, "storage_align", {0, 1, 2});
        }
        if (flags & MS_SPACE_REORDER) {
            if (d.in_dtype != MS_F32 && d.in_dtype != MS_F8E4M3 && !is_conv2d(d.kind)) add_cat(out, MS_SLOT_REORDER, "reorder", {0, 1, 2, 3});
            else add_cat(out, MS_SLOT_REORDER, "reorder", {0, 1, 2});
        }
        if (flags & MS_SPACE_CACHE_WRITE) add_cat(out, MS_SLOT_CACHE_WRITE, "cache_write", {0, 1});
        if (flags & MS_SPACE_COMPUTE_AT) add_cat(out, MS_SLOT_COMPUTE_AT, "compute_at", {0, 1, 2, 3, 4});
        if (flags & MS_SPACE_RFACTOR) add_cat(out, MS_SLOT_RFACTOR, "rfactor", {1, 2, 4, 8});
        if (is_conv2d(d.kind)) {
            // candidates that no trace of this operator can use keep their position (stored decisions are indices)
            // but get weight 0: vector widths that do not divide the channel counts, and the resident-patch modes
            // when no intrinsic's k divides Cin
            for (int i = 0; i < out->n_slots; ++i) {
                ms_slot &sl = out->slots[i];
                for (int c = 0; c < sl.n_candidates; ++c) {
                    if (sl.slot_id == MS_SLOT_VECTORIZE && (d.dims[3] / op->nb) % sl.candidates[c]) sl.weight[c] = 0;
                    if (sl.slot_id == MS_SLOT_VECTORIZE_B && op->N % sl.candidates[c]) sl.weight[c] = 0;
                    if (sl.slot_id == MS_SLOT_COMPUTE_AT && sl.candidates[c] > 0 &&
                        ((d.dims[3] / op->nb) % 8 || is_3d(op)))
                        sl.weight[c] = 0;
                    if (sl.slot_id == MS_SLOT_COMPUTE_AT && (flags & MS_SPACE_TAP_ROWS))
                        sl.weight[c] = sl.candidates[c] == 0 || (d.stride * d.dims[3] * op->in_size) % 4 == 0 ? 1 : 0;
                }
            }
        }
        return MS_OK;
    }
    flags &= ~(MS_SPACE_CACHE_WRITE | MS_SPACE_COMPUTE_AT);
    out->flags = flags;
    if (is_conv2d(d.kind))
        return fail(MS_ERR_UNSUPPORTED, "ms_space_describe: conv2d needs the tensorize module (fp16/bf16 inputs)");
    if (d.in_dtype == MS_F8E4M3)
        return fail(MS_ERR_UNSUPPORTED, "ms_space_describe: 8-bit float inputs need the tensorize module");
    out->family = MS_FAM_GEMM_ALU;
    add_tile(out, MS_SLOT_TILE_I, "i", op->M);
    add_tile(out, MS_SLOT_TILE_J, "j", op->N);
    add_tile(out, MS_SLOT_TILE_K, "k", op->K);
    if (flags & MS_SPACE_UNROLL) add_cat(out, MS_SLOT_UNROLL, "unroll", {0, 16, 64});
    if (flags & MS_SPACE_CACHE_READ) add_cat(out, MS_SLOT_CACHE_READ, "cache_read", {0, 1, 2});
    if (flags & MS_SPACE_VECTORIZE) {
        add_cat(out, MS_SLOT_VECTORIZE, "vectorize", {1, 2, 4});
        add_cat(out, MS_SLOT_VECTORIZE_B, "vectorize_b", {1, 2, 4});
    }
    if (flags & MS_SPACE_STORAGE_ALIGN) add_cat(out, MS_SLOT_STORAGE_ALIGN, "storage_align", {0, 1});
    if (flags & MS_SPACE_REORDER) add_cat(out, MS_SLOT_REORDER, "reorder", {0, 1, 2});
    return MS_OK;
}

// ---------------------------------------------------------------- modules as data (Section 3.2)

namespace {
struct Module {
    const char *name;
    const char *primitives;
    int32_t location;
    uint32_t flag, requires_;
};
// canonical order = the order in which ms_space_describe lays out the slots the modules contribute
const Module kModules[] = {
    {"multi-level-tiling", "sample-perfect-tile, split, reorder, bind (4 factors per loop)", MS_LOC_BLOCK, 0u, 0u},
    {"use-mfma", "sample-categorical, blockize, tensorize (matrix-core intrinsic; tiles counted in its units)", MS_LOC_BLOCK, MS_SPACE_TENSORIZE, 0u},
    {"use-mfma-f32", "sample-categorical, blockize, tensorize (fp32 matrix-core intrinsics, opt-in)", MS_LOC_BLOCK, MS_SPACE_TENSORIZE_F32, 0u},
    {"unroll", "sample-categorical, unroll (budget 0, 16, 64)", MS_LOC_BLOCK, MS_SPACE_UNROLL, 0u},
    {"rfactor", "sample-categorical, rfactor (k0 across workgroups, workspace)", MS_LOC_BLOCK, MS_SPACE_RFACTOR, MS_SPACE_TENSORIZE},
    {"cache-read", "sample-categorical, cache-read, set-scope, compute-at (staging scheme of the operands)", MS_LOC_READS, MS_SPACE_CACHE_READ, 0u},
    {"vectorize", "sample-categorical, vectorize (global load width per operand)", MS_LOC_READS, MS_SPACE_VECTORIZE, 0u},
    {"compute-location", "sample-compute-location, compute-at (loop that holds the cache-read of the activations)", MS_LOC_READS, MS_SPACE_COMPUTE_AT, MS_SPACE_TENSORIZE},
    {"filter-row-layout", "transform-layout (reduction as filter rows, opt-in)", MS_LOC_READS, MS_SPACE_TAP_ROWS, MS_SPACE_TENSORIZE},
    {"storage-align", "sample-categorical, storage-align (padding / swizzle of the LDS planes)", MS_LOC_LDS, MS_SPACE_STORAGE_ALIGN, 0u},
    {"cache-write", "sample-categorical, cache-write, reverse-compute-at (result tile staged in LDS)", MS_LOC_WRITE, MS_SPACE_CACHE_WRITE, MS_SPACE_TENSORIZE},
    {"reorder-grid", "sample-categorical, reorder, bind (workgroup loop order, XCD grouping, persistent loop)", MS_LOC_LAUNCH, MS_SPACE_REORDER, 0u},
};
constexpr int kNumModules = (int)(sizeof kModules / sizeof kModules[0]);
static_assert(kNumModules <= MS_MAX_MODULES, "module table fits the public limit");

// does the module change the space of this operator, given what has been applied?  (ms_space_describe drops the bits
// that do not apply; a bit that survives it took effect)
bool module_takes_effect(const ms_op *op, uint32_t before, const Module &m)
{
    if (!m.flag) return true;
    ms_space sp;
    if (ms_space_describe(op, before | m.flag, &sp) != MS_OK) return false;
    return (sp.flags & m.flag) != 0;
}
} // namespace

extern "C" int32_t ms_module_count(void) { return kNumModules; }

extern "C" int32_t ms_module_get(int32_t index, ms_module_info *out)
{
    if (!out || index < 0 || index >= kNumModules) return fail(MS_ERR_BAD_ARG, "ms_module_get: no module %d", index);
    memset(out, 0, sizeof *out);
    snprintf(out->name, sizeof out->name, "%s", kModules[index].name);
    snprintf(out->primitives, sizeof out->primitives, "%s", kModules[index].primitives);
    out->location = kModules[index].location;
    out->flag = kModules[index].flag;
    out->requires = kModules[index].requires_;
    return MS_OK;
}

extern "C" int32_t ms_space_compose(const ms_op *op, const int32_t *modules, int32_t n, uint32_t *applied_mask, ms_space *out)
{
    if (!op || !modules || !out || n < 1 || n > MS_MAX_MODULES) return fail(MS_ERR_BAD_ARG, "ms_space_compose: bad argument");
    if (modules[0] != 0) return fail(MS_ERR_BAD_ARG, "ms_space_compose: the list must start with %s: every kernel family is built on it", kModules[0].name);
    uint32_t mask = 0, listed = 0;
    for (int i = 0; i < n; ++i) {
        if (modules[i] < 0 || modules[i] >= kNumModules) return fail(MS_ERR_BAD_ARG, "ms_space_compose: no module %d", modules[i]);
        const Module &m = kModules[modules[i]];
        if (i > 0 && modules[i] == 0) return fail(MS_ERR_BAD_ARG, "ms_space_compose: %s listed twice", m.name);
        if (m.flag && (listed & m.flag)) return fail(MS_ERR_BAD_ARG, "ms_space_compose: %s listed twice", m.name);
        if ((m.requires_ & listed) != m.requires_) {
            for (int j = 0; j < kNumModules; ++j)
                if (kModules[j].flag & m.requires_ & ~listed)
                    return fail(MS_ERR_BAD_ARG, "ms_space_compose: %s needs %s earlier in the list", m.name, kModules[j].name);
        }
        listed |= m.flag;
        if (module_takes_effect(op, mask, m)) mask |= m.flag;
    }
    int32_t rc = ms_space_describe(op, mask, out);
    if (rc != MS_OK) return rc;
    if (applied_mask) *applied_mask = out->flags;
    return MS_OK;
}

extern "C" int32_t ms_space_stochastic_compose(const ms_op *op, const int32_t *module_set, int32_t n, uint64_t seed, int32_t *applied,
                                               int32_t *n_applied, ms_space *out)
{
    if (!op || !module_set || !applied || !n_applied || !out || n < 0 || n > MS_MAX_MODULES)
        return fail(MS_ERR_BAD_ARG, "ms_space_stochastic_compose: bad argument");
    bool in_set[MS_MAX_MODULES] = {false}, done[MS_MAX_MODULES] = {false};
    for (int i = 0; i < n; ++i) {
        if (module_set[i] < 0 || module_set[i] >= kNumModules) return fail(MS_ERR_BAD_ARG, "ms_space_stochastic_compose: no module %d", module_set[i]);
        in_set[module_set[i]] = true;
    }
    Rng rng(mix64(seed ^ 0x53C0A705E5ull));
    int na = 0;
    uint32_t mask = 0;
    // the program starts as the untiled block; tiling it creates the other locations
    applied[na++] = 0;
    done[0] = true;
    {
        // operators without a vector-ALU kernel family (convolutions, 8-bit float inputs) exist on the matrix cores
        // only: for them the hardware-specific module is part of the base, provided the set offers it
        ms_space probe;
        if (ms_space_describe(op, 0, &probe) != MS_OK) {
            if (!in_set[1] || ms_space_describe(op, kModules[1].flag, &probe) != MS_OK)
                return fail(MS_ERR_UNSUPPORTED, "ms_space_stochastic_compose: the operator needs %s, which the module set lacks or which does not apply", kModules[1].name);
            applied[na++] = 1;
            done[1] = true;
            mask |= kModules[1].flag;
        }
    }
    int queue[8] = {MS_LOC_BLOCK, MS_LOC_READS, MS_LOC_LDS, MS_LOC_WRITE, MS_LOC_LAUNCH}, nq = 5, head = 0;
    while (head < nq) { // while locations are not exhausted
        const int loc = queue[head]; // next-location(program)
        int cand[MS_MAX_MODULES], nc = 0;
        for (int j = 1; j < kNumModules; ++j) {
            const Module &m = kModules[j];
            if (!in_set[j] || done[j] || m.location != loc) continue;
            if ((m.requires_ & mask) != m.requires_) continue;
            if (!module_takes_effect(op, mask, m)) continue;
            cand[nc++] = j;
        }
        const int pick = (int)rng.below((uint64_t)nc + 1); // m ~ Sample(modules); outcome nc = identity
        if (pick == nc) {
            ++head; // the location is retired
            continue;
        }
        const int j = cand[pick];
        applied[na++] = j; // program <- m(location, program); the changed location stays at the head of the list
        done[j] = true;
        mask |= kModules[j].flag;
    }
    *n_applied = na;
    return ms_space_compose(op, applied, na, nullptr, out);
}

// number of ordered n-tuples with product e: prod over primes C(a+n-1, n-1)
static double log10_tiles(int64_t e, int n)
{
    double lg = 0;
    for (int64_t p = 2; e > 1; ++p) {
        if (p * p > e) p = e;
        int a = 0;
        while (e % p == 0) {
            e /= p;
            ++a;
        }
        if (a) {
            double c = 1;
            for (int i = 1; i <= n - 1; ++i) c = c * (a + i) / i;
            lg += log10(c);
        }
    }
    return lg;
}

extern "C" int32_t ms_space_log10_size(const ms_space *space, double *out)
{
    if (!space_ok(space) || !out) return fail(MS_ERR_BAD_ARG, "ms_space_log10_size: bad argument");
    // dependent tiles: average over the controlling choices would need a sum; report the
    // size as log10 of sum over choices of the product of dependent tile counts times the rest
    double rest = 0;
    int ctl = -1;
    for (int i = 0; i < space->n_slots; ++i) {
        const ms_slot &s = space->slots[i];
        if (s.kind == MS_SLOT_PERFECT_TILE && s.depends_on >= 0) ctl = s.depends_on;
    }
    for (int i = 0; i < space->n_slots; ++i) {
        const ms_slot &s = space->slots[i];
        if (i == ctl) continue;
        if (s.kind == MS_SLOT_CATEGORICAL) rest += log10((double)s.n_candidates);
        else if (s.depends_on < 0) rest += log10_tiles(s.extent, s.n_factors);
    }
    if (ctl < 0) {
        *out = rest;
        return MS_OK;
    }
    double sum = 0;
    for (int c = 0; c < space->slots[ctl].n_candidates; ++c) {
        double lg = 0;
        for (int i = 0; i < space->n_slots; ++i) {
            const ms_slot &s = space->slots[i];
            if (s.kind == MS_SLOT_PERFECT_TILE && s.depends_on == ctl) lg += log10_tiles(s.extent_by_choice[c], s.n_factors);
        }
        sum += pow(10.0, lg);
    }
    *out = rest + log10(sum);
    return MS_OK;
}

// ---------------------------------------------------------------- sampling

// Uniform over ordered n-tuples with product `extent`: the exponent a of each
// prime is spread over the n positions as a uniformly random weak composition
// (a random (n-1)-subset of a+n-1 places marks the bars).
static void sample_tile(Rng &rng, int64_t extent, int n, int64_t *f)
{
    for (int i = 0; i < n; ++i) f[i] = 1;
    int64_t e = extent;
    for (int64_t p = 2; e > 1; ++p) {
        if (p * p > e) p = e;
        int a = 0;
        while (e % p == 0) {
            e /= p;
            ++a;
        }
        if (!a) continue;
        int places = a + n - 1;
        int idx[64 + MS_MAX_FACTORS];
        for (int i = 0; i < places; ++i) idx[i] = i;
        // choose n-1 bar places
        for (int i = 0; i < n - 1; ++i) {
            int j = i + (int)rng.below((uint64_t)(places - i));
            std::swap(idx[i], idx[j]);
        }
        std::sort(idx, idx + (n - 1));
        int prev = -1;
        for (int i = 0; i < n; ++i) {
            int bar = i < n - 1 ? idx[i] : places;
            int stars = bar - prev - 1;
            for (int s = 0; s < stars; ++s) f[i] *= p;
            prev = bar;
        }
    }
}

static int sample_cat(Rng &rng, const ms_slot &s)
{
    uint64_t tot = 0;
    for (int c = 0; c < s.n_candidates; ++c) tot += (uint64_t)s.weight[c];
    uint64_t r = rng.below(tot);
    for (int c = 0; c < s.n_candidates; ++c) {
        if (r < (uint64_t)s.weight[c]) return c;
        r -= (uint64_t)s.weight[c];
    }
    return s.n_candidates - 1;
}

static int32_t sample_with(const ms_space *space, Rng &rng, ms_trace *out)
{
    memset(out, 0, sizeof *out);
    out->n = space->n_slots;
    for (int i = 0; i < space->n_slots; ++i) {
        const ms_slot &s = space->slots[i];
        ms_decision &d = out->d[i];
        d.slot_id = s.slot_id;
        d.kind = s.kind;
        if (s.kind == MS_SLOT_CATEGORICAL) {
            d.n = 1;
            d.v[0] = sample_cat(rng, s);
        } else {
            int64_t e = slot_extent(space, out, i);
            if (e < 1) return fail(MS_ERR_BAD_ARG, "ms_trace_sample: slot %d has no extent", i);
            d.n = s.n_factors;
            sample_tile(rng, e, s.n_factors, d.v);
        }
    }
    return MS_OK;
}

extern "C" int32_t ms_trace_sample(const ms_space *space, uint64_t seed, uint64_t index, ms_trace *out)
{
    if (!space_ok(space) || !out) return fail(MS_ERR_BAD_ARG, "ms_trace_sample: bad argument");
    Rng rng(mix64(mix64(seed) ^ (index * 0xD1342543DE82EF95ull + 1)));
    return sample_with(space, rng, out);
}

extern "C" int32_t ms_trace_sample_valid(const ms_op *op, const ms_space *space, uint64_t seed, uint64_t index,
                                         int32_t max_tries, ms_trace *out)
{
    if (!op || !space_ok(space) || !out || max_tries < 1) return fail(MS_ERR_BAD_ARG, "ms_trace_sample_valid: bad argument");
    for (int32_t t = 0; t < max_tries; ++t) {
        Rng rng(mix64(mix64(mix64(seed) ^ (index * 0xD1342543DE82EF95ull + 1)) + (uint64_t)t * 0x2545F4914F6CDD1Dull));
        int32_t rc = sample_with(space, rng, out);
        if (rc != MS_OK) return rc;
        if (ms_trace_validate(op, space, out, nullptr) == MS_OK) return MS_OK;
    }
    return fail(MS_ERR_INVALID_TRACE, "ms_trace_sample_valid: no valid trace in %d draws (last: %s)", max_tries, ms_last_error());
}

static int smallest_prime(int64_t v)
{
    for (int64_t p = 2; p * p <= v; ++p)
        if (v % p == 0) return (int)p;
    return (int)v;
}

extern "C" int32_t ms_trace_mutate(const ms_space *space, const ms_trace *in, uint64_t seed, ms_trace *out)
{
    if (!space_ok(space) || !in || !out) return fail(MS_ERR_BAD_ARG, "ms_trace_mutate: bad argument");
    if (in->n != space->n_slots) return fail(MS_ERR_INVALID_TRACE, "ms_trace_mutate: trace has %d decisions, space %d", in->n, space->n_slots);
    ms_trace t = *in;
    Rng rng(mix64(seed ^ 0xA0761D6478BD642Full));
    // slots that can change
    int cand[MS_MAX_SLOTS], nc = 0;
    for (int i = 0; i < space->n_slots; ++i) {
        const ms_slot &s = space->slots[i];
        if (s.kind == MS_SLOT_CATEGORICAL) {
            if (s.n_candidates > 1) cand[nc++] = i;
        } else {
            int64_t e = slot_extent(space, &t, i);
            if (e > 1 && s.n_factors > 1) cand[nc++] = i;
        }
    }
    if (nc == 0) return fail(MS_ERR_UNSUPPORTED, "ms_trace_mutate: the space has a single point");
    int pos = cand[rng.below((uint64_t)nc)];
    const ms_slot &s = space->slots[pos];
    ms_decision &d = t.d[pos];
    if (s.kind == MS_SLOT_CATEGORICAL) {
        int64_t old = d.v[0];
        int64_t nv = (int64_t)rng.below((uint64_t)(s.n_candidates - 1));
        if (nv >= old) ++nv;
        d.v[0] = nv;
        // tiles counted in units of the old choice are redrawn
        for (int i = pos + 1; i < space->n_slots; ++i) {
            const ms_slot &dep = space->slots[i];
            if (dep.kind == MS_SLOT_PERFECT_TILE && dep.depends_on == pos) {
                int64_t e = slot_extent(space, &t, i);
                if (e < 1) return fail(MS_ERR_BAD_ARG, "ms_trace_mutate: dependent slot without extent");
                sample_tile(rng, e, dep.n_factors, t.d[i].v);
            }
        }
    } else {
        // move one prime factor from a position that has one to another position
        int src[MS_MAX_FACTORS], ns = 0;
        for (int i = 0; i < d.n; ++i)
            if (d.v[i] > 1) src[ns++] = i;
        if (ns == 0) return fail(MS_ERR_INVALID_TRACE, "ms_trace_mutate: tile of extent 1");
        int a = src[rng.below((uint64_t)ns)];
        int b = (int)rng.below((uint64_t)(d.n - 1));
        if (b >= a) ++b;
        // pick one of the primes of v[a] (with multiplicity)
        int64_t v = d.v[a];
        int primes[64], np = 0;
        while (v > 1) {
            int p = smallest_prime(v);
            primes[np++] = p;
            v /= p;
        }
        int p = primes[rng.below((uint64_t)np)];
        d.v[a] /= p;
        d.v[b] *= p;
    }
    *out = t;
    return MS_OK;
}

// ---------------------------------------------------------------- text form

static void appendf(std::string &s, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    s += buf;
}

extern "C" int32_t ms_trace_to_text(const ms_op *op, const ms_space *space, const ms_trace *trace, char *buf, size_t cap,
                                    size_t *needed)
{
    if (!op || !space_ok(space) || !trace) return fail(MS_ERR_BAD_ARG, "ms_trace_to_text: bad argument");
    if (trace->n != space->n_slots) return fail(MS_ERR_INVALID_TRACE, "ms_trace_to_text: trace/space length mismatch");
    std::string s;
    appendf(s, "# op=%s in=%s out=%s M=%" PRId64 " N=%" PRId64 " K=%" PRId64 " batch=%" PRId64 "\n", op_kind_name(op->user.kind),
            dtype_name(op->d.in_dtype), dtype_name(op->d.out_dtype), op->M, op->N, op->K, op->nb);
    // sampling instructions with their decisions
    for (int i = 0; i < space->n_slots; ++i) {
        const ms_slot &sl = space->slots[i];
        const ms_decision &d = trace->d[i];
        if (sl.kind == MS_SLOT_CATEGORICAL) {
            appendf(s, "v%d = sample-categorical(slot=%s, candidates=[", i, sl.name);
            for (int c = 0; c < sl.n_candidates; ++c) appendf(s, "%s%" PRId64, c ? ", " : "", sl.candidates[c]);
            s += "], weights=[";
            for (int c = 0; c < sl.n_candidates; ++c) appendf(s, "%s%d", c ? ", " : "", sl.weight[c]);
            appendf(s, "]) # decision: %" PRId64 "\n", d.v[0]);
        } else {
            int64_t e = slot_extent(space, trace, i);
            for (int f = 0; f < sl.n_factors; ++f) appendf(s, "%s%s%d", f ? ", " : "", sl.name, f);
            appendf(s, " = sample-perfect-tile(slot=%s, extent=%" PRId64 ", n=%d) # decision: [", sl.name, e, sl.n_factors);
            for (int f = 0; f < d.n; ++f) appendf(s, "%s%" PRId64, f ? ", " : "", d.v[f]);
            s += "]\n";
        }
    }
    // transformation instructions they parameterise (informational on read-back)
    ms_variant_params p;
    if (ms_trace_validate(op, space, trace, &p) == MS_OK) {
        if (p.mfma) appendf(s, "tensorize(block=C, intrin=mfma_%dx%dx%d)\n", p.tile_unit[0], p.tile_unit[1], p.tile_unit[2]);
        const char *nm[4] = {"i", "j", "c", "k"};
        const int32_t *tl[4] = {p.ti, p.tj, p.tc, p.tk};
        for (int l = 0; l < 4; ++l) {
            if (!tl[l][0]) continue;
            appendf(s, "%s0, %s1, %s2, %s3 = split(loop=%s, factors=[%d, %d, %d, %d])\n", nm[l], nm[l], nm[l], nm[l], nm[l],
                    tl[l][0], tl[l][1], tl[l][2], tl[l][3]);
        }
        if (p.family == MS_FAM_REDUCE) {
            s += "reorder(i0, i1, i2, i3, k0, k1, k2, k3)\nbind(i0, blockIdx.x)\n";
            appendf(s, "bind(fuse(i2, k2), threadIdx.x)  # k2: cross-thread reduction over %d lanes (wavefront shuffles%s)\n", p.tk[2],
                    p.tk[2] > 64 ? ", LDS across wavefronts" : "");
            appendf(s, "vectorize(k3)\nunroll(k1)\n");
            if (p.cache_read) appendf(s, "cache-read(buffer=X, scope=registers, compute-at=i3)  # one pass over global memory\n");
            appendf(s, "# workgroup=%d threads, grid=%d, lds=%d B, values/lane=%d\n", p.threads, p.grid[0] * p.grid[1] * p.grid[2], p.lds_bytes,
                    p.acc_per_thread);
        } else if (p.family == MS_FAM_DWCONV) {
            s += "reorder(i0, j0, c0, i1, j1, c1, i2, j2, c2, i3, j3, c3, kh, kw)\n";
            s += "bind(fuse(i0, j0, c0), blockIdx.x)\nbind(fuse(i2, j2, c2), threadIdx.x)\nvectorize(c3)\n";
        } else {
            s += "reorder(i0, j0, k0, i2, j2, k1, k2, k3, i1, j1, i3, j3)\n";
            if (p.reorder == 3) appendf(s, "bind(fuse(i0, j0), persistent workgroup loop, one workgroup per compute unit)\n");
            else appendf(s, "bind(fuse(%s), blockIdx.x)\n", p.reorder == 1 ? "j0, i0" : "i0, j0");
            appendf(s, "bind(fuse(i2, j2), %s)\n", p.mfma ? "wavefront" : "threadIdx.x");
        }
        if (p.family == MS_FAM_REDUCE) {
            // everything was said above
        } else {
        if (p.cache_read) {
            if (p.cache_read >= 8)
                appendf(s, "cache-read(buffers=[A, B], scope=lds, at=k0, stages=%d, prefetch_distance=%d, direct_to_lds=1)\n"
                           "annotate(block=C, key=wave_groups, value=ping_pong_on_the_ring)  # slots of k3 steps: one group reads, the other multiplies\n",
                        p.cache_read - 6, p.cache_read - 7);
            else if (p.cache_read >= 5)
                appendf(s, "cache-read(buffers=[A, B], scope=lds, at=k0, stages=%d, prefetch_distance=%d, direct_to_lds=1)\n", p.cache_read - 3, p.cache_read - 4);
            else if (p.compute_at >= 2)
                appendf(s, "%sbind(fuse(i0, j0), persistent workgroup loop over runs of consecutive tiles)\n"
                           "cache-read(buffer=W, scope=%s, compute-at=root of the tile loop, all k steps resident)\n"
                           "cache-read(buffer=X, scope=lds, compute-at=fuse(i0, j0), input rows of the tile with zero halo, prefetch_distance=%d)\n",
                        p.compute_at == 3 ? "annotate(block=C, key=helper_wavefronts, value=4)  # global loads and stores of the tile loop\n" : "",
                        p.compute_at == 4 ? "registers (through an LDS staging buffer)" : "lds", p.cache_read >= 2 ? 1 : 0);
            else if (p.compute_at)
                appendf(s, "cache-read(buffer=X, scope=lds, compute-at=fuse(i0, j0), input rows of the tile with zero halo)\n"
                           "cache-read(buffer=W, scope=lds, compute-at=k0, stages=%d, prefetch_distance=%d)\n",
                        p.cache_read >= 2 ? 2 : 1, p.cache_read == 3 ? 2 : (p.cache_read >= 2 ? 1 : 0));
            else
                appendf(s, "cache-read(buffers=[A, B], scope=lds, compute-at=k0, stages=%d, prefetch_distance=%d)\n", p.cache_read >= 2 ? 2 : 1, p.cache_read == 3 ? 2 : (p.cache_read >= 2 ? 1 : 0));
            if (p.cache_read == 4) appendf(s, "annotate(block=C, key=wave_groups, value=ping_pong)\n");
            appendf(s, "storage-align(scope=lds, pad_bytes=%d, swizzle=%d)\n", p.lds_pad ? 16 : 0, p.lds_pad == 2 || p.lds_pad == 3);
            if (p.lds_pad == 3) appendf(s, "transform-layout(buffer=B.lds, row-major k-rows, fragments through transposing LDS loads)\n");
            if (p.lds_pad == 4) appendf(s, "transform-layout(buffer=B.lds, row-major k-rows padded by 32 bytes, fragments through transposing LDS loads)\n");
        }
        if (p.cache_write) appendf(s, "cache-write(buffer=C, scope=lds%s)\n", p.cache_read >= 8 ? ", per wavefront" : "");
        if (p.rfactor > 1) appendf(s, "rfactor(loop=k0, factor=%d)  # partial sums in the workspace, second kernel adds them in order\n", p.rfactor);
        if (p.vec > 1) appendf(s, "vectorize(global loads of A, width=%d)\n", p.vec);
        if (p.vec_b > 1) appendf(s, "vectorize(global loads of B, width=%d)\n", p.vec_b);
        appendf(s, "unroll(k1, factor=%d)\nunroll(k2, factor=%d)\n", p.unroll_k1, p.unroll_k2);
        appendf(s, "# workgroup=%d threads, grid=%d, lds=%d B, acc/lane=%d\n", p.threads, p.grid[0] * p.grid[1] * p.grid[2], p.lds_bytes,
                p.acc_per_thread);
        }
    } else {
        appendf(s, "# invalid: %s\n", ms_last_error());
    }
    if (needed) *needed = s.size() + 1;
    if (buf && cap) {
        size_t n = std::min(cap - 1, s.size());
        memcpy(buf, s.data(), n);
        buf[n] = 0;
    }
    return MS_OK;
}

extern "C" int32_t ms_trace_from_text(const ms_space *space, const char *text, ms_trace *out)
{
    if (!space_ok(space) || !text || !out) return fail(MS_ERR_BAD_ARG, "ms_trace_from_text: bad argument");
    memset(out, 0, sizeof *out);
    int pos = 0;
    const char *p = text;
    while (*p) {
        const char *eol = strchr(p, '\n');
        std::string line(p, eol ? (size_t)(eol - p) : strlen(p));
        p = eol ? eol + 1 : p + line.size();
        bool cat = line.find("sample-categorical(") != std::string::npos;
        bool tile = line.find("sample-perfect-tile(") != std::string::npos;
        if (!cat && !tile) continue;
        if (pos >= space->n_slots) return fail(MS_ERR_INVALID_TRACE, "ms_trace_from_text: more sampling instructions than slots");
        const ms_slot &sl = space->slots[pos];
        if ((cat && sl.kind != MS_SLOT_CATEGORICAL) || (tile && sl.kind != MS_SLOT_PERFECT_TILE))
            return fail(MS_ERR_INVALID_TRACE, "ms_trace_from_text: instruction %d has the wrong kind for slot %s", pos, sl.name);
        std::string want = std::string("slot=") + sl.name;
        size_t at = line.find(want);
        if (at == std::string::npos || (at + want.size() < line.size() && line[at + want.size()] != ',' && line[at + want.size()] != ')'))
            return fail(MS_ERR_INVALID_TRACE, "ms_trace_from_text: instruction %d is not for slot %s", pos, sl.name);
        size_t dec = line.find("# decision:");
        if (dec == std::string::npos) return fail(MS_ERR_INVALID_TRACE, "ms_trace_from_text: instruction %d has no decision", pos);
        ms_decision &d = out->d[pos];
        d.slot_id = sl.slot_id;
        d.kind = sl.kind;
        const char *q = line.c_str() + dec + 11;
        int n = 0;
        while (*q) {
            while (*q && !(*q == '-' || (*q >= '0' && *q <= '9'))) ++q;
            if (!*q) break;
            char *end;
            long long v = strtoll(q, &end, 10);
            if (end == q) break;
            if (n >= MS_MAX_FACTORS) return fail(MS_ERR_INVALID_TRACE, "ms_trace_from_text: too many values in instruction %d", pos);
            d.v[n++] = v;
            q = end;
        }
        int expect = cat ? 1 : sl.n_factors;
        if (n != expect) return fail(MS_ERR_INVALID_TRACE, "ms_trace_from_text: instruction %d has %d values, expected %d", pos, n, expect);
        d.n = n;
        ++pos;
    }
    if (pos != space->n_slots) return fail(MS_ERR_INVALID_TRACE, "ms_trace_from_text: truncated trace: %d of %d sampling instructions", pos, space->n_slots);
    out->n = pos;
    return MS_OK;
}

// ---------------------------------------------------------------- limits / misc

extern "C" int32_t ms_get_limits(ms_limits *out)
{
    if (!out) return fail(MS_ERR_BAD_ARG, "ms_get_limits: NULL argument");
    *out = g_limits;
    return MS_OK;
}

extern "C" int32_t ms_set_limits(const ms_limits *in)
{
    if (!in || in->max_threads < 1 || in->max_lds_bytes < 0 || in->max_acc_per_thread < 1 || in->wave_size != 64 || in->max_waves < 1)
        return fail(MS_ERR_BAD_ARG, "ms_set_limits: bad limits");
    g_limits = *in;
    return MS_OK;
}

extern "C" int32_t ms_version(void) { return MS_ABI_VERSION; }
extern "C" const char *ms_last_error(void) { return ms::g_err; }
