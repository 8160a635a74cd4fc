// Trace interpreter and validator: decisions -> kernel template parameters
// (the split / reorder / bind / cache-read / unroll / vectorize / tensorize
// schedule of Table 2, applied in a fixed order per kernel family), plus the
// hardware-limit checks of the paper's "Trace validation" paragraph.
// Host only.
#include "ms_internal.h"

#include <algorithm>
#include <cinttypes>
#include <cstdio>
#include <cstring>

using namespace ms;

namespace {

struct Reject {
    int32_t code;
};

int32_t reject(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
int32_t reject(const char *fmt, ...)
{
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    return fail(MS_ERR_INVALID_TRACE, "invalid trace: %s", buf);
}

int64_t cat_value(const ms_space *sp, const ms_trace *t, int32_t slot_id, int64_t dflt)
{
    int pos;
    const ms_slot *s = find_slot(sp, slot_id, &pos);
    if (!s) return dflt;
    return s->candidates[t->d[pos].v[0]];
}

bool get_tile(const ms_space *sp, const ms_trace *t, int32_t slot_id, int32_t *f)
{
    int pos;
    const ms_slot *s = find_slot(sp, slot_id, &pos);
    if (!s) return false;
    for (int i = 0; i < 4; ++i) f[i] = (int32_t)t->d[pos].v[i];
    return true;
}

uint64_t hash_params(const ms_op *op, const ms_variant_params *p)
{
    uint64_t h = 0x243F6A8885A308D3ull;
    auto add = [&](uint64_t v) { h = mix64(h ^ mix64(v)); };
    const ms_op_desc &d = op->d;
    add((uint64_t)d.kind);
    add((uint64_t)d.in_dtype);
    add((uint64_t)d.out_dtype);
    add((uint64_t)d.stride);
    add((uint64_t)d.pad);
    if (op->pad_h != d.pad && (is_conv2d(d.kind))) add(0x1D00000000ull + (uint64_t)op->pad_h); // 1-D convolutions only
    if (is_3d(op)) {
        add(0x3D00000000ull + (uint64_t)op->depth);
        add((uint64_t)op->kd);
    }
    add((uint64_t)d.dilation);
    add((uint64_t)d.has_bias);
    add((uint64_t)d.relu);
    for (int i = 0; i < 8; ++i) add((uint64_t)d.dims[i]);
    for (int i = 0; i < 3; ++i) {
        add((uint64_t)d.a_strides[i]);
        add((uint64_t)d.b_strides[i]);
    }
    add((uint64_t)p->family);
    add((uint64_t)p->mfma);
    for (int i = 0; i < 4; ++i) {
        add((uint64_t)p->ti[i]);
        add((uint64_t)p->tj[i]);
        add((uint64_t)p->tc[i]);
        add((uint64_t)p->tk[i]);
    }
    add((uint64_t)p->cache_read);
    add((uint64_t)p->vec);
    add((uint64_t)p->vec_b);
    add((uint64_t)p->cache_write);
    add((uint64_t)p->unroll_k1); // the unroll budget itself is not part of the key: the two factors it
    add((uint64_t)p->unroll_k2); // resolves to select the code, and budgets that resolve alike give one kernel
    add((uint64_t)p->lds_pad);
    add((uint64_t)p->reorder);
    add((uint64_t)p->compute_at);
    if (p->tap_rows) add(0x7A9ull);
    if (p->rfactor > 1) add(0x4F0000ull + (uint64_t)p->rfactor);
    return h;
}

void unroll_factors(ms_variant_params *p)
{
    // budget = number of innermost iterations that may be unrolled; k3 is always unrolled
    int32_t u = p->unroll;
    int32_t k1 = p->tk[1], k2 = p->tk[2], k3 = p->tk[3];
    if (u <= 0) {
        p->unroll_k1 = 1;
        p->unroll_k2 = 1;
        return;
    }
    p->unroll_k2 = std::min(k2, std::max(1, u / k3));
    if (p->unroll_k2 == k2 && (int64_t)k2 * k3 <= u)
        p->unroll_k1 = std::min(k1, std::max(1, u / (k2 * k3)));
    else
        p->unroll_k1 = 1;
    // keep the unrolled body within the instruction cache: at most 4096
    // multiply-accumulate (or matrix-core) instructions per lane
    int64_t per_iter = (int64_t)std::max(1, p->acc_per_thread) * k3;
    if (p->mfma) per_iter = (int64_t)p->ti[1] * p->ti[3] * p->tj[1] * p->tj[3] * k3 * 16;
    while (p->unroll_k1 > 1 && per_iter * p->unroll_k2 * p->unroll_k1 > 4096) p->unroll_k1 = (p->unroll_k1 + 1) / 2;
    while (p->unroll_k2 > 1 && per_iter * p->unroll_k2 > 4096) p->unroll_k2 = (p->unroll_k2 + 1) / 2;
}

} // namespace

extern "C" int32_t ms_trace_validate(const ms_op *op, const ms_space *space, const ms_trace *trace, ms_variant_params *out)
{
    if (!op || !space || !trace) return fail(MS_ERR_BAD_ARG, "ms_trace_validate: NULL argument");
    if (space->n_slots < 1 || space->n_slots > MS_MAX_SLOTS) return fail(MS_ERR_BAD_ARG, "ms_trace_validate: bad space");
    if (trace->n != space->n_slots)
        return reject("trace has %d decisions, the space has %d sampling instructions (truncated?)", trace->n, space->n_slots);
    // well-formedness of every decision, read or not
    for (int i = 0; i < space->n_slots; ++i) {
        const ms_slot &s = space->slots[i];
        const ms_decision &d = trace->d[i];
        if (d.slot_id != s.slot_id) return reject("decision %d is for slot id %d, expected %d (%s)", i, d.slot_id, s.slot_id, s.name);
        if (d.kind != s.kind) return reject("decision %d (%s) has the wrong kind", i, s.name);
        if (s.kind == MS_SLOT_CATEGORICAL) {
            if (d.n != 1) return reject("categorical %s carries %d values", s.name, d.n);
            if (d.v[0] < 0 || d.v[0] >= s.n_candidates)
                return reject("categorical %s: index %" PRId64 " outside [0,%d)", s.name, d.v[0], s.n_candidates);
            if (s.weight[d.v[0]] <= 0) return reject("categorical %s: candidate %" PRId64 " has zero probability", s.name, d.v[0]);
        } else {
            if (d.n != s.n_factors) return reject("tile %s carries %d factors, expected %d", s.name, d.n, s.n_factors);
            int64_t e = slot_extent(space, trace, i);
            if (e < 1) return reject("tile %s: extent undefined", s.name);
            int64_t prod = 1;
            for (int f = 0; f < d.n; ++f) {
                if (d.v[f] < 1) return reject("tile %s: factor %d is %" PRId64, s.name, f, d.v[f]);
                if (d.v[f] > e) return reject("tile %s: factor %d = %" PRId64 " exceeds the extent %" PRId64, s.name, f, d.v[f], e);
                prod *= d.v[f];
                if (prod > e) break;
            }
            if (prod != e) return reject("tile %s: factors multiply to %" PRId64 ", loop extent is %" PRId64, s.name, prod, e);
        }
    }

    ms_variant_params p;
    memset(&p, 0, sizeof p);
    p.family = space->family;
    const ms_op_desc &d = op->d;
    const ms_limits &L = g_limits;
    p.unroll = (int32_t)cat_value(space, trace, MS_SLOT_UNROLL, 0);
    p.vec = (int32_t)cat_value(space, trace, MS_SLOT_VECTORIZE, 1);
    p.vec_b = (int32_t)cat_value(space, trace, MS_SLOT_VECTORIZE_B, 1);
    p.cache_write = (int32_t)cat_value(space, trace, MS_SLOT_CACHE_WRITE, 0);
    p.lds_pad = (int32_t)cat_value(space, trace, MS_SLOT_STORAGE_ALIGN, 0);
    p.tap_rows = (space->flags & MS_SPACE_TAP_ROWS) && d.kind == MS_OP_CONV2D_NHWC && op->nb == 1 && !is_3d(op) && d.dilation == 1 ? 1 : 0;
    p.reorder = (int32_t)cat_value(space, trace, MS_SLOT_REORDER, 0);
    p.compute_at = (int32_t)cat_value(space, trace, MS_SLOT_COMPUTE_AT, 0);
    p.rfactor = (int32_t)cat_value(space, trace, MS_SLOT_RFACTOR, 1);

    if (space->family == MS_FAM_GEMM_ALU || space->family == MS_FAM_GEMM_MFMA) {
        if (!get_tile(space, trace, MS_SLOT_TILE_I, p.ti) || !get_tile(space, trace, MS_SLOT_TILE_J, p.tj) ||
            !get_tile(space, trace, MS_SLOT_TILE_K, p.tk))
            return fail(MS_ERR_BAD_ARG, "ms_trace_validate: the space lacks a tile slot");
        p.cache_read = (int32_t)cat_value(space, trace, MS_SLOT_CACHE_READ, 1);
        int es = op->in_size;
        if (space->family == MS_FAM_GEMM_ALU) {
            p.mfma = MS_MFMA_NONE;
            p.tile_unit[0] = p.tile_unit[1] = p.tile_unit[2] = 1;
        } else {
            p.mfma = (int32_t)cat_value(space, trace, MS_SLOT_TENSORIZE, 0);
            mfma_dims(p.mfma, &p.tile_unit[0], &p.tile_unit[1], &p.tile_unit[2]);
            if (p.tile_unit[0] != p.tile_unit[1] || (p.tile_unit[0] != 16 && p.tile_unit[0] != 32))
                return reject("tensorize: unknown intrinsic %d", p.mfma);
        }
        int64_t bm = (int64_t)p.ti[1] * p.ti[2] * p.ti[3] * p.tile_unit[0];
        int64_t bn = (int64_t)p.tj[1] * p.tj[2] * p.tj[3] * p.tile_unit[1];
        int64_t bk = (int64_t)p.tk[1] * p.tk[2] * p.tk[3] * p.tile_unit[2];
        if (bm > 4096 || bn > 4096 || bk > 4096) return reject("workgroup tile %" PRId64 "x%" PRId64 "x%" PRId64 " is beyond any register/LDS budget", bm, bn, bk);
        p.block_m = (int32_t)bm;
        p.block_n = (int32_t)bn;
        p.block_k = (int32_t)bk;
        int64_t g = (int64_t)p.ti[0] * p.tj[0];
        if (g > 0x7fffffff / std::max<int64_t>(1, op->nb)) return reject("grid of %" PRId64 " workgroups overflows", g);
        p.grid[0] = (int32_t)g;
        p.grid[1] = 1;
        p.grid[2] = (int32_t)op->nb;
        int64_t units = (int64_t)p.ti[2] * p.tj[2];
        int64_t acc;
        if (p.mfma) {
            // conv2d with helper wavefronts (compute_at 3): four more, one per SIMD, that only move data
            if (p.compute_at == 3) units += 4;
            if (units > L.max_waves) return reject("%" PRId64 " wavefronts per workgroup, the limit is %d", units, L.max_waves);
            p.waves = (int32_t)units;
            p.threads = p.waves * L.wave_size;
            acc = (int64_t)p.ti[1] * p.ti[3] * p.tj[1] * p.tj[3] * (p.tile_unit[0] * p.tile_unit[1] / L.wave_size);
        } else {
            if (units > L.max_threads) return reject("%" PRId64 " threads per workgroup, the limit is %d", units, L.max_threads);
            p.threads = (int32_t)units;
            p.waves = (p.threads + L.wave_size - 1) / L.wave_size;
            acc = (int64_t)p.ti[1] * p.ti[3] * p.tj[1] * p.tj[3];
        }
        if (p.threads > L.max_threads) return reject("%d threads per workgroup, the limit is %d", p.threads, L.max_threads);
        if (acc > L.max_acc_per_thread) return reject("%" PRId64 " accumulators per lane, the register budget is %d", acc, L.max_acc_per_thread);
        p.acc_per_thread = (int32_t)acc;
        unroll_factors(&p);
        // cache-read: LDS footprint
        int64_t lds = 0;
        if (p.mfma) {
            int kp = p.tile_unit[2] / (L.wave_size / p.tile_unit[0]); // k elements one lane feeds per intrinsic
            int64_t padb = p.lds_pad ? 16 : 0;
            // fragments of more than 16 bytes lie in LDS as 16-byte halves, each in a (padded) plane of its own
            const int split = kp * es > 16 ? kp * es / 16 : 1;
            int64_t rowsA = split * (bm * (kp / split) * es + padb), rowsB = split * (bn * (kp / split) * es + padb);
            lds = (int64_t)(p.cache_read >= 2 ? 2 : 1) * (bk / kp) * (rowsA + rowsB);
            if (p.lds_pad == 3 || p.lds_pad == 4) {
                // B row-major in LDS (dense k-rows of bn elements, granules swizzled), fragments through the transposing loads
                if (is_conv2d(d.kind) || !(d.b_strides[2] == 1 && d.b_strides[1] != 1)) return reject("storage_align 3, 4 (row-major B in LDS) is for GEMMs whose B is contiguous along j");
                if (!((es == 2 && (kp == 4 || kp == 8)) || (es == 1 && (kp == 8 || kp == 16 || kp == 32))))
                    return reject("storage_align 3, 4 needs fragments of whole transposing loads: 4 or 8 k per lane of 2-byte, 8, 16 or 32 k per lane of 1-byte inputs");
                if (p.cache_read < 1 || p.cache_read > 4) return reject("storage_align 3, 4 applies to register staging (cache_read 1..4)");
                if (p.vec_b * es != 16) return reject("storage_align 3, 4 moves B in 16-byte vectors: vectorize_b must be %d", 16 / es);
                if (d.b_strides[1] % (16 / es) || d.b_strides[0] % (16 / es)) return reject("storage_align 3, 4 needs 16-byte aligned rows of B");
                // 4: rows of B padded by 32 bytes instead of swizzled
                lds = (int64_t)(p.cache_read >= 2 ? 2 : 1) * ((bk / kp) * rowsA + bk * (bn * es + (p.lds_pad == 4 ? 32 : 0)));
            }
            if (p.cache_read >= 5) {
                // direct-to-LDS ring: dense tiles, no padding (the swizzle replaces it)
                const int ce = 16 / es; // elements per 16-byte chunk
                if (!((es == 2 && kp == 8) || (es == 1 && kp == 16)))
                    return reject("direct-to-LDS staging needs 16-byte fragments: 2-byte inputs with 8 k per lane or 1-byte inputs with 16 k per lane");
                if (bk * es != 64 && bk * es != 128 && bk * es != 256) return reject("direct-to-LDS staging needs a k tile of 64, 128 or 256 bytes, not %" PRId64, bk * es);
                if (d.a_strides[2] != 1 || d.a_strides[1] % ce || d.a_strides[0] % ce) return reject("direct-to-LDS staging needs 16-byte aligned rows of A");
                if (d.b_strides[1] == 1 && d.b_strides[2] != 1) {
                    if (d.b_strides[2] % ce || d.b_strides[0] % ce) return reject("direct-to-LDS staging needs 16-byte aligned rows of B");
                } else if (d.b_strides[2] == 1) {
                    if (d.b_strides[1] % ce || d.b_strides[0] % ce) return reject("direct-to-LDS staging needs 16-byte aligned rows of B");
                    if (bn % 16) return reject("direct-to-LDS staging reads B in groups of 16 columns");
                } else {
                    return reject("direct-to-LDS staging needs B contiguous along k or j");
                }
                if (p.lds_pad) return reject("direct-to-LDS staging has its own swizzle: storage_align must be 0");
                // the j-contiguous B tile is rounded up to whole 1 KiB load instructions
                int64_t btile = d.b_strides[2] == 1 ? ((bk * (bn / ce) + 63) / 64) * 1024 : bn * bk * es;
                const int stages = p.cache_read >= 8 ? p.cache_read - 6 : p.cache_read - 3;
                lds = (int64_t)stages * (bm * bk * es + btile);
                if (p.cache_read >= 8) {
                    // ping-pong on the ring: two groups of wavefronts one phase apart under persistent workgroups
                    if (p.reorder != 3) return reject("ping-pong on the ring (cache_read 8, 9, 10) runs under persistent workgroups: reorder must be 3");
                    if (p.waves % 2) return reject("ping-pong on the ring needs an even number of wavefronts, not %d", p.waves);
                    if (p.tk[1] != 1) return reject("ping-pong on the ring: a k0 step is k2 slots of k3 intrinsic steps, k1 must be 1");
                    // a slot's fragments and the accumulators are all live; 64 more registers hold the LDS addresses of the
                    // fragments, the load offsets and the epilogue's temporaries (what the compiler needed for a
                    // 128 x 64 wave tile: 247 registers with 128 accumulators and 48 fragment registers)
                    const int64_t fr = kp * es / 4 > 0 ? kp * es / 4 : 1;
                    const int64_t fragr = ((int64_t)p.ti[1] * p.ti[3] + (int64_t)p.tj[1] * p.tj[3]) * p.tk[3] * fr;
                    const int64_t have = 512 / ((p.waves + 3) / 4);
                    if (fragr + acc + 64 > have)
                        return reject("ping-pong on the ring: %" PRId64 " fragment + %" PRId64 " accumulator + 64 other registers per lane exceed the %" PRId64
                                      " a wavefront can have", fragr, acc, have);
                    // the k2 slots are always unrolled, whatever the budget: one kernel, one key
                    p.unroll_k1 = 1;
                    p.unroll_k2 = p.tk[2];
                }
            }
            if (is_conv2d(d.kind) && op->K % p.tile_unit[2] && !p.tap_rows) {
                // the k split covers the reduction rounded up to the intrinsic's k; only the im2col loader pads with zeros
                if (p.compute_at) return reject("KH*KW*Cin = %" PRId64 " is not a multiple of the intrinsic's k = %d: compute_at must be 0", op->K, p.tile_unit[2]);
                if (p.cache_read >= 5) return reject("a padded reduction cannot be staged directly to LDS");
            }
            if (is_3d(op) && p.compute_at) return reject("3-D convolution: compute_at must be 0 (the resident patch is a set of image rows)");
            if (p.tap_rows) {
                // the reduction as KH runs of KW * Cin contiguous elements, each rounded up to the intrinsic's k
                if (p.cache_read >= 5) return reject("filter-row layout: no direct-to-LDS staging");
                if (p.compute_at >= 1 && (d.stride * d.dims[3] * es) % 4) return reject("filter-row layout with a resident patch: pixels of an output row must start at multiples of 4 bytes");
            }
            if (p.compute_at) {
                // conv2d with the activations' cache-read under the workgroup tile loop: the input rows of
                // the tile (zero halo included) are resident, only the weights are staged per k step
                if (!is_conv2d(d.kind)) return reject("compute_location applies to conv2d only");
                if (p.compute_at == 1 && p.cache_read > 3) return reject("with the input patch resident only the weights are staged per k step: cache_read 1, 2 or 3");
                if (p.compute_at == 2 && p.cache_read > 2) return reject("with resident weights cache_read is 1 (patch loaded between tiles) or 2 (next patch prefetched)");
                if (p.compute_at == 3 && (p.cache_read != 2 || !p.cache_write))
                    return reject("helper wavefronts prefetch the patch and write the staged tile: cache_read 2 and cache_write 1");
                if (p.compute_at >= 2 && p.reorder != 0) return reject("persistent workgroups with resident weights walk the tile list in order: reorder must be 0");
                int64_t cin = d.dims[3] / op->nb, ohw = op->OH * op->OW; // channels of one group
                if (cin % p.tile_unit[2] && !p.tap_rows) return reject("resident input patch: Cin = %" PRId64 " is not a multiple of the intrinsic's k = %d", cin, p.tile_unit[2]);
                if (ohw % bm) return reject("resident input patch: the %" PRId64 "-pixel tile straddles images of %" PRId64 " output pixels", bm, ohw);
                int64_t rows = bm % op->OW == 0 ? bm / op->OW : (op->OW + bm - 2) / op->OW + 1;
                int64_t pr = (rows - 1) * d.stride + d.dilation * (d.dims[5] - 1) + 1, pw = (op->OW - 1) * d.stride + d.dilation * (d.dims[6] - 1) + 1;
                int64_t ps = cin * es + (p.lds_pad ? 16 : 0);
                if (p.tap_rows) {
                    // dense pixels (a run crosses pixel boundaries), and the pixels that the padding of the last run reads
                    const int64_t run = d.dims[6] * cin, kr = (run + p.tile_unit[2] - 1) / p.tile_unit[2] * p.tile_unit[2];
                    ps = cin * es;
                    pw += (kr - run + cin - 1) / cin;
                    if ((pw * ps) % 4) pw += 1; // rows start at multiples of 4 bytes (2-byte elements, odd Cin)
                }
                int64_t patch = pr * pw * ps;
                lds = (int64_t)(p.cache_read >= 2 ? 2 : 1) * (bk / kp) * rowsB + patch;
                if (p.compute_at >= 2) lds = (int64_t)p.tk[0] * (bk / kp) * rowsB + patch; // all k steps of the weights
                if (p.compute_at == 4) {
                    // weights in registers: LDS holds one k step of them as a staging buffer
                    lds = (bk / kp) * rowsB + patch;
                    if (p.cache_read > 2) return reject("with the weights in registers cache_read is 1 (patch loaded between tiles) or 2 (next patch prefetched)");
                }
                if ((cin * es) % 16 && p.lds_pad && !p.tap_rows) return reject("resident input patch: padded pixels need Cin * element size to be a multiple of 16 bytes");
                if (d.dims[0] * d.dims[1] * d.dims[2] * d.dims[3] > 0x7fffffff / es) return reject("resident input patch: one instance of X exceeds 32-bit byte offsets");
            }
            if (p.reorder == 3 && p.cache_read < 5) return reject("persistent workgroups (reorder 3) are built on direct-to-LDS staging (cache_read 5, 6, 7)");
            if (p.rfactor > 1) {
                // the reduction of one output tile shared by rfactor workgroups: whole runs of k0 steps each
                if (p.tk[0] % p.rfactor) return reject("rfactor %d does not divide the %d steps of the k0 loop", p.rfactor, p.tk[0]);
                if (p.reorder == 3 || p.compute_at >= 2) return reject("persistent workgroups own the whole reduction of their tiles: rfactor must be 1");
                if (p.cache_write) return reject("rfactor writes partial sums straight from the accumulators: cache_write must be 0");
                if (g * p.rfactor > 0x7fffffff / std::max<int64_t>(1, op->nb)) return reject("grid of %" PRId64 " workgroups overflows", g * p.rfactor);
                p.grid[0] = (int32_t)(g * p.rfactor);
            }
            if (p.cache_write) {
                // the output tile reuses the operand buffers: rows of bn outputs padded by 16 bytes
                int64_t ctile = bm * (bn * op->out_size + 16);
                if (p.cache_read >= 8) {
                    // one staging area per wavefront: the rows of one intrinsic tile across the wavefront's j3 adjacent tiles
                    const int64_t wrow = (int64_t)p.tj[3] * p.tile_unit[1] * op->out_size;
                    if (wrow % 16) return reject("cache_write on the ring: a wavefront's staged rows of %" PRId64 " bytes are not whole 16-byte chunks", wrow);
                    lds += (int64_t)p.waves * p.tile_unit[0] * wrow;
                } else if (p.reorder == 3 || p.compute_at >= 2) lds += ctile; // persistent workgroups keep their operands alive during the epilogue
                else if (ctile > lds) lds = ctile;
                if ((op->N * op->out_size) % 16) return reject("cache_write needs output rows that are multiples of 16 bytes");
            }
            // fragment operands of one k step for the whole wave tile live in registers too
            int64_t frag = ((int64_t)p.ti[1] * p.ti[3] + (int64_t)p.tj[1] * p.tj[3]) * p.tk[3] * (kp * es / 4 > 0 ? kp * es / 4 : 1);
            // registers that carry a tile from global memory to LDS; with two buffers they are live across the k step
            int64_t stage = (bm * bk * es / 4 + p.threads - 1) / p.threads + (bn * bk * es / 4 + p.threads - 1) / p.threads;
            if (p.cache_read >= 5) stage = 0;
            if (p.compute_at) stage = (bn * bk * es / 4 + p.threads - 1) / p.threads;
            if (p.compute_at == 3) {
                // only the helpers carry the patch, over 256 lanes
                int64_t rows = bm % op->OW == 0 ? bm / op->OW : (op->OW + bm - 2) / op->OW + 1;
                int64_t pr = (rows - 1) * d.stride + d.dilation * (d.dims[5] - 1) + 1, pw = (op->OW - 1) * d.stride + d.dilation * (d.dims[6] - 1) + 1;
                stage = std::max(stage, (pr * pw * d.dims[3] * es / 4 + 255) / 256);
            }
            if (p.compute_at == 2 && p.cache_read == 2) {
                // the next tile's patch waits in registers during the k loop
                int64_t rows = bm % op->OW == 0 ? bm / op->OW : (op->OW + bm - 2) / op->OW + 1;
                int64_t pr = (rows - 1) * d.stride + d.dilation * (d.dims[5] - 1) + 1, pw = (op->OW - 1) * d.stride + d.dilation * (d.dims[6] - 1) + 1;
                stage = std::max(stage, (pr * pw * d.dims[3] * es / 4 + p.threads - 1) / p.threads);
            }
            int64_t live = p.cache_read == 3 ? frag + 2 * stage : (p.cache_read >= 2 ? frag + stage : std::max(frag, stage));
            if (p.compute_at == 4) {
                // weight fragments of the wavefront's columns for every k step, A fragments of two steps
                int64_t fr = kp * es / 4 > 0 ? kp * es / 4 : 1;
                int64_t breg = (int64_t)p.tj[1] * p.tj[3] * ((int64_t)p.tk[0] * p.tk[1] * p.tk[2] * p.tk[3]) * fr; // every MFMA k step of the reduction
                int64_t areg = 2 * (int64_t)p.ti[1] * p.ti[3] * fr;
                int64_t pre = 0;
                if (p.cache_read == 2) {
                    int64_t rows = bm % op->OW == 0 ? bm / op->OW : (op->OW + bm - 2) / op->OW + 1;
                    int64_t pr = (rows - 1) * d.stride + d.dilation * (d.dims[5] - 1) + 1, pw = (op->OW - 1) * d.stride + d.dilation * (d.dims[6] - 1) + 1;
                    pre = (pr * pw * d.dims[3] * es / 4 + p.threads - 1) / p.threads;
                }
                int64_t have = 512 / ((p.waves + 3) / 4);
                if (breg + areg + pre + acc + 24 > have)
                    return reject("weights in registers: %" PRId64 " weight + %" PRId64 " operand + %" PRId64 " prefetch + %" PRId64
                                  " accumulator registers per lane exceed the %" PRId64 " a wavefront can have", breg, areg, pre, acc, have);
                frag = 0; // accounted for above
                stage = 0;
                live = 0;
            }
            if (p.cache_read == 4) {
                if (p.waves % 2) return reject("ping-pong wave groups need an even number of wavefronts, not %d", p.waves);
                if (p.tk[1] != 1 || p.tk[2] != 1) return reject("ping-pong wave groups need k1 = k2 = 1 (a tile's fragments are read in one phase)");
            }
            // a SIMD's 512 registers per lane are shared by the workgroup's wavefronts resident on it
            int64_t budget = 512 / ((p.waves + 3) / 4);
            // only the ping-pong schedule needs every fragment of a tile live at once; elsewhere the
            // compiler sequences the fragment reads, so the estimate is allowed to overshoot by half
            if (p.cache_read != 4) budget += budget / 2;
            if (live + acc > budget)
                return reject("%" PRId64 " fragment + %" PRId64 " staging + %" PRId64 " accumulator registers per lane exceed the %" PRId64
                              " a wavefront can have with %d wavefronts per workgroup", frag, stage, acc, budget, p.waves);
        } else if (p.cache_read) {
            int stages = p.cache_read;
            lds = (int64_t)stages * 4 * (bm * (bk + (p.lds_pad ? 4 : 0)) + bk * (bn + (p.lds_pad ? 4 : 0)));
            int64_t frag = ((int64_t)p.ti[1] * p.ti[3] + (int64_t)p.tj[1] * p.tj[3]) * p.tk[3];
            if (frag + acc > 448) return reject("%" PRId64 " operand + %" PRId64 " accumulator registers per lane exceed the register file", frag, acc);
        } else {
            if (p.lds_pad) return reject("storage_align without cache_read has nothing to pad");
            int64_t frag = ((int64_t)p.ti[1] * p.ti[3] + (int64_t)p.tj[1] * p.tj[3]) * p.tk[3];
            if (frag + acc > 448) return reject("%" PRId64 " operand + %" PRId64 " accumulator registers per lane exceed the register file", frag, acc);
        }
        if (lds > L.max_lds_bytes) return reject("LDS tile needs %" PRId64 " bytes, the limit is %d", lds, L.max_lds_bytes);
        p.lds_bytes = (int32_t)lds;
        // vectorize: alignment and divisibility of the global loads, per operand
        if (p.vec > 1) {
            int v = p.vec;
            if (v * es > 16) return reject("vector of %d x %d bytes is wider than a 16-byte load", v, es);
            if (is_conv2d(d.kind)) {
                if ((d.dims[3] / op->nb) % v) return reject("vector width %d does not divide Cin = %" PRId64 " (per group)", v, d.dims[3] / op->nb);
                if (bk % v) return reject("vector width %d does not divide the k tile %" PRId64, v, bk);
            } else {
                if (d.a_strides[2] != 1) return reject("vector loads of A need k contiguous");
                if (bk % v || d.a_strides[1] % v || (op->nb > 1 && d.a_strides[0] % v))
                    return reject("vector width %d breaks alignment of A (k tile %" PRId64 ", row stride %" PRId64 ")", v, bk, d.a_strides[1]);
            }
        }
        if (p.vec_b > 1) {
            int v = p.vec_b;
            if (v * es > 16) return reject("vector of %d x %d bytes is wider than a 16-byte load", v, es);
            if (is_conv2d(d.kind)) {
                if (op->N % v) return reject("vector width %d does not divide Cout = %" PRId64 " (per group)", v, op->N);
                if (bn % v) return reject("vector width %d does not divide the j tile %" PRId64, v, bn);
            } else if (d.b_strides[2] == 1) { // vector along j
                if (bn % v || d.b_strides[1] % v || (op->nb > 1 && d.b_strides[0] % v))
                    return reject("vector width %d breaks alignment of B (j tile %" PRId64 ", row stride %" PRId64 ")", v, bn, d.b_strides[1]);
            } else if (d.b_strides[1] == 1) { // vector along k
                if (bk % v || d.b_strides[2] % v || (op->nb > 1 && d.b_strides[0] % v))
                    return reject("vector width %d breaks alignment of B (k tile %" PRId64 ", column stride %" PRId64 ")", v, bk, d.b_strides[2]);
            } else {
                return reject("vector loads of B need j or k contiguous");
            }
        }
    } else if (space->family == MS_FAM_DWCONV) {
        if (!get_tile(space, trace, MS_SLOT_TILE_I, p.ti) || !get_tile(space, trace, MS_SLOT_TILE_J, p.tj) ||
            !get_tile(space, trace, MS_SLOT_TILE_C, p.tc))
            return fail(MS_ERR_BAD_ARG, "ms_trace_validate: the space lacks a tile slot");
        p.cache_read = (int32_t)cat_value(space, trace, MS_SLOT_CACHE_READ, 0);
        p.tile_unit[0] = p.tile_unit[1] = p.tile_unit[2] = 1;
        int64_t boh = (int64_t)p.ti[1] * p.ti[2] * p.ti[3], bow = (int64_t)p.tj[1] * p.tj[2] * p.tj[3],
                bc = (int64_t)p.tc[1] * p.tc[2] * p.tc[3];
        p.block_m = (int32_t)boh;
        p.block_n = (int32_t)bow;
        p.block_k = (int32_t)bc;
        int64_t threads = (int64_t)p.ti[2] * p.tj[2] * p.tc[2];
        if (threads > L.max_threads) return reject("%" PRId64 " threads per workgroup, the limit is %d", threads, L.max_threads);
        p.threads = (int32_t)threads;
        p.waves = (p.threads + L.wave_size - 1) / L.wave_size;
        // registers of one thread: the I3 x J3 output patch, its input patch and the taps, VC channels each
        int vc = p.tc[3] % 4 == 0 ? 4 : (p.tc[3] % 2 == 0 ? 2 : 1);
        int64_t patch_h = (int64_t)(p.ti[3] - 1) * d.stride + d.dims[4], patch_w = (int64_t)(p.tj[3] - 1) * d.stride + d.dims[5];
        int64_t acc = (int64_t)p.ti[3] * p.tj[3] * vc;
        int64_t regs = acc + (patch_h * patch_w + d.dims[4] * d.dims[5]) * vc;
        if (regs > L.max_acc_per_thread) return reject("%" PRId64 " registers for the output and input patch exceed the register budget %d", regs, L.max_acc_per_thread);
        p.acc_per_thread = (int32_t)acc;
        int64_t g = (int64_t)p.ti[0] * p.tj[0] * p.tc[0];
        if (g > 0x7fffffff / std::max<int64_t>(1, d.dims[0])) return reject("grid of %" PRId64 " workgroups overflows", g);
        p.grid[0] = (int32_t)g;
        p.grid[1] = 1;
        p.grid[2] = (int32_t)d.dims[0];
        p.vec = vc;
        if (p.cache_read) {
            int64_t ih = (boh - 1) * d.stride + d.dims[4], iw = (bow - 1) * d.stride + d.dims[5];
            int64_t lds = ih * iw * bc * 4;
            if (lds > L.max_lds_bytes) return reject("LDS halo tile needs %" PRId64 " bytes, the limit is %d", lds, L.max_lds_bytes);
            p.lds_bytes = (int32_t)lds;
        }
        p.tk[0] = 1;
        p.tk[1] = (int32_t)d.dims[4];
        p.tk[2] = (int32_t)d.dims[5];
        p.tk[3] = 1;
        p.unroll_k1 = p.unroll_k2 = p.unroll > 0 ? 0 : 1; // 0 = full unroll of the tap loops
    } else if (space->family == MS_FAM_REDUCE) {
        if (!get_tile(space, trace, MS_SLOT_TILE_I, p.ti) || !get_tile(space, trace, MS_SLOT_TILE_K, p.tk))
            return fail(MS_ERR_BAD_ARG, "ms_trace_validate: the space lacks a tile slot");
        p.cache_read = (int32_t)cat_value(space, trace, MS_SLOT_CACHE_READ, 0);
        if (d.kind == MS_OP_NORM) p.cache_read = 0; // a single pass anyway
        p.tile_unit[0] = p.tile_unit[1] = p.tile_unit[2] = 1;
        const int es = op->in_size;
        const int64_t k0 = p.tk[0], k1 = p.tk[1], k2 = p.tk[2], k3 = p.tk[3];
        if (k3 * es > 16 || (k3 & (k3 - 1))) return reject("vector of %" PRId64 " elements: a load moves 1, 2, 4, ... elements and at most 16 bytes", k3);
        if (op->out_size * k3 > 16) return reject("vector of %" PRId64 " output elements exceeds 16 bytes", k3);
        if (k2 > L.max_threads || (k2 & (k2 - 1))) return reject("%" PRId64 " lanes per row: the cross-thread reduction needs a power of two up to %d", k2, L.max_threads);
        if (d.kind == MS_OP_NORM && k2 < 64 && op->K > 4096)
            return reject("%" PRId64 " lanes would each sum %" PRId64 " squares in one fp32 chain; at least one wavefront per row", k2, op->K / k2);
        int64_t threads = (int64_t)p.ti[2] * k2;
        if (threads > L.max_threads) return reject("%" PRId64 " threads per workgroup, the limit is %d", threads, L.max_threads);
        if (threads % L.wave_size) return reject("%" PRId64 " threads per workgroup is not a whole number of wavefronts", threads);
        p.threads = (int32_t)threads;
        p.waves = p.threads / L.wave_size;
        if (k1 > 64) return reject("%" PRId64 " loads in flight per lane", k1);
        // values a lane holds at once: the rows of its group that are processed together, all of the lane's
        // share of them when the row stays in registers between the passes
        int64_t live = (int64_t)p.ti[3] * k1 * k3 * (p.cache_read ? k0 : 1);
        const int budget = std::min(L.max_acc_per_thread, 128); // the loaded vectors and the exponentials are live together
        if (live > budget) return reject("%" PRId64 " values per lane exceed the register budget %d", live, budget);
        if (p.cache_read && k0 * k1 > 64) return reject("%" PRId64 " loads per lane and row in a fully unrolled pass", k0 * k1);
        p.acc_per_thread = (int32_t)live;
        p.block_m = (int32_t)std::min<int64_t>((int64_t)p.ti[1] * p.ti[2] * p.ti[3], 0x7fffffff);
        p.block_n = 1;
        p.block_k = (int32_t)std::min<int64_t>(op->K, 0x7fffffff);
        p.vec = (int32_t)k3;
        p.grid[0] = p.ti[0];
        p.grid[1] = 1;
        p.grid[2] = 1;
        // partial results of the wavefronts of a group meet in LDS (maximum and sum use it in turn)
        p.lds_bytes = k2 > L.wave_size ? (int32_t)(p.waves * p.ti[3] * 4) : 0;
        p.unroll_k1 = (int32_t)k1;
        p.unroll_k2 = 1;
    } else {
        return fail(MS_ERR_BAD_ARG, "ms_trace_validate: unknown family %d", space->family);
    }
    p.key = hash_params(op, &p);
    if (out) *out = p;
    return MS_OK;
}

namespace ms {

static std::string def(const char *name, int64_t v)
{
    char buf[96];
    snprintf(buf, sizeof buf, "-D%s=%" PRId64, name, v);
    return buf;
}

static int dt_code(int32_t dt) { return dt; }

int32_t make_kernel_spec(const ms_op *op, const ms_variant_params *p, KernelSpec *out)
{
    const ms_op_desc &d = op->d;
    KernelSpec k;
    k.entry = "ms_kernel";
    k.block[0] = (unsigned)p->threads;
    k.block[1] = k.block[2] = 1;
    k.grid[0] = (unsigned)p->grid[0];
    k.grid[1] = (unsigned)p->grid[1];
    k.grid[2] = (unsigned)p->grid[2];
    k.lds_dynamic = 0;
    auto &D = k.defines;
    D.push_back(def("IN_DT", dt_code(d.in_dtype)));
    D.push_back(def("OUT_DT", dt_code(d.out_dtype)));
    const char *tn[4] = {"I", "J", "C", "K"};
    const int32_t *tl[4] = {p->ti, p->tj, p->tc, p->tk};
    for (int l = 0; l < 4; ++l)
        for (int f = 0; f < 4; ++f) {
            char nm[8];
            snprintf(nm, sizeof nm, "%s%d", tn[l], f);
            D.push_back(def(nm, tl[l][f] ? tl[l][f] : 1));
        }
    D.push_back(def("NTHREADS", p->threads));
    D.push_back(def("CACHE_READ", p->cache_read));
    D.push_back(def("VEC", p->vec));
    D.push_back(def("VEC_B", p->vec_b > 0 ? p->vec_b : 1));
    D.push_back(def("CACHE_WRITE", p->cache_write));
    D.push_back(def("UNROLL_K1", p->unroll_k1));
    D.push_back(def("UNROLL_K2", p->unroll_k2));
    D.push_back(def("LDS_PAD", p->lds_pad));
    D.push_back(def("REORDER", p->reorder));
    D.push_back(def("COMPUTE_AT", p->compute_at));
    D.push_back(def("HELPER_WAVES", p->compute_at == 3 ? 4 : 0));
    D.push_back(def("RFACTOR", p->rfactor > 1 ? p->rfactor : 1));
    if (p->family == MS_FAM_GEMM_ALU || p->family == MS_FAM_GEMM_MFMA) {
        D.push_back(def("DIM_B", op->nb));
        D.push_back(def("DIM_M", op->M));
        D.push_back(def("DIM_N", op->N));
        D.push_back(def("DIM_K", op->K));
        bool conv = is_conv2d(d.kind);
        D.push_back(def("IS_CONV", conv ? 1 : 0));
        if (conv) {
            D.push_back(def("CV_N", d.dims[0]));
            D.push_back(def("CV_H", d.dims[1]));
            D.push_back(def("CV_W", d.dims[2]));
            D.push_back(def("CV_CIN", d.dims[3] / op->nb)); // channels a group reduces over
            D.push_back(def("CV_XC", d.dims[3]));           // channels per pixel of X
            D.push_back(def("CV_COUT", d.dims[4]));
            D.push_back(def("LDC", d.dims[4]));             // output channels per pixel of Y = bias values per instance
            D.push_back(def("C_BATCH", op->N));             // a group's outputs start op->N channels after the previous group's
            D.push_back(def("CV_KH", d.dims[5]));
            D.push_back(def("CV_KW", d.dims[6]));
            D.push_back(def("CV_OH", op->OH));
            D.push_back(def("CV_OW", op->OW));
            D.push_back(def("CV_STRIDE", d.stride));
            D.push_back(def("CV_PAD", d.pad));
            D.push_back(def("CV_PAD_H", op->pad_h));
            D.push_back(def("CV_D", op->depth));
            D.push_back(def("CV_KD", op->kd));
            D.push_back(def("CV_OD", op->OD));
            D.push_back(def("CV_DIL", d.dilation));
            D.push_back(def("CV_TRANSPOSED", d.kind == MS_OP_CONV2D_TRANSPOSED_NHWC ? 1 : 0));
            D.push_back(def("CV_TAPROWS", p->tap_rows));
            D.push_back(def("CV_KR", (d.dims[6] * d.dims[3] + p->tile_unit[2] - 1) / p->tile_unit[2] * p->tile_unit[2]));
            D.push_back(def("HAS_BIAS", d.has_bias ? 1 : 0));
            D.push_back(def("RELU", d.relu ? 1 : 0));
            // implicit GEMM view: A rows are output pixels, B = W as [K][N]
            D.push_back(def("SA_B", d.dims[3] / op->nb)); // channel offset of a group
            D.push_back(def("SA_I", 0));
            D.push_back(def("SA_K", 1));
            D.push_back(def("SB_B", op->N));              // column offset of a group in W [K][Cout]
            D.push_back(def("SB_K", d.dims[4]));
            D.push_back(def("SB_J", 1));
            D.push_back(def("A_INST", d.dims[0] * op->depth * d.dims[1] * d.dims[2] * d.dims[3]));
            D.push_back(def("B_INST", op->K * op->N * op->nb));
        } else {
            D.push_back(def("HAS_BIAS", 0));
            D.push_back(def("RELU", 0));
            D.push_back(def("SA_B", d.a_strides[0]));
            D.push_back(def("SA_I", d.a_strides[1]));
            D.push_back(def("SA_K", d.a_strides[2]));
            D.push_back(def("SB_B", d.b_strides[0]));
            D.push_back(def("SB_K", d.b_strides[1]));
            D.push_back(def("SB_J", d.b_strides[2]));
            int64_t ab, bb;
            ms_op_tensor_bytes(op, 0, &ab);
            ms_op_tensor_bytes(op, 1, &bb);
            D.push_back(def("A_INST", ab / op->in_size));
            D.push_back(def("B_INST", bb / op->in_size));
        }
        if (p->family == MS_FAM_GEMM_MFMA) {
            k.template_name = "gemm_mfma.hip";
            D.push_back(def("MI_M", p->tile_unit[0]));
            D.push_back(def("MI_N", p->tile_unit[1]));
            D.push_back(def("MI_K", p->tile_unit[2]));
        } else {
            k.template_name = "gemm_alu.hip";
        }
    } else if (p->family == MS_FAM_REDUCE) {
        k.template_name = "reduce.hip";
        D.push_back(def("RD_OP", d.kind == MS_OP_NORM ? 1 : 0));
        D.push_back(def("RD_ROWS", op->M));
        D.push_back(def("RD_LEN", op->K));
    } else {
        k.template_name = "dwconv.hip";
        D.push_back(def("CV_N", d.dims[0]));
        D.push_back(def("CV_H", d.dims[1]));
        D.push_back(def("CV_W", d.dims[2]));
        D.push_back(def("CV_C", d.dims[3]));
        D.push_back(def("CV_KH", d.dims[4]));
        D.push_back(def("CV_KW", d.dims[5]));
        D.push_back(def("CV_OH", op->OH));
        D.push_back(def("CV_OW", op->OW));
        D.push_back(def("CV_STRIDE", d.stride));
        D.push_back(def("CV_PAD", d.pad));
    }
    *out = k;
    return MS_OK;
}

} // namespace ms

extern "C" int32_t ms_variant_kernel_text(const ms_op *op, const ms_variant_params *p, char *buf, size_t cap, size_t *needed)
{
    if (!op || !p) return fail(MS_ERR_BAD_ARG, "ms_variant_kernel_text: NULL argument");
    KernelSpec k;
    int32_t rc = make_kernel_spec(op, p, &k);
    if (rc != MS_OK) return rc;
    std::string s = k.template_name + "\n";
    for (auto &d : k.defines) s += d + "\n";
    if (needed) *needed = s.size() + 1;
    if (buf && cap) {
        size_t n = std::min(cap - 1, s.size());
        memcpy(buf, s.data(), n);
        buf[n] = 0;
    }
    return MS_OK;
}

// Index of the four-level split: ((x0*f1 + x1)*f2 + x2)*f3 + x3.
static inline int64_t split_index(const int32_t *f, int64_t x0, int64_t x1, int64_t x2, int64_t x3)
{
    return ((x0 * f[1] + x1) * f[2] + x2) * f[3] + x3;
}

extern "C" int32_t ms_variant_coverage(const ms_op *op, const ms_variant_params *p, int32_t *counts, int64_t out_elems)
{
    if (!op || !p || !counts) return fail(MS_ERR_BAD_ARG, "ms_variant_coverage: NULL argument");
    int64_t ob;
    ms_op_tensor_bytes(op, -1, &ob);
    if (out_elems != ob / op->out_size) return fail(MS_ERR_BAD_ARG, "ms_variant_coverage: out_elems %" PRId64 " != %" PRId64, out_elems, ob / op->out_size);
    memset(counts, 0, sizeof(int32_t) * (size_t)out_elems);
    if (p->family == MS_FAM_GEMM_ALU || p->family == MS_FAM_GEMM_MFMA) {
        int um = p->tile_unit[0], un = p->tile_unit[1];
        for (int64_t b = 0; b < op->nb; ++b)
            for (int64_t wg = 0; wg < p->grid[0] / std::max(1, p->rfactor); ++wg) { // output tiles (rfactor workgroups share one)
                int64_t i0, j0;
                if (p->reorder == 1) {
                    j0 = wg / p->ti[0];
                    i0 = wg % p->ti[0];
                } else {
                    i0 = wg / p->tj[0];
                    j0 = wg % p->tj[0];
                }
                for (int64_t t = 0; t < (int64_t)p->ti[2] * p->tj[2]; ++t) { // thread or wavefront
                    int64_t ti = t / p->tj[2], tj = t % p->tj[2];
                    for (int64_t r1 = 0; r1 < p->ti[1]; ++r1)
                        for (int64_t r3 = 0; r3 < p->ti[3]; ++r3)
                            for (int64_t c1 = 0; c1 < p->tj[1]; ++c1)
                                for (int64_t c3 = 0; c3 < p->tj[3]; ++c3) {
                                    int64_t iu = split_index(p->ti, i0, r1, ti, r3);
                                    int64_t ju = split_index(p->tj, j0, c1, tj, c3);
                                    for (int a = 0; a < um; ++a)
                                        for (int c = 0; c < un; ++c) {
                                            int64_t i = iu * um + a, j = ju * un + c;
                                            if (i >= op->M || j >= op->N) return fail(MS_ERR_INVALID_TRACE, "coverage: index out of range");
                                            if (is_conv2d(op->d.kind)) ++counts[i * (op->N * op->nb) + b * op->N + j]; // groups interleave per pixel
                                            else ++counts[(b * op->M + i) * op->N + j];
                                        }
                                }
                }
            }
    } else if (p->family == MS_FAM_REDUCE) {
        const bool per_element = op->d.kind == MS_OP_SOFTMAX;
        for (int64_t wg = 0; wg < p->grid[0]; ++wg)
            for (int64_t r1 = 0; r1 < p->ti[1]; ++r1)
                for (int64_t g = 0; g < p->ti[2]; ++g)
                    for (int64_t r3 = 0; r3 < p->ti[3]; ++r3) {
                        int64_t row = split_index(p->ti, wg, r1, g, r3);
                        if (row >= op->M) return fail(MS_ERR_INVALID_TRACE, "coverage: index out of range");
                        if (!per_element) {
                            ++counts[row];
                            continue;
                        }
                        for (int64_t q0 = 0; q0 < p->tk[0]; ++q0)
                            for (int64_t q1 = 0; q1 < p->tk[1]; ++q1)
                                for (int64_t t = 0; t < p->tk[2]; ++t)
                                    for (int64_t q3 = 0; q3 < p->tk[3]; ++q3) {
                                        int64_t k = split_index(p->tk, q0, q1, t, q3);
                                        if (k >= op->K) return fail(MS_ERR_INVALID_TRACE, "coverage: index out of range");
                                        ++counts[row * op->K + k];
                                    }
                    }
    } else {
        const ms_op_desc &d = op->d;
        int64_t C = d.dims[3];
        for (int64_t n = 0; n < d.dims[0]; ++n)
            for (int64_t wg = 0; wg < p->grid[0]; ++wg) {
                int64_t c0 = wg % p->tc[0], j0 = wg / p->tc[0] % p->tj[0], i0 = wg / ((int64_t)p->tc[0] * p->tj[0]);
                for (int64_t t = 0; t < p->threads; ++t) {
                    int64_t tc = t % p->tc[2], tj = t / p->tc[2] % p->tj[2], ti = t / ((int64_t)p->tc[2] * p->tj[2]);
                    for (int64_t r1 = 0; r1 < p->ti[1]; ++r1)
                        for (int64_t r3 = 0; r3 < p->ti[3]; ++r3)
                            for (int64_t q1 = 0; q1 < p->tj[1]; ++q1)
                                for (int64_t q3 = 0; q3 < p->tj[3]; ++q3)
                                    for (int64_t s1 = 0; s1 < p->tc[1]; ++s1)
                                        for (int64_t s3 = 0; s3 < p->tc[3]; ++s3) {
                                            int64_t oh = split_index(p->ti, i0, r1, ti, r3);
                                            int64_t ow = split_index(p->tj, j0, q1, tj, q3);
                                            int64_t c = split_index(p->tc, c0, s1, tc, s3);
                                            if (oh >= op->OH || ow >= op->OW || c >= C) return fail(MS_ERR_INVALID_TRACE, "coverage: index out of range");
                                            ++counts[((n * op->OH + oh) * op->OW + ow) * C + c];
                                        }
                }
            }
    }
    return MS_OK;
}

extern "C" int32_t ms_variant_reduction_coverage(const ms_op *op, const ms_variant_params *p, int32_t *counts, int64_t k_elems, int64_t *needed)
{
    if (!op || !p) return fail(MS_ERR_BAD_ARG, "ms_variant_reduction_coverage: NULL argument");
    const bool dw = p->family == MS_FAM_DWCONV;
    const int unit = dw ? 1 : std::max(1, p->tile_unit[2]);
    const int64_t len = dw ? (int64_t)op->d.dims[4] * op->d.dims[5] : (int64_t)p->tk[0] * p->tk[1] * p->tk[2] * p->tk[3] * unit;
    if (needed) *needed = len;
    if (!counts) return needed ? MS_OK : fail(MS_ERR_BAD_ARG, "ms_variant_reduction_coverage: NULL argument");
    if (k_elems != len) return fail(MS_ERR_BAD_ARG, "ms_variant_reduction_coverage: k_elems %" PRId64 " != %" PRId64, k_elems, len);
    // the interpreted reduction covers the operator's K, padded by less than one intrinsic where a convolution rounds it up
    if (!dw && !p->tap_rows && (len < op->K || len - op->K >= unit))
        return fail(MS_ERR_INVALID_TRACE, "reduction coverage: the split covers %" PRId64 " positions, the operator reduces over %" PRId64, len, op->K);
    memset(counts, 0, sizeof(int32_t) * (size_t)len);
    if (dw) {
        for (int64_t kh = 0; kh < p->tk[1]; ++kh)
            for (int64_t kw = 0; kw < p->tk[2]; ++kw) {
                int64_t k = kh * op->d.dims[5] + kw;
                if (k >= len) return fail(MS_ERR_INVALID_TRACE, "reduction coverage: index out of range");
                ++counts[k];
            }
        return MS_OK;
    }
    const int rf = std::max(1, p->rfactor);
    if (p->tk[0] % rf) return fail(MS_ERR_INVALID_TRACE, "reduction coverage: rfactor does not divide k0");
    const int64_t run = p->tk[0] / rf; // k0 steps of one workgroup
    for (int64_t s = 0; s < rf; ++s)
        for (int64_t q0 = s * run; q0 < (s + 1) * run; ++q0)
            for (int64_t q1 = 0; q1 < p->tk[1]; ++q1)
                for (int64_t q2 = 0; q2 < p->tk[2]; ++q2)
                    for (int64_t q3 = 0; q3 < p->tk[3]; ++q3)
                        for (int u = 0; u < unit; ++u) {
                            int64_t k = split_index(p->tk, q0, q1, q2, q3) * unit + u;
                            if (k < 0 || k >= len) return fail(MS_ERR_INVALID_TRACE, "reduction coverage: index out of range");
                            ++counts[k];
                        }
    return MS_OK;
}
