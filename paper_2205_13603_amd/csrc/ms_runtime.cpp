// Variant handles, launch and measurement (the only part of libms that talks
// to the GPU).
#include "ms_internal.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

using namespace ms;

struct ms_variant {
    ms_op op;
    ms_variant_params p;
    KernelSpec spec;
    std::vector<char> *code; // owned by the cache
    hipModule_t mod;
    hipFunction_t fn;
    hipFunction_t fn_reduce; // second kernel of an rfactor launch, else null
    int device;              // device the module is loaded on, -1 = not loaded
    int compute_units;       // of that device
};

#define HIP_TRY(call)                                                                               \
    do {                                                                                            \
        hipError_t e_ = (call);                                                                     \
        if (e_ != hipSuccess) return fail(MS_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_));      \
    } while (0)

extern "C" int32_t ms_variant_build(const ms_op *op, const ms_space *space, const ms_trace *trace, ms_variant **out)
{
    if (!op || !space || !trace || !out) return fail(MS_ERR_BAD_ARG, "ms_variant_build: NULL argument");
    *out = nullptr;
    ms_variant_params p;
    int32_t rc = ms_trace_validate(op, space, trace, &p);
    if (rc != MS_OK) return rc;
    ms_variant *v = new (std::nothrow) ms_variant();
    if (!v) return fail(MS_ERR_NOMEM, "ms_variant_build: out of memory");
    v->op = *op;
    v->p = p;
    v->mod = nullptr;
    v->fn = nullptr;
    v->fn_reduce = nullptr;
    v->device = -1;
    rc = make_kernel_spec(op, &p, &v->spec);
    if (rc == MS_OK) rc = jit_get_code(v->spec, p.key, &v->code);
    if (rc != MS_OK) {
        delete v;
        return rc;
    }
    *out = v;
    return MS_OK;
}

extern "C" void ms_variant_destroy(ms_variant *v)
{
    if (!v) return;
    if (v->mod) (void)hipModuleUnload(v->mod);
    delete v;
}

// rfactor partial results of one instance: [rfactor][batch][M][N] accumulator values (fp32 or int32)
static size_t workspace_per_instance(const ms_variant *v)
{
    if (v->p.rfactor <= 1) return 0;
    return (size_t)v->p.rfactor * (size_t)v->op.nb * (size_t)v->op.M * (size_t)v->op.N * 4u;
}

extern "C" int32_t ms_variant_info(const ms_variant *v, ms_variant_params *params, size_t *workspace_bytes)
{
    if (!v) return fail(MS_ERR_BAD_ARG, "ms_variant_info: NULL variant");
    if (params) *params = v->p;
    if (workspace_bytes) *workspace_bytes = workspace_per_instance(v);
    return MS_OK;
}

// The code object's metadata is a MessagePack map in an ELF note; each kernel entry holds ".vgpr_count", ".agpr_count",
// ... as a short string key followed by an unsigned integer.  Reads the value behind the first occurrence of `key`
// that lies after `from` (the position of the kernel's ".name" entry), -1 if absent.
static long meta_uint(const std::vector<char> &blob, const char *key, size_t from)
{
    const size_t kl = strlen(key);
    for (size_t i = from; i + kl + 1 < blob.size(); ++i) {
        if (memcmp(&blob[i], key, kl) != 0) continue;
        if (i == 0 || (unsigned char)blob[i - 1] != (0xa0u | kl)) continue; // a fixstr of exactly this length
        const unsigned char *p = (const unsigned char *)&blob[i + kl];
        const size_t left = blob.size() - (i + kl);
        if (p[0] <= 0x7f) return p[0];
        if (p[0] == 0xcc && left >= 2) return p[1];
        if (p[0] == 0xcd && left >= 3) return (p[1] << 8) | p[2];
        if (p[0] == 0xce && left >= 5) return ((long)p[1] << 24) | (p[2] << 16) | (p[3] << 8) | p[4];
        return -1;
    }
    return -1;
}

extern "C" int32_t ms_variant_resources_get(const ms_variant *v, ms_variant_resources *out)
{
    if (!v || !out) return fail(MS_ERR_BAD_ARG, "ms_variant_resources_get: NULL argument");
    memset(out, 0, sizeof *out);
    const std::vector<char> &blob = *v->code;
    // the entry of the main kernel: its symbol is "<entry>.kd"
    const std::string sym = v->spec.entry + ".kd";
    size_t at = std::string::npos;
    for (size_t i = 0; i + sym.size() <= blob.size(); ++i)
        if (memcmp(&blob[i], sym.data(), sym.size()) == 0 && i > 0 && (unsigned char)blob[i - 1] == (0xa0u | sym.size())) {
            at = i;
            break;
        }
    if (at == std::string::npos) return fail(MS_ERR_UNSUPPORTED, "ms_variant_resources_get: no metadata entry for %s", sym.c_str());
    // the keys of one kernel's map are sorted, so those before ".symbol" precede it in the blob: scan from the start of
    // this kernel's map, which begins at the last ".agpr_count" (its first key) before the symbol
    size_t start = 0;
    for (size_t i = 0; i + 11 < at; ++i)
        if (memcmp(&blob[i], ".agpr_count", 11) == 0) start = i > 0 ? i - 1 : 0;
    const long vg = meta_uint(blob, ".vgpr_count", start), ag = meta_uint(blob, ".agpr_count", start), sg = meta_uint(blob, ".sgpr_count", start);
    const long sc = meta_uint(blob, ".private_segment_fixed_size", start), sp = meta_uint(blob, ".vgpr_spill_count", start);
    const long ld = meta_uint(blob, ".group_segment_fixed_size", start);
    if (vg < 0 || sg < 0) return fail(MS_ERR_UNSUPPORTED, "ms_variant_resources_get: register counts not found in the code object");
    out->vgprs = (int32_t)vg;
    out->agprs = (int32_t)(ag < 0 ? 0 : ag);
    out->sgprs = (int32_t)sg;
    out->scratch_bytes = (int32_t)(sc < 0 ? 0 : sc);
    out->spilled_vgprs = (int32_t)(sp < 0 ? 0 : sp);
    out->lds_bytes = (int32_t)(ld < 0 ? 0 : ld);
    return MS_OK;
}

extern "C" int32_t ms_prebuild(const ms_op *op, const ms_space *space, const ms_trace *traces, int32_t n, int32_t threads,
                               int32_t *n_built)
{
    if (!op || !space || (!traces && n > 0) || n < 0) return fail(MS_ERR_BAD_ARG, "ms_prebuild: bad argument");
    threads = std::max(1, std::min(threads, 64));
    std::atomic<int> next(0), built(0);
    auto work = [&]() {
        for (;;) {
            int i = next.fetch_add(1);
            if (i >= n) break;
            ms_variant_params p;
            if (ms_trace_validate(op, space, &traces[i], &p) != MS_OK) continue;
            KernelSpec spec;
            std::vector<char> *code;
            if (make_kernel_spec(op, &p, &spec) == MS_OK && jit_get_code(spec, p.key, &code) == MS_OK) built.fetch_add(1);
        }
    };
    std::vector<std::thread> pool;
    for (int t = 1; t < threads; ++t) pool.emplace_back(work);
    work();
    for (auto &t : pool) t.join();
    if (n_built) *n_built = built.load();
    return MS_OK;
}

static int32_t ensure_loaded(ms_variant *v)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (v->device == dev) return MS_OK;
    if (v->mod) {
        (void)hipModuleUnload(v->mod);
        v->mod = nullptr;
        v->device = -1;
    }
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(MS_ERR_UNSUPPORTED, "device %d is %s; kernels are built for gfx950 only", dev, prop.gcnArchName);
    if ((size_t)v->p.lds_bytes > prop.sharedMemPerBlock)
        return fail(MS_ERR_HIP, "variant needs %d bytes of LDS, the device offers %zu per workgroup", v->p.lds_bytes, (size_t)prop.sharedMemPerBlock);
    HIP_TRY(hipModuleLoadData(&v->mod, v->code->data()));
    HIP_TRY(hipModuleGetFunction(&v->fn, v->mod, v->spec.entry.c_str()));
    v->fn_reduce = nullptr;
    if (v->p.rfactor > 1) HIP_TRY(hipModuleGetFunction(&v->fn_reduce, v->mod, "ms_rfactor_reduce"));
    v->device = dev;
    v->compute_units = prop.multiProcessorCount;
    return MS_OK;
}

// ---------------------------------------------------------------- launch without allocation
//
// Workspace of ms_variant_launch_static: one array per GPU, in the library's own device image, held until the
// process ends.  In host code the array's name is only a stand-in; its address on a device comes from
// hipGetSymbolAddress with that device current, once per device, and that pointer is what kernels receive.
static __device__ __align__(256) unsigned char scratch[MS_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices]; // per device, null until ms_variant_prepare ran on it

int32_t scratch_on_current_device(bool resolve, void **out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(MS_ERR_UNSUPPORTED, "device index %d is beyond the %d this library keeps a workspace for", dev, kMaxDevices);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        if (!resolve) return fail(MS_ERR_BAD_ARG, "ms_variant_launch_static: call ms_variant_prepare on device %d first (set-up may allocate, this call must not)", dev);
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(MS_ERR_HIP, "hipGetSymbolAddress returned a null workspace");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MS_OK;
}
} // namespace



extern "C" int32_t ms_variant_prepare(ms_variant *v)
{
    if (!v) return fail(MS_ERR_BAD_ARG, "ms_variant_prepare: NULL variant");
    int32_t rc = ensure_loaded(v);
    if (rc != MS_OK) return rc;
    void *ptr = nullptr;
    return scratch_on_current_device(true, &ptr);
}

extern "C" int32_t ms_variant_launch_static(ms_variant *v, const void *const *inputs, void *const *outputs, int32_t instances, void *stream)
{
    if (!v || !inputs || !outputs) return fail(MS_ERR_BAD_ARG, "ms_variant_launch_static: NULL argument");
    if (instances < 1) return fail(MS_ERR_BAD_ARG, "ms_variant_launch_static: instances = %d", instances);
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (v->device != dev || !v->fn) return fail(MS_ERR_BAD_ARG, "ms_variant_launch_static: call ms_variant_prepare on device %d first (loading a kernel allocates)", dev);
    const size_t need = workspace_per_instance(v) * (size_t)instances;
    if (need > (size_t)MS_STATIC_WORKSPACE_BYTES)
        return fail(MS_ERR_BAD_ARG, "ms_variant_launch_static: %d instances need a workspace of %zu bytes, the built-in one holds %zu",
                    instances, need, (size_t)MS_STATIC_WORKSPACE_BYTES);
    void *ws = nullptr;
    if (need) {
        int32_t rc = scratch_on_current_device(false, &ws);
        if (rc != MS_OK) return rc;
    }
    // every partial sum the second kernel reads is written by the first kernel of the same call: nothing to clear
    return ms_variant_launch(v, inputs, outputs, ws, instances, stream);
}

extern "C" int32_t ms_variant_launch(ms_variant *v, const void *const *inputs, void *const *outputs, void *workspace,
                                     int32_t instances, void *stream)
{
    if (!v || !inputs || !outputs) return fail(MS_ERR_BAD_ARG, "ms_variant_launch: NULL argument");
    if (instances < 1) return fail(MS_ERR_BAD_ARG, "ms_variant_launch: instances = %d", instances);
    if (v->p.rfactor > 1 && !workspace)
        return fail(MS_ERR_BAD_ARG, "ms_variant_launch: the variant splits its reduction over %d workgroups and needs a workspace of %zu bytes per instance",
                    v->p.rfactor, workspace_per_instance(v));
    if (v->p.rfactor > 1 && ((uintptr_t)workspace & 15u)) return fail(MS_ERR_BAD_ARG, "ms_variant_launch: the workspace must be 16-byte aligned");
    const bool one_input = v->p.family == MS_FAM_REDUCE;
    if (!inputs[0] || (!one_input && !inputs[1]) || !outputs[0]) return fail(MS_ERR_BAD_ARG, "ms_variant_launch: NULL tensor pointer");
    uint64_t gz = (uint64_t)v->spec.grid[2] * (uint64_t)instances;
    if (gz > 65535ull * 32768ull || (uint64_t)v->spec.grid[0] * gz > 0x7fffffffull)
        return fail(MS_ERR_BAD_ARG, "ms_variant_launch: %d instances overflow the grid", instances);
    int32_t rc = ensure_loaded(v);
    if (rc != MS_OK) return rc;
    const void *in0 = inputs[0], *in1 = one_input ? nullptr : inputs[1];
    const void *in2 = nullptr;
    if (is_conv2d(v->op.d.kind) && v->op.d.has_bias) {
        in2 = inputs[2];
        if (!in2) return fail(MS_ERR_BAD_ARG, "ms_variant_launch: the op has a bias but inputs[2] is NULL");
    }
    void *o = outputs[0];
    int32_t inst = instances;
    void *ws = workspace;
    void *args[] = {&in0, &in1, &in2, &o, &inst, &ws}; // kernels without a workspace declare the first five only
    // grid z carries batch x instances; fold overflow beyond 65535 into y
    unsigned gy = 1, gzz = (unsigned)gz;
    if (gz > 65535) {
        // kernels recover z = blockIdx.z * gridDim.y + blockIdx.y
        gy = 32768;
        while (gy > 1 && gz % gy) gy >>= 1;
        gzz = (unsigned)(gz / gy);
        if (gzz > 65535) return fail(MS_ERR_BAD_ARG, "ms_variant_launch: %d instances overflow the grid", instances);
    }
    unsigned gx = v->spec.grid[0];
    if (v->p.family == MS_FAM_GEMM_MFMA && v->p.reorder == 3) {
        // persistent workgroups: one per compute unit (fewer if there are fewer tiles), each loops over its tiles
        uint64_t total = (uint64_t)v->spec.grid[0] * gz;
        gx = (unsigned)std::min<uint64_t>(total, (uint64_t)std::max(1, v->compute_units));
        gy = 1;
        gzz = 1;
    }
    if (v->p.family == MS_FAM_GEMM_MFMA && v->p.compute_at >= 2) {
        // persistent workgroups with resident weights: as many as fit the compute units' LDS, each owns a run of tiles
        uint64_t total = (uint64_t)v->spec.grid[0] * gz;
        uint64_t per_cu = std::max<uint64_t>(1, std::min<uint64_t>(4, (160u * 1024u) / (uint64_t)std::max(1, v->p.lds_bytes)));
        gx = (unsigned)std::min<uint64_t>(total, per_cu * (uint64_t)std::max(1, v->compute_units));
        gy = 1;
        gzz = 1;
    }
    HIP_TRY(hipModuleLaunchKernel(v->fn, gx, gy, gzz, v->spec.block[0], 1, 1, v->spec.lds_dynamic, (hipStream_t)stream, args, nullptr));
    if (v->p.rfactor > 1) {
        // stream order makes the partial sums visible to the kernel that adds them: 4 outputs per thread
        const uint64_t quads = (uint64_t)instances * (uint64_t)v->op.nb * (uint64_t)v->op.M * (uint64_t)(v->op.N / 4);
        const uint64_t blocks = (quads + 255) / 256;
        if (blocks > 0x7fffffffull) return fail(MS_ERR_BAD_ARG, "ms_variant_launch: %d instances overflow the grid of the reduction", instances);
        const void *wsc = workspace;
        void *rargs[] = {&wsc, &in2, &o, &inst};
        HIP_TRY(hipModuleLaunchKernel(v->fn_reduce, (unsigned)blocks, 1, 1, 256, 1, 1, 0, (hipStream_t)stream, rargs, nullptr));
    }
    return MS_OK;
}

namespace {

// The one timing routine: `launch` is called warm-up + repeats x launches_per_repeat times on `stream`;
// each repeat is bracketed by two HIP events on that stream.  Fills min / median / mean per launch.
template <class Launch>
int32_t timed_repeats(Launch &&launch, const ms_measure_cfg *cfg, hipStream_t s, ms_measure_result *out, const char *who)
{
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail(MS_ERR_HIP, "hipEventCreate failed");
    }
    int32_t rc = MS_OK;
    std::vector<double> us;
    for (int i = 0; i < cfg->warmup && rc == MS_OK; ++i) rc = launch();
    if (rc == MS_OK && hipStreamSynchronize(s) != hipSuccess) rc = fail(MS_ERR_HIP, "%s: warm-up failed: %s", who, hipGetErrorString(hipGetLastError()));
    for (int r = 0; r < cfg->repeats && rc == MS_OK; ++r) {
        hipError_t e = hipEventRecord(e0, s);
        for (int l = 0; l < cfg->launches_per_repeat && rc == MS_OK; ++l) rc = launch();
        if (rc != MS_OK) break;
        if (e == hipSuccess) e = hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms_elapsed = 0;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms_elapsed, e0, e1);
        if (e != hipSuccess) {
            rc = fail(MS_ERR_HIP, "%s: %s", who, hipGetErrorString(e));
            break;
        }
        us.push_back((double)ms_elapsed * 1000.0 / cfg->launches_per_repeat);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != MS_OK) return rc;
    std::sort(us.begin(), us.end());
    out->n = (int32_t)us.size();
    out->min_us = us.front();
    out->median_us = us.size() % 2 ? us[us.size() / 2] : 0.5 * (us[us.size() / 2 - 1] + us[us.size() / 2]);
    double sum = 0;
    for (double x : us) sum += x;
    out->mean_us = sum / us.size();
    return MS_OK;
}

} // namespace

extern "C" int32_t ms_measure(ms_variant *v, const ms_bufset *sets, int32_t n_sets, const ms_measure_cfg *cfg, void *stream,
                              ms_measure_result *out)
{
    if (!v || !sets || !cfg || !out || n_sets < 1) return fail(MS_ERR_BAD_ARG, "ms_measure: bad argument");
    if (cfg->repeats < 1 || cfg->launches_per_repeat < 1 || cfg->warmup < 0 || cfg->instances < 1)
        return fail(MS_ERR_BAD_ARG, "ms_measure: bad configuration");
    memset(out, 0, sizeof *out);
    int set = 0;
    auto launch = [&]() -> int32_t {
        const ms_bufset &b = sets[set];
        set = (set + 1) % n_sets;
        void *outs[1] = {b.output};
        return ms_variant_launch(v, b.inputs, outs, b.workspace, cfg->instances, stream);
    };
    int32_t rc = timed_repeats(launch, cfg, (hipStream_t)stream, out, "ms_measure");
    if (rc != MS_OK) return rc;
    double f, b;
    ms_op_work(&v->op, &f, &b);
    out->flop = f * cfg->instances;
    out->bytes = b * cfg->instances;
    return MS_OK;
}

extern "C" int32_t ms_device_info_get(ms_device_info *out)
{
    if (!out) return fail(MS_ERR_BAD_ARG, "ms_device_info_get: NULL argument");
    memset(out, 0, sizeof *out);
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    snprintf(out->name, sizeof out->name, "%s", prop.name);
    snprintf(out->arch, sizeof out->arch, "%s", prop.gcnArchName);
    out->compute_units = prop.multiProcessorCount;
    out->wave_size = prop.warpSize;
    out->lds_bytes_per_block = (int32_t)prop.sharedMemPerBlock;
    out->max_threads_per_block = prop.maxThreadsPerBlock;
    out->clock_khz = prop.clockRate;
    out->mem_clock_khz = prop.memoryClockRate;
    out->mem_bus_bits = prop.memoryBusWidth;
    out->l2_bytes = prop.l2CacheSize;
    out->global_mem_bytes = (int64_t)prop.totalGlobalMem;
    return MS_OK;
}

// ---------------------------------------------------------------- calibration

namespace {

struct CalibKernel {
    hipModule_t mod = nullptr;
    hipFunction_t fn = nullptr;
};

int32_t load_calib(const std::vector<std::string> &defs, uint64_t key, CalibKernel *out)
{
    KernelSpec spec;
    spec.template_name = "calib.hip";
    spec.defines = defs;
    spec.entry = "ms_calib_kernel";
    std::vector<char> *code;
    int32_t rc = jit_get_code(spec, key, &code);
    if (rc != MS_OK) return rc;
    HIP_TRY(hipModuleLoadData(&out->mod, code->data()));
    HIP_TRY(hipModuleGetFunction(&out->fn, out->mod, "ms_calib_kernel"));
    return MS_OK;
}

int32_t time_launches(hipFunction_t fn, unsigned grid, void **args, hipStream_t s, int reps, double *best_ms, unsigned block = 256)
{
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    HIP_TRY(hipEventCreate(&e1));
    double best = 1e30;
    int32_t rc = MS_OK;
    for (int r = 0; r < reps + 1 && rc == MS_OK; ++r) { // first repeat is the warm-up
        hipError_t e = hipEventRecord(e0, s);
        if (e == hipSuccess) e = hipModuleLaunchKernel(fn, grid, 1, 1, block, 1, 1, 0, s, args, nullptr);
        if (e == hipSuccess) e = hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms_el = 0;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms_el, e0, e1);
        if (e != hipSuccess) rc = fail(MS_ERR_HIP, "calibration launch: %s", hipGetErrorString(e));
        else if (r > 0 && ms_el < best) best = ms_el;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *best_ms = best;
    return rc;
}

} // namespace

extern "C" int32_t ms_calibrate_mfma(int32_t in_dtype, int32_t mfma_code, const void *operands, void *scratch, void *stream, double *tflops)
{
    if (!scratch || !tflops) return fail(MS_ERR_BAD_ARG, "ms_calibrate_mfma: NULL argument");
    static const int f16_codes[] = {161616, 323208, 161632, 323216}, i8_codes[] = {161632, 323216, 161664, 323232},
                     f32_codes[] = {161604, 323202, 161604, 323202};
    static const int f8_codes[] = {161632, 323216, 1616128, 323264}; // 1616128: the 16x16x128 intrinsic (three-digit k)
    const int *codes = in_dtype == MS_I8 ? i8_codes : (in_dtype == MS_F32 ? f32_codes : (in_dtype == MS_F8E4M3 ? f8_codes : f16_codes));
    if (in_dtype != MS_F16 && in_dtype != MS_BF16 && in_dtype != MS_I8 && in_dtype != MS_F32 && in_dtype != MS_F8E4M3)
        return fail(MS_ERR_BAD_ARG, "ms_calibrate_mfma: bad dtype");
    bool ok = false;
    for (int i = 0; i < 4; ++i) ok = ok || codes[i] == mfma_code;
    if (!ok) return fail(MS_ERR_BAD_ARG, "ms_calibrate_mfma: no intrinsic %d for %s", mfma_code, dtype_name(in_dtype));
    int m, n, k;
    mfma_dims(mfma_code, &m, &n, &k);
    std::vector<std::string> defs = {"-DMODE=0", "-DCAL_DT=" + std::to_string(in_dtype), "-DMI_M=" + std::to_string(m),
                                     "-DMI_N=" + std::to_string(n), "-DMI_K=" + std::to_string(k)};
    CalibKernel ck;
    int32_t rc = load_calib(defs, mix64(0xCA11B0ull ^ (uint64_t)mfma_code * 131 ^ (uint64_t)in_dtype), &ck);
    if (rc != MS_OK) return rc;
    int dev = 0;
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    unsigned grid = (unsigned)prop.multiProcessorCount * 2; // 2 workgroups x 4 waves per CU = 2 waves per SIMD
    int iters = 20000;
    const void *src = operands;
    void *args[] = {&src, &src, &src, &scratch, &iters};
    double ms_best = 0;
    rc = time_launches(ck.fn, grid, args, (hipStream_t)stream, 3, &ms_best);
    (void)hipModuleUnload(ck.mod);
    if (rc != MS_OK) return rc;
    double insts = (double)grid * 4 * iters * 8;
    *tflops = insts * 2.0 * m * n * k / (ms_best * 1e-3) / 1e12;
    return MS_OK;
}

extern "C" int32_t ms_calibrate_stream(int32_t mode, const void *src, void *dst, size_t bytes, void *stream, double *gbs)
{
    if (!src || !dst || !gbs) return fail(MS_ERR_BAD_ARG, "ms_calibrate_stream: NULL argument");
    if (mode < 1 || mode > 4 || bytes == 0 || bytes % 4096 || bytes / 4096 > 0x7fffffffull)
        return fail(MS_ERR_BAD_ARG, "ms_calibrate_stream: mode must be 1, 2, 3 or 4 and bytes a multiple of 4096");
    // kernel modes: 1 copy, 2 read, 6 write, 7 copy in small chunks (3, 4, 5 are the LDS, L2 and timer kernels)
    std::vector<std::string> defs = {"-DMODE=" + std::to_string(mode == 3 ? 6 : (mode == 4 ? 7 : mode)), "-DCAL_DT=0"};
    CalibKernel ck;
    int32_t rc = load_calib(defs, mix64(0xCA11B1ull ^ (uint64_t)mode), &ck);
    if (rc != MS_OK) return rc;
    int dev = 0;
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    unsigned grid = (unsigned)prop.multiProcessorCount * 16;
    int n16_by_256 = (int)(bytes / 4096);
    if (mode == 4) grid = (unsigned)(bytes / 1024); // one 64-lane workgroup per KiB
    void *args[] = {&src, &src, &src, &dst, &n16_by_256};
    double ms_best = 0;
    rc = time_launches(ck.fn, grid, args, (hipStream_t)stream, 5, &ms_best, mode == 4 ? 64u : 256u);
    (void)hipModuleUnload(ck.mod);
    if (rc != MS_OK) return rc;
    *gbs = (double)bytes * (mode == 1 || mode == 4 ? 2.0 : 1.0) / (ms_best * 1e-3) / 1e9;
    return MS_OK;
}

extern "C" int32_t ms_calibrate_lds(void *scratch, void *stream, double *bytes_per_clk_per_cu, double *gbs)
{
    if (!scratch || !bytes_per_clk_per_cu || !gbs) return fail(MS_ERR_BAD_ARG, "ms_calibrate_lds: NULL argument");
    std::vector<std::string> defs = {"-DMODE=3", "-DCAL_DT=0"};
    CalibKernel ck;
    int32_t rc = load_calib(defs, mix64(0xCA11B3ull), &ck);
    if (rc != MS_OK) return rc;
    int dev = 0;
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    unsigned grid = (unsigned)prop.multiProcessorCount * 2;
    int iters = 20000;
    const void *src = nullptr;
    void *args[] = {&src, &src, &src, &scratch, &iters};
    double ms_best = 0;
    rc = time_launches(ck.fn, grid, args, (hipStream_t)stream, 3, &ms_best);
    (void)hipModuleUnload(ck.mod);
    if (rc != MS_OK) return rc;
    double bytes = (double)grid * 256 * 16.0 * 8 * iters;
    *gbs = bytes / (ms_best * 1e-3) / 1e9;
    *bytes_per_clk_per_cu = bytes / (ms_best * 1e-3) / ((double)prop.clockRate * 1e3) / prop.multiProcessorCount;
    return MS_OK;
}

extern "C" int32_t ms_calibrate_l2(const void *src, void *scratch, void *stream, double *gbs)
{
    if (!src || !scratch || !gbs) return fail(MS_ERR_BAD_ARG, "ms_calibrate_l2: NULL argument");
    std::vector<std::string> defs = {"-DMODE=4", "-DCAL_DT=0"};
    CalibKernel ck;
    int32_t rc = load_calib(defs, mix64(0xCA11B4ull), &ck);
    if (rc != MS_OK) return rc;
    int dev = 0;
    hipDeviceProp_t prop;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipGetDeviceProperties(&prop, dev));
    unsigned grid = (unsigned)prop.multiProcessorCount * 8;
    int reps = 2000;
    void *args[] = {&src, &src, &src, &scratch, &reps};
    double ms_best = 0;
    rc = time_launches(ck.fn, grid, args, (hipStream_t)stream, 3, &ms_best);
    (void)hipModuleUnload(ck.mod);
    if (rc != MS_OK) return rc;
    *gbs = (double)grid * 256 * 16.0 * 8 * reps / (ms_best * 1e-3) / 1e9;
    return MS_OK;
}

extern "C" int32_t ms_calibrate_timer(double target_us, const ms_measure_cfg *cfg, void *scratch, void *stream, ms_measure_result *out)
{
    if (!cfg || !out || !scratch) return fail(MS_ERR_BAD_ARG, "ms_calibrate_timer: NULL argument");
    if (!(target_us >= 1.0) || target_us > 20000.0) return fail(MS_ERR_BAD_ARG, "ms_calibrate_timer: target of %g us outside [1, 20000]", target_us);
    if (cfg->repeats < 1 || cfg->launches_per_repeat < 1 || cfg->warmup < 0) return fail(MS_ERR_BAD_ARG, "ms_calibrate_timer: bad configuration");
    memset(out, 0, sizeof *out);
    int dev = 0, khz = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) return fail(MS_ERR_UNSUPPORTED, "ms_calibrate_timer: the device reports no wall clock rate");
    std::vector<std::string> defs = {"-DMODE=5", "-DCAL_DT=0"};
    CalibKernel ck;
    int32_t rc = load_calib(defs, mix64(0xCA11B5ull), &ck);
    if (rc != MS_OK) return rc;
    int ticks = (int)(target_us * (double)khz / 1000.0 + 0.5);
    const void *none = nullptr;
    void *args[] = {&none, &none, &none, &scratch, &ticks};
    hipStream_t s = (hipStream_t)stream;
    auto launch = [&]() -> int32_t {
        HIP_TRY(hipModuleLaunchKernel(ck.fn, 1, 1, 1, 64, 1, 1, 0, s, args, nullptr));
        return MS_OK;
    };
    rc = timed_repeats(launch, cfg, s, out, "ms_calibrate_timer");
    (void)hipModuleUnload(ck.mod);
    return rc;
}
