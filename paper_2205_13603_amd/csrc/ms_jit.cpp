// Run-time compilation of kernel templates for gfx950 through hiprtc, with an
// in-memory and an on-disk cache of code objects.  Compilation needs no GPU.
#include "ms_internal.h"

#include <dlfcn.h>
#include <hip/hiprtc.h>
#include <sys/stat.h>
#include <unistd.h>

#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>

namespace ms {

static std::mutex g_mu;
static std::map<uint64_t, std::unique_ptr<std::vector<char>>> g_codes;
static std::map<std::string, std::string> g_sources;
static std::string g_cache_dir;
static bool g_cache_dir_set = false;
static int64_t g_n_compiled = 0, g_n_disk = 0, g_n_mem = 0;

// Version of the run-time compiler this process is bound to.  A process that loaded PyTorch first runs PyTorch's
// copy of the compiler library, one that did not runs the system's; the two generate different code for the same
// source, so the version is part of every cache key: a code object is only ever reused by the compiler that made it.
static uint64_t compiler_id()
{
    int major = 0, minor = 0;
    if (hiprtcVersion(&major, &minor) != HIPRTC_SUCCESS) return 0;
    return ((uint64_t)(uint32_t)major << 32) | (uint32_t)minor;
}

std::string kernels_dir()
{
    const char *env = getenv("MS_KERNELS_DIR");
    if (env && *env) return env;
    Dl_info info;
    if (dladdr((void *)&kernels_dir, &info) && info.dli_fname) {
        std::string p = info.dli_fname;
        size_t slash = p.rfind('/');
        std::string dir = slash == std::string::npos ? "." : p.substr(0, slash);
        return dir + "/csrc/kernels";
    }
    return "csrc/kernels";
}

static std::string cache_dir()
{
    if (g_cache_dir_set) return g_cache_dir;
    const char *env = getenv("MS_CACHE_DIR");
    if (env) return env;
    Dl_info info;
    if (dladdr((void *)&kernels_dir, &info) && info.dli_fname) {
        std::string p = info.dli_fname;
        size_t slash = p.rfind('/');
        std::string dir = slash == std::string::npos ? "." : p.substr(0, slash);
        return dir + "/kcache";
    }
    return "";
}

static bool read_file(const std::string &path, std::string *out)
{
    FILE *f = fopen(path.c_str(), "rb");
    if (!f) return false;
    std::string s;
    char buf[65536];
    size_t n;
    while ((n = fread(buf, 1, sizeof buf, f)) > 0) s.append(buf, n);
    fclose(f);
    *out = s;
    return true;
}

static uint64_t hash_bytes(const std::string &s)
{
    uint64_t h = 0xcbf29ce484222325ull;
    for (unsigned char c : s) {
        h ^= c;
        h *= 0x100000001b3ull;
    }
    return mix64(h);
}

static int32_t get_source(const std::string &name, std::string *src)
{
    {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_sources.find(name);
        if (it != g_sources.end()) {
            *src = it->second;
            return MS_OK;
        }
    }
    std::string dir = kernels_dir();
    std::string body, common;
    if (!read_file(dir + "/" + name, &body)) return fail(MS_ERR_COMPILE, "kernel template %s/%s not found", dir.c_str(), name.c_str());
    if (!read_file(dir + "/common.h", &common)) return fail(MS_ERR_COMPILE, "kernel header %s/common.h not found", dir.c_str());
    // hiprtc sees one translation unit: the shared header is spliced in
    std::string marker = "#include \"common.h\"";
    size_t at = body.find(marker);
    if (at != std::string::npos) body.replace(at, marker.size(), common);
    std::lock_guard<std::mutex> lk(g_mu);
    g_sources[name] = body;
    *src = body;
    return MS_OK;
}

int32_t jit_get_code(const KernelSpec &spec, uint64_t key, std::vector<char> **code_out)
{
    std::string src;
    int32_t rc = get_source(spec.template_name, &src);
    if (rc != MS_OK) return rc;
    std::string opts_joined;
    for (auto &d : spec.defines) opts_joined += d + " ";
    // developer knob: extra -D options for experiments with a private copy of the templates
    std::vector<std::string> extra;
    if (const char *env = getenv("MS_EXTRA_DEFINES")) {
        std::string e(env), tok;
        for (size_t i = 0; i <= e.size(); ++i) {
            if (i == e.size() || e[i] == ' ') {
                if (!tok.empty()) extra.push_back(tok);
                tok.clear();
            } else {
                tok += e[i];
            }
        }
        for (auto &x : extra) opts_joined += x + " ";
    }
    uint64_t k = mix64(key ^ hash_bytes(src) ^ mix64(hash_bytes(opts_joined)) ^ mix64(0xC0DE000000000000ull ^ compiler_id()));
    {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_codes.find(k);
        if (it != g_codes.end()) {
            ++g_n_mem;
            *code_out = it->second.get();
            return MS_OK;
        }
    }
    std::string dir = cache_dir();
    char fname[64];
    snprintf(fname, sizeof fname, "/%016" PRIx64 ".hsaco", k);
    std::unique_ptr<std::vector<char>> code(new std::vector<char>());
    if (!dir.empty()) {
        std::string blob;
        if (read_file(dir + fname, &blob) && blob.size() > 64) {
            code->assign(blob.begin(), blob.end());
            std::lock_guard<std::mutex> lk(g_mu);
            ++g_n_disk;
        }
    }
    if (code->empty()) {
        hiprtcProgram prog;
        hiprtcResult r = hiprtcCreateProgram(&prog, src.c_str(), spec.template_name.c_str(), 0, nullptr, nullptr);
        if (r != HIPRTC_SUCCESS) return fail(MS_ERR_COMPILE, "hiprtcCreateProgram: %s", hiprtcGetErrorString(r));
        std::vector<std::string> opts = spec.defines;
        for (auto &x : extra) opts.push_back(x);
        // developer knob: the full target id (e.g. gfx950:sramecc+:xnack-) instead of the generic one
        const char *arch_env = getenv("MS_OFFLOAD_ARCH");
        opts.push_back(std::string("--offload-arch=") + (arch_env && *arch_env ? arch_env : "gfx950"));
        opts.push_back("-O3");
        opts.push_back("-std=c++17");
        // no fast-math: results must not depend on reassociation
        // scalar fp32 code only: the packed fp32 forms are kept out of generated code
        opts.push_back("-Xclang");
        opts.push_back("-target-feature");
        opts.push_back("-Xclang");
        opts.push_back("-packed-fp32-ops");
        std::vector<const char *> copts;
        for (auto &o : opts) copts.push_back(o.c_str());
        r = hiprtcCompileProgram(prog, (int)copts.size(), copts.data());
        if (r != HIPRTC_SUCCESS) {
            size_t ls = 0;
            hiprtcGetProgramLogSize(prog, &ls);
            std::string log(ls, '\0');
            if (ls) hiprtcGetProgramLog(prog, &log[0]);
            hiprtcDestroyProgram(&prog);
            if (log.size() > 3000) log.resize(3000);
            return fail(MS_ERR_COMPILE, "compiling %s [%s] failed: %s\n%s", spec.template_name.c_str(), opts_joined.c_str(),
                        hiprtcGetErrorString(r), log.c_str());
        }
        size_t cs = 0;
        hiprtcGetCodeSize(prog, &cs);
        code->resize(cs);
        hiprtcGetCode(prog, code->data());
        hiprtcDestroyProgram(&prog);
        {
            std::lock_guard<std::mutex> lk(g_mu);
            ++g_n_compiled;
        }
        if (!dir.empty()) {
            mkdir(dir.c_str(), 0777);
            char tmpn[96];
            snprintf(tmpn, sizeof tmpn, "%s.tmp.%d.%" PRIx64, fname, (int)getpid(), (uint64_t)(uintptr_t)code.get());
            std::string tmp = dir + tmpn;
            FILE *f = fopen(tmp.c_str(), "wb");
            if (f) {
                bool ok = fwrite(code->data(), 1, code->size(), f) == code->size();
                ok = fclose(f) == 0 && ok;
                if (ok) rename(tmp.c_str(), (dir + fname).c_str());
                else unlink(tmp.c_str());
            }
        }
    }
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_codes.find(k);
    if (it == g_codes.end()) it = g_codes.emplace(k, std::move(code)).first;
    *code_out = it->second.get();
    return MS_OK;
}

} // namespace ms

extern "C" int32_t ms_jit_stats(int64_t *compiled, int64_t *from_disk, int64_t *from_memory, int32_t *compiler_major, int32_t *compiler_minor)
{
    std::lock_guard<std::mutex> lk(ms::g_mu);
    if (compiled) *compiled = ms::g_n_compiled;
    if (from_disk) *from_disk = ms::g_n_disk;
    if (from_memory) *from_memory = ms::g_n_mem;
    const uint64_t id = ms::compiler_id();
    if (compiler_major) *compiler_major = (int32_t)(id >> 32);
    if (compiler_minor) *compiler_minor = (int32_t)(id & 0xffffffffu);
    return MS_OK;
}

extern "C" int32_t ms_set_cache_dir(const char *path)
{
    std::lock_guard<std::mutex> lk(ms::g_mu);
    ms::g_cache_dir = path ? path : "";
    ms::g_cache_dir_set = true;
    return MS_OK;
}
