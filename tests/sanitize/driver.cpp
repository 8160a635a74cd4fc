// Exercises the host logic of libms and the C oracle under -fsanitize=address,undefined: every call the CPU tests
// make from Python, in bulk, including the error paths (truncated traces, bad text, tiny limits, NULL arguments).
// Exit status 0 = every check held; the sanitizers abort the program on the first finding.
#include "../../include/ms.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

extern "C" int ms_oracle_bmm(int dtype, int64_t nb, int64_t M, int64_t N, int64_t K, const void *A, int64_t sAb, int64_t sAi, int64_t sAk,
                             const void *B, int64_t sBb, int64_t sBk, int64_t sBj, double *C);

#define CHECK(x)                                                               \
    do {                                                                       \
        if (!(x)) {                                                            \
            fprintf(stderr, "%s:%d: CHECK failed: %s (last error: %s)\n", __FILE__, __LINE__, #x, ms_last_error()); \
            exit(1);                                                           \
        }                                                                      \
    } while (0)

static double fake_latency(const ms_variant_params *p, void *)
{
    // smooth, with an optimum at a 64 x 64 x 16 workgroup tile and 256 threads
    double a = std::log2((double)p->block_m) - 6, b = std::log2((double)p->block_n) - 6, c = std::log2((double)p->block_k) - 4;
    double t = std::log2((double)p->threads) - 8;
    return 1.0 + a * a + b * b + 0.5 * c * c + 0.25 * t * t + (p->cache_read == 0 ? 2.0 : 0.0);
}

static ms_op *make_op(int which)
{
    ms_op_desc d;
    memset(&d, 0, sizeof d);
    switch (which) {
    case 0: d.kind = MS_OP_GEMM; d.in_dtype = MS_F32; d.out_dtype = MS_F32; d.dims[0] = d.dims[1] = d.dims[2] = 128; break;
    case 1: d.kind = MS_OP_GEMM; d.in_dtype = MS_F16; d.out_dtype = MS_F16; d.dims[0] = 1024; d.dims[1] = 1024; d.dims[2] = 1024; break;
    case 2: d.kind = MS_OP_BMM_NT; d.in_dtype = MS_F16; d.out_dtype = MS_F16; d.dims[0] = 12; d.dims[1] = 128; d.dims[2] = 128; d.dims[3] = 64; break;
    case 3: d.kind = MS_OP_GEMM; d.in_dtype = MS_I8; d.out_dtype = MS_I32; d.dims[0] = d.dims[1] = d.dims[2] = 512; break;
    case 4:
        d.kind = MS_OP_CONV2D_NHWC; d.in_dtype = MS_F16; d.out_dtype = MS_F16; d.stride = 1; d.pad = 1; d.has_bias = 1; d.relu = 1;
        d.dims[0] = 1; d.dims[1] = 56; d.dims[2] = 56; d.dims[3] = 64; d.dims[4] = 64; d.dims[5] = 3; d.dims[6] = 3;
        break;
    case 5:
        d.kind = MS_OP_DWCONV2D_NHWC; d.in_dtype = MS_F32; d.out_dtype = MS_F32; d.stride = 2; d.pad = 1;
        d.dims[0] = 1; d.dims[1] = 56; d.dims[2] = 56; d.dims[3] = 144; d.dims[4] = 3; d.dims[5] = 3;
        break;
    case 6: d.kind = MS_OP_SOFTMAX; d.in_dtype = MS_F32; d.out_dtype = MS_F32; d.dims[0] = 1; d.dims[1] = 256; d.dims[2] = 256; break;
    case 7: d.kind = MS_OP_CONV1D_NWC; d.in_dtype = MS_F16; d.out_dtype = MS_F16; d.stride = 2; d.pad = 1; d.has_bias = 1; d.relu = 1;
        d.dims[0] = 1; d.dims[1] = 256; d.dims[2] = 64; d.dims[3] = 128; d.dims[4] = 3; break;
    default:
        d.kind = MS_OP_CONV3D_NDHWC; d.in_dtype = MS_F16; d.out_dtype = MS_F16; d.stride = 2; d.pad = 3; d.has_bias = 1; d.relu = 1;
        d.dims[0] = 1; d.dims[1] = 8; d.dims[2] = 32; d.dims[3] = 32; d.dims[4] = 3; d.dims[5] = 64; d.dims[6] = 7;
    }
    ms_op *op = nullptr;
    CHECK(ms_op_create(&d, &op) == MS_OK && op);
    return op;
}

int main()
{
    CHECK(ms_version() == MS_ABI_VERSION);
    // error paths must return codes, never touch freed or foreign memory
    CHECK(ms_op_create(nullptr, nullptr) == MS_ERR_BAD_ARG);
    CHECK(ms_trace_validate(nullptr, nullptr, nullptr, nullptr) == MS_ERR_BAD_ARG);
    ms_op_destroy(nullptr);
    const uint32_t masks[] = {MS_SPACE_DEFAULT, 0u, MS_SPACE_DEFAULT | MS_SPACE_RFACTOR, MS_SPACE_TENSORIZE | MS_SPACE_UNROLL, 0x7ffu};
    long valid = 0, invalid = 0;
    for (int which = 0; which < 9; ++which) {
        ms_op *op = make_op(which);
        ms_loop loops[MS_MAX_LOOPS];
        int32_t nl = 0;
        CHECK(ms_op_loops(op, loops, &nl) == MS_OK && nl >= 2);
        double flop, bytes;
        CHECK(ms_op_work(op, &flop, &bytes) == MS_OK && flop > 0 && bytes > 0);
        for (uint32_t mask : masks) {
            ms_space sp;
            int32_t rc = ms_space_describe(op, mask, &sp);
            if (rc != MS_OK) continue; // e.g. a convolution without the matrix-core module
            double lg;
            CHECK(ms_space_log10_size(&sp, &lg) == MS_OK && lg >= 0);
            for (uint64_t i = 0; i < 200; ++i) {
                ms_trace t, m, back;
                CHECK(ms_trace_sample(&sp, 7, i, &t) == MS_OK);
                ms_variant_params p;
                rc = ms_trace_validate(op, &sp, &t, &p);
                CHECK(rc == MS_OK || rc == MS_ERR_INVALID_TRACE);
                (rc == MS_OK ? valid : invalid)++;
                CHECK(ms_trace_mutate(&sp, &t, i * 31 + 5, &m) == MS_OK);
                size_t need = 0;
                CHECK(ms_trace_to_text(op, &sp, &t, nullptr, 0, &need) == MS_OK && need > 1);
                std::vector<char> buf(need);
                CHECK(ms_trace_to_text(op, &sp, &t, buf.data(), need, nullptr) == MS_OK);
                CHECK(ms_trace_from_text(&sp, buf.data(), &back) == MS_OK && memcmp(&back, &t, sizeof t) == 0);
                // truncated text, a buffer one byte short, a trace with a decision cut off
                std::string cut(buf.data(), need / 2);
                (void)ms_trace_from_text(&sp, cut.c_str(), &back);
                std::vector<char> small(need > 8 ? need - 7 : 1);
                CHECK(ms_trace_to_text(op, &sp, &t, small.data(), small.size(), nullptr) == MS_OK);
                ms_trace shorter = t;
                shorter.n -= 1;
                CHECK(ms_trace_validate(op, &sp, &shorter, nullptr) == MS_ERR_INVALID_TRACE);
                if (rc == MS_OK && i < 40) {
                    int64_t ob = 0, kn = 0;
                    CHECK(ms_op_tensor_bytes(op, -1, &ob) == MS_OK);
                    ms_op_desc dd;
                    CHECK(ms_op_get_desc(op, &dd) == MS_OK);
                    const int osz = dd.out_dtype == MS_F16 || dd.out_dtype == MS_BF16 ? 2 : 4;
                    std::vector<int32_t> counts((size_t)(ob / osz));
                    CHECK(ms_variant_coverage(op, &p, counts.data(), (int64_t)counts.size()) == MS_OK);
                    for (int32_t c : counts) CHECK(c == 1);
                    CHECK(ms_variant_reduction_coverage(op, &p, nullptr, 0, &kn) == MS_OK && kn > 0);
                    std::vector<int32_t> kc((size_t)kn);
                    CHECK(ms_variant_reduction_coverage(op, &p, kc.data(), kn, nullptr) == MS_OK);
                    for (int32_t c : kc) CHECK(c == 1);
                    double f[128];
                    int32_t nf = 0;
                    CHECK(ms_variant_features(op, &p, f, 128, &nf) == MS_OK && nf > 10);
                    size_t kt = 0;
                    CHECK(ms_variant_kernel_text(op, &p, nullptr, 0, &kt) == MS_OK && kt > 10);
                    std::vector<char> ktb(kt);
                    CHECK(ms_variant_kernel_text(op, &p, ktb.data(), kt, nullptr) == MS_OK);
                }
            }
        }
        // modules as data
        int32_t all[MS_MAX_MODULES], applied[MS_MAX_MODULES], na = 0;
        const int nm = ms_module_count();
        for (int i = 0; i < nm; ++i) all[i] = i;
        for (uint64_t seed = 0; seed < 50; ++seed) {
            ms_space sp;
            int32_t rc = ms_space_stochastic_compose(op, all, nm, seed, applied, &na, &sp);
            CHECK(rc == MS_OK && na >= 1 && na <= nm);
        }
        ms_op_destroy(op);
    }
    CHECK(valid > 1000 && invalid > 100);
    // tiny limits force rejections on every path
    ms_limits lim, keep;
    CHECK(ms_get_limits(&keep) == MS_OK);
    lim = keep;
    lim.max_threads = 64;
    lim.max_lds_bytes = 1024;
    lim.max_acc_per_thread = 4;
    CHECK(ms_set_limits(&lim) == MS_OK);
    {
        ms_op *op = make_op(1);
        ms_space sp;
        CHECK(ms_space_describe(op, MS_SPACE_DEFAULT, &sp) == MS_OK);
        ms_trace t;
        CHECK(ms_trace_sample_valid(op, &sp, 1, 0, 50, &t) == MS_ERR_INVALID_TRACE); // and the message must not have been formatted into itself
        CHECK(strlen(ms_last_error()) < 2000);
        ms_op_destroy(op);
    }
    CHECK(ms_set_limits(&keep) == MS_OK);
    // the search on a synthetic latency, with and without the cost model
    for (int model = 0; model < 2; ++model) {
        ms_op *op = make_op(0);
        ms_space sp;
        CHECK(ms_space_describe(op, MS_SPACE_DEFAULT, &sp) == MS_OK);
        ms_search_cfg cfg;
        ms_search_cfg_default(&cfg);
        cfg.trials = 160;
        cfg.seed = 11;
        cfg.cost_model = model;
        ms_search_result res;
        CHECK(ms_search(op, &sp, &cfg, nullptr, 0, nullptr, fake_latency, nullptr, nullptr, nullptr, &res) == MS_OK);
        CHECK(res.n_measured == 160 && res.best_us >= 1.0 && res.best_us < 3.0);
        ms_op_destroy(op);
    }
    // boosted trees: fit and predict
    {
        ms_cost_model *m = nullptr;
        CHECK(ms_cost_model_create(30, 3, 0.3, 2, &m) == MS_OK);
        std::vector<double> X(200 * 3), y(200), out(200);
        for (int i = 0; i < 200; ++i) {
            X[i * 3] = i % 7;
            X[i * 3 + 1] = (i * 5) % 11;
            X[i * 3 + 2] = i % 2;
            y[i] = X[i * 3] * 2 - X[i * 3 + 1] + 3 * X[i * 3 + 2];
        }
        CHECK(ms_cost_model_fit(m, X.data(), y.data(), 200, 3) == MS_OK);
        CHECK(ms_cost_model_predict(m, X.data(), 200, 3, out.data()) == MS_OK);
        double err = 0;
        for (int i = 0; i < 200; ++i) err += std::fabs(out[i] - y[i]);
        CHECK(err / 200 < 0.5);
        CHECK(ms_cost_model_predict(m, X.data(), 200, 2, out.data()) != MS_OK);
        ms_cost_model_destroy(m);
    }
    // the oracle's plain loops under the sanitizers as well: a small fp32 product, A = identity
    {
        const int n = 24;
        std::vector<float> A(n * n, 0.f), Bm(n * n);
        for (int i = 0; i < n; ++i) A[i * n + i] = 1.f;
        for (int i = 0; i < n * n; ++i) Bm[i] = (float)(i % 13) - 6.f;
        std::vector<double> Cc(n * n);
        CHECK(ms_oracle_bmm(0, 1, n, n, n, A.data(), 0, n, 1, Bm.data(), 0, n, 1, Cc.data()) == 0);
        for (int i = 0; i < n * n; ++i) CHECK(Cc[i] == (double)Bm[i]);
    }
    printf("sanitized host checks ok: %ld valid and %ld rejected traces\n", valid, invalid);
    return 0;
}
