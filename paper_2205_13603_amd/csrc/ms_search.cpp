// Evolutionary search over traces (Section 4 of arXiv 2205.13603, "End-to-end
// search"): sample traces from the probabilistic program, then explore by
// mutating sampling decisions; the validator rejects proposals outside the
// hardware limits; every surviving candidate is measured on the device, and
// selection / acceptance follow the posterior of Eq. 1, exp(-f) up to an
// annealed temperature, with the measured latency f (no learned cost model).
#include "ms_internal.h"

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <map>
#include <vector>

using namespace ms;

extern "C" void ms_search_cfg_default(ms_search_cfg *cfg)
{
    if (!cfg) return;
    memset(cfg, 0, sizeof *cfg);
    cfg->seed = 0;
    cfg->trials = 256;
    cfg->init_population = 32;
    cfg->population = 16;
    cfg->children = 16;
    cfg->eps_permille = 100;
    cfg->compile_threads = 8;
    cfg->temperature0 = 1.0;
    cfg->temperature1 = 0.1;
    cfg->measure.warmup = 2;
    cfg->measure.repeats = 5;
    cfg->measure.launches_per_repeat = 20;
    cfg->measure.instances = 1;
}

namespace {

struct Member {
    ms_trace trace;
    double us;
    uint64_t key;
};

struct Search {
    const ms_op *op;
    const ms_space *space;
    const ms_search_cfg *cfg;
    const ms_bufset *sets;
    int32_t n_sets;
    void *stream;
    ms_latency_fn fake;
    void *fake_user;
    ms_trial_cb cb;
    void *cb_user;
    ms_search_result *res;
    std::map<uint64_t, double> seen;
    std::vector<double> curve; // latency of each measured trial
    bool stop = false;

    // returns latency in us, or < 0 when the candidate produced no measurement
    double evaluate(const ms_trace &t, uint64_t *key_out)
    {
        ms_variant_params p;
        if (ms_trace_validate(op, space, &t, &p) != MS_OK) {
            ++res->n_invalid;
            return -1;
        }
        *key_out = p.key;
        if (seen.count(p.key)) {
            ++res->n_duplicate;
            return -2;
        }
        double us = -1;
        int32_t status = MS_OK;
        if (fake) {
            us = fake(&p, fake_user);
            if (!(us > 0)) status = MS_ERR_HIP;
        } else {
            ms_variant *v = nullptr;
            status = ms_variant_build(op, space, &t, &v);
            if (status == MS_OK) {
                ms_measure_result mr;
                status = ms_measure(v, sets, n_sets, &cfg->measure, stream, &mr);
                if (status == MS_OK) us = mr.median_us;
            }
            ms_variant_destroy(v);
        }
        seen[p.key] = us;
        ms_trial tr;
        memset(&tr, 0, sizeof tr);
        tr.trace = t;
        tr.key = p.key;
        tr.status = status;
        if (status != MS_OK || !(us > 0)) {
            ++res->n_failed;
            tr.index = res->n_measured;
            tr.us = -1;
            tr.best_us = res->best_us;
            if (cb && cb(&tr, cb_user)) stop = true;
            return -1;
        }
        ++res->n_measured;
        curve.push_back(us);
        if (res->best_us <= 0 || us < res->best_us) {
            res->best_us = us;
            res->best_trace = t;
        }
        tr.index = res->n_measured;
        tr.us = us;
        tr.best_us = res->best_us;
        if (cb && cb(&tr, cb_user)) stop = true;
        return us;
    }
};

double unit_uniform(Rng &rng) { return (double)rng.below(1ull << 53) / (double)(1ull << 53); }

} // namespace

extern "C" int32_t ms_search(const ms_op *op, const ms_space *space, const ms_search_cfg *cfg, const ms_bufset *sets, int32_t n_sets,
                             void *stream, ms_latency_fn fake_latency, void *fake_user, ms_trial_cb cb, void *cb_user,
                             ms_search_result *out)
{
    if (!op || !space || !cfg || !out) return fail(MS_ERR_BAD_ARG, "ms_search: NULL argument");
    if (!fake_latency && (!sets || n_sets < 1)) return fail(MS_ERR_BAD_ARG, "ms_search: no buffer sets to measure on");
    if (cfg->trials < 1 || cfg->init_population < 1 || cfg->population < 1 || cfg->children < 1 || cfg->eps_permille < 0 ||
        cfg->eps_permille > 1000 || !(cfg->temperature0 > 0) || !(cfg->temperature1 > 0))
        return fail(MS_ERR_BAD_ARG, "ms_search: bad configuration");
    auto t_start = std::chrono::steady_clock::now();
    memset(out, 0, sizeof *out);
    Search S;
    S.op = op;
    S.space = space;
    S.cfg = cfg;
    S.sets = sets;
    S.n_sets = n_sets;
    S.stream = stream;
    S.fake = fake_latency;
    S.fake_user = fake_user;
    S.cb = cb;
    S.cb_user = cb_user;
    S.res = out;
    Rng rng(mix64(cfg->seed ^ 0x5851F42D4C957F2Dull));
    std::vector<Member> pop;
    uint64_t sample_index = 0;
    const int64_t max_proposals = (int64_t)cfg->trials * 200 + 10000;
    int64_t proposals = 0;

    auto insert_member = [&](const ms_trace &t, double us, uint64_t key) {
        Member m;
        m.trace = t;
        m.us = us;
        m.key = key;
        pop.push_back(m);
        std::sort(pop.begin(), pop.end(), [](const Member &a, const Member &b) { return a.us < b.us; });
        if ((int)pop.size() > cfg->population) pop.resize((size_t)cfg->population);
    };

    // initial population: draws from the prior P(tau)
    {
        std::vector<ms_trace> batch;
        int want = std::min(cfg->init_population, cfg->trials);
        while (out->n_measured < want && !S.stop && proposals < max_proposals) {
            batch.clear();
            int need = want - out->n_measured;
            for (int tries = 0; (int)batch.size() < need && tries < need * 1000; ++tries) {
                ms_trace t;
                int32_t rc = ms_trace_sample(space, cfg->seed, sample_index++, &t);
                if (rc != MS_OK) return rc;
                ++proposals;
                if (ms_trace_validate(op, space, &t, nullptr) == MS_OK) batch.push_back(t);
                else ++out->n_invalid;
            }
            if (batch.empty()) return fail(MS_ERR_INVALID_TRACE, "ms_search: the sampler produced no valid trace");
            if (!fake_latency) ms_prebuild(op, space, batch.data(), (int32_t)batch.size(), cfg->compile_threads, nullptr);
            for (auto &t : batch) {
                if (S.stop || out->n_measured >= want) break;
                uint64_t key = 0;
                double us = S.evaluate(t, &key);
                if (us > 0) insert_member(t, us, key);
            }
        }
    }
    if (pop.empty()) return fail(MS_ERR_HIP, "ms_search: no candidate of the initial population could be measured (%s)", ms_last_error());

    // generations
    while (out->n_measured < cfg->trials && !S.stop && proposals < max_proposals) {
        double progress = (double)out->n_measured / (double)cfg->trials;
        double T = cfg->temperature0 * pow(cfg->temperature1 / cfg->temperature0, progress);
        double fbest = out->best_us;
        // parents drawn with probability proportional to exp(-f / (T f_best))
        std::vector<double> cum(pop.size());
        double tot = 0;
        for (size_t i = 0; i < pop.size(); ++i) {
            tot += exp(-(pop[i].us - fbest) / (T * fbest));
            cum[i] = tot;
        }
        struct Child {
            ms_trace t;
            int parent; // -1 = fresh sample
        };
        std::vector<Child> kids;
        for (int c = 0; c < cfg->children && proposals < max_proposals; ++c) {
            Child k;
            ++proposals;
            if ((int)rng.below(1000) < cfg->eps_permille) {
                if (ms_trace_sample(space, cfg->seed, sample_index++, &k.t) != MS_OK) continue;
                k.parent = -1;
            } else {
                double u = unit_uniform(rng) * tot;
                size_t pi = (size_t)(std::lower_bound(cum.begin(), cum.end(), u) - cum.begin());
                if (pi >= pop.size()) pi = pop.size() - 1;
                if (ms_trace_mutate(space, &pop[pi].trace, rng.next(), &k.t) != MS_OK) continue;
                k.parent = (int)pi;
            }
            kids.push_back(k);
        }
        if (!fake_latency) {
            std::vector<ms_trace> batch;
            for (auto &k : kids) batch.push_back(k.t);
            ms_prebuild(op, space, batch.data(), (int32_t)batch.size(), cfg->compile_threads, nullptr);
        }
        std::vector<Member> snapshot = pop; // parents as they were when the children were proposed
        for (auto &k : kids) {
            if (S.stop || out->n_measured >= cfg->trials) break;
            uint64_t key = 0;
            double us = S.evaluate(k.t, &key);
            if (!(us > 0)) continue;
            bool accept = (int)pop.size() < cfg->population || us < pop.back().us;
            if (!accept && k.parent >= 0) {
                double a = exp(-(us - snapshot[(size_t)k.parent].us) / (T * out->best_us));
                accept = unit_uniform(rng) < a;
                if (accept && (int)pop.size() >= cfg->population) pop.pop_back(); // replaces the worst member
            }
            if (accept) insert_member(k.t, us, key);
        }
    }
    // first trial within 1 % of the final best
    out->best_trial = 0;
    for (size_t i = 0; i < S.curve.size(); ++i)
        if (S.curve[i] <= out->best_us * 1.01) {
            out->best_trial = (int32_t)i + 1;
            break;
        }
    out->wall_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t_start).count();
    return MS_OK;
}
