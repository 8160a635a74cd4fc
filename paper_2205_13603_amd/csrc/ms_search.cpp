// Evolutionary search over traces (Section 4 of arXiv 2205.13603, "End-to-end
// search"): sample traces from the probabilistic program, then explore by
// mutating sampling decisions; the validator rejects proposals outside the
// hardware limits; every surviving candidate is measured on the device, and
// selection / acceptance follow the posterior of Eq. 1, exp(-f) up to an
// annealed temperature, with the measured latency f.  With cfg->cost_model the
// generation proposes model_candidates times as many children, a cost model
// fitted to all measurements so far (log2 of the latency as a function of the
// variant's features) predicts each, an annealed Metropolis-Hastings step on
// the predictions decides which children stay, and only the best predicted
// ones are measured: the paper's search, with boosted trees of this library.
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
    cfg->cost_model = 0;
    cfg->model_candidates = 8;
    cfg->model_min_trials = 48;
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
    std::vector<double> feat;  // features of each measured trial, row-major
    std::vector<double> target; // log2 of its latency
    int32_t n_feat = 0;
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
        if (cfg->cost_model) {
            double fv[128];
            int32_t nf = 0;
            if (ms_variant_features(op, &p, fv, 128, &nf) == MS_OK && (n_feat == 0 || nf == n_feat)) {
                n_feat = nf;
                feat.insert(feat.end(), fv, fv + nf);
                target.push_back(log2(us));
            }
        }
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
    if (cfg->cost_model && (cfg->model_candidates < 1 || cfg->model_candidates > 1024 || cfg->model_min_trials < 4))
        return fail(MS_ERR_BAD_ARG, "ms_search: bad cost-model configuration");
    const bool pretrained = cfg->cost_model && cfg->pretrain_n > 0;
    if (pretrained && (!cfg->pretrain_X || !cfg->pretrain_y || cfg->pretrain_d < 1 || cfg->pretrain_d > 128))
        return fail(MS_ERR_BAD_ARG, "ms_search: pre-training rows without arrays or with a bad width");
    ms_cost_model *model = nullptr;
    if (cfg->cost_model) {
        int32_t rc = ms_cost_model_create(60, 4, 0.3, 2, &model);
        if (rc != MS_OK) return rc;
    }
    struct ModelGuard {
        ms_cost_model *m;
        ~ModelGuard() { ms_cost_model_destroy(m); }
    } model_guard{model};
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
    if (pretrained) {
        for (int64_t i = 0; i < (int64_t)cfg->pretrain_n * cfg->pretrain_d; ++i)
            if (!std::isfinite(cfg->pretrain_X[i])) return fail(MS_ERR_BAD_ARG, "ms_search: pre-training feature %lld is not finite", (long long)i);
        for (int32_t i = 0; i < cfg->pretrain_n; ++i)
            if (!std::isfinite(cfg->pretrain_y[i])) return fail(MS_ERR_BAD_ARG, "ms_search: pre-training target %d is not finite", i);
        S.n_feat = cfg->pretrain_d;
        S.feat.assign(cfg->pretrain_X, cfg->pretrain_X + (size_t)cfg->pretrain_n * cfg->pretrain_d);
        S.target.assign(cfg->pretrain_y, cfg->pretrain_y + cfg->pretrain_n);
    }
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

    if (pretrained) {
        // the rows must be as wide as this operator's feature vectors (looked up on the first valid draw; the draws
        // themselves are made again below)
        for (uint64_t probe = 0; probe < 4096; ++probe) {
            ms_trace t;
            ms_variant_params p;
            if (ms_trace_sample(space, cfg->seed, probe, &t) != MS_OK) break;
            if (ms_trace_validate(op, space, &t, &p) != MS_OK) continue;
            int32_t nf = 0;
            if (ms_variant_features(op, &p, nullptr, 0, &nf) == MS_OK && nf != S.n_feat)
                return fail(MS_ERR_BAD_ARG, "ms_search: pre-training rows have %d features, this operator's variants %d", S.n_feat, nf);
            break;
        }
    }
    // initial population: draws from the prior P(tau); a pre-trained model picks half of them from a larger draw
    const int want_init = std::min(cfg->init_population, cfg->trials);
    if (pretrained && cfg->pretrain_n >= cfg->model_min_trials) {
        if (ms_cost_model_fit(model, S.feat.data(), S.target.data(), (int32_t)S.target.size(), S.n_feat) != MS_OK) return MS_ERR_BAD_ARG;
        struct Drawn {
            ms_trace t;
            double pred;
        };
        std::vector<Drawn> drawn;
        std::map<uint64_t, bool> have;
        const int pool = want_init * cfg->model_candidates;
        for (int tries = 0; (int)drawn.size() < pool && tries < pool * 1000; ++tries) {
            Drawn d;
            int32_t rc = ms_trace_sample(space, cfg->seed, sample_index++, &d.t);
            if (rc != MS_OK) return rc;
            ++proposals;
            ms_variant_params p;
            if (ms_trace_validate(op, space, &d.t, &p) != MS_OK) {
                ++out->n_invalid;
                continue;
            }
            if (have.count(p.key)) {
                ++out->n_duplicate;
                continue;
            }
            double fv[128];
            int32_t nf = 0;
            if (ms_variant_features(op, &p, fv, 128, &nf) != MS_OK) continue;
            if (nf != S.n_feat) return fail(MS_ERR_BAD_ARG, "ms_search: pre-training rows have %d features, this operator's variants %d", S.n_feat, nf);
            if (ms_cost_model_predict(model, fv, 1, nf, &d.pred) != MS_OK) continue;
            have[p.key] = true;
            drawn.push_back(d);
        }
        std::vector<size_t> by_pred(drawn.size());
        for (size_t i = 0; i < drawn.size(); ++i) by_pred[i] = i;
        std::stable_sort(by_pred.begin(), by_pred.end(), [&](size_t a, size_t b) { return drawn[a].pred < drawn[b].pred; });
        std::vector<bool> taken(drawn.size(), false);
        std::vector<ms_trace> batch;
        for (size_t r = 0; r < by_pred.size() && (int)batch.size() < (want_init + 1) / 2; ++r) {
            taken[by_pred[r]] = true;
            batch.push_back(drawn[by_pred[r]].t);
        }
        for (size_t i = 0; i < drawn.size() && (int)batch.size() < want_init; ++i)
            if (!taken[i]) batch.push_back(drawn[i].t);
        if (!fake_latency && !batch.empty()) ms_prebuild(op, space, batch.data(), (int32_t)batch.size(), cfg->compile_threads, nullptr);
        for (auto &t : batch) {
            if (S.stop || out->n_measured >= want_init) break;
            uint64_t key = 0;
            double us = S.evaluate(t, &key);
            if (us > 0) insert_member(t, us, key);
        }
    }
    {
        std::vector<ms_trace> batch;
        int want = want_init;
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
        auto propose = [&](Child *k) -> bool {
            ++proposals;
            if ((int)rng.below(1000) < cfg->eps_permille) {
                if (ms_trace_sample(space, cfg->seed, sample_index++, &k->t) != MS_OK) return false;
                k->parent = -1;
            } else {
                double u = unit_uniform(rng) * tot;
                size_t pi = (size_t)(std::lower_bound(cum.begin(), cum.end(), u) - cum.begin());
                if (pi >= pop.size()) pi = pop.size() - 1;
                if (ms_trace_mutate(space, &pop[pi].trace, rng.next(), &k->t) != MS_OK) return false;
                k->parent = (int)pi;
            }
            return true;
        };
        const bool use_model = model && (int32_t)S.target.size() >= cfg->model_min_trials && S.n_feat > 0;
        if (!use_model) {
            for (int c = 0; c < cfg->children && proposals < max_proposals; ++c) {
                Child k;
                if (propose(&k)) kids.push_back(k);
            }
        } else {
            // the model sees every measurement so far; targets are log2(latency)
            if (ms_cost_model_fit(model, S.feat.data(), S.target.data(), (int32_t)S.target.size(), S.n_feat) != MS_OK) return MS_ERR_BAD_ARG;
            struct Scored {
                Child k;
                double pred;
                uint64_t key;
            };
            std::vector<Scored> cand;
            std::map<uint64_t, bool> in_batch;
            // Candidates come from several rounds of mutation: in the first round the parents are measured
            // members of the population, in later rounds also candidates accepted so far (their cost is the
            // predicted one), so that the model can lead the search more than one decision away.
            const int want = cfg->children * cfg->model_candidates;
            const int rounds = 3;
            for (int round = 0; round < rounds; ++round) {
                const int goal = want * (round + 1) / rounds;
                const size_t n_prev = cand.size();
                for (int c = 0; c < want * 4 && (int)cand.size() < goal && proposals < max_proposals; ++c) {
                    Scored sc;
                    double parent_cost = -1;
                    if (round > 0 && n_prev > 0 && rng.below(2) == 0) {
                        ++proposals;
                        const Scored &src = cand[(size_t)rng.below(n_prev)];
                        if (ms_trace_mutate(space, &src.k.t, rng.next(), &sc.k.t) != MS_OK) continue;
                        sc.k.parent = src.k.parent; // the measured ancestor (-1: a fresh sample)
                        parent_cost = exp2(src.pred);
                    } else {
                        if (!propose(&sc.k)) continue;
                        if (sc.k.parent >= 0) parent_cost = pop[(size_t)sc.k.parent].us;
                    }
                    ms_variant_params p;
                    if (ms_trace_validate(op, space, &sc.k.t, &p) != MS_OK) {
                        ++out->n_invalid;
                        continue;
                    }
                    if (S.seen.count(p.key) || in_batch.count(p.key)) {
                        ++out->n_duplicate;
                        continue;
                    }
                    double fv[128];
                    int32_t nf = 0;
                    if (ms_variant_features(op, &p, fv, 128, &nf) != MS_OK || nf != S.n_feat) continue;
                    if (ms_cost_model_predict(model, fv, 1, nf, &sc.pred) != MS_OK) continue;
                    // annealed Metropolis-Hastings on the predicted cost: a child predicted slower than its parent
                    // survives with probability exp(-(f^_child - f_parent) / (T f_best)), latencies in microseconds
                    if (parent_cost > 0) {
                        const double fc = exp2(sc.pred);
                        if (fc > parent_cost && !(unit_uniform(rng) < exp(-(fc - parent_cost) / (T * fbest)))) continue;
                    }
                    sc.key = p.key;
                    in_batch[p.key] = true;
                    cand.push_back(sc);
                }
            }
            // Half of the generation's measurements go to the best predicted candidates, the other half to
            // candidates in the order they were proposed (the plain search's own distribution): a model that
            // is wrong about a region it has not seen must not be able to keep the search out of it.
            // Fresh samples keep their share of the slots.
            std::vector<size_t> by_pred(cand.size());
            for (size_t i = 0; i < cand.size(); ++i) by_pred[i] = i;
            std::stable_sort(by_pred.begin(), by_pred.end(), [&](size_t a, size_t b) { return cand[a].pred < cand[b].pred; });
            int fresh_quota = (cfg->children * cfg->eps_permille + 999) / 1000;
            std::vector<bool> taken(cand.size(), false);
            auto take = [&](size_t i) {
                kids.push_back(cand[i].k);
                taken[i] = true;
            };
            for (size_t i = 0; i < cand.size() && fresh_quota > 0 && (int)kids.size() < cfg->children; ++i)
                if (cand[i].k.parent < 0) {
                    take(i);
                    --fresh_quota;
                }
            const int by_model = ((int)cfg->children - (int)kids.size() + 1) / 2 + (int)kids.size();
            for (size_t r = 0; r < by_pred.size() && (int)kids.size() < by_model; ++r)
                if (!taken[by_pred[r]]) take(by_pred[r]);
            for (size_t i = 0; i < cand.size() && (int)kids.size() < cfg->children; ++i)
                if (!taken[i]) take(i);
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
