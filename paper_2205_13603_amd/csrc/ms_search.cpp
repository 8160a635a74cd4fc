// Evolutionary search over traces (Section 4 of arXiv 2205.13603) on measured latency.
#include "ms_internal.h"

using namespace ms;

extern "C" void ms_search_cfg_default(ms_search_cfg *cfg)
{
    if (!cfg) return;
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

extern "C" int32_t ms_search(const ms_op *, const ms_space *, const ms_search_cfg *, const ms_bufset *, int32_t, void *,
                             ms_latency_fn, void *, ms_trial_cb, void *, ms_search_result *)
{
    return fail(MS_ERR_UNSUPPORTED, "ms_search: not built yet");
}
