// Stand-ins for the part of libms that talks to the compiler and the GPU, so that the host logic (operator
// definitions, space, sampler, mutation, text form, interpreter, validator, cost model, search on a synthetic
// latency) links into a CPU-only program built with the address and undefined-behaviour sanitizers.
#include "../../include/ms.h"

extern "C" int32_t ms_variant_build(const ms_op *, const ms_space *, const ms_trace *, ms_variant **out)
{
    if (out) *out = nullptr;
    return MS_ERR_UNSUPPORTED;
}
extern "C" void ms_variant_destroy(ms_variant *) {}
extern "C" int32_t ms_measure(ms_variant *, const ms_bufset *, int32_t, const ms_measure_cfg *, void *, ms_measure_result *) { return MS_ERR_UNSUPPORTED; }
extern "C" int32_t ms_prebuild(const ms_op *, const ms_space *, const ms_trace *, int32_t, int32_t, int32_t *n_built)
{
    if (n_built) *n_built = 0;
    return MS_OK;
}
