"""Every sampled trace computes the operator: 64 valid traces per configuration from the seeded sampler (256 for
config 2, the number of trials its configuration names), each run
at the configuration's full shape and compared with the oracle element by element (int8 bit for bit); each variant
is launched twice into poisoned outputs and the two results must be identical (Section 2: all programs of S(e0) are
semantically equal; Section 4, "Trace validation": what the validator lets through must run)."""
import numpy as np
import pytest

from oracle import compare
from oracle.workloads import oracle_run
from paper_2205_13603_amd import binding as B
from paper_2205_13603_amd.workloads import WORKLOADS, OUT_SHAPE, BOUND, workload_inputs
from gpu_util import run_variant

pytestmark = pytest.mark.gpu

N_TRACES = 64
N_TRACES_OF = {"c2_gemm_f16_1024": 256}
# (workload, module mask of the space, seed of the trace stream)
CONFIGS = [
    ("c1_gemm_f32_128", B.SPACE_UNROLL, 11),       # config 1 as stated: tiles + unroll, vector ALUs
    ("c1_gemm_f32_128", B.SPACE_DEFAULT, 12),      # the full vector-ALU space
    ("c2_gemm_f16_1024", B.SPACE_DEFAULT, 13),
    ("c3_conv_f16_56x56x64", B.SPACE_DEFAULT, 14),
    ("c4a_bmm_nt_f16", B.SPACE_DEFAULT, 15),
    ("c4b_bmm_nn_f16", B.SPACE_DEFAULT, 16),
    ("c4c_gemm_i8_512", B.SPACE_DEFAULT, 17),
    ("c5a_dw_f32_112x112x32", B.SPACE_DEFAULT, 18),
    ("c5b_dw_f32_56x56x144", B.SPACE_DEFAULT, 19),
]


@pytest.mark.parametrize("name,flags,seed", CONFIGS, ids=["%s-%x" % (c[0], c[1]) for c in CONFIGS])
def test_sampled_traces(name, flags, seed):
    mk, _ = WORKLOADS[name]
    op = mk()
    space = op.space(flags)
    ins = workload_inputs(name, 0)
    shape, odt = OUT_SHAPE[name]
    rtol = None if odt == "i32" else (compare.RTOL_F32 if BOUND[name][1] == "f32" else compare.RTOL_HALF)
    ref = None
    keys = set()
    n_traces = N_TRACES_OF.get(name, N_TRACES)
    for idx in range(n_traces):
        t = B.trace_sample_valid(op, space, seed, idx)
        keys.add(B.trace_validate(op, space, t).key)
        print(name, "trace", idx, t.decisions(), flush=True)
        got = run_variant(op, space, t, ins, odt, shape)
        if got is None:
            continue
        if ref is None:
            ref = np.asarray(oracle_run(name, ins)).reshape(shape)
        if odt == "i32":
            compare.assert_int_equal(got, ref, "%s trace %d" % (name, idx))
        else:
            compare.assert_float_close(got, ref, rtol, "%s trace %d" % (name, idx))
    assert len(keys) >= n_traces // 2, "the sampler keeps drawing the same kernels"
