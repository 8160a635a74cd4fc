"""The search on the device (Section 4, "End-to-end search", Eq. 1): ms_search measures real candidates, and every
candidate it measures is rebuilt from the trace the trial callback receives, launched into a poisoned output and
compared with the oracle.  A search ranks on latency alone, so a variant that is fast because it is wrong must be
caught here."""
import numpy as np
import pytest

from oracle import compare
from oracle.workloads import oracle_run
from paper_2205_13603_amd import binding as B, devmem, tuned
from paper_2205_13603_amd.workloads import WORKLOADS, OUT_SHAPE, BOUND, workload_inputs

pytestmark = pytest.mark.gpu

TRIALS = 32


def _search(name, seed, trials, init_population, cost_model=0, check=True, pretrain=None):
    import torch
    mk, _ = WORKLOADS[name]
    op = mk()
    space = op.space()
    R = 2
    ins = [workload_inputs(name, 200 + r) for r in range(R)]
    shape, odt = OUT_SHAPE[name]
    dev = [devmem.to_device(np.stack([ins[r][k] for r in range(R)])) for k in range(len(ins[0]))]
    out = devmem.empty_output(shape, odt, R, poison=True)
    stream = devmem.current_stream()
    sets = [([d.data_ptr() for d in dev], out.data_ptr())]
    refs = [np.asarray(oracle_run(name, x)).reshape(shape) for x in ins] if check else None
    rtol = None if odt == "i32" else (compare.RTOL_F32 if BOUND[name][1] == "f32" else compare.RTOL_HALF)
    trials_seen = []
    errors = []

    def on_trial(t):
        trials_seen.append((t.index, t.status, t.us, t.key))
        if t.status != 0 or not check:
            return 0
        try:
            trace = t.trace.copy()
            v = B.Variant(op, space, trace)  # the kernel the search just measured (in the library's cache)
            assert v.params().key == t.key
            chk = devmem.empty_output(shape, odt, R, poison=True)
            v.launch([d.data_ptr() for d in dev], chk.data_ptr(), instances=R, stream=stream)
            got = devmem.to_host(chk, odt)
            for r in range(R):
                what = "%s search trial %d %s instance %d" % (name, t.index, trace.decisions(), r)
                if odt == "i32":
                    compare.assert_int_equal(got[r], refs[r], what)
                else:
                    compare.assert_float_close(got[r], refs[r], rtol, what)
        except Exception as e:  # an exception must not unwind through the C callback
            errors.append(repr(e)[:2000])
            return 1  # stop the search at the first mismatch
        return 0

    cfg = B.search_cfg_default()
    cfg.seed, cfg.trials, cfg.init_population = seed, trials, init_population
    cfg.population, cfg.children = 8, 8
    cfg.compile_threads = 16
    cfg.cost_model, cfg.model_min_trials = cost_model, 12
    cfg.measure = B.ms_measure_cfg(1, 3, 3, R)
    rows = tuned.pretraining_rows(op, space, tuned.pretraining_logs(name, "filling")) if pretrain else None
    if pretrain:
        assert len(rows[1]) >= 256, "stored trial logs of %s" % name
    res = B.search(op, space, cfg, bufsets=sets, stream=stream, on_trial=on_trial, pretrain=rows)
    torch.cuda.synchronize()
    return res, trials_seen, errors


@pytest.mark.parametrize("name", ["c2_gemm_f16_1024", "c3_conv_f16_56x56x64", "c5a_dw_f32_112x112x32", "c4c_gemm_i8_512"])
def test_every_measured_candidate_of_a_real_search_matches_the_oracle(name):
    if not devmem.gpu_available():
        pytest.skip("the search measures on the device")
    res, seen, errors = _search(name, seed=5, trials=TRIALS, init_population=12)
    assert not errors, errors[0]
    ok = [s for s in seen if s[1] == 0]
    assert res.n_measured == TRIALS == len(ok)
    assert res.n_failed == 0, "candidates the validator let through failed to build or launch"
    assert [s[0] for s in ok] == list(range(1, TRIALS + 1))
    assert len({s[3] for s in ok}) == TRIALS, "one kernel was measured twice"
    assert res.best_us == min(s[2] for s in ok) and 1 <= res.best_trial <= TRIALS
    print(name, "best %.2f us at trial %d" % (res.best_us, res.best_trial), flush=True)


def test_same_seed_same_initial_population():
    """The initial population is drawn from the prior with the seeded counter generator: two searches with one
    seed measure the same kernels in the same order, whatever the latencies were."""
    if not devmem.gpu_available():
        pytest.skip("the search measures on the device")
    name = "c5a_dw_f32_112x112x32"
    a = _search(name, seed=9, trials=8, init_population=8, check=False)[1]
    b = _search(name, seed=9, trials=8, init_population=8, check=False)[1]
    c = _search(name, seed=10, trials=8, init_population=8, check=False)[1]
    assert [s[3] for s in a] == [s[3] for s in b]
    assert [s[3] for s in a] != [s[3] for s in c]


def test_model_guided_search_measures_correct_kernels():
    """The cost-model branch of the search (Section 4): proposals are ranked by the boosted trees fitted to the
    measurements so far; what it then measures is checked against the oracle like any other candidate."""
    if not devmem.gpu_available():
        pytest.skip("the search measures on the device")
    res, seen, errors = _search("c5b_dw_f32_56x56x144", seed=3, trials=40, init_population=12, cost_model=1)
    assert not errors, errors[0]
    assert res.n_measured == 40 and res.n_failed == 0


def test_pretrained_model_picks_a_better_initial_population():
    """The model fitted beforehand on the stored trial logs of the workload (Section 4 allows a model trained before the search)
    chooses half of the initial population from 8x as many draws: the better half of the 12 kernels it measures first
    is faster than the better half of the 12 random draws the plain search starts with (same seed), and every kernel is
    checked against the oracle."""
    if not devmem.gpu_available():
        pytest.skip("the search measures on the device")
    name = "c5a_dw_f32_112x112x32"
    res, seen, errors = _search(name, seed=6, trials=24, init_population=12, cost_model=1, pretrain=True)
    assert not errors, errors[0]
    assert res.n_measured == 24 and res.n_failed == 0
    plain = _search(name, seed=6, trials=12, init_population=12, check=False)[1]
    first = sorted(s[2] for s in seen[:12] if s[1] == 0)[:6]
    base = sorted(s[2] for s in plain if s[1] == 0)[:6]
    print("pre-trained", first, "plain", base, flush=True)
    assert sum(first) < sum(base)
