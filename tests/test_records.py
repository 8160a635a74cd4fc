"""Stored tuning records (best traces of earlier searches): every workload has at least one that still parses and
validates in the search space named by its module mask, so bench.py always has a candidate besides the fresh search."""
import pytest

from paper_2205_13603_amd import binding as B, tuned


@pytest.mark.parametrize("name", sorted(tuned.WORKLOADS))
def test_records_parse_in_their_own_space(name):
    mk, instances = tuned.WORKLOADS[name]
    op = mk()
    recs = tuned.load_records(name, "filling")
    assert recs, "no stored record for %s" % name
    assert all(a["us"] <= b["us"] for a, b in zip(recs, recs[1:]))      # best first
    usable = tuned.records_with_traces(name, op, limit=len(recs), protocol="filling")
    assert usable, "no record of %s is valid in today's space" % name
    best_rec, space, trace = usable[0]
    assert best_rec is recs[0] or best_rec["us"] <= 1.25 * recs[0]["us"], "the best records of %s no longer parse" % name
    p = B.trace_validate(op, space, trace)
    assert p.threads >= 64 and p.key != 0
    # the text form of a record is the exact round trip of its trace
    again = B.trace_from_text(space, B.trace_to_text(op, space, trace))
    assert bytes(again) == bytes(trace)
    assert instances >= 1


@pytest.mark.parametrize("name", ["c1_gemm_f32_128", "c2_gemm_f16_1024", "c3_conv_f16_56x56x64", "c4a_bmm_nt_f16", "c4b_bmm_nn_f16",
                                  "c4c_gemm_i8_512", "c5a_dw_f32_112x112x32", "c5b_dw_f32_56x56x144"])
def test_best_records_compile_without_spills_and_with_the_lds_the_validator_counted(name):
    """What the compiler made of the record the benchmark times (from the code object's metadata, no GPU): no scratch
    memory, registers within what the workgroup's wavefronts can share, and exactly the LDS bytes the validator
    charged the trace with."""
    mk, _ = tuned.WORKLOADS[name]
    op = mk()
    rec, space, trace = tuned.records_with_traces(name, op, limit=1, protocol="filling")[0]
    v = B.Variant(op, space, trace)
    p, r = v.params(), v.resources()
    assert r.scratch_bytes == 0 and r.spilled_vgprs == 0, "the best record of %s spills %d registers" % (name, r.spilled_vgprs)
    assert r.lds_bytes == p.lds_bytes
    waves_per_simd = (p.waves + 3) // 4
    assert 0 < r.vgprs + r.agprs <= 512 // waves_per_simd


def test_stored_trial_logs_give_pretraining_rows():
    """The trial logs kept next to the records (plain 256-trial searches, seeds 1-3, of the eight configurations) are the
    cost model's pre-training data: every logged trial still validates in today's space of its workload, its feature
    vector has the width the search expects, and leaving out the log of the seed being run leaves the other two."""
    import numpy as np
    from paper_2205_13603_amd.workloads import WORKLOADS
    names = [n for n in WORKLOADS if n.startswith("c")]
    assert len(names) == 8
    for name in names:
        logs = tuned.pretraining_logs(name, "filling")
        assert len(logs) == 3, (name, logs)
        assert len(tuned.pretraining_logs(name, "filling", exclude_seed=2)) == 2
        op = WORKLOADS[name][0]()
        sp = op.space(0xFF)
        X, y = tuned.pretraining_rows(op, sp, logs)
        assert X.shape[0] == y.shape[0] >= 700, (name, X.shape)       # 3 x 256 trials, all still valid
        p = B.trace_validate(op, sp, B.trace_sample_valid(op, sp, 1, 0))
        assert X.shape[1] == len(B.variant_features(op, p))
        assert np.all(np.isfinite(X)) and np.all(np.isfinite(y)) and y.min() > 0   # log2 of microseconds above 1
    assert tuned.pretraining_logs("x3_softmax_f32_256x256", "filling") == []
