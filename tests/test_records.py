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
