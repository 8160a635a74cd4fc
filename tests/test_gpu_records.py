"""GPU parity of every stored tuning record.

bench.py times the best of these traces, so each one must compute its operator (Section 2: every program of the
space is semantically equal to e0): every record of every workload is rebuilt in the space named by its module mask
and run at the workload's full shape on three instances with distinct data (one launch), element by element against
the oracle; int32 results bit for bit.  Every launch is repeated and the two results must be identical."""
import numpy as np
import pytest

from oracle import compare
from oracle.workloads import oracle_run
from paper_2205_13603_amd import binding as B, tuned
from paper_2205_13603_amd.workloads import WORKLOADS, OUT_SHAPE, BOUND, workload_inputs
from gpu_util import run_variant_distinct

pytestmark = pytest.mark.gpu

INSTANCES = 3  # odd: the launch-wide tile order of the XCD-grouped variants is then not a multiple of 8


def tolerance(name):
    shape, odt = OUT_SHAPE[name]
    if odt == "i32":
        return None
    return compare.RTOL_F32 if BOUND[name][1] == "f32" else compare.RTOL_HALF


@pytest.mark.parametrize("name", sorted(WORKLOADS))
def test_every_record_matches_the_oracle(name):
    mk, _ = WORKLOADS[name]
    op = mk()
    recs = tuned.load_records(name)
    usable = tuned.records_with_traces(name, op, limit=len(recs))
    assert usable, "no usable record for %s" % name
    ins = [workload_inputs(name, 100 + r) for r in range(INSTANCES)]
    shape, odt = OUT_SHAPE[name]
    refs = None
    for n, (rec, space, trace) in enumerate(usable):
        print(name, "record", n, "flags", hex(space.flags), "us", rec.get("us"), trace.decisions(), flush=True)
        got = run_variant_distinct(op, space, trace, ins, odt, shape)
        if got is None:
            continue
        if refs is None:
            refs = [oracle_run(name, x) for x in ins]
        for r in range(INSTANCES):
            what = "%s record %d instance %d" % (name, n, r)
            if odt == "i32":
                compare.assert_int_equal(got[r], refs[r].reshape(shape), what)
            else:
                compare.assert_float_close(got[r], np.asarray(refs[r]).reshape(shape), tolerance(name), what)
