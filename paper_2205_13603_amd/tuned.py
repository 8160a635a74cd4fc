"""Tuning records: the best traces earlier searches found, kept as text next to the package (one file per
workload, the linearised trace of Section 4 plus the measured latency), one line per record.  Records are only candidates: they are re-measured before use."""
import json
import os

from . import binding as B
from .workloads import WORKLOADS  # noqa: F401  (name -> (op factory, instances of one device-filling launch))

HERE = os.path.dirname(os.path.abspath(__file__))
RECORD_DIR = os.path.join(HERE, "tuned_records")


def record_path(name):
    return os.path.join(RECORD_DIR, name + ".jsonl")


def load_records(name, protocol=None):
    """List of dicts {trace: text, us: float, protocol: "filling" | "steady", mode: str, ...}, best first.
    `protocol` keeps the records measured that way (records without the field are device-filling ones)."""
    path = record_path(name)
    if not os.path.exists(path):
        return []
    recs = [json.loads(line) for line in open(path) if line.strip()]
    if protocol is not None:
        recs = [r for r in recs if r.get("protocol", "filling") == protocol]
    return sorted(recs, key=lambda r: r.get("us", 1e30))


SEARCHES = os.path.join(RECORD_DIR, "searches.jsonl")


def load_searches(name, trials=256):
    """Summaries of the stored `trials`-trial searches of a workload (one line per run of the tuning command)."""
    if not os.path.exists(SEARCHES):
        return []
    rows = [json.loads(line) for line in open(SEARCHES) if line.strip()]
    return [r for r in rows if r.get("workload") == name and r.get("trials") == trials]


def append_record(name, rec):
    os.makedirs(RECORD_DIR, exist_ok=True)
    with open(record_path(name), "a") as f:
        f.write(json.dumps(rec, sort_keys=True) + "\n")


def records_with_traces(name, op, limit=4, protocol=None):
    """[(record dict, space, parsed trace)] of the stored records that still parse and validate, best first.
    Every record names the module mask of the space it was found in (`flags`), so each gets its own space."""
    out = []
    spaces = {}
    for rec in load_records(name, protocol)[:limit]:
        flags = int(rec.get("flags", B.SPACE_DEFAULT))
        try:
            if flags not in spaces:
                spaces[flags] = op.space(flags)
            space = spaces[flags]
            t = B.trace_from_text(space, rec["trace"])
            B.trace_validate(op, space, t)
            out.append((rec, space, t))
        except B.MsError:
            continue
    return out


def precompile_all(threads=4):
    n = 0
    for name, (mk, _) in WORKLOADS.items():
        op = mk()
        for protocol in ("filling", "steady"):
            for _, space, t in records_with_traces(name, op, protocol=protocol):
                n += B.prebuild(op, space, [t], threads)
    return n
