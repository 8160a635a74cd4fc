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


def pretraining_rows(op, space, log_paths):
    """(X, y) for the search's cost model from the trial logs the tuning command writes: the feature vector of
    every measured trial whose trace still validates in `space`, and log2 of its latency in microseconds.  The
    logs must be of the same workload and measurement protocol as the search that uses the rows."""
    import math
    import numpy as np
    X, y = [], []
    for path in log_paths:
        for line in open(path):
            if not line.strip():
                continue
            r = json.loads(line)
            if r.get("status") != 0 or not r.get("us", 0) > 0:
                continue
            try:
                p = B.trace_validate(op, space, B.trace_from_decisions(space, r["decisions"]))
            except (B.MsError, ValueError):
                continue
            X.append(B.variant_features(op, p))
            y.append(math.log2(r["us"]))
    return np.array(X, dtype=np.float64).reshape(len(y), -1), np.array(y, dtype=np.float64)


PRETRAIN_DIR = os.path.join(RECORD_DIR, "logs")


def pretraining_logs(name, protocol, exclude_seed=None):
    """Stored trial logs of a workload under a protocol (written by the tuning command, kept next to the records)."""
    if not os.path.isdir(PRETRAIN_DIR):
        return []
    pre = "%s.%s.s" % (name, protocol)
    out = []
    for f in sorted(os.listdir(PRETRAIN_DIR)):
        if f.startswith(pre) and f.endswith(".log.jsonl"):
            if exclude_seed is not None and f == "%s%d.log.jsonl" % (pre, exclude_seed):
                continue
            out.append(os.path.join(PRETRAIN_DIR, f))
    return out


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
