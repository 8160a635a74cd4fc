"""Tuning records: the best traces earlier searches found, kept as text next to the package (one file per
workload, the linearised trace of Section 4 plus the measured latency), and the workload table shared by
bench.py and the tuning command.  Records are only candidates: they are re-measured before use."""
import json
import os

from . import binding as B

HERE = os.path.dirname(os.path.abspath(__file__))
RECORD_DIR = os.path.join(HERE, "tuned_records")

# name -> (op factory, instances of one device-filling launch)
WORKLOADS = {
    "c1_gemm_f32_128": (lambda: B.gemm_op(128, 128, 128, "f32"), 4096),
    "c2_gemm_f16_1024": (lambda: B.gemm_op(1024, 1024, 1024, "f16"), 64),
    "x2_gemm_f8_1024": (lambda: B.gemm_op(1024, 1024, 1024, "f8", "f16"), 64),
    "c3_conv_f16_56x56x64": (lambda: B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1), 512),
    "c4a_bmm_nt_f16": (lambda: B.bmm_op(12, 128, 128, 64, True, "f16"), 1024),
    "c4b_bmm_nn_f16": (lambda: B.bmm_op(12, 128, 64, 128, False, "f16"), 1024),
    "c4c_gemm_i8_512": (lambda: B.gemm_op(512, 512, 512, "i8"), 512),
    "c5a_dw_f32_112x112x32": (lambda: B.dwconv2d_op(1, 112, 112, 32, stride=1, pad=1), 512),
    "c5b_dw_f32_56x56x144": (lambda: B.dwconv2d_op(1, 56, 56, 144, stride=2, pad=1), 512),
    "x5_cbr_f16_224x224x3": (lambda: B.conv2d_op(1, 224, 224, 3, 64, 7, 7, stride=2, pad=3), 256),
    "x5b_cbr_f16_224x224x4": (lambda: B.conv2d_op(1, 224, 224, 4, 64, 7, 7, stride=2, pad=3), 256),
    "x6_t2d_f16_4x4x512": (lambda: B.conv2d_transposed_op(1, 4, 4, 512, 256, 4, 4, stride=2, pad=1), 128),
    "x7_grp_f16_56x56x64_g4": (lambda: B.conv2d_op(1, 56, 56, 64, 128, 3, 3, stride=2, pad=1, groups=4), 512),
    "x8_gemm_nt_f16_1024": (lambda: B.bmm_op(1, 1024, 1024, 1024, True, "f16"), 64),
    "x9_c1d_f16_256x64": (lambda: B.conv1d_op(1, 256, 64, 128, 3, stride=2, pad=1), 4096),
    "x10_c3d_f16_16x224x224x3": (lambda: B.conv3d_op(1, 16, 224, 224, 3, 64, 7, stride=2, pad=3), 8),
    "x11_gemm_bf16_1024": (lambda: B.gemm_op(1024, 1024, 1024, "bf16"), 64),
    "x12_conv_bf16_56x56x64": (lambda: B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1, in_dtype="bf16"), 512),
    "x3_softmax_f32_256x256": (lambda: B.softmax_op(1, 256, 256), 2048),
    "x4_norm_f32_256x256": (lambda: B.norm_op(1, 256, 256), 2048),
}


def record_path(name):
    return os.path.join(RECORD_DIR, name + ".jsonl")


def load_records(name):
    """List of dicts {trace: text, us: float, mode: str, ...}, best first."""
    path = record_path(name)
    if not os.path.exists(path):
        return []
    recs = [json.loads(line) for line in open(path) if line.strip()]
    return sorted(recs, key=lambda r: r.get("us", 1e30))


def append_record(name, rec):
    os.makedirs(RECORD_DIR, exist_ok=True)
    with open(record_path(name), "a") as f:
        f.write(json.dumps(rec, sort_keys=True) + "\n")


def records_with_traces(name, op, limit=4):
    """[(record dict, space, parsed trace)] of the stored records that still parse and validate, best first.
    Every record names the module mask of the space it was found in (`flags`), so each gets its own space."""
    out = []
    spaces = {}
    for rec in load_records(name)[:limit]:
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
        for _, space, t in records_with_traces(name, op):
            n += B.prebuild(op, space, [t], threads)
    return n
