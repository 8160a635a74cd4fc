"""Tune one workload on the GPU: run the evolutionary search over traces and store the best as a record.

    python -m paper_2205_13603_amd.tune --workload c2_gemm_f16_1024 --trials 256 --out tuned_out

Writes <out>/<workload>.jsonl (best record, appendable to tuned_records/) and <out>/<workload>.log.jsonl
(every trial: index, status, latency, best so far, trace text) so that a search can be inspected or resumed.
"""
import argparse
import json
import os
import sys
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--trials", type=int, default=256)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--instances", type=int, default=0)
    ap.add_argument("--flags", type=lambda s: int(s, 0), default=0xFF, help="search-space module mask (0xff = default, 0x1ff = with fp32 tensorize)")
    ap.add_argument("--out", default="tuned_out")
    ap.add_argument("--cost-model", action="store_true", help="let the learned cost model pick which proposals are measured")
    ap.add_argument("--model-candidates", type=int, default=8, help="proposals scored per measured candidate")
    ap.add_argument("--seed-records", action="store_true", help="measure stored records first (reported, not part of the search)")
    ap.add_argument("--measure", default="1,3,3", help="warm-up launches, repeats, launches per repeat of every trial; a long "
                    "warm-up (e.g. 150,3,20) times candidates at the clocks of a sustained run instead of just after an idle gap")
    args = ap.parse_args()

    import torch
    from . import binding as B, devmem, tuned
    from .workloads import workload_inputs, OUT_SHAPE

    devmem.require_gpu()
    mk, default_r = tuned.WORKLOADS[args.workload]
    R = args.instances or default_r
    op = mk()
    space = op.space(args.flags)
    base = [workload_inputs(args.workload, s) for s in range(min(4, R))]
    dev_in = []
    for k in range(len(base[0])):
        parts = [devmem.to_device(b[k]) for b in base]
        reps = (R + len(parts) - 1) // len(parts)
        dev_in.append(torch.stack(parts * reps)[:R].contiguous())
    shape, odt = OUT_SHAPE[args.workload]
    dev_out = devmem.empty_output(shape, odt, R)
    sets = [([t.data_ptr() for t in dev_in], dev_out.data_ptr())]
    os.makedirs(args.out, exist_ok=True)
    log = open(os.path.join(args.out, args.workload + ".log.jsonl"), "w")
    t0 = time.time()

    curve = []  # (trial index, best latency so far)

    def on_trial(t):
        if t.status == 0:
            curve.append((t.index, t.best_us))
        rec = {"trial": t.index, "status": t.status, "us": t.us, "best_us": t.best_us, "key": "%016x" % t.key,
               "decisions": t.trace.decisions(), "t": round(time.time() - t0, 2)}
        log.write(json.dumps(rec) + "\n")
        log.flush()
        if t.status == 0 and t.index % 8 == 0:
            print("trial %d: %.2f us, best %.2f us (%.1f s)" % (t.index, t.us, t.best_us, time.time() - t0), flush=True)
        return 0

    cfg = B.search_cfg_default()
    cfg.seed, cfg.trials = args.seed, args.trials
    cfg.cost_model, cfg.model_candidates = int(args.cost_model), args.model_candidates
    wu, reps, lpr = (int(x) for x in args.measure.split(","))
    cfg.measure = B.ms_measure_cfg(wu, reps, lpr, R)
    res = B.search(op, space, cfg, bufsets=sets, stream=devmem.current_stream(), on_trial=on_trial)
    flop, byts = op.work()
    rec = {"workload": args.workload, "trace": B.trace_to_text(op, space, res.best_trace), "us": res.best_us,
           "mode": "device-filling, %d instances" % R, "tflops": flop * R / res.best_us / 1e6, "gbs": byts * R / res.best_us / 1e3,
           "trials": res.n_measured, "trials_to_best": res.best_trial, "invalid": res.n_invalid, "failed": res.n_failed,
           "duplicate": res.n_duplicate, "search_seconds": round(res.wall_seconds, 1), "seed": args.seed, "flags": args.flags,
           # first measured trial whose best-so-far latency is within 1 % of the final best
           "trials_to_within_1pct": next((i for i, b in curve if b <= 1.01 * res.best_us), res.best_trial)}
    with open(os.path.join(args.out, args.workload + ".jsonl"), "a") as f:
        f.write(json.dumps(rec, sort_keys=True) + "\n")
    print(json.dumps({k: v for k, v in rec.items() if k != "trace"}))
    print(rec["trace"])


if __name__ == "__main__":
    main()
