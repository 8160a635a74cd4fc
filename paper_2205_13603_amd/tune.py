"""Tune one workload on the GPU: run the evolutionary search over traces and store the best as a record.

    python -m paper_2205_13603_amd.tune --workload c2_gemm_f16_1024 --trials 256 --out tuned_out
    python -m paper_2205_13603_amd.tune --workload c2_gemm_f16_1024 --protocol steady --flags 0x4ff

Two measurement protocols (what a trial's latency is):
  filling  one launch over R instances of the workload (the device-filling batch): kernel quality against the roofline
  steady   back-to-back launches of ONE instance, rotating over R distinct buffer sets whose footprint exceeds the
           last-level cache: the workload at its own shape, dispatch gaps included
Writes <out>/<workload>.jsonl (best record, appendable to tuned_records/), <out>/<workload>.<protocol>.s<seed>.log.jsonl
(every trial: index, status, latency, best so far, decisions) and one summary line per run to <out>/searches.jsonl.
Such trial logs are what `--cost-model --pretrain` fits the cost model on before a later search of the same workload
and protocol starts (Section 4 allows a model trained before the search); `--pretrain stored` takes the logs under tuned_records/logs.
"""
import argparse
import json
import os
import time


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--trials", type=int, default=256)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--instances", type=int, default=0, help="instances of a device-filling launch / rotating buffer sets of the steady protocol")
    ap.add_argument("--protocol", choices=["filling", "steady"], default="filling")
    ap.add_argument("--flags", type=lambda s: int(s, 0), default=0xFF,
                    help="search-space module mask (0xff = default, 0x1ff = with fp32 tensorize, 0x4ff = with rfactor)")
    ap.add_argument("--modules", default="", help="build the space with Compose from this comma-separated ordered module list "
                    "(names of `binding.modules()`, starting with multi-level-tiling) instead of --flags")
    ap.add_argument("--compose-seed", type=int, default=-1, help="build the space with Stochastic-Compose over the modules of "
                    "--modules (or of --flags) with this seed")
    ap.add_argument("--out", default="tuned_out")
    ap.add_argument("--cost-model", action="store_true", help="let the learned cost model pick which proposals are measured")
    ap.add_argument("--model-candidates", type=int, default=8, help="proposals scored per measured candidate")
    ap.add_argument("--pretrain", default="", help="with --cost-model: pre-train the model on trial logs of earlier searches of this "
                    "workload and protocol; a comma-separated list of *.log.jsonl files, or 'stored' for the logs kept with the "
                    "records (the one of this very seed left out)")
    ap.add_argument("--measure", default="", help="warm-up launches, repeats, launches per repeat of every trial (default 1,3,3 for "
                    "filling; 8,3,<sets> for steady); a long warm-up (e.g. 150,3,20) times candidates at the clocks of a sustained run")
    ap.add_argument("--compile-threads", type=int, default=16)
    args = ap.parse_args()

    import torch
    from . import binding as B, devmem, tuned
    from .workloads import workload_inputs, OUT_SHAPE

    devmem.require_gpu()
    mk, default_r = tuned.WORKLOADS[args.workload]
    R = args.instances or default_r
    op = mk()
    composed = None
    if args.modules or args.compose_seed >= 0:
        names = [n for n in args.modules.split(",") if n] or [m["name"] for m in B.modules() if m["flag"] == 0 or (m["flag"] & args.flags)]
        if args.compose_seed >= 0:
            space, composed = B.space_stochastic_compose(op, names, args.compose_seed)
        else:
            space, _ = B.space_compose(op, names)
            composed = names
        args.flags = space.flags
        print("space composed of", composed, "-> module mask 0x%x" % space.flags, flush=True)
    else:
        space = op.space(args.flags)
    base = [workload_inputs(args.workload, s) for s in range(min(4, R))]
    dev_in = []
    for k in range(len(base[0])):
        parts = [devmem.to_device(b[k]) for b in base]
        reps = (R + len(parts) - 1) // len(parts)
        dev_in.append(torch.stack(parts * reps)[:R].contiguous())
    shape, odt = OUT_SHAPE[args.workload]
    dev_out = devmem.empty_output(shape, odt, R)
    # workspace for variants that split the reduction (rfactor <= 8): partial sums of every instance of a launch
    ws = None
    if args.flags & B.SPACE_RFACTOR:
        per_instance = 8 * dev_out[0].numel() * 4
        ws = torch.empty(per_instance * (R if args.protocol == "filling" else 1), dtype=torch.uint8, device="cuda")
    wsp = ws.data_ptr() if ws is not None else None
    if args.protocol == "filling":
        sets = [([t.data_ptr() for t in dev_in], dev_out.data_ptr(), wsp)]
        inst = R
        wu, reps, lpr = 1, 3, 3
    else:
        sets = [([t[r].data_ptr() for t in dev_in], dev_out[r].data_ptr(), wsp) for r in range(R)]
        inst = 1
        wu, reps, lpr = 8, 3, max(R, 32)
    if args.measure:
        wu, reps, lpr = (int(x) for x in args.measure.split(","))
    os.makedirs(args.out, exist_ok=True)
    log = open(os.path.join(args.out, "%s.%s.s%d.log.jsonl" % (args.workload, args.protocol, args.seed)), "w")
    t0 = time.time()

    curve = []  # (trial index, best latency so far)

    def on_trial(t):
        if t.status == 0:
            curve.append((t.index, t.best_us))
        rec = {"trial": t.index, "status": t.status, "us": t.us, "best_us": t.best_us, "key": "%016x" % t.key,
               "decisions": t.trace.decisions(), "t": round(time.time() - t0, 2)}
        log.write(json.dumps(rec) + "\n")
        log.flush()
        if t.status == 0 and t.index % 16 == 0:
            print("trial %d: %.2f us, best %.2f us (%.1f s)" % (t.index, t.us, t.best_us, time.time() - t0), flush=True)
        return 0

    cfg = B.search_cfg_default()
    cfg.seed, cfg.trials = args.seed, args.trials
    cfg.compile_threads = args.compile_threads
    cfg.cost_model, cfg.model_candidates = int(args.cost_model), args.model_candidates
    cfg.measure = B.ms_measure_cfg(wu, reps, lpr, inst)
    pretrain, pretrain_logs = None, []
    if args.pretrain:
        if not args.cost_model:
            raise SystemExit("--pretrain needs --cost-model")
        pretrain_logs = (tuned.pretraining_logs(args.workload, args.protocol, exclude_seed=args.seed) if args.pretrain == "stored"
                         else [p for p in args.pretrain.split(",") if p])
        pretrain = tuned.pretraining_rows(op, space, pretrain_logs)
        print("cost model pre-trained on %d trials of %d logs" % (len(pretrain[1]), len(pretrain_logs)), flush=True)
        if len(pretrain[1]) == 0:
            raise SystemExit("--pretrain: no usable trial in %s" % pretrain_logs)
    res = B.search(op, space, cfg, bufsets=sets, stream=devmem.current_stream(), on_trial=on_trial, pretrain=pretrain)
    flop, byts = op.work()
    mode = "device-filling, %d instances" % R if args.protocol == "filling" else "steady state, 1 instance, %d rotating buffer sets" % R
    rec = {"workload": args.workload, "trace": B.trace_to_text(op, space, res.best_trace), "us": res.best_us, "protocol": args.protocol,
           "mode": mode, "tflops": flop * inst / res.best_us / 1e6, "gbs": byts * inst / res.best_us / 1e3,
           "trials": res.n_measured, "trials_to_best": res.best_trial, "invalid": res.n_invalid, "failed": res.n_failed,
           "duplicate": res.n_duplicate, "search_seconds": round(res.wall_seconds, 1), "seed": args.seed, "flags": args.flags,
           "cost_model": int(args.cost_model), "pretrain_trials": int(len(pretrain[1])) if pretrain else 0,
           "pretrain_logs": [os.path.basename(p) for p in pretrain_logs], "modules": composed, "compiler": list(B.jit_stats()["compiler"]),
           # first measured trial whose best-so-far latency is within 1 % of the final best
           "trials_to_within_1pct": next((i for i, b in curve if b <= 1.01 * res.best_us), res.best_trial)}
    with open(os.path.join(args.out, args.workload + ".jsonl"), "a") as f:
        f.write(json.dumps(rec, sort_keys=True) + "\n")
    with open(os.path.join(args.out, "searches.jsonl"), "a") as f:
        f.write(json.dumps({k: v for k, v in rec.items() if k != "trace"}, sort_keys=True) + "\n")
    print(json.dumps({k: v for k, v in rec.items() if k != "trace"}))
    print(rec["trace"])


if __name__ == "__main__":
    main()
