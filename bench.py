#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

One "step" = one launch of the best variant found for the workload over a batch of R independent
instances of the workload's shape (per-instance tiling exactly as the trace says), inputs resident
in HBM.  Before the timed region the hot path up to that point runs untimed: the operator is
defined, the space described, candidates (stored tuning records plus a fresh seeded search of
--trials measured candidates) are validated, compiled and measured, and the fastest is kept.

Prints ONE JSON line (see the keys below).  `value` is the throughput of the K timed steps (the device-filling
protocol, named in `value_protocol`).  Next to it, at top level, `steady_state`: back-to-back launches of ONE
instance at the workload's own shape over rotating buffer sets larger than the last-level cache, with the variant
tuned for that protocol and the floor max(launch gap, ideal time) it is bounded by.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

METRIC = "best-variant TFLOP/s per operator (% of MFMA/HBM roofline); trials to reach it"

# published MI355X peaks: dense MFMA TFLOP/s (TOP/s) by input type, fp32 vector TFLOP/s, HBM GB/s
PEAK_MFMA = {"f16": 2500.0, "bf16": 2500.0, "i8": 5000.0, "f32": 157.3, "f8": 5000.0}
PEAK_FP32_VECTOR = 157.3
PEAK_HBM_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-ms", type=float, default=100.0,
                    help="untimed launches of the chosen variant for this long before the warm-up steps: after the host-side "
                         "oracle check the idle device has dropped its clocks and needs tens of ms of load to raise them")
    ap.add_argument("--workload", default="c2_gemm_f16_1024")
    ap.add_argument("--instances", type=int, default=0, help="instances per launch (0 = the workload's default)")
    ap.add_argument("--trials", type=int, default=16, help="measured candidates of the fresh search")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-records", action="store_true", help="ignore stored tuning records")
    ap.add_argument("--record-index", type=int, default=-1,
                    help="consider only this stored record (0 = the best stored latency): fixes the variant, e.g. for counter runs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-steady", action="store_true", help="skip the steady-state block (profiling runs: only the timed variant's launches remain)")
    ap.add_argument("--trace-file", default="", help="time exactly this trace (text form) instead of searching")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (every figure is single-GPU)" % args.gpus,
              file=sys.stderr)
        return 2

    import torch
    from paper_2205_13603_amd import binding as B, devmem, tuned
    from paper_2205_13603_amd.workloads import workload_inputs, OUT_SHAPE, BOUND, PROFILE_NAME
    from oracle import compare
    from oracle.workloads import oracle_run

    devmem.require_gpu()
    name = args.workload
    mk, default_r = tuned.WORKLOADS[name]
    R = args.instances or default_r
    op = mk()
    space = op.space()
    flop1, bytes1 = op.work()
    stream = devmem.current_stream()

    # ---- inputs: R instances resident in HBM (4 distinct seeds, tiled), one output per instance
    base = [workload_inputs(name, args.seed + s) for s in range(min(4, R))]
    dev_in = []
    for k in range(len(base[0])):
        parts = [devmem.to_device(b[k]) for b in base]
        reps = (R + len(parts) - 1) // len(parts)
        dev_in.append(torch.stack(parts * reps)[:R].contiguous())
    shape, odt = OUT_SHAPE[name]
    dev_out = devmem.empty_output(shape, odt, R, poison=True)
    in_ptrs = [t.data_ptr() for t in dev_in]
    full_set = [(in_ptrs, dev_out.data_ptr())]
    # one buffer set per instance, for the single-instance protocols (rotating over > last-level-cache bytes)
    inst_sets = [([t[r].data_ptr() for t in dev_in], dev_out[r].data_ptr()) for r in range(R)]

    # ---- the oracle's result for the distinct inputs (and, from the same calls, the CPU baseline)
    t_or = time.time()
    refs = [oracle_run(name, b) for b in base]
    oracle_runs = len(base)
    if not args.no_cpu_baseline:
        # the CPU baseline is the oracle as it stands: keep timing whole instances until about 10 s of CPU work are
        # sampled (at most 64 more runs; cheap operators finish far earlier and are then timed on all of those runs)
        while time.time() - t_or < 10.0 and oracle_runs < len(base) + 64:
            oracle_run(name, base[oracle_runs % len(base)])
            oracle_runs += 1
    oracle_seconds = (time.time() - t_or) / oracle_runs
    rtol = compare.RTOL_F32 if odt == "f32" and BOUND[name][1] == "f32" else compare.RTOL_HALF

    def check(got, rows, what):
        """got[r] against the oracle for the instances `rows` (instance r holds input set r mod len(base))"""
        for r in rows:
            ref = np.asarray(refs[r % len(base)]).reshape(shape)
            if odt == "i32":
                compare.assert_int_equal(got[r], ref, "%s instance %d" % (what, r))
            else:
                compare.assert_float_close(got[r], ref, rtol, "%s instance %d" % (what, r))

    # ---- candidates: stored records + fresh search, all measured now in the timed configuration
    t_search0 = time.time()
    mcfg = dict(warmup=10, repeats=5, launches_per_repeat=10, instances=R)
    best = (None, float("inf"), "none", None)
    record_search = None
    search_info = {"trials": 0, "trials_to_best": None, "invalid": 0, "failed": 0, "duplicate": 0}

    settled = False

    def settle(v, ms):
        """Untimed launches for `ms` milliseconds: raises the clocks of a device that has been idle."""
        t0, n = time.perf_counter(), 0
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(20):
                v.launch(in_ptrs, dev_out.data_ptr(), instances=R, stream=stream)
            torch.cuda.synchronize()
            n += 20
        return n

    def consider(trace, origin, rec=None, sp=None):
        nonlocal best, record_search, settled
        sp = sp if sp is not None else space
        try:
            v = B.Variant(op, sp, trace)
            if not settled:  # the candidates are ranked at the clocks they will be timed at
                settle(v, args.settle_ms)
                settled = True
            us = v.measure(full_set, stream=stream, **mcfg).median_us
        except B.MsError as e:
            print("candidate from %s failed: %s" % (origin, str(e)[:200]), file=sys.stderr)
            return
        if us < best[1]:
            best = (trace, us, origin, sp)
            if rec is not None:  # statistics of the search that found this record
                record_search = {k: rec.get(k) for k in ("trials", "trials_to_best", "invalid", "failed", "duplicate", "seed")}

    if args.trace_file:
        consider(B.trace_from_text(space, open(args.trace_file).read()), "file")
    else:
        if not args.no_records:
            # the headline runs in the space the configuration names: records found with an opt-in module in the space
            # (fp32 operators on the fp32 matrix cores) are timed separately below, never as `value`
            usable = [(rec, sp, t) for rec, sp, t in tuned.records_with_traces(name, op, limit=8, protocol="filling")
                      if not (sp.flags & B.SPACE_TENSORIZE_F32)]
            for idx, (rec, sp, t) in enumerate(usable[:4]):
                if args.record_index < 0 or idx == args.record_index:
                    consider(t, "record", rec, sp)
        if args.trials > 0:
            cfg = B.search_cfg_default()
            cfg.seed, cfg.trials = args.seed, args.trials
            cfg.init_population = min(cfg.init_population, max(1, args.trials // 2))
            cfg.measure = B.ms_measure_cfg(**mcfg)
            # a search ranks on latency alone: every candidate it measures is also run on the first instances and compared
            # with the oracle (the kernel is in the library's cache by then), and a mismatch ends the benchmark
            n_chk = min(R, len(base))
            chk = devmem.empty_output(shape, odt, n_chk, poison=True)
            wrong = []

            def on_trial(t):
                if t.status != 0:
                    return 0
                try:
                    vt = B.Variant(op, space, t.trace.copy())
                    chk.fill_({"bf16": 0x7FC0, "i32": -123456789}.get(odt, float("nan")))
                    vt.launch(in_ptrs, chk.data_ptr(), instances=n_chk, stream=stream)
                    check(devmem.to_host(chk, odt).reshape((n_chk,) + tuple(shape)), range(n_chk), "search trial %d" % t.index)
                except Exception as e:  # must not unwind through the C callback
                    wrong.append(repr(e)[:500])
                    return 1
                return 0

            # with stored trial logs of the workload the search's cost model is fitted on them before the first
            # trial (Section 4 allows a model trained beforehand), so even a short search starts from good candidates
            logs = tuned.pretraining_logs(name, "filling")
            rows = tuned.pretraining_rows(op, space, logs) if logs else None
            if rows is not None and len(rows[1]) >= cfg.model_min_trials:
                cfg.cost_model = 1
            else:
                rows = None
            res = B.search(op, space, cfg, bufsets=full_set, stream=stream, on_trial=on_trial, pretrain=rows)
            if wrong:
                print("bench.py: a candidate of the search does not match the oracle: %s" % wrong[0], file=sys.stderr)
                return 1
            search_info = {"trials": res.n_measured, "trials_to_best": res.best_trial, "invalid": res.n_invalid,
                           "failed": res.n_failed, "duplicate": res.n_duplicate, "checked_against_oracle": res.n_measured,
                           "best_us": res.best_us, "cost_model": "pre-trained on %d stored trials" % len(rows[1]) if rows is not None else "off"}
            if res.best_us < best[1]:
                best = (res.best_trace, res.best_us, "search", space)
    if best[0] is None:
        print("bench.py: no candidate could be measured", file=sys.stderr)
        return 1
    search_seconds = time.time() - t_search0
    trace = best[0]
    v = B.Variant(op, best[3], trace)
    params = v.params()

    # ---- correctness of the variant about to be timed: sampled instances against the oracle
    dev_out.fill_({"bf16": 0x7FC0, "i32": -123456789}.get(odt, float("nan")))
    v.launch(in_ptrs, dev_out.data_ptr(), instances=R, stream=stream)
    got = devmem.to_host(dev_out, odt)
    check(got, sorted({0, 1 % R, R // 2, R - 1}), "timed variant")

    # ---- timed region: clock settling, W warm-up steps, then exactly K steps between synchronisations
    settle_launches = settle(v, args.settle_ms)
    for _ in range(args.warmup):
        v.launch(in_ptrs, dev_out.data_ptr(), instances=R, stream=stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    res = v.measure(full_set, warmup=0, repeats=1, launches_per_repeat=args.steps, instances=R, stream=stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_us = res.mean_us  # HIP events around the K launches on the launch stream / K
    ms_per_step = wall * 1e3 / args.steps

    bound, in_dt = BOUND[name]
    if bound == "hbm":
        unit, work = "GB/s", bytes1 * R / 1e9
        peak = PEAK_HBM_GBS
    else:
        unit, work = "TFLOP/s", flop1 * R / 1e12
        peak = PEAK_MFMA[in_dt] if bound == "mfma" else PEAK_FP32_VECTOR
    value = work * args.steps / wall
    achieved = work / (kernel_us * 1e-6)

    # ---- what the device attains on the bounding resource, measured now with the same clocks: the register-resident
    # issue loop of the variant's intrinsic fed with operands of this workload, or the plain copy kernel
    attainable = None
    try:
        if bound == "mfma" and params.mfma:
            scratch = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
            attainable = B.calibrate_mfma(in_dt, params.mfma, scratch.data_ptr(), dev_in[0].data_ptr(), stream=stream)
        elif bound == "hbm":
            nb = 1 << 30
            src = torch.ones(nb, dtype=torch.uint8, device="cuda")
            dst = torch.empty(nb, dtype=torch.uint8, device="cuda")
            attainable = max(B.calibrate_stream(m, src.data_ptr(), dst.data_ptr(), nb, stream=stream) for m in (1, 4))
            del src, dst
    except B.MsError as e:
        print("calibration failed: %s" % str(e)[:200], file=sys.stderr)

    # ---- the workload at its own shape: one instance per launch
    per1 = (bytes1 / 1e9) if bound == "hbm" else (flop1 / 1e12)
    l1 = v.measure(inst_sets[:1], warmup=5, repeats=100, launches_per_repeat=1, instances=1, stream=stream)
    # steady state: candidates are the records tuned under that protocol (their space may include rfactor, whose
    # partial sums go to a workspace) and the device-filling variant; all measured now, the fastest is reported
    ws = torch.empty(8 * dev_out[0].numel() * 4, dtype=torch.uint8, device="cuda")
    steady_sets = [(ins, out, ws.data_ptr()) for ins, out in inst_sets]
    lpr = max(200, R) if not args.no_steady else 2
    steady = {"us": v.measure(steady_sets, warmup=20 if not args.no_steady else 0, repeats=5 if not args.no_steady else 1, launches_per_repeat=lpr, instances=1, stream=stream).median_us,
              "variant_from": "the device-filling variant", "rfactor": 1, "record_search": None}
    filling_variant_steady_us = steady["us"]
    if not args.no_records and not args.trace_file and not args.no_steady:
        for rec, sp, t in tuned.records_with_traces(name, op, limit=4, protocol="steady"):
            try:
                vs = B.Variant(op, sp, t)
                us = vs.measure(steady_sets, warmup=20, repeats=5, launches_per_repeat=lpr, instances=1, stream=stream).median_us
            except B.MsError as e:
                print("steady-state record failed: %s" % str(e)[:200], file=sys.stderr)
                continue
            if us < steady["us"]:
                steady = {"us": us, "variant_from": "record tuned under the steady-state protocol", "rfactor": vs.params().rfactor,
                          "record_search": {k: rec.get(k) for k in ("trials", "trials_to_best", "seed", "flags")}}
    # the floor: back-to-back launches of a kernel that does nothing for 1 us cost the launch gap, and no kernel is
    # faster than its work at the published peak
    scratch_b = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    gap_us = max(0.0, B.calibrate_timer(1.0, scratch_b.data_ptr(), warmup=20, repeats=5, launches_per_repeat=200, stream=stream).median_us - 1.0)
    ideal_us = per1 / peak * 1e6
    # the opt-in fp32 matrix-core space of an fp32 operator: reported beside the headline, never as it
    opt_in = None
    if BOUND[name] == ("alu", "f32") and not args.no_records and not args.trace_file:
        for rec, sp, t in tuned.records_with_traces(name, op, limit=8, protocol="filling"):
            if sp.flags & B.SPACE_TENSORIZE_F32:
                try:
                    vo = B.Variant(op, sp, t)
                    uo = vo.measure(full_set, warmup=20, repeats=5, launches_per_repeat=20, instances=R, stream=stream).median_us
                except B.MsError:
                    continue
                opt_in = {"space": "with the opt-in module that tensorizes fp32 operators onto the fp32 matrix-core intrinsics",
                          "kernel_us": uo, "tflops": flop1 * R / uo / 1e6, "bound": "mfma", "peak": PEAK_MFMA["f32"],
                          "frac": flop1 * R / uo / 1e6 / PEAK_MFMA["f32"]}
                break

    # HBM bytes per launch from the committed rocprofv3 counter summary, if it is of this very variant
    traffic, traffic_source = None, None
    # (one summary per profiled record of the workload: ms_kernel_<family>_<workload>.txt and ..._record<i>.txt)
    import glob
    stem = os.path.join(ROOT, "profiles", "ms_kernel_%s" % PROFILE_NAME.get(name, name))
    for prof in [stem + ".txt"] + sorted(glob.glob(stem + "_record*.txt")):
        if R != default_r or not os.path.exists(prof):
            continue
        fields = dict(line.split(":", 1) for line in open(prof) if line.startswith(("traffic_bytes_per_launch:", "variant_key:")))
        if fields.get("variant_key", "").strip() == "%016x" % params.key and "traffic_bytes_per_launch" in fields:
            traffic = float(fields["traffic_bytes_per_launch"])
            traffic_source = "profiles/%s: rocprofv3 FETCH_SIZE + WRITE_SIZE of this very variant (matched by key), not measured in this run" % os.path.basename(prof)
            break

    out = {
        "metric": METRIC, "value": value, "unit": unit,
        "value_protocol": "device-filling: one launch over %d instances of the workload's shape" % R, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_launches": settle_launches,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": in_dt, "data": "synthetic",
        "config": {"workload": "%s x %d instances per launch (device-filling batch; per-instance tiling as traced)" % (name, R),
                   "instances": R, "best_from": best[2], "search": search_info, "record_search": record_search if best[2] == "record" else None,
                   "search_seconds": round(search_seconds, 1),
                   "variant": {"mfma": params.mfma, "block": [params.block_m, params.block_n, params.block_k],
                               "waves": params.waves, "lds_bytes": params.lds_bytes, "cache_read": params.cache_read,
                               "vec": params.vec, "reorder": params.reorder, "lds_pad": params.lds_pad,
                               "ti": list(params.ti), "tj": list(params.tj), "tk": list(params.tk), "tc": list(params.tc),
                               "unroll": params.unroll}},
        "roofline": {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                     "traffic": traffic, "traffic_source": traffic_source, "kernel_us": kernel_us,
                     "attainable": attainable, "frac_of_attainable": (achieved / attainable) if attainable else None,
                     "attainable_kind": {"mfma": "register-resident loop of the variant's intrinsic on this workload's operand values",
                                         "hbm": "1 GiB copy kernel (the faster of two launch shapes), bytes read + written"}.get(bound) if attainable else None},
        # vector-ALU kernels here issue one fp32 FMA per lane and clock (the packed two-FMA forms are compiled out):
        # 256 CUs x 64 lanes x 2 flop x 2.4 GHz = 78.6 TFLOP/s is what such code can reach; the published 157.3 counts the packed form
        "alu_unpacked": ({"peak": PEAK_FP32_VECTOR / 2, "frac": achieved / (PEAK_FP32_VECTOR / 2)} if bound == "alu" else None),
        "steady_state": {"protocol": "back-to-back launches of ONE instance, %d per repeat, rotating over %d buffer sets (%.0f MB, beyond the last-level cache)"
                                     % (lpr, R, bytes1 * R / 1e6),
                         "us_per_launch": steady["us"], "value": per1 / (steady["us"] * 1e-6), "unit": unit,
                         "frac": per1 / (steady["us"] * 1e-6) / peak, "variant_from": steady["variant_from"], "rfactor": steady["rfactor"],
                         "record_search": steady["record_search"], "device_filling_variant_us": filling_variant_steady_us,
                         "floor_us": max(gap_us, ideal_us), "launch_gap_us": gap_us, "ideal_us_at_published_peak": ideal_us,
                         "single_launch_us": l1.median_us},
    }
    out["config"]["search_256"] = [{k: r.get(k) for k in ("protocol", "seed", "us", "trials_to_best", "trials_to_within_1pct", "best_us_at", "cost_model", "pretrain_trials", "flags")}
                                   for r in tuned.load_searches(name, 256)]
    out["config"]["headline_variant_from"] = ("stored record of a %s-trial search (seed %s)" % (record_search.get("trials"), record_search.get("seed"))
                                              if best[2] == "record" and record_search else best[2])
    if opt_in:
        out["opt_in_fp32_matrix_cores"] = opt_in
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        out["cpu_baseline"] = {"value": per1 / oracle_seconds, "unit": unit, "cores": O.threads(), "kind": "oracle",
                               "sample": "whole instances of the workload, mean of %d runs (%.3f ms each)" % (oracle_runs, oracle_seconds * 1e3)}
        # two more figures of the same plain loops, each on a bounded sample (about 3 s): one thread; and all threads with
        # the running sum kept in the operator's own precision instead of double (a build of its own, never used for parity)
        def timed(budget_s):
            t0, n = time.time(), 0
            while n == 0 or (time.time() - t0 < budget_s and n < 16):
                oracle_run(name, base[n % len(base)])
                n += 1
            return (time.time() - t0) / n, n
        O.set_threads(1)
        s1, n1 = timed(3.0)
        O.set_threads(0)
        out["cpu_baseline"]["single_thread"] = {"value": per1 / s1, "unit": unit, "cores": 1, "sample": "%d whole instances" % n1}
        if odt != "i32":
            O.use_build("f32acc")
            try:
                sf, nf = timed(3.0)
                out["cpu_baseline"]["float_accumulate"] = {"value": per1 / sf, "unit": unit, "cores": O.threads(),
                                                           "sample": "%d whole instances; same loops built with a float running sum" % nf}
            finally:
                O.use_build("f64")
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
