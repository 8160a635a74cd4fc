"""Measure what this device attains: MFMA issue loops per intrinsic and streaming copy/read.

    python -m paper_2205_13603_amd.calibrate [--copy-mib 2048] [--quick]

Prints one JSON object.  The streaming copy (kernel `ms_calib_kernel`, a known byte count) is also the
reference that hardware byte counters are scaled by.
"""
import argparse
import json


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--copy-mib", type=int, default=2048)
    ap.add_argument("--quick", action="store_true", help="stream kernels only")
    args = ap.parse_args()
    import torch
    from . import binding as B, devmem
    devmem.require_gpu()
    out = {}
    info = B.device_info()
    out["device"] = {"name": info.name.decode(), "arch": info.arch.decode(), "compute_units": info.compute_units,
                     "lds_bytes_per_block": info.lds_bytes_per_block, "clock_khz": info.clock_khz,
                     "mem_clock_khz": info.mem_clock_khz, "mem_bus_bits": info.mem_bus_bits, "l2_bytes": info.l2_bytes,
                     "global_mem_bytes": info.global_mem_bytes}
    n = args.copy_mib << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    out["stream"] = {"bytes": n, "copy_gbs_read_plus_write": B.calibrate_stream(1, src.data_ptr(), dst.data_ptr(), n),
                     "read_gbs": B.calibrate_stream(2, src.data_ptr(), dst.data_ptr(), n),
                     "write_gbs": B.calibrate_stream(3, src.data_ptr(), dst.data_ptr(), n),
                     "copy_small_chunks_gbs": B.calibrate_stream(4, src.data_ptr(), dst.data_ptr(), n)}
    if not args.quick:
        scratch = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
        bpc, gbs = B.calibrate_lds(scratch.data_ptr())
        out["l2_read_gbs"] = B.calibrate_l2(src.data_ptr(), scratch.data_ptr())
        out["lds_read"] = {"bytes_per_clk_per_cu_at_nominal_clock": bpc, "gbs": gbs}
        rnd = (torch.randn(32768, device="cuda") * 0.1)
        ops = {"f16": rnd.half(), "bf16": rnd.bfloat16(), "i8": torch.randint(-128, 128, (32768,), device="cuda", dtype=torch.int8),
               "f32": torch.rand(32768, device="cuda") * 2 - 1,
               "f8": rnd.clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8)}
        codes = {"f16": [161616, 323208, 161632, 323216], "bf16": [161616, 323208, 161632, 323216],
                 "i8": [161632, 323216, 161664, 323232], "f32": [161604, 323202], "f8": [161632, 323216, 1616128, 323264]}
        t = B.calibrate_timer(1000.0, scratch.data_ptr(), repeats=7)
        out["timer_check"] = {"target_us": 1000.0, "measured_min_us": t.min_us, "measured_median_us": t.median_us}
        out["mfma_tflops"] = {}
        for dt in ("f16", "bf16", "i8", "f32", "f8"):
            for c in codes[dt]:
                out["mfma_tflops"]["%s_%d" % (dt, c)] = {
                    "small_int_operands": B.calibrate_mfma(dt, c, scratch.data_ptr()),
                    "random_operands": B.calibrate_mfma(dt, c, scratch.data_ptr(), ops[dt].data_ptr())}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
