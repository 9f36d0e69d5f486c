"""Measures the two machine ceilings the perturbation pass is rated against and prints them as a markdown
summary (and, with --json FILE, as JSON): the bare in-place read-modify-write stream in GB/s and the
vector-instruction issue rate in cycles per wave64 instruction and SIMD.

    python -m paper_2601_12917_amd.ceilings [--json ceilings.json]

Argument marshalling and arithmetic on the measured times only; the kernels are in csrc/ceilings.hip.
"""
import argparse
import json
import sys

import numpy as np

OPS = ["v_fma_f32", "v_xor_b32", "v_bitop3_b32", "v_mad_u64_u32", "v_mul_hi_u32", "v_mul_lo_u32", "v_cvt_f32_u32", "v_rsq_f32",
       "v_add_u32", "v_lshrrev_b32", "v_cndmask_b32", "v_mul_f32", "v_add_f32", "v_log_f32", "v_cvt_pk_bf16_f32", "v_sqrt_f32", "v_mov_b32", "v_mfma_f32_32x32x16_bf16", "v_mfma_f32_32x32x2_f32"]
N_VECTOR_OPS = 17                     # the entries before the two matrix instructions
MFMA_FLOPS = 2.0 * 32 * 32 * 16
MFMA_F32_FLOPS = 2.0 * 32 * 32 * 2


def issue_rate(lib, B, torch, op, ilp, waves_per_simd, iters=512, n_cu=None):
    """(cycles per wave instruction per SIMD, shader clock in GHz, wave-instructions per second over the chip).
    The waves of a SIMD finish far apart (the arbiter favours the oldest), so the rate is taken over the span from
    the first wave's start to the last wave's end; the clock is each wave's own cycles over its own real time."""
    n_cu = n_cu or torch.cuda.get_device_properties(0).multi_processor_count
    blocks = n_cu * waves_per_simd             # a block is 4 waves, one per SIMD of the CU it lands on
    out = torch.zeros(4 * 4 * blocks, dtype=torch.int64, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    for _ in range(3):
        B.check(lib.zgr_debug_issue_rate(op, ilp, blocks, iters, out.data_ptr(), st))
    torch.cuda.synchronize()
    r = out.cpu().numpy().reshape(-1, 4)
    cyc, t0, t1 = r[:, 0].astype(np.float64), r[:, 1].astype(np.float64), r[:, 2].astype(np.float64)
    ghz = float(np.median(cyc / ((t1 - t0) / 100e6))) / 1e9
    span_s = (t1.max() - t0.min()) / 100e6
    n_inst = iters * 64.0
    rate = n_cu * 4 * waves_per_simd * n_inst / span_s
    cpi = span_s * ghz * 1e9 / (n_inst * waves_per_simd)
    return cpi, ghz, rate


GEN_PARTS = ["Philox4x32-10 call", "two radii", "two (cos, sin) pairs", "two Box-Muller pairs", "whole generator: Philox call + two Box-Muller pairs",
             "the two table look-ups alone"]


def generator_rate(lib, B, torch, part, waves_per_simd, iters=1024, n_cu=None):
    """(cycles per call and SIMD, shader clock GHz): a call is what one lane does for 4 Gaussians."""
    n_cu = n_cu or torch.cuda.get_device_properties(0).multi_processor_count
    blocks = n_cu * waves_per_simd
    out = torch.zeros(4 * 4 * blocks, dtype=torch.int64, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    for _ in range(3):
        B.check(lib.zgr_debug_generator_rate(part, blocks, iters, out.data_ptr(), st))
    torch.cuda.synchronize()
    r = out.cpu().numpy().reshape(-1, 4)
    cyc, t0, t1 = r[:, 0].astype(np.float64), r[:, 1].astype(np.float64), r[:, 2].astype(np.float64)
    ghz = float(np.median(cyc / ((t1 - t0) / 100e6))) / 1e9
    span_s = (t1.max() - t0.min()) / 100e6
    return span_s * ghz * 1e9 / (iters * waves_per_simd), ghz


def stream_rate(lib, B, torch, nbytes, dtype, mode, blocks, reps=5):
    buf = torch.zeros(nbytes // 2, dtype=torch.bfloat16, device="cuda:0") if dtype == 1 else torch.zeros(nbytes // 4, dtype=torch.float32, device="cuda:0")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    run = lambda: B.check(lib.zgr_debug_rmw(buf.data_ptr(), nbytes, dtype, 1e-3, mode, blocks, sink.data_ptr(), st))
    for _ in range(2):
        run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    moved = nbytes * (2 if mode == 0 else 1)
    return moved / (ms * 1e-3) / 1e9, ms


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--json", default=None)
    args = ap.parse_args()
    import torch
    from . import binding as B
    lib = B.lib()
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    res = {"device": torch.cuda.get_device_name(0), "compute_units": n_cu, "stream": [], "issue": []}
    print("## Bare in-place stream (16-byte vectors, grid-stride blocks of 256 threads)\n")
    print("| data | bytes | mode | blocks | ms | GB/s (read + written) |\n|---|---:|---|---:|---:|---:|")
    for dtype, dname in ((1, "bf16"), (0, "fp32")):
        for nbytes in (1 << 29, 1 << 31):
            for mode, mname in ((0, "read-modify-write"), (1, "read only"), (2, "write only")):
                for blocks in (n_cu * 8, n_cu * 32):
                    if dtype == 0 and (mode != 0 or nbytes != 1 << 31):
                        continue
                    gbs, ms = stream_rate(lib, B, torch, nbytes, dtype, mode, blocks)
                    res["stream"].append({"dtype": dname, "bytes": nbytes, "mode": mname, "blocks": blocks, "ms": ms, "gbs": gbs})
                    print(f"| {dname} | {nbytes} | {mname} | {blocks} | {ms:.3f} | {gbs:.0f} |")
    print("\n## Vector-instruction issue rate (cycles per wave64 instruction and SIMD; shader cycle counter s_memtime, clock from the 100 MHz s_memrealtime)\n")
    print("| instruction | chains per wave | waves per SIMD | cycles / instruction | shader clock GHz | T wave-instr/s (chip) |\n|---|---:|---:|---:|---:|---:|")
    for op, name in enumerate(OPS[:N_VECTOR_OPS]):
        for ilp, wps in ((1, 1), (4, 1), (1, 4), (4, 4), (1, 8), (4, 8)):
            if name not in ("v_fma_f32", "v_xor_b32", "v_mad_u64_u32") and (ilp, wps) not in ((1, 1), (4, 8), (1, 8)):
                continue
            cpi, ghz, rate = issue_rate(lib, B, torch, op, ilp, wps, n_cu=n_cu)
            res["issue"].append({"op": name, "ilp": ilp, "waves_per_simd": wps, "cycles_per_instruction": cpi, "shader_ghz": ghz, "wave_instr_per_s": rate})
            print(f"| {name} | {ilp} | {wps} | {cpi:.2f} | {ghz:.2f} | {rate / 1e12:.3f} |")
    print("\n## The matrix core alone (v_mfma_f32_32x32x16_bf16 on register operands of random bf16; dense peak quoted at 2.4 GHz: 2500 TFLOP/s)\n")
    print("| accumulators per wave | waves per SIMD | cycles / instruction | shader clock GHz | TFLOP/s (chip) |\n|---:|---:|---:|---:|---:|")
    res["mfma"] = []
    for ilp, wps in ((1, 1), (4, 1), (2, 2), (4, 2)):
        cpi, ghz, rate = issue_rate(lib, B, torch, N_VECTOR_OPS, ilp, wps, iters=4096, n_cu=n_cu)
        res["mfma"].append({"ilp": ilp, "waves_per_simd": wps, "cycles_per_instruction": cpi, "shader_ghz": ghz, "tflops": rate * MFMA_FLOPS / 1e12})
        print(f"| {ilp} | {wps} | {cpi:.2f} | {ghz:.2f} | {rate * MFMA_FLOPS / 1e12:.0f} |")
    print("\n## The fp32 matrix instruction alone (v_mfma_f32_32x32x2_f32 on register operands of random fp32; dense peak quoted at 2.4 GHz: 157.3 TFLOP/s)\n")
    print("| accumulators per wave | waves per SIMD | cycles / instruction | shader clock GHz | TFLOP/s (chip) |\n|---:|---:|---:|---:|---:|")
    res["mfma_f32"] = []
    for ilp, wps in ((1, 1), (4, 1), (4, 2), (4, 3)):
        cpi, ghz, rate = issue_rate(lib, B, torch, N_VECTOR_OPS + 1, ilp, wps, iters=2048, n_cu=n_cu)
        res["mfma_f32"].append({"ilp": ilp, "waves_per_simd": wps, "cycles_per_instruction": cpi, "shader_ghz": ghz, "tflops": rate * MFMA_F32_FLOPS / 1e12})
        print(f"| {ilp} | {wps} | {cpi:.2f} | {ghz:.2f} | {rate * MFMA_F32_FLOPS / 1e12:.0f} |")
    print("\n## The Gaussian generator's parts alone (cycles per call and SIMD; a call is one lane's work for 4 Gaussians, 64 lanes per wave)\n")
    print("| part | waves per SIMD | cycles / call | shader clock GHz |\n|---|---:|---:|---:|")
    res["generator"] = []
    for part, name in enumerate(GEN_PARTS):
        for wps in (8, 4, 2):
            cyc, ghz = generator_rate(lib, B, torch, part, wps, n_cu=n_cu)
            res["generator"].append({"part": name, "waves_per_simd": wps, "cycles_per_call": cyc, "shader_ghz": ghz})
            print(f"| {name} | {wps} | {cyc:.0f} | {ghz:.2f} |")
    if args.json:
        json.dump(res, open(args.json, "w"), indent=1)


if __name__ == "__main__":
    sys.exit(main())
