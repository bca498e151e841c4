#!/usr/bin/env python3
"""Micro-benchmarks of what bounds the GEMMs (HIP-event timing, no profiler):

  python3 microbench.py ingest
      the rate at which a compute unit takes tile data in (exe_probe_ingest): L2-resident regions against the bytes in
      flight, streams from HBM with loads to registers / direct-to-LDS loads, ordinary / nontemporal, and the row-major
      operand-tile pattern at the row strides of K = 5120, 8192 and 20480.
  python3 microbench.py decode_gemm [--rows 16,64,153,256] [--lib PATH]
      the four projections of an OPT-13B layer (QKV, out, FFN1, FFN2) at decode row counts, split-K reductions included,
      with the weights rotating through HBM-resident copies; --lib takes a measurement variant of the library built by
      `python -m paper_2404_07947_amd.build --ablate N` (N: 1 no MFMA, 2 no activation loads, 4 no weight loads, sums
      combine), whose results are meaningless and whose timing isolates a part of the kernel.
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import torch

import paper_2404_07947_amd as exe
import paper_2404_07947_amd.binding as binding

DEV = "cuda:0"
OPT_GEMMS = ((15360, 5120, "qkv"), (5120, 5120, "out"), (20480, 5120, "ffn1"), (5120, 20480, "ffn2"))
MODES = {0: "registers", 1: "registers nt", 2: "LDS", 3: "LDS nt"}


def ingest():
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    row = lambda name, bps: print(f"| {name} | {bps / 1e12:.2f} | {bps / cus / 1e9:.1f} |", flush=True)
    print("L2-resident: 64 KB per workgroup read 400 times, direct-to-LDS loads\n")
    print("| waves x loads per batch (KB in flight per CU) | TB/s | GB/s per CU |\n|---|---:|---:|")
    for waves, lpb in ((1, 2), (1, 4), (1, 8), (1, 16), (2, 8), (4, 4), (4, 8), (8, 8)):
        row(f"{waves} x {lpb} ({waves * lpb}-{2 * waves * lpb})", exe.exe_probe_ingest(2, 64 << 10, 400, waves, lpb))
    print("\nHBM stream: 4 MB per workgroup read once\n")
    print("| loads | waves x loads per batch | TB/s | GB/s per CU |\n|---|---|---:|---:|")
    for mode in (0, 1, 2, 3):
        for waves, lpb in ((1, 4), (1, 8), (4, 4), (4, 8), (8, 8)):
            bps = exe.exe_probe_ingest(mode, 4 << 20, 1, waves, lpb)
            print(f"| {MODES[mode]} | {waves} x {lpb} | {bps / 1e12:.2f} | {bps / cus / 1e9:.1f} |", flush=True)
    print("\nOperand-tile pattern from HBM: a 128-row panel per workgroup, 8 rows x 128 bytes per wave-load, against the same bytes contiguous\n")
    print("| K (row stride) | loads | row-major TB/s | contiguous TB/s |\n|---:|---|---:|---:|")
    for K in (5120, 8192, 20480):
        for mode in (2, 3):
            a = exe.exe_probe_ingest(mode, 0, 1, 4, 4, 2 * K)
            b = exe.exe_probe_ingest(mode, 128 * 2 * K, 1, 4, 4)
            print(f"| {K} ({2 * K} B) | {MODES[mode]} | {a / 1e12:.2f} | {b / 1e12:.2f} |", flush=True)


def decode_gemm(rows, iters=40, copies=6):
    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters * 1e3
    print("| rows | " + " | ".join(f"{n} us (plan)" for _, _, n in OPT_GEMMS) + " | layer us | weights TB/s |\n|---:|" + "---:|" * 6)
    for M in rows:
        cells, layer = [], 0.0
        for N, K, _ in OPT_GEMMS:
            A = torch.randn((M, K), device=DEV).to(torch.bfloat16)
            Ws = [(torch.randn((N, K), device=DEV) * 0.02).to(torch.bfloat16) for _ in range(copies)]
            bias = torch.randn((N,), device=DEV).to(torch.bfloat16)
            out = torch.empty((M, N), device=DEV, dtype=torch.bfloat16)
            ws = torch.zeros(exe.exe_op_gemm_workspace(1, M, N, K) // 4 + 16, device=DEV, dtype=torch.float32)
            i = [0]

            def once():
                i[0] = (i[0] + 1) % copies
                exe.exe_op_gemm(1, M, N, K, A, Ws[i[0]], bias, 0, 1.0, 0, out, ws)
            t = timed(once)
            layer += t
            p = exe.exe_op_gemm_plan(1, M, N, K)
            cells.append(f"{t:.1f} ({exe.GEMM_CFG_NAMES[p['cfg']]} /{p['splits']})")
            del A, Ws, out, ws
        w_bytes = sum(N * K * 2 for N, K, _ in OPT_GEMMS)
        print(f"| {M} | " + " | ".join(cells) + f" | {layer:.1f} | {w_bytes / layer / 1e6:.2f} |", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["ingest", "decode_gemm"])
    ap.add_argument("--rows", default="16,64,153,256")
    ap.add_argument("--lib", default=None, help="a measurement variant of the library (python -m paper_2404_07947_amd.build --ablate N)")
    args = ap.parse_args()
    if args.lib:
        path = os.path.abspath(args.lib)
        binding.lib_path = lambda: path
    print(f"# {exe.exe_version()}  {binding.lib_path()}", flush=True)
    if args.what == "ingest":
        ingest()
    else:
        decode_gemm([int(x) for x in args.rows.split(",")])


if __name__ == "__main__":
    main()
