#!/usr/bin/env python3
"""Micro-benchmarks of what bounds the GEMMs (HIP-event timing, no profiler):

  python3 microbench.py ingest
      the rate at which a compute unit takes tile data in (exe_probe_ingest): L2-resident regions against the bytes in
      flight, streams from HBM with loads to registers / direct-to-LDS loads, ordinary / nontemporal, and the row-major
      operand-tile pattern at the row strides of K = 5120, 8192 and 20480.
  python3 microbench.py decode_gemm [--rows 16,64,153,256] [--lib PATH]
      the four projections of an OPT-13B layer (QKV, out, FFN1, FFN2) at decode row counts, split-K reductions included,
      with the weights rotating through HBM-resident copies; --lib takes a measurement variant of the library built by
      `python -m paper_2404_07947_amd.build --variant ablateN -DEXE_GEMM_ABLATE=N` (N: 1 no MFMA, 2 no activation loads, 4 no weight loads, 32 no epilogue, sums
      combine), whose results are meaningless and whose timing isolates a part of the kernel.
  python3 microbench.py encode_gemm [--rows 16020,16384] [--lib PATH]
      the same four projections at encode row counts; --lib e.g. a variant with the loads of a k-tile issued later
      or earlier (`build --variant late -DEXE_GEMM_ISSUE_AT=1`).
  python3 microbench.py two_streams
      one decode layer's attention and projections for the whole batch on one stream, against two half-batches on
      one stream and on two streams (one a phase ahead, so that one half's attention could run beside the other
      half's projections).
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


def encode_gemm(rows, iters=8):
    # the first launches after start-up run 8-10 % slow (clocks, first touches): spend them on a throw-away shape
    A = torch.randn((8192, 5120), device=DEV).to(torch.bfloat16)
    W = (torch.randn((5120, 5120), device=DEV) * 0.02).to(torch.bfloat16)
    out = torch.empty((8192, 5120), device=DEV, dtype=torch.bfloat16)
    for _ in range(40):
        exe.exe_op_gemm(1, 8192, 5120, 5120, A, W, None, -1, 1.0, 0, out, None)
    torch.cuda.synchronize()
    del A, W, out
    print("| rows | " + " | ".join(f"{n} us (TFLOP/s)" for _, _, n in OPT_GEMMS) + " | all TFLOP/s |\n|---:|" + "---:|" * 5)
    for M in rows:
        cells, tot, fl = [], 0.0, 0.0
        for N, K, _ in OPT_GEMMS:
            A = torch.randn((M, K), device=DEV).to(torch.bfloat16)
            Ws = [(torch.randn((N, K), device=DEV) * 0.02).to(torch.bfloat16) for _ in range(2)]
            bias = torch.randn((N,), device=DEV).to(torch.bfloat16)
            out = torch.empty((M, N), device=DEV, dtype=torch.bfloat16)
            ws = torch.zeros(exe.exe_op_gemm_workspace(1, M, N, K) // 4 + 16, device=DEV, dtype=torch.float32)
            for i in range(2):
                exe.exe_op_gemm(1, M, N, K, A, Ws[i], bias, 0, 1.0, 0, out, ws)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for i in range(iters):
                exe.exe_op_gemm(1, M, N, K, A, Ws[i % 2], bias, 0, 1.0, 0, out, ws)
            b.record()
            torch.cuda.synchronize()
            t = a.elapsed_time(b) / iters * 1e3
            tot += t
            fl += 2.0 * M * N * K
            cells.append(f"{t:.1f} ({2.0 * M * N * K / t / 1e6:.0f})")
            del A, Ws, out, ws
        print(f"| {M} | " + " | ".join(cells) + f" | {fl / tot / 1e6:.0f} |", flush=True)


def two_streams(layers=20):
    import numpy as np
    import workload as wl
    H, dh = 40, 128
    lens_all = (wl.workload_opt13b(256).in_len + 64).astype(np.int32)
    shapes = [(N, K) for N, K, _ in OPT_GEMMS]
    wsets = [[(torch.randn((N, K), device=DEV) * 0.02).to(torch.bfloat16) for N, K in shapes] for _ in range(3)]

    def attention(lens):
        lens = np.asarray(lens, dtype=np.int32)
        B = len(lens)
        caps = ((lens + 8) // 8 * 8).astype(np.int64)
        offs = np.concatenate([[0], np.cumsum(2 * H * caps * dh)])[:-1].astype(np.int64)
        pool = torch.empty(int((2 * H * caps * dh).sum()), dtype=torch.bfloat16, device=DEV).normal_()
        q = torch.randn((B, H * dh), device=DEV).to(torch.bfloat16)
        out = torch.empty_like(q)
        t = lambda a, dt: torch.tensor(a, dtype=dt, device=DEV)
        args = (1, B, q, H * dh, pool, t(offs, torch.int64), t(caps, torch.int32), t(lens, torch.int32), t(lens - 1, torch.int32),
                H, dh, 1.0 / np.sqrt(dh), None, 0, out)
        return lambda s: exe.exe_op_decode_attention(*args, stream=s)

    def projections(M):
        As = [torch.randn((M, K), device=DEV).to(torch.bfloat16) for _, K in shapes]
        outs = [torch.empty((M, N), device=DEV, dtype=torch.bfloat16) for N, _ in shapes]
        wss = [torch.zeros(exe.exe_op_gemm_workspace(1, M, N, K) // 4 + 16, device=DEV, dtype=torch.float32) for N, K in shapes]
        turn = [0]

        def run(s):
            turn[0] += 1
            W = wsets[turn[0] % 3]
            for i, (N, K) in enumerate(shapes):
                exe.exe_op_gemm(1, M, N, K, As[i], W[i], None, -1, 1.0, 0, outs[i], wss[i], stream=s)
        return run

    def timed(fn):
        fn(2)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn(layers)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / layers * 1e3
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    print("| batch | attention us | projections us | one stream us | two halves, one stream us | two halves, two streams us |\n|---:|" + "---:|" * 5)
    for B in (256, 128, 64):
        h = B // 2
        att, gem = attention(lens_all[:B]), projections(B)
        att_a, att_b, gem_a, gem_b = attention(lens_all[:h]), attention(lens_all[h:B]), projections(h), projections(h)
        cur = torch.cuda.current_stream()

        def whole(L):
            for _ in range(L):
                att(None)
                gem(None)

        def halves(L):
            for _ in range(L):
                att_a(None)
                gem_a(None)
                att_b(None)
                gem_b(None)

        def streams(L):
            s1.wait_stream(cur)
            s2.wait_stream(cur)
            gem_b(s2)                                  # the second half starts a phase ahead
            for _ in range(L):
                att_a(s1)
                gem_a(s1)
                att_b(s2)
                gem_b(s2)
            cur.wait_stream(s1)
            cur.wait_stream(s2)
        only_att = lambda L: [att(None) for _ in range(L)]
        only_gem = lambda L: [gem(None) for _ in range(L)]
        print(f"| {B} | {timed(only_att):.1f} | {timed(only_gem):.1f} | {timed(whole):.1f} | {timed(halves):.1f} | {timed(streams):.1f} |", flush=True)
        del att, gem, att_a, att_b, gem_a, gem_b


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["ingest", "decode_gemm", "encode_gemm", "two_streams"])
    ap.add_argument("--rows", default=None)
    ap.add_argument("--lib", default=None, help="a measurement variant of the library (python -m paper_2404_07947_amd.build --variant ...)")
    args = ap.parse_args()
    if args.lib:
        path = os.path.abspath(args.lib)
        binding.lib_path = lambda: path
    print(f"# {exe.exe_version()}  {binding.lib_path()}", flush=True)
    rows = lambda dflt: [int(x) for x in (args.rows or dflt).split(",")]
    if args.what == "ingest":
        ingest()
    elif args.what == "decode_gemm":
        decode_gemm(rows("16,64,153,256"))
    elif args.what == "encode_gemm":
        encode_gemm(rows("16020,16384"))
    else:
        two_streams()


if __name__ == "__main__":
    main()
