#!/usr/bin/env python3
"""Runs the dominant kernels once each at their bench shapes (OPT-13B, configs[1]), next to a plain device copy
of known size, so that one `rocprofv3 --pmc ...` run can attribute hardware counters per launch:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o t -- python3 kernel_probe.py
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir> -o t -- python3 kernel_probe.py
    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES GRBM_GUI_ACTIVE ... -- python3 kernel_probe.py

The copy (1 GiB read, 1 GiB written) gives the factor between the traffic counters and real bytes.  Prints the
algorithmic bytes and flops of every probe, in launch order, so the counter values can be set against them.
`--set` picks a subset: encode (the four projection GEMMs at the first encode batch's token count), prefill,
decode_attn, decode_gemm (the four projections at 64, 153 and 256 rows), all (default).
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import numpy as np
import torch

import paper_2404_07947_amd as exe
import workload as wl

DEV = "cuda:0"
OPT_GEMMS = ((15360, 5120, "qkv"), (5120, 5120, "out"), (20480, 5120, "ffn1"), (5120, 20480, "ffn2"))


def gemm_once(M, N, K, name, out_mode):
    A = torch.randn((M, K), device=DEV).to(torch.bfloat16)
    W = (torch.randn((N, K), device=DEV) * 0.02).to(torch.bfloat16)
    b = torch.randn((N,), device=DEV).to(torch.bfloat16)
    out = torch.zeros((M, N), dtype=torch.float32 if out_mode else torch.bfloat16, device=DEV)
    ws = torch.empty(max(exe.exe_op_gemm_workspace(1, M, N, K) // 4, 1), dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    exe.exe_op_gemm(1, M, N, K, A, W, b, 0 if out_mode == 0 else -1, 1.0, out_mode, out, ws)
    torch.cuda.synchronize()
    ob = M * N * (2 if out_mode == 0 else 8)
    print(f"gemm {name} M={M} N={N} K={K}: reads {(M * K + N * K) * 2 + (M * N * 4 if out_mode else 0)} bytes, "
          f"writes {M * N * (2 if out_mode == 0 else 4)} bytes, {2 * M * N * K} flops (algorithmic bytes {(M * K + N * K) * 2 + ob})",
          flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--set", default="all", choices=["all", "encode", "prefill", "decode_attn", "decode_gemm"])
    args = ap.parse_args()
    want = lambda s: args.set in ("all", s)
    torch.manual_seed(0)
    # calibration copy: 1 GiB in, 1 GiB out
    src = torch.empty(1 << 29, dtype=torch.bfloat16, device=DEV).normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    print("copy: reads 1073741824 bytes, writes 1073741824 bytes", flush=True)
    del src, dst

    job = wl.workload_opt13b(256)
    H, dh = 40, 128
    if want("encode"):
        # the projections of one layer at the token count of the bench's first encode batch (QKV and FFN1 store
        # bf16, the out-projection and FFN2 accumulate into the float residual stream)
        T = int(job.in_len[:32].sum())
        for (N, K, name) in OPT_GEMMS:
            gemm_once(T, N, K, name, 1 if name in ("out", "ffn2") else 0)
    if want("decode_gemm"):
        for M in (64, 153, 256):
            for (N, K, name) in OPT_GEMMS:
                gemm_once(M, N, K, name, 1 if name in ("out", "ffn2") else 0)
    if want("decode_attn"):
        # decode attention at batch 256 with the bench job's K/V lengths after 64 decode steps
        lens = (job.in_len + 64).astype(np.int32)
        caps = ((lens + 8) // 8 * 8).astype(np.int64)
        offs = np.concatenate([[0], np.cumsum(2 * H * caps * dh)])[:-1].astype(np.int64)
        pool = torch.empty(int((2 * H * caps * dh).sum()), dtype=torch.bfloat16, device=DEV).normal_()
        q = torch.randn((256, H * dh), device=DEV).to(torch.bfloat16)
        out = torch.empty_like(q)
        t = lambda a, dt: torch.tensor(a, dtype=dt, device=DEV)
        torch.cuda.synchronize()
        exe.exe_op_decode_attention(1, 256, q, H * dh, pool, t(offs, torch.int64), t(caps, torch.int32), t(lens, torch.int32),
                                    t(lens - 1, torch.int32), H, dh, 1.0 / np.sqrt(dh), None, 0, out)
        torch.cuda.synchronize()
        print(f"decode_attn B=256 sum(L)={int(lens.sum())}: reads {int(lens.sum()) * 2 * H * dh * 2 + 256 * H * dh * 2} bytes, "
              f"writes {256 * H * dh * 2} bytes", flush=True)
        del pool
    if want("prefill"):
        # prefill attention of the first encode batch (32 sequences)
        il = job.in_len[:32]
        cu = np.concatenate([[0], np.cumsum(il)]).astype(np.int32)
        Tq = int(cu[-1])
        qkv = torch.randn((Tq, 3 * H * dh), device=DEV).to(torch.bfloat16)
        ctx = torch.empty((Tq, H * dh), dtype=torch.bfloat16, device=DEV)
        torch.cuda.synchronize()
        exe.exe_op_prefill_attention(1, cu, qkv, H, dh, 1.0 / np.sqrt(dh), 1, None, 0, ctx)
        torch.cuda.synchronize()
        fl = float(sum(2.0 * H * dh * int(L) * (int(L) + 1) for L in il))
        print(f"prefill_attn T={Tq}: reads {Tq * 3 * H * dh * 2} bytes, writes {Tq * H * dh * 2} bytes, {fl:.0f} flops", flush=True)


if __name__ == "__main__":
    main()
