"""Runs the dominant kernels once each at their bench shapes, next to a plain device copy of known size, so
that `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` can attribute HBM traffic per launch:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o t -- python3 paper_2404_07947_amd/traffic_probe.py
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir> -o t -- python3 paper_2404_07947_amd/traffic_probe.py

The copy (1 GiB read, 1 GiB written) gives the factor between the counter and real bytes.  Prints the
algorithmic bytes of every probe so the counter values can be set against them.
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import numpy as np
import torch

import paper_2404_07947_amd as exe
import workload as wl

DEV = "cuda:0"


def main():
    torch.manual_seed(0)
    # 1. calibration copy: 1 GiB in, 1 GiB out
    src = torch.empty(1 << 29, dtype=torch.bfloat16, device=DEV).normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    print("copy: reads 1073741824 bytes, writes 1073741824 bytes")
    del src, dst

    # 2. encode GEMMs of one OPT-13B layer at T = 16701 tokens (the bench's first encode batch)
    T = 16701
    for (N, K, name) in ((15360, 5120, "qkv"), (5120, 5120, "out"), (20480, 5120, "ffn1"), (5120, 20480, "ffn2")):
        A = torch.randn((T, K), device=DEV).to(torch.bfloat16)
        W = (torch.randn((N, K), device=DEV) * 0.02).to(torch.bfloat16)
        b = torch.randn((N,), device=DEV).to(torch.bfloat16)
        out = torch.empty((T, N), dtype=torch.bfloat16, device=DEV)
        # (the rows beyond whole rounds of tiles go to a second launch, which may use split-K partials)
        ws = torch.empty(max(exe.exe_op_gemm_workspace(1, T, N, K) // 4, 1), dtype=torch.float32, device=DEV)
        exe.exe_op_gemm(1, T, N, K, A, W, b, 0, 1.0, 0, out, ws)
        torch.cuda.synchronize()
        print(f"gemm {name} M={T} N={N} K={K}: reads {(T * K + N * K) * 2} bytes, writes {T * N * 2} bytes")
        del A, W, b, out, ws

    # 3. decode attention at batch 256 with the bench job's K/V lengths after 64 decode steps
    job = wl.workload_opt13b(256)
    H, dh = 40, 128
    lens = (job.in_len + 64).astype(np.int32)
    caps = ((lens + 8) // 8 * 8).astype(np.int64)
    offs = np.concatenate([[0], np.cumsum(2 * H * caps * dh)])[:-1].astype(np.int64)
    pool = torch.empty(int((2 * H * caps * dh).sum()), dtype=torch.bfloat16, device=DEV).normal_()
    q = torch.randn((256, H * dh), device=DEV).to(torch.bfloat16)
    out = torch.empty_like(q)
    t = lambda a, dt: torch.tensor(a, dtype=dt, device=DEV)
    exe.exe_op_decode_attention(1, 256, q, H * dh, pool, t(offs, torch.int64), t(caps, torch.int32), t(lens, torch.int32),
                                t(lens - 1, torch.int32), H, dh, 1.0 / np.sqrt(dh), None, 0, out)
    torch.cuda.synchronize()
    print(f"decode_attn B=256 sum(L)={int(lens.sum())}: reads {int(lens.sum()) * 2 * H * dh * 2 + 256 * H * dh * 2} bytes, "
          f"writes {256 * H * dh * 2} bytes")
    del pool

    # 4. prefill attention of the first encode batch (32 sequences)
    il = job.in_len[:32]
    cu = np.concatenate([[0], np.cumsum(il)]).astype(np.int32)
    Tq = int(cu[-1])
    qkv = torch.randn((Tq, 3 * H * dh), device=DEV).to(torch.bfloat16)
    ctx = torch.empty((Tq, H * dh), dtype=torch.bfloat16, device=DEV)
    exe.exe_op_prefill_attention(1, cu, qkv, H, dh, 1.0 / np.sqrt(dh), 1, None, 0, ctx)
    torch.cuda.synchronize()
    print(f"prefill_attn T={Tq}: reads {Tq * 3 * H * dh * 2} bytes, writes {Tq * H * dh * 2} bytes")


if __name__ == "__main__":
    main()
