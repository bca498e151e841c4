#!/usr/bin/env python3
"""Benchmark of the whole hot path at the OPT-13B shape (configs[1]) on one MI355X.

One "step" = one pass of the whole path over one synthetic job: B0 sequences are encoded in batches of 32
(inputs ~ N(512,128) clipped to [64,1024]) and then decoded together, one token per live sequence per
iteration, until every sequence has produced its forced output length (~ N(128,32) clipped to [16,256]);
finished sequences leave the batch.  Inputs (weights, token ids, lengths) are resident before timing starts.

Prints ONE JSON line.  `value` = (input tokens encoded + tokens generated) / wall time of the timed steps;
encode and decode rates are given separately, with the per-kernel-class roofline figures measured with HIP
events on the library's stream in an extra instrumented pass, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_BF16 = 2.5e15      # dense bf16 MFMA flop/s, MI355X
PEAK_HBM = 8.0e12            # bytes/s


def run_job(m, job, shape, timed_kernels=None, decode_sample_every=1):
    """One full pass.  Returns (encode_s, decode_s, n_in_tokens, n_generated, n_decode_steps)."""
    import workload as wl
    n = job.n
    ids = np.arange(n, dtype=np.int32)
    off = job.offsets()
    cur = np.zeros(n, dtype=np.int32)
    reserve = (job.in_len + job.out_len).astype(np.int32)
    t_enc = 0.0
    for b0 in range(0, n, job.encode_batch):
        sl = slice(b0, min(n, b0 + job.encode_batch))
        if timed_kernels is not None:
            m.kernel_timing(True)
        t0 = time.perf_counter()
        cur[sl] = m.encode(ids[sl], job.in_len[sl], job.tokens[off[sl.start]:off[sl.stop]], reserve_lengths=reserve[sl])
        t_enc += time.perf_counter() - t0
        if timed_kernels is not None:
            accumulate(timed_kernels["encode"], m.kernel_times())
            m.kernel_timing(False)
    generated = n            # the encode calls emitted token #1 of every sequence
    t_dec = 0.0
    steps = wl.n_decode_steps(job.out_len, True)
    alive_prev = ids
    for step in range(1, steps + 1):
        alive = wl.alive_at_step(job.out_len, step, True)
        if len(alive) < len(alive_prev):
            gone = np.setdiff1d(alive_prev, alive)
            m.seq_release(gone)
        alive_prev = alive
        sample = timed_kernels is not None and (step - 1) % decode_sample_every == 0
        if sample:
            m.kernel_timing(True)
        t0 = time.perf_counter()
        cur[alive] = m.decode_step(alive, cur[alive], job.in_len[alive] + step)
        t_dec += time.perf_counter() - t0
        if sample:
            accumulate(timed_kernels["decode"], m.kernel_times())
            m.kernel_timing(False)
        generated += len(alive)
    m.seq_release(alive_prev)
    return t_enc, t_dec, int(job.in_len.sum()), generated, steps


def accumulate(acc, rows):
    for r in rows:
        a = acc.setdefault(r["kind"], {"launches": 0, "ms": 0.0, "bytes": 0.0, "flops": 0.0})
        for k in ("launches", "ms", "bytes", "flops"):
            a[k] += r[k]


def roofline_entry(kind, a):
    """Achieved rate of one kernel class against the roofline that bounds it."""
    if a["launches"] == 0 or a["ms"] <= 0:
        return None
    sec = a["ms"] * 1e-3
    mfma = kind in ("gemm_tile", "prefill_attn")
    if mfma:
        ach, peak, unit = a["flops"] / sec / 1e12, PEAK_MFMA_BF16 / 1e12, "TFLOP/s"
    else:
        ach, peak, unit = a["bytes"] / sec / 1e9, PEAK_HBM / 1e9, "GB/s"
    return {"kernel": kind, "bound": "mfma" if mfma else "hbm", "achieved": round(ach, 2), "peak": peak, "unit": unit,
            "frac": round(ach / peak, 4), "traffic": None, "launches": int(a["launches"]),
            "avg_ms": round(a["ms"] / a["launches"], 5), "total_ms": round(a["ms"], 2)}


def cpu_baseline(shape, weights_dev, job):
    """The oracle (float build, as it stands) on a bounded sample: ONE of the 40 layers at full width, the two
    shortest sequences of the job, encode + 4 decode steps; rate divided by the layer count."""
    import oracle
    import workload as wl
    s1 = shape.replace(n_layers=1)
    names = [n for n, _, _ in wl.weight_specs(shape)]
    keep = [n for n, _, _ in wl.weight_specs(s1)]
    w1 = [weights_dev[names.index(n)].float().cpu() for n in keep]
    o = oracle.Oracle(s1, w1, "float")
    pick = np.argsort(job.in_len)[:2]
    t0 = time.perf_counter()
    tokens = 0
    for j, i in enumerate(pick):
        t, _ = o.encode(j, job.seq_tokens(int(i)))
        tokens += int(job.in_len[i]) + 1
        for _ in range(4):
            t, _ = o.decode(j, t)
            tokens += 1
    dt = time.perf_counter() - t0
    per_layer = tokens / dt
    return {"value": round(per_layer / shape.n_layers, 3), "unit": "tokens/s", "cores": o.threads, "kind": "oracle",
            "sample": f"1 of {shape.n_layers} layers at full OPT-13B width, 2 shortest sequences "
                      f"({[int(job.in_len[i]) for i in pick]} input tokens) encode + 4 decode steps: {tokens} tokens in "
                      f"{dt:.1f} s = {per_layer:.1f} tokens/s per layer; value = that / {shape.n_layers} "
                      f"(extrapolated from 1 of {shape.n_layers} layers), float arithmetic, OpenMP"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--decode-batch", type=int, default=256, help="B0: sequences decoded together (32..256)")
    ap.add_argument("--layers", type=int, default=40, help="debugging only: fewer layers is NOT the benchmark")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; every figure is one MI355X's throughput. "
              "Multi-GPU runs (--gpus > 1) are not part of it.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2404_07947_amd as exe
    import workload as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    shape = wl.opt13b_shape(args.layers)
    job = wl.workload_opt13b(args.decode_batch)
    t0 = time.perf_counter()
    weights = wl.make_weights(shape, wl.BASE_SEED + 1, device="cuda:0")
    torch.cuda.synchronize()
    print(f"[bench] weights {wl.n_params(shape) / 1e9:.2f} G params generated in {time.perf_counter() - t0:.1f} s",
          file=sys.stderr, flush=True)
    kv_tok = shape.n_layers * 2 * shape.inner * 2
    need_tokens = int(((job.in_len + job.out_len + 8) // 8 * 8).sum())
    cfg = exe.config_from_shape(shape, kv_pool_bytes=need_tokens * kv_tok, max_seqs=job.n,
                                max_batch_tokens=job.encode_batch * 1024, max_batch_seqs=max(job.n, job.encode_batch))
    stream = torch.cuda.Stream()
    m = exe.Model(cfg, weights, stream=stream)
    print(f"[bench] K/V pool {need_tokens * kv_tok / 1e9:.1f} GB for {job.n} sequences, {need_tokens} positions",
          file=sys.stderr, flush=True)

    for i in range(args.warmup):
        r = run_job(m, job, shape)
        print(f"[bench] warmup {i}: encode {r[0]:.3f} s decode {r[1]:.3f} s", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    t_enc = t_dec = 0.0
    t_start = time.perf_counter()
    for i in range(args.steps):
        e, d, n_in, n_gen, n_steps = run_job(m, job, shape)
        t_enc += e
        t_dec += d
        print(f"[bench] step {i}: encode {e:.3f} s decode {d:.3f} s", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    total = time.perf_counter() - t_start
    K = args.steps
    out = {
        "metric": "encode & decode tokens/s per MI355X at OPT-13B shape (value = input tokens encoded + tokens "
                  "generated per second of the whole job; encode and decode rates listed separately); % MFMA/HBM roofline",
        "value": round(K * (n_in + n_gen) / total, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K,
        "warmup": args.warmup, "ms_per_step": round(1e3 * total / K, 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"configs[1] OPT-13B shape ({shape.n_layers} layers, d 5120, 40 heads, FFN 20480, vocab "
                               f"50272), bf16 random init: {job.n // job.encode_batch} encode batches of "
                               f"{job.encode_batch} (inputs N(512,128) in [64,1024]) then shrinking decode from "
                               f"B0={job.n} (outputs N(128,32) in [16,256], forced)",
                   "decode_batch": job.n, "encode_batch": job.encode_batch, "input_tokens": n_in,
                   "generated_tokens": n_gen, "decode_iterations": n_steps, "layers": shape.n_layers},
        "encode_tokens_per_s": round(K * n_in / t_enc, 1),
        "decode_tokens_per_s": round(K * (n_gen - job.n) / t_dec, 1),
        "encode_s_per_step": round(t_enc / K, 4), "decode_s_per_step": round(t_dec / K, 4),
        "decode_ms_per_iteration": round(1e3 * t_dec / K / n_steps, 3),
    }
    if not args.no_roofline:
        acc = {"encode": {}, "decode": {}}
        run_job(m, job, shape, timed_kernels=acc, decode_sample_every=8)
        kernels = {}
        for phase in ("encode", "decode"):
            rows = [roofline_entry(k, a) for k, a in acc[phase].items()]
            kernels[phase] = sorted([r for r in rows if r], key=lambda r: -r["total_ms"])
        # the dominant kernel of the job: the class with the most time in its phase, weighted by the phase's
        # share of the step (decode was sampled every 8th iteration)
        enc_top, dec_top = kernels["encode"][0], kernels["decode"][0]
        dom = enc_top if enc_top["total_ms"] >= dec_top["total_ms"] * 8 else dec_top
        out["roofline"] = {k: dom[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
        out["roofline"]["kernel"] = dom["kernel"]
        out["roofline"]["avg_ms"] = dom["avg_ms"]
        out["roofline_kernels"] = kernels
        # whole-phase figures: encode flops against MFMA peak, decode bytes against HBM peak
        enc_flops = sum(a["flops"] for a in acc["encode"].values())
        dec_bytes = sum(a["bytes"] for a in acc["decode"].values())
        dec_sampled_s = None
        out["encode_frac_of_mfma_peak"] = round(enc_flops / (t_enc / K) / PEAK_MFMA_BF16, 4)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, weights, job)
    m.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
