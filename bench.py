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


def run_job(m, job, shape, timed_kernels=None, decode_sample_every=1, hidden=None):
    """One full pass.  Returns (encode_s, decode_s, n_in_tokens, n_generated, n_decode_steps).
    Decoder-only models emit generated token 1 from the encode call; encoder-decoder models start decoding
    from token id 0.  `hidden` = (encode hidden states [sum in_len, d], decode hidden states [n, d]) for
    models without an embedding (they return hidden states; nothing is fed back)."""
    import workload as wl
    dec_only = shape.arch == wl.ARCH_DECODER_ONLY
    has_tok = bool(shape.has_embed)
    n = job.n
    ids = np.arange(n, dtype=np.int32)
    off = job.offsets()
    cur = np.zeros(n, dtype=np.int32)
    reserve = (job.in_len + job.out_len).astype(np.int32) if dec_only else job.out_len.astype(np.int32)
    t_enc = 0.0
    for b0 in range(0, n, job.encode_batch):
        sl = slice(b0, min(n, b0 + job.encode_batch))
        if timed_kernels is not None:
            m.kernel_timing(True)
        t0 = time.perf_counter()
        r = m.encode(ids[sl], job.in_len[sl], job.tokens[off[sl.start]:off[sl.stop]] if has_tok else None,
                     reserve_lengths=reserve[sl], hidden_in=None if has_tok else hidden[0][off[sl.start]:off[sl.stop]],
                     want_tokens=has_tok and dec_only, out_device=None if has_tok else hidden[2][off[sl.start]:off[sl.stop]])
        t_enc += time.perf_counter() - t0
        if has_tok and dec_only:
            cur[sl] = r
        if timed_kernels is not None:
            accumulate(timed_kernels["encode"], m.kernel_times())
            m.kernel_timing(False)
    generated = n if dec_only else 0     # decoder-only: the encode calls emitted token 1 of every sequence
    t_dec = 0.0
    steps = wl.n_decode_steps(job.out_len, dec_only)
    alive_prev = ids
    for step in range(1, steps + 1):
        alive = wl.alive_at_step(job.out_len, step, dec_only)
        if len(alive) < len(alive_prev):
            m.seq_release(np.setdiff1d(alive_prev, alive))
        alive_prev = alive
        kv = job.in_len[alive] + step if dec_only else np.full(len(alive), step, dtype=np.int32)
        hid_in = hid_out = None
        if not has_tok:
            hid_in, hid_out = hidden[1][: len(alive)], hidden[3][: len(alive)]
        sample = timed_kernels is not None and (step - 1) % decode_sample_every == 0
        if sample:
            m.kernel_timing(True)
        t0 = time.perf_counter()
        r = m.decode_step(alive, cur[alive] if has_tok else None, kv, hidden_in=hid_in, want_tokens=has_tok, out_device=hid_out)
        t_dec += time.perf_counter() - t0
        if has_tok:
            cur[alive] = r
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


# HBM-side bytes (rocprofv3 FETCH_SIZE x 2 + WRITE_SIZE, factors from a plain copy) per algorithmic byte, measured
# per kernel at the OPT-13B bench shapes by a separate counter run (profiles/traffic_opt13b_kernels.md gives the
# command and the table; regenerate it whenever a kernel it covers changes).  gemm_skinny: at the job's mean decode
# batch of 153 rows (1.20 at 64 rows, 1.51 at 256: the split-K partial sums).  A class not listed reports null.
TRAFFIC_RATIO = {"gemm_tile": 6.04, "gemm_skinny": 1.38, "decode_attn": 1.0, "cross_attn": 1.0, "prefill_attn": 1.02}


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
    ratio = TRAFFIC_RATIO.get(kind)
    return {"kernel": kind, "bound": "mfma" if mfma else "hbm", "achieved": round(ach, 2), "peak": peak, "unit": unit,
            "frac": round(ach / peak, 4),
            "traffic": None if ratio is None else round(ratio * a["bytes"] / a["launches"]),
            "algorithmic_bytes_per_launch": round(a["bytes"] / a["launches"]),
            "algorithmic_flops_per_launch": round(a["flops"] / a["launches"]),
            "launches": int(a["launches"]), "avg_ms": round(a["ms"] / a["launches"], 5), "total_ms": round(a["ms"], 2)}


def cpu_baseline(shape, weights_dev, job):
    """The oracle (float build, as it stands) on a bounded sample: ONE of the decoder layers at full width, the
    first sequences of the job up to about 6000 input tokens, encode + 4 decode steps each; the measured
    per-layer rate is divided by the layer count."""
    import oracle
    import workload as wl
    if shape.arch != wl.ARCH_DECODER_ONLY or not shape.has_embed:
        return None
    s1 = shape.replace(n_layers=1)
    names = [n for n, _, _ in wl.weight_specs(shape)]
    keep = [n for n, _, _ in wl.weight_specs(s1)]
    w1 = [weights_dev[names.index(n)].float().cpu() for n in keep]
    o = oracle.Oracle(s1, w1, "float")
    pick, tot = [], 0
    for i in range(job.n):
        pick.append(i)
        tot += int(job.in_len[i])
        if tot >= 6000:
            break
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
            "sample": f"1 of {shape.n_layers} layers at full width, the job's first {len(pick)} sequences "
                      f"({tot} input tokens) encode + 4 decode steps each: {tokens} tokens in {dt:.1f} s = "
                      f"{per_layer:.1f} tokens/s per layer; value = that / {shape.n_layers} (extrapolated from 1 of "
                      f"{shape.n_layers} layers), float arithmetic, OpenMP"}


WORKLOADS = {
    # name: (shape factory, job factory, default B0, description)
    "opt13b": ("configs[1] OPT-13B shape ({L} layers, d 5120, 40 heads, FFN 20480, vocab 50272), bf16 random init: "
               "{nb} encode batches of {eb} (inputs N(512,128) in [64,1024]) then shrinking decode from B0={n} "
               "(outputs N(128,32) in [16,256], forced)"),
    "t5_11b": ("configs[2] T5-11B shape ({L}+{LD} layers, d 1024, 128 heads of 128, FFN 65536, vocab 32128), bf16 random "
               "init: {nb} encode batches of {eb} (inputs N(768,192) in [128,1024]) then shrinking decode from B0={n} "
               "with cross-attention + relative-position bias (outputs N(64,16) in [8,128], forced)"),
    "gpt3_share": ("configs[3] one GPU's share of a GPT-3-175B shape ({L} layers, d 12288, 96 heads, FFN 49152), hidden "
                   "states in and out, bf16 random init: {nb} encode batches of {eb} (inputs N(1024,256) in [128,2048]) "
                   "then shrinking decode from B0={n} (outputs N(256,64) in [32,512], forced)"),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="opt13b",
                    help="opt13b is the benchmark (BASELINE metric); the others are secondary measurements")
    ap.add_argument("--decode-batch", type=int, default=0, help="B0: sequences decoded together (default per workload)")
    ap.add_argument("--layers", type=int, default=0, help="debugging only: fewer layers is NOT the benchmark")
    ap.add_argument("--rra", type=int, default=0, metavar="N_D",
                    help="also run the refilled (RRA) schedule: 3 x B0 requests, decode batch B0, N_D decode iterations "
                         "between encoding phases (secondary figures under the key \"rra\")")
    ap.add_argument("--kv-block", type=int, default=0, metavar="POSITIONS",
                    help="paged K/V pool with blocks of this many positions (default 0: one extent per sequence, the "
                         "configuration the headline is measured in)")
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
    if args.workload == "opt13b":
        shape = wl.opt13b_shape(args.layers or 40)
        job = wl.workload_opt13b(args.decode_batch or 256)
        max_in = 1024
    elif args.workload == "t5_11b":
        shape = wl.t5_11b_shape(args.layers or 24, args.layers or 24)
        job = wl.workload_t5(args.decode_batch or 64)
        max_in = 1024
    else:
        shape = wl.gpt3_175b_share_shape(args.layers or 12)
        job = wl.workload_gpt3_share(args.decode_batch or 256)
        max_in = 2048
    dec_only = shape.arch == wl.ARCH_DECODER_ONLY
    t0 = time.perf_counter()
    weights = wl.make_weights(shape, wl.BASE_SEED + 1, device="cuda:0")
    torch.cuda.synchronize()
    print(f"[bench] weights {wl.n_params(shape) / 1e9:.2f} G params generated in {time.perf_counter() - t0:.1f} s",
          file=sys.stderr, flush=True)
    n_kv_layers = shape.n_layers if dec_only else shape.n_dec_layers
    kv_tok = n_kv_layers * 2 * shape.inner * 2
    if dec_only:
        need_tokens = int(((job.in_len + job.out_len + 8) // 8 * 8).sum())
    else:
        need_tokens = int(((job.in_len + 8) // 8 * 8).sum() + ((job.out_len + 8) // 8 * 8).sum())
    if args.rra:
        need_tokens = int(need_tokens * 1.3)          # refilled batches fragment the pool: leave slack
    cfg = exe.config_from_shape(shape, kv_pool_bytes=need_tokens * kv_tok, max_seqs=job.n,
                                max_batch_tokens=job.encode_batch * max_in, max_batch_seqs=max(job.n, job.encode_batch),
                                kv_block_size=args.kv_block)
    hidden = None
    if not shape.has_embed:
        # (before the K/V pool is allocated: the generator's float temporaries are returned to the device first)
        T = int(job.in_len.sum())
        hidden = (wl.random_hidden(11, T, shape.d_model, shape.dtype, "cuda:0"),
                  wl.random_hidden(12, job.n, shape.d_model, shape.dtype, "cuda:0"),
                  torch.empty((T, shape.d_model), dtype=torch.bfloat16, device="cuda:0"),
                  torch.empty((job.n, shape.d_model), dtype=torch.bfloat16, device="cuda:0"))
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
    stream = torch.cuda.Stream()
    m = exe.Model(cfg, weights, stream=stream)
    print(f"[bench] K/V pool {need_tokens * kv_tok / 1e9:.1f} GB for {job.n} sequences, {need_tokens} positions",
          file=sys.stderr, flush=True)

    for i in range(args.warmup):
        r = run_job(m, job, shape, hidden=hidden)
        print(f"[bench] warmup {i}: encode {r[0]:.3f} s decode {r[1]:.3f} s", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    t_enc = t_dec = 0.0
    t_start = time.perf_counter()
    for i in range(args.steps):
        e, d, n_in, n_gen, n_steps = run_job(m, job, shape, hidden=hidden)
        t_enc += e
        t_dec += d
        print(f"[bench] step {i}: encode {e:.3f} s decode {d:.3f} s", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    total = time.perf_counter() - t_start
    K = args.steps
    n_dec_tokens = n_gen - job.n if dec_only else n_gen       # tokens produced by decode iterations
    out = {
        "metric": "encode & decode tokens/s per MI355X at OPT-13B shape (value = input tokens encoded + tokens "
                  "generated per second of the whole job; encode and decode rates listed separately); % MFMA/HBM roofline",
        "value": round(K * (n_in + n_gen) / total, 1), "unit": "tokens/s", "n_gpus": 1, "steps": K,
        "warmup": args.warmup, "ms_per_step": round(1e3 * total / K, 2), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOADS[args.workload].format(L=shape.n_layers, LD=shape.n_dec_layers,
                                                               nb=-(-job.n // job.encode_batch), eb=job.encode_batch, n=job.n),
                   "decode_batch": job.n, "encode_batch": job.encode_batch, "input_tokens": n_in,
                   "generated_tokens": n_gen, "decode_iterations": n_steps, "layers": shape.n_layers + shape.n_dec_layers,
                   "kv_block_size": args.kv_block},
        "encode_tokens_per_s": round(K * n_in / t_enc, 1),
        "decode_tokens_per_s": round(K * n_dec_tokens / t_dec, 1),
        "encode_s_per_step": round(t_enc / K, 4), "decode_s_per_step": round(t_dec / K, 4),
        "decode_ms_per_iteration": round(1e3 * t_dec / K / n_steps, 3),
    }
    if args.workload != "opt13b":
        out["metric"] = out["metric"].replace("at OPT-13B shape", f"at the {args.workload} shape (secondary workload)")
    if not args.no_roofline:
        every = 8
        acc = {"encode": {}, "decode": {}}
        run_job(m, job, shape, timed_kernels=acc, decode_sample_every=every, hidden=hidden)
        kernels = {}
        for phase in ("encode", "decode"):
            rows = [roofline_entry(k, a) for k, a in acc[phase].items()]
            kernels[phase] = sorted([r for r in rows if r], key=lambda r: -r["total_ms"])
        # the dominant kernel class of the job: most time over the whole step (decode classes were sampled every
        # `every`-th iteration, so their totals are scaled up)
        enc_top, dec_top = kernels["encode"][0], kernels["decode"][0]
        dom = enc_top if enc_top["total_ms"] >= dec_top["total_ms"] * every else dec_top
        out["roofline"] = {k: dom[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
        out["roofline"].update(kernel=dom["kernel"], avg_ms=dom["avg_ms"],
                               algorithmic_bytes_per_launch=dom["algorithmic_bytes_per_launch"],
                               algorithmic_flops_per_launch=dom["algorithmic_flops_per_launch"])
        out["roofline_kernels"] = kernels
        out["roofline_decode_sampling"] = f"decode classes timed on every {every}th iteration"
        enc_flops = sum(a["flops"] for a in acc["encode"].values())
        out["encode_frac_of_mfma_peak"] = round(enc_flops / (t_enc / K) / PEAK_MFMA_BF16, 4)
        # what this machine sustains with nothing but loads / nothing but MFMAs, measured now (the fractions above stay
        # against the nominal peaks)
        torch.cuda.synchronize()
        pk = exe.exe_probe_peaks()
        ach = {"hbm": pk["hbm_read_bytes_per_s"] / 1e9, "mfma": pk["mfma_bf16_flops_per_s"] / 1e12}
        out["achievable"] = {"hbm_read_GBps": round(ach["hbm"], 1), "mfma_bf16_TFLOPs": round(ach["mfma"], 1),
                             "how": "streaming read of 4 GiB; back-to-back 16x16x32 bf16 MFMAs on every CU"}
        out["roofline"]["frac_of_achievable"] = round(dom["achieved"] / ach[dom["bound"]], 4)
    if args.rra and shape.has_embed:
        rng = np.random.default_rng(wl.BASE_SEED + 17)
        big = {"opt13b": wl.workload_opt13b, "t5_11b": wl.workload_t5}[args.workload](3 * job.n, seed=wl.BASE_SEED + 17)
        _, st = m.run_rra(job.n, args.rra, big.in_len, big.out_len, big.tokens, max_encode_batch=job.encode_batch)
        out["rra"] = {"schedule": f"RRA, {big.n} requests queued at time 0, decode batch {job.n}, N_D = {args.rra}, "
                                  f"encode batches of at most {job.encode_batch}",
                      "tokens_per_s": round((st["encoded_tokens"] + st["generated_tokens"]) / st["wall_s"], 1),
                      "generated_tokens_per_s": round(st["generated_tokens"] / st["wall_s"], 1),
                      "sequences_per_s": round(big.n / st["wall_s"], 2),
                      **{k: (round(v, 4) if isinstance(v, float) else v) for k, v in st.items()}}
    if not args.no_cpu_baseline:
        cb = cpu_baseline(shape, weights, job)
        if cb:
            out["cpu_baseline"] = cb
    m.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
