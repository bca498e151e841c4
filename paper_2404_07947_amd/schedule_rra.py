"""Profile -> simulate -> schedule -> run, on one MI355X at the OPT-13B shape.

The model's own latency table (exe_profile) feeds the schedule simulator; the branch-and-bound search
(exe_sched_rra) picks the decode batch B_D and the number of decode iterations N_D between encoding phases for each
latency bound; exe_run_rra then executes that configuration on a queue of synthetic requests and the simulated
throughput and latency are printed next to the measured ones.

    python -m paper_2404_07947_amd.schedule_rra [--layers 40] [--requests 768] [--bounds 3,4,6,0] [--markdown]

Input lengths ~ Normal(512, 128) clipped to [64, 1024], output lengths ~ Normal(128, 32) clipped to [16, 256]
(the benchmark's recipe); the latency bound applies to a query of 200 output tokens (about the 99th percentile);
bound 0 means unbounded.
"""
import argparse
import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=40)
    ap.add_argument("--requests", type=int, default=768)
    ap.add_argument("--bounds", default="3,4,6,0", help="latency bounds in seconds for a 200-token answer; 0 = none")
    ap.add_argument("--max-batch", type=int, default=256)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--markdown", action="store_true")
    args = ap.parse_args()
    import numpy as np
    import torch
    import paper_2404_07947_amd as exe
    import workload as wl

    shape = wl.opt13b_shape(args.layers)
    weights = wl.make_weights(shape, wl.BASE_SEED + 1, device="cuda:0")
    job = wl.workload_opt13b(args.requests, seed=wl.BASE_SEED + 17)
    kv_tok = shape.n_layers * 2 * shape.inner * 2
    # room for max_batch live sequences of average length with slack for spread and fragmentation (admission waits
    # when the pool is full); about 190 GB at 40 layers and a batch of 256
    need_tokens = int(args.max_batch * 700 * 1.3)
    enc_batch = 32
    cfg = exe.config_from_shape(shape, kv_pool_bytes=need_tokens * kv_tok, max_seqs=args.max_batch,
                                max_batch_tokens=enc_batch * 1024, max_batch_seqs=max(args.max_batch, enc_batch))
    m = exe.Model(cfg, weights, stream=torch.cuda.Stream())
    t0 = time.perf_counter()
    rows = m.profile(0, [1, 2, 4, 8, 16, 32], [128, 512, 1024], n_steps=args.steps)
    rows += m.profile(1, [1, 8, 32, 64, 128, 192, 256], [256, 640, 1024], n_steps=args.steps)
    print(f"[schedule] profiled {len(rows)} table rows in {time.perf_counter() - t0:.1f} s", file=sys.stderr, flush=True)
    table = exe.make_sim_table(rows, shape.n_layers, shape.n_layers)
    p_in = wl.clipped_normal_pmf(512, 128, 64, 1024)
    p_out = wl.clipped_normal_pmf(128, 32, 16, 256)
    latency_len = 200
    results = []
    for bound_s in [float(x) for x in args.bounds.split(",")]:
        bound_ms = bound_s * 1e3 if bound_s > 0 else 1e12
        plan = exe.exe_sched_rra(table, p_in, p_out, (8, args.max_batch), (4, 64), latency_len, bound_ms,
                                 eps_throughput=100.0, eps_latency_ms=50.0)
        if not plan["search"]["found"]:
            results.append({"latency_bound_s": bound_s, "found": False, "evaluations": plan["search"]["evaluations"]})
            continue
        bd, nd, sim = plan["decode_batch"], plan["n_decode"], plan["sim"]
        _, st = m.run_rra(bd, nd, job.in_len, job.out_len, job.tokens, max_encode_batch=enc_batch)
        results.append({
            "latency_bound_s": bound_s, "found": True, "decode_batch": bd, "n_decode": nd,
            "evaluations": plan["search"]["evaluations"], "grid_points": (args.max_batch - 7) * 61,
            "sim_encode_batch": round(sim["b_e"], 2), "sim_generated_tok_s": round(sim["throughput_tok_s"], 1),
            "sim_latency_200_s": round(sim["latency_ms"] / 1e3, 3),
            "run_generated_tok_s": round(st["generated_tokens"] / st["wall_s"], 1),
            "run_sequences_s": round(job.n / st["wall_s"], 2), "run_mean_decode_batch": round(st["mean_decode_batch"], 1),
            "run_latency_p50_s": round(st["latency_p50_s"], 3), "run_latency_p99_s": round(st["latency_p99_s"], 3),
            "run_latency_max_s": round(st["latency_max_s"], 3),
        })
        print(f"[schedule] bound {bound_s} s: B_D {bd} N_D {nd}: simulated {sim['throughput_tok_s']:.0f} tok/s, "
              f"ran {st['generated_tokens'] / st['wall_s']:.0f} tok/s", file=sys.stderr, flush=True)
    if args.markdown:
        print("| latency bound (200 tokens) | B_D | N_D | points evaluated / grid | simulated tok/s | measured tok/s | "
              "simulated latency s | measured latency p50 / p99 / max s | mean decode batch |")
        print("|---|---:|---:|---:|---:|---:|---:|---:|---:|")
        for r in results:
            if not r["found"]:
                print(f"| {r['latency_bound_s']} s | - | - | {r['evaluations']} | no configuration meets the bound | | | | |")
                continue
            print(f"| {r['latency_bound_s'] or 'none'} s | {r['decode_batch']} | {r['n_decode']} | {r['evaluations']} / {r['grid_points']} | "
                  f"{r['sim_generated_tok_s']} | {r['run_generated_tok_s']} | {r['sim_latency_200_s']} | "
                  f"{r['run_latency_p50_s']} / {r['run_latency_p99_s']} / {r['run_latency_max_s']} | {r['run_mean_decode_batch']} |")
    else:
        for r in results:
            print(json.dumps(r))
    m.close()


if __name__ == "__main__":
    main()
