"""Latency-profile sweep (configs[4]): exe_profile over encode batches at a fixed input length and decode
batches x K/V lengths, uniform and ragged, at the OPT-13B shape.  Prints the table a scheduler consumes
(per-layer attention / rest-of-layer latency, head, extrapolated full step) as JSON lines or Markdown.

    python -m paper_2404_07947_amd.profile_sweep [--markdown] [--steps 20] [--shape opt13b|gpt3_share]

--shape gpt3_share profiles one layer of configs[3] (d 12288, 96 heads, FFN 49152; hidden states in and out, so no
head) at its decode batch of 512, whose full-depth K/V does not fit one GPU: one layer's does.
"""
import argparse
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--markdown", action="store_true")
    ap.add_argument("--shape", choices=["opt13b", "gpt3_share"], default="opt13b")
    args = ap.parse_args()
    import torch
    import paper_2404_07947_amd as exe
    from paper_2404_07947_amd.binding import LengthDist
    import workload as wl

    rows = []
    if args.shape == "opt13b":
        shape = wl.opt13b_shape(1)                  # the profiler runs a single layer; weights of one layer suffice
        weights = wl.make_weights(shape, wl.BASE_SEED + 4, device="cuda:0")
        kv_tok = 2 * shape.inner * 2
        cfg = exe.config_from_shape(shape, kv_pool_bytes=1024 * 2056 * kv_tok + (1 << 20), max_seqs=8,
                                    max_batch_tokens=32 * 512, max_batch_seqs=1024)
        m = exe.Model(cfg, weights)
        rows += m.profile(0, [1, 2, 4, 8, 16, 32], [512], n_steps=args.steps)
        rows += m.profile(1, [1, 8, 32, 128, 512, 1024], [256, 1024, 2048], n_steps=args.steps)
        rows += m.profile(1, [1, 8, 32, 128, 512, 1024], [1024], dist=LengthDist(1, 0.0, 256.0, 64, 2048, 20240431),
                          n_steps=args.steps)
        depth = 40
    else:
        shape = wl.gpt3_175b_share_shape(1)
        weights = wl.make_weights(shape, wl.BASE_SEED + 5, device="cuda:0")
        kv_tok = 2 * shape.inner * 2
        cfg = exe.config_from_shape(shape, kv_pool_bytes=512 * 2568 * kv_tok + (1 << 20), max_seqs=8,
                                    max_batch_tokens=8 * 2048, max_batch_seqs=512)
        m = exe.Model(cfg, weights)
        rows += m.profile(0, [1, 2, 4, 8], [1024, 2048], n_steps=args.steps)
        rows += m.profile(1, [64, 128, 256, 320, 512], [1152, 2048, 2560], n_steps=args.steps)
        rows += m.profile(1, [512], [1280], dist=LengthDist(1, 0.0, 264.0, 160, 2560, 20240432), n_steps=args.steps)
        depth = 12
    for r in rows:
        r[f"full_step_ms_{depth}_layers"] = depth * (r["attn_ms_per_layer"] + r["rest_ms_per_layer"]) + r["head_ms"]
    if args.markdown:
        print(f"| phase | batch | length | ragged | tokens | attn ms/layer | rest ms/layer | head ms | std ms | {depth}-layer step ms |")
        print("|---|---:|---:|---:|---:|---:|---:|---:|---:|---:|")
        for r in rows:
            print(f"| {'encode' if r['phase'] == 0 else 'decode'} | {r['batch']} | {r['length']} | {r['ragged']} | "
                  f"{r['total_tokens']} | {r['attn_ms_per_layer']:.4f} | {r['rest_ms_per_layer']:.4f} | {r['head_ms']:.4f} | "
                  f"{r['std_ms']:.4f} | {r[f'full_step_ms_{depth}_layers']:.2f} |")
    else:
        for r in rows:
            print(json.dumps(r))
    m.close()


if __name__ == "__main__":
    main()
