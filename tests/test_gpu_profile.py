"""exe_profile: the latency-vs-batch table (attention vs rest of layer) through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2404_07947_amd as exe
import workload as wl
from gpu_util import DEV, kv_bytes_per_token

pytestmark = pytest.mark.gpu


def make_model(shape, pool_tokens, max_batch_tokens=8192, max_batch_seqs=64):
    w = [t.to(DEV) for t in wl.make_weights(shape, 31)]
    cfg = exe.config_from_shape(shape, kv_pool_bytes=pool_tokens * kv_bytes_per_token(shape), max_seqs=16,
                                max_batch_tokens=max_batch_tokens, max_batch_seqs=max_batch_seqs)
    return exe.Model(cfg, w)


def test_profile_table_decoder_only():
    shape = wl.tiny_shape().replace(name="prof", dtype=wl.DTYPE_BF16, d_model=1024, n_heads=8, head_dim=128,
                                    d_ff=4096, max_pos=4096, n_layers=2)
    m = make_model(shape, pool_tokens=64 * 1100)
    dec = m.profile(1, [1, 8, 64], [128, 2048], n_steps=5)
    assert [(r["batch"], r["length"]) for r in dec] == [(1, 128), (1, 2048), (8, 128), (8, 2048), (64, 128), (64, 2048)]
    for r in dec:
        assert r["phase"] == 1 and r["ragged"] == 0 and r["n_timed"] == 5
        assert r["total_tokens"] == r["batch"] * r["length"]
        assert r["attn_ms_per_layer"] > 0 and r["rest_ms_per_layer"] > 0 and r["head_ms"] > 0
        layer = r["attn_ms_per_layer"] + r["rest_ms_per_layer"]
        assert abs(r["full_step_ms"] - (shape.n_layers * layer + r["head_ms"])) < 1e-3 * r["full_step_ms"] + 1e-4
    # 16x the K/V bytes must cost more attention time at the largest batch
    assert dec[5]["attn_ms_per_layer"] > 2 * dec[4]["attn_ms_per_layer"]
    enc = m.profile(0, [1, 4], [256, 1024], n_steps=3)
    assert len(enc) == 4 and all(r["phase"] == 0 for r in enc)
    assert enc[3]["attn_ms_per_layer"] > enc[2]["attn_ms_per_layer"]         # quadratic in length
    assert enc[3]["rest_ms_per_layer"] > enc[0]["rest_ms_per_layer"]         # 16x the tokens
    # ragged rows: deterministic in the seed, total within the clip range
    dist = exe.binding.LengthDist(1, 0.0, 256.0, 64, 2048, 7)
    r1 = m.profile(1, [32], [1024], dist=dist, n_steps=2)
    r2 = m.profile(1, [32], [1024], dist=dist, n_steps=2)
    assert r1[0]["ragged"] == 1 and r1[0]["total_tokens"] == r2[0]["total_tokens"]
    assert 32 * 64 <= r1[0]["total_tokens"] <= 32 * 2048 and r1[0]["total_tokens"] != 32 * 1024
    # the pool is returned, and the model still works
    assert m.kv_stats()["used_bytes"] == 0
    t = m.encode([0], [5], [1, 2, 3, 4, 5])
    with pytest.raises(exe.ExeError) as e:
        m.profile(1, [1], [16], n_steps=1)                     # a live sequence
    assert e.value.code == -4
    m.seq_release([0])
    with pytest.raises(exe.ExeError) as e:
        m.profile(1, [64], [4096], n_steps=1)                  # one layer of this row does not fit the pool
    assert e.value.code == -3 and m.kv_stats()["used_bytes"] == 0
    with pytest.raises(exe.ExeError) as e:
        m.profile(0, [64], [1024], n_steps=1)                  # more tokens than the workspace
    assert e.value.code == -1
    m.close()


def test_profile_table_encoder_decoder():
    shape = wl.small_t5_shape(wl.DTYPE_BF16).replace(head_dim=128, n_heads=4, d_model=512, d_ff=1024)
    m = make_model(shape, pool_tokens=16 * 4096)
    dec = m.profile(1, [4, 16], [256, 1024], n_steps=3)
    assert len(dec) == 4 and all(r["attn_ms_per_layer"] > 0 and r["rest_ms_per_layer"] > 0 for r in dec)
    enc = m.profile(0, [2], [512], n_steps=3)
    assert enc[0]["head_ms"] > 0 and enc[0]["attn_ms_per_layer"] > 0
    assert m.kv_stats()["used_bytes"] == 0
    m.close()
