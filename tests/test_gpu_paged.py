"""Paged K/V pool (exe_config_t.kv_block_size > 0; Section 2: paging applied to the key/value memorization cache).
The same parity bar as the extent pool: logits and greedy tokens against the oracle; plus what paging is for: a
sequence takes blocks as it grows, released blocks serve other sequences at once, admission is all or nothing, and
the hand-over format does not depend on which pool either side uses."""
import numpy as np
import pytest

import paper_2404_07947_amd as exe
import workload as wl
from gpu_util import kv_bytes_per_token, make_pair
from test_gpu_model import BF16_TOL, F32_TOL, run_decoder_only

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block", [8, 64])
def test_tiny_config_logits_and_tokens_paged(block):
    job = wl.workload_tiny()
    run_decoder_only(wl.tiny_shape(), wl.BASE_SEED, job.in_len, 16, F32_TOL, check_tokens=True, kv_block_size=block)


def test_small_bf16_ragged_with_release_paged():
    shape = wl.tiny_shape().replace(name="small_bf16", dtype=wl.DTYPE_BF16, max_pos=512, n_layers=3)
    run_decoder_only(shape, 5, [1, 37, 128, 129, 300, 64], 6, BF16_TOL, release_at={3: [1, 4], 5: [0]}, kv_block_size=16)


def test_small_bf16_head128_paged():
    shape = wl.tiny_shape().replace(name="small_bf16_h128", dtype=wl.DTYPE_BF16, max_pos=512, head_dim=128,
                                    n_heads=2, act=wl.ACT_RELU)
    run_decoder_only(shape, 6, [5, 200, 131], 4, BF16_TOL, kv_block_size=64)


def test_opt13b_width_two_layers_paged():
    run_decoder_only(wl.opt13b_shape(2), 7, [40, 7, 65], 2, BF16_TOL, real="float", kv_block_size=64)


def oracle_tokens(o, toks, steps):
    t, _ = o.encode(0, toks)
    seq = [t]
    for _ in range(steps):
        t, _ = o.decode(0, t)
        seq.append(t)
    o.release(0)
    return seq


def test_blocks_are_taken_as_sequences_grow_and_reused_after_release():
    shape = wl.tiny_shape()
    block = 8
    m, o, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=128, max_seqs=8, max_batch_tokens=256, max_batch_seqs=8,
                        kv_block_size=block)
    per_block = block * kv_bytes_per_token(shape)
    st = m.kv_stats()
    assert st["pool_bytes"] == 16 * per_block and st["used_bytes"] == 0
    rng = np.random.default_rng(51)
    in_len = np.array([5, 8, 9, 20], dtype=np.int32)             # 1 + 1 + 2 + 3 = 7 blocks
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    off = np.concatenate([[0], np.cumsum(in_len)])
    steps = 10
    want = [oracle_tokens(o, toks[off[i]:off[i + 1]], steps) for i in range(4)]
    ids = np.arange(4)
    cur = m.encode(ids, in_len, toks)
    assert m.kv_stats()["used_bytes"] == 7 * per_block
    got = [[int(t)] for t in cur]
    for s in range(1, steps + 1):
        cur = m.decode_step(ids, cur, in_len + s)
        for i in range(4):
            got[i].append(int(cur[i]))
        blocks = sum((int(L) + s + block - 1) // block for L in in_len)
        assert m.kv_stats()["used_bytes"] == blocks * per_block    # exactly the blocks the lengths need
    assert got == want
    # 16 blocks in all: a request that does not fit is refused whole, one that fits after a release is admitted
    used = m.kv_stats()["used_bytes"] // per_block
    big = int((16 - used) * block + 1)
    btoks = wl.random_tokens(rng, big + 3, shape.vocab)
    with pytest.raises(exe.ExeError) as e:
        m.encode([4, 5], [3, big], btoks)
    assert e.value.code == -3 and m.kv_stats()["used_bytes"] == used * per_block and m.kv_stats()["live_seqs"] == 4
    m.seq_release([3])
    m.encode([4, 5], [3, big], btoks)
    assert m.kv_stats()["live_seqs"] == 5
    # the pool is full now or nearly: a decode step that needs more blocks than are free changes nothing
    st = m.kv_stats()
    free_blocks = (st["pool_bytes"] - st["used_bytes"]) // per_block
    lens = {i: m.seq_length(i) for i in [0, 1, 2, 4, 5]}
    need = [i for i in lens if lens[i] % block == 0]
    if len(need) > free_blocks:
        with pytest.raises(exe.ExeError) as e:
            m.decode_step(list(lens), [1] * len(lens), [lens[i] + 1 for i in lens])
        assert e.value.code == -3 and m.kv_stats() == st and all(m.seq_length(i) == lens[i] for i in lens)
    # reserve ahead / give back
    m.seq_release([4, 5])
    before = m.kv_stats()["used_bytes"]
    m.seq_reserve(0, m.seq_length(0) + 3 * block)
    assert m.kv_stats()["used_bytes"] == before + 3 * per_block
    m.seq_reserve(0, m.seq_length(0))
    assert m.kv_stats()["used_bytes"] == before
    assert m.kv_compact() == 0
    m.close()


@pytest.mark.parametrize("src_block,dst_block", [(8, 0), (0, 16), (16, 8)])
def test_hand_over_between_pools_of_different_kinds(src_block, dst_block):
    shape = wl.tiny_shape()
    a, o, wd = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=1024, max_seqs=8, max_batch_tokens=512, max_batch_seqs=8,
                         kv_block_size=src_block)
    cfg = exe.config_from_shape(shape, kv_pool_bytes=1024 * kv_bytes_per_token(shape), max_seqs=8, max_batch_tokens=512,
                                max_batch_seqs=8, kv_block_size=dst_block)
    b = exe.Model(cfg, wd)
    rng = np.random.default_rng(52)
    L, steps_a, steps_total = 21, 4, 11
    toks = wl.random_tokens(rng, L, shape.vocab)
    want = oracle_tokens(o, toks, steps_total)
    cur = a.encode([2], [L], toks)
    got = [int(cur[0])]
    for s in range(1, steps_a + 1):
        cur = a.decode_step([2], cur, [L + s])
        got.append(int(cur[0]))
    buf, st = a.seq_export(2)
    assert st == {"kv_len": L + steps_a, "cross_len": 0} and buf.nbytes == kv_bytes_per_token(shape) * st["kv_len"]
    b.seq_import(5, buf, st, reserve_length=L + steps_total + 1)
    buf2, st2 = b.seq_export(5)
    assert st2 == st and np.array_equal(buf, buf2)
    for s in range(steps_a + 1, steps_total + 1):
        cur = b.decode_step([5], cur, [L + s])
        got.append(int(cur[0]))
    assert got == want
    a.close(); b.close()


def test_rra_schedule_on_a_paged_pool_gives_the_same_tokens():
    shape = wl.tiny_shape()
    rng = np.random.default_rng(5)
    n = 13
    in_len = wl.uniform_lengths(rng, n, 4, 24)
    out_len = rng.integers(1, 9, size=n).astype(np.int32)
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    res = []
    for block in (0, 8):
        m, _, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=2048, max_seqs=16, max_batch_tokens=256, max_batch_seqs=8,
                            kv_block_size=block)
        got, st = m.run_rra(4, 3, in_len, out_len, toks, max_encode_batch=4)
        assert m.kv_stats()["used_bytes"] == 0 and m.kv_stats()["live_seqs"] == 0
        res.append((got.tolist(), st["decode_iterations"], st["encode_phases"]))
        m.close()
    assert res[0] == res[1]            # (the extent run is checked against the oracle in test_gpu_rra.py)


def test_profile_on_a_paged_model():
    # exe_profile times a single layer on an empty pool; a paged model lends it the same memory
    shape = wl.tiny_shape()
    m, _, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=4096, max_seqs=16, max_batch_tokens=1024, max_batch_seqs=16,
                        kv_block_size=16)
    rows = m.profile(1, [2, 4], [16, 32], n_steps=3)
    assert len(rows) == 4 and all(r["full_step_ms"] > 0 for r in rows)
    assert m.kv_stats()["used_bytes"] == 0
    m.close()


def test_paged_pool_configuration_errors():
    shape = wl.tiny_shape()
    w = wl.make_weights(shape, wl.BASE_SEED)
    from gpu_util import DEV
    wd = [t.to(DEV) for t in w]
    for bad in (3, 12, 8192):
        cfg = exe.config_from_shape(shape, kv_pool_bytes=1 << 20, max_seqs=4, max_batch_tokens=64, max_batch_seqs=4, kv_block_size=bad)
        with pytest.raises(exe.ExeError) as e:
            exe.Model(cfg, wd)
        assert e.value.code == -1
    t5 = wl.small_t5_shape(wl.DTYPE_BF16)
    wt = [t.to(DEV) for t in wl.make_weights(t5, wl.BASE_SEED)]
    cfg = exe.config_from_shape(t5, kv_pool_bytes=1 << 24, max_seqs=4, max_batch_tokens=64, max_batch_seqs=4, kv_block_size=16)
    with pytest.raises(exe.ExeError) as e:
        exe.Model(cfg, wt)
    assert e.value.code == -7
