"""K/V hand-over (exe_seq_export / exe_seq_import; Section 3 "XRunner", WAA scheduling): a sequence encoded and partly
decoded by one model instance continues on another one after its key/value entries went through host memory.
The tokens must be the oracle's greedy tokens of that sequence, the exported bytes must survive the round trip
unchanged, and failures must leave the importing model as it was."""
import numpy as np
import pytest

import paper_2404_07947_amd as exe
import workload as wl
from gpu_util import DEV, kv_bytes_per_token, make_pair

pytestmark = pytest.mark.gpu


def second_model(shape, weights_dev, pool_tokens=4096, max_seqs=16):
    cfg = exe.config_from_shape(shape, kv_pool_bytes=pool_tokens * kv_bytes_per_token(shape), max_seqs=max_seqs,
                                max_batch_tokens=1024, max_batch_seqs=16)
    return exe.Model(cfg, weights_dev)


def test_decoder_only_hand_over_matches_oracle_tokens():
    shape = wl.tiny_shape()
    a, o, wd = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=4096, max_seqs=16, max_batch_tokens=1024, max_batch_seqs=16)
    b = second_model(shape, wd)
    rng = np.random.default_rng(21)
    n, steps_a, steps_total = 5, 3, 9
    in_len = wl.uniform_lengths(rng, n, 3, 40)
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    off = np.concatenate([[0], np.cumsum(in_len)])
    want = []
    for i in range(n):                                   # the oracle: every sequence on its own, no hand-over
        t, _ = o.encode(0, toks[off[i]:off[i + 1]])
        seq = [t]
        for _ in range(steps_total):
            t, _ = o.decode(0, t)
            seq.append(t)
        o.release(0)
        want.append(seq)
    ids = np.arange(n)
    cur = a.encode(ids, in_len, toks)
    got = [[int(t)] for t in cur]
    for s in range(1, steps_a + 1):
        cur = a.decode_step(ids, cur, in_len + s)
        for i in range(n):
            got[i].append(int(cur[i]))
    moved, new_ids = [1, 3], [7, 2]
    for i, j in zip(moved, new_ids):
        buf, st = a.seq_export(i)
        assert st == {"kv_len": int(in_len[i]) + steps_a, "cross_len": 0}
        assert buf.nbytes == kv_bytes_per_token(shape) * st["kv_len"]
        b.seq_import(j, buf, st, reserve_length=int(in_len[i]) + steps_total + 1)
        buf2, st2 = b.seq_export(j)
        assert st2 == st and np.array_equal(buf, buf2)             # byte-exact round trip
        assert b.seq_length(j) == st["kv_len"]
    a.seq_release(moved)
    stay = [i for i in range(n) if i not in moved]
    cur_a, cur_b = cur[stay], cur[moved]
    for s in range(steps_a + 1, steps_total + 1):
        cur_a = a.decode_step(stay, cur_a, in_len[stay] + s)
        cur_b = b.decode_step(new_ids, cur_b, in_len[moved] + s)
        for k, i in enumerate(stay):
            got[i].append(int(cur_a[k]))
        for k, i in enumerate(moved):
            got[i].append(int(cur_b[k]))
    assert got == want
    assert b.kv_stats()["live_seqs"] == 2 and a.kv_stats()["live_seqs"] == 3
    a.close(); b.close()


def test_encoder_decoder_hand_over_right_after_encoding():
    # the WAA case proper: the encoding side never decodes; cross K/V entries travel, self-attention entries are empty
    shape = wl.small_t5_shape(wl.DTYPE_BF16)
    a, _, wd = make_pair(shape, wl.BASE_SEED + 3, "float", pool_tokens=4096, max_seqs=16, max_batch_tokens=1024, max_batch_seqs=16)
    b = second_model(shape, wd)
    rng = np.random.default_rng(22)
    in_len = np.array([17, 64, 5], dtype=np.int32)
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    a.encode([0, 1, 2], in_len, toks, want_tokens=False)
    for i in range(3):
        buf, st = a.seq_export(i)
        assert st == {"kv_len": 0, "cross_len": int(in_len[i])}
        b.seq_import(i + 4, buf, st)
    steps = 12
    ref, got = [], []
    cur_a = np.zeros(3, dtype=np.int32)
    cur_b = np.zeros(3, dtype=np.int32)
    for s in range(1, steps + 1):
        cur_a = a.decode_step([0, 1, 2], cur_a, np.full(3, s))
        cur_b = b.decode_step([4, 5, 6], cur_b, np.full(3, s))
        ref.append(cur_a.tolist()); got.append(cur_b.tolist())
    assert got == ref                                     # same kernels on the same entries: the same tokens
    buf_a, st_a = a.seq_export(1)
    buf_b, st_b = b.seq_export(5)
    assert st_a == st_b == {"kv_len": steps, "cross_len": 64} and np.array_equal(buf_a, buf_b)
    a.close(); b.close()


def test_hand_over_errors_change_nothing():
    shape = wl.tiny_shape()
    a, _, wd = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=96, max_seqs=4, max_batch_tokens=256, max_batch_seqs=4)
    toks = wl.random_tokens(np.random.default_rng(1), 30, shape.vocab)
    a.encode([0], [30], toks, reserve_lengths=[64])          # 64 of the pool's 96 positions
    buf, st = a.seq_export(0)
    before = a.kv_stats()
    for call, code in [(lambda: a.seq_export(1), -4), (lambda: a.seq_export(9), -4),
                       (lambda: a.seq_import(0, buf, st), -4),                          # id is live
                       (lambda: a.seq_import(1, buf[:-1], st), -1),                     # buffer too small
                       (lambda: a.seq_import(1, buf, {"kv_len": 0, "cross_len": 0}), -5),
                       (lambda: a.seq_import(1, buf, {"kv_len": 30, "cross_len": 4}), -5),
                       (lambda: a.seq_import(1, buf, st, reserve_length=8), -5),
                       (lambda: a.seq_import(1, buf, st, reserve_length=40), -3)]:      # 32 positions left
        with pytest.raises(exe.ExeError) as e:
            call()
        assert e.value.code == code
    assert a.kv_stats() == before
    a.seq_import(1, buf, st, reserve_length=32)
    assert a.kv_stats()["live_seqs"] == 2 and a.kv_stats()["used_bytes"] == a.kv_stats()["pool_bytes"]
    a.close()
