"""Extent relocation and compaction (exe_seq_reserve / exe_kv_compact; Section 3 "XRunner": early termination
comes with the compaction of the key/value cache entries of terminated queries).  Moving a sequence's entries must
not change anything a caller can observe: the tokens stay the oracle's greedy tokens, the exported bytes stay the
same, and the pool's free space becomes one piece."""
import numpy as np
import pytest

import paper_2404_07947_amd as exe
import workload as wl
from gpu_util import kv_bytes_per_token, make_pair

pytestmark = pytest.mark.gpu


def oracle_tokens(o, toks, off, i, steps):
    t, _ = o.encode(0, toks[off[i]:off[i + 1]])
    seq = [t]
    for _ in range(steps):
        t, _ = o.decode(0, t)
        seq.append(t)
    o.release(0)
    return seq


def test_reserve_lets_a_sequence_outgrow_its_first_extent():
    shape = wl.tiny_shape()
    m, o, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=2048, max_seqs=16, max_batch_tokens=1024, max_batch_seqs=16)
    rng = np.random.default_rng(31)
    n, steps_total = 5, 12
    in_len = wl.uniform_lengths(rng, n, 3, 30)
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    off = np.concatenate([[0], np.cumsum(in_len)])
    want = [oracle_tokens(o, toks, off, i, steps_total) for i in range(n)]
    ids = np.arange(n)
    tight = (in_len + 7) // 8 * 8                           # capacities are multiples of 8: no room beyond this
    cur = m.encode(ids, in_len, toks, reserve_lengths=tight)
    got = [[int(t)] for t in cur]
    step = 0
    grown = False
    while step < steps_total:
        step += 1
        try:
            nxt = m.decode_step(ids, cur, in_len + step)
        except exe.ExeError as e:
            assert e.code == -3 and not grown               # a reservation is exhausted: nothing was decoded
            before = [m.seq_export(int(i)) for i in ids]
            for i in ids:
                m.seq_reserve(int(i), int(in_len[i]) + steps_total + 1)
            after = [m.seq_export(int(i)) for i in ids]
            for (b0, s0), (b1, s1) in zip(before, after):
                assert s0 == s1 and np.array_equal(b0, b1)  # the entries moved unchanged
            grown = True
            step -= 1
            continue
        cur = nxt
        for i in range(n):
            got[i].append(int(cur[i]))
    assert grown and got == want
    # shrinking returns capacity
    used = m.kv_stats()["used_bytes"]
    m.seq_reserve(0, int(in_len[0]) + steps_total)
    assert m.kv_stats()["used_bytes"] <= used
    m.close()


@pytest.mark.parametrize("arch", ["decoder_only", "encoder_decoder"])
def test_compaction_keeps_tokens_and_joins_the_free_space(arch):
    encdec = arch == "encoder_decoder"
    shape = wl.small_t5_shape(wl.DTYPE_BF16) if encdec else wl.tiny_shape()
    m, o, _ = make_pair(shape, wl.BASE_SEED + (3 if encdec else 0), "float", pool_tokens=4096, max_seqs=16,
                        max_batch_tokens=1024, max_batch_seqs=16)
    rng = np.random.default_rng(32)
    n, steps_a, steps_total = 8, 3, 9
    in_len = wl.uniform_lengths(rng, n, 4, 48)
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    ids = np.arange(n)
    start = np.zeros(n, dtype=np.int32)

    def run(model, compact):
        if encdec:
            model.encode(ids, in_len, toks, want_tokens=False)
            cur, out = start.copy(), [[] for _ in range(n)]
            base = np.zeros(n, dtype=np.int32)
        else:
            cur = model.encode(ids, in_len, toks)
            out = [[int(t)] for t in cur]
            base = in_len
        live = list(range(n))
        for s in range(1, steps_total + 1):
            nxt = model.decode_step(ids[live], cur, base[live] + s)
            for k, i in enumerate(live):
                out[i].append(int(nxt[k]))
            cur = nxt
            if s == steps_a:
                gone = [i for i in live if i % 2 == 1]      # every other sequence terminates early: holes
                model.seq_release(gone)
                keep = [k for k, i in enumerate(live) if i % 2 == 0]
                live = [live[k] for k in keep]
                cur = cur[keep]
                if compact:
                    st0 = model.kv_stats()
                    exported = [model.seq_export(i) for i in live]
                    moved = model.kv_compact()
                    st1 = model.kv_stats()
                    assert moved > 0 and st1["used_bytes"] == st0["used_bytes"] and st1["live_seqs"] == st0["live_seqs"]
                    assert st0["largest_free_bytes"] < st0["pool_bytes"] - st0["used_bytes"]
                    assert st1["largest_free_bytes"] == st1["pool_bytes"] - st1["used_bytes"]
                    for i, (b0, s0) in zip(live, exported):
                        b1, s1 = model.seq_export(i)
                        assert s0 == s1 and np.array_equal(b0, b1)
                    assert model.kv_compact() == 0            # nothing left to move
        return out

    got = run(m, True)
    if encdec:
        # same kernels on the same entries: the run without compaction is the reference
        m.seq_release([i for i in range(n) if i % 2 == 0])
        ref = run(m, False)
        assert got == ref
    else:
        off = np.concatenate([[0], np.cumsum(in_len)])
        for i in range(n):
            want = oracle_tokens(o, toks, off, i, steps_total)
            assert got[i] == want[:len(got[i])]
    m.close()


def test_relocation_errors_change_nothing():
    shape = wl.tiny_shape()
    m, _, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=96, max_seqs=4, max_batch_tokens=256, max_batch_seqs=4)
    toks = wl.random_tokens(np.random.default_rng(1), 30, shape.vocab)
    m.encode([0], [30], toks, reserve_lengths=[40])
    before = m.kv_stats()
    for call, code in [(lambda: m.seq_reserve(1, 40), -4), (lambda: m.seq_reserve(9, 40), -4),
                       (lambda: m.seq_reserve(0, 29), -5),                               # below the current length
                       (lambda: m.seq_reserve(0, 65), -5),                               # beyond the position table (64)
                       (lambda: m.seq_reserve(0, 64), -3)]:                              # 40 + 64 > 96 positions
        with pytest.raises(exe.ExeError) as e:
            call()
        assert e.value.code == code
        assert m.kv_stats() == before and m.seq_length(0) == 30
    m.seq_reserve(0, 48)                                                                 # fits beside the old extent
    assert m.kv_stats()["used_bytes"] == 48 * kv_bytes_per_token(shape)
    m.close()


@pytest.mark.parametrize("first_reserve,moves", [(32, True), (8, False)])
def test_compaction_moves_an_extent_over_itself_in_pieces_or_leaves_it(first_reserve, moves):
    # a long extent behind a short released one: the move overlaps its own source and goes in 1024 / 32 = 32 pieces;
    # behind an extent of 8 positions it would take 128 pieces, more than the limit of 64, and the extent stays
    shape = wl.tiny_shape().replace(name="tiny_long", max_pos=1024)
    m, o, _ = make_pair(shape, wl.BASE_SEED + 9, "float", pool_tokens=2048, max_seqs=8, max_batch_tokens=256, max_batch_seqs=8)
    rng = np.random.default_rng(33)
    L = 40
    toks = wl.random_tokens(rng, 5 + L, shape.vocab)
    steps = 6
    t, _ = o.encode(0, toks[5:])
    want = [t]
    for _ in range(steps):
        t, _ = o.decode(0, t)
        want.append(t)
    m.encode([0], [5], toks[:5], reserve_lengths=[first_reserve])
    cur = m.encode([1], [L], toks[5:], reserve_lengths=[1024])
    got = [int(cur[0])]
    for s in range(1, 4):
        cur = m.decode_step([1], cur, [L + s])
        got.append(int(cur[0]))
    m.seq_release([0])
    buf0, st0 = m.seq_export(1)
    moved = m.kv_compact()
    st = m.kv_stats()
    if moves:
        assert moved == 1024 * kv_bytes_per_token(shape)
        assert st["largest_free_bytes"] == st["pool_bytes"] - st["used_bytes"]
    else:
        assert moved == 0 and st["largest_free_bytes"] < st["pool_bytes"] - st["used_bytes"]
    buf1, st1 = m.seq_export(1)
    assert st0 == st1 and np.array_equal(buf0, buf1)
    for s in range(4, steps + 1):
        cur = m.decode_step([1], cur, [L + s])
        got.append(int(cur[0]))
    assert got == want
    # the free list is consistent: a sequence that needs the whole remainder is admitted exactly when it is one piece
    free_tokens = (st["pool_bytes"] - st["used_bytes"]) // kv_bytes_per_token(shape)
    t2 = wl.random_tokens(rng, 3, shape.vocab)
    if moves:
        m.encode([2], [3], t2, reserve_lengths=[int(free_tokens)])
        assert m.kv_stats()["used_bytes"] == st["pool_bytes"]
    else:
        with pytest.raises(exe.ExeError) as e:
            m.encode([2], [3], t2, reserve_lengths=[int(free_tokens)])
        assert e.value.code == -3
    m.close()
