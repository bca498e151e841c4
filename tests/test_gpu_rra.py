"""exe_run_rra: the RRA schedule (encode once, N_D decode iterations, refill with as many queries as completed)
on one GPU.  Sequences are independent, so every request's tokens must equal the oracle's greedy decoding of
that request alone; the schedule's counters must equal an independent simulation written from the paper's
description (Section 4, "RRA Scheduling")."""
import numpy as np
import pytest

import paper_2404_07947_amd as exe
import workload as wl
from gpu_util import make_pair

pytestmark = pytest.mark.gpu


def simulate_rra(in_len, out_len, BD, ND):
    """Counters of the schedule: the first encoding phase fills the decode batch; every later one admits as many
    queries as completed since the previous one; a query produces one token at its encoding (decoder-only)
    and one per decode iteration, and leaves when it has produced its forced output length."""
    n = len(in_len)
    nxt, live, finished = 0, {}, 0
    completed = BD
    phases = iters = batch_sum = gen = 0
    slot = 0
    while finished < n:
        want = min(completed, BD - len(live), n - nxt)
        if want > 0:
            phases += 1
        completed = 0
        for _ in range(want):
            gen += 1
            if out_len[nxt] == 1:
                finished += 1
                completed += 1
            else:
                live[slot] = [nxt, 1]
                slot += 1
            nxt += 1
        if not live:
            if nxt >= n:
                break
            completed = BD
            continue
        for _ in range(ND):
            if not live:
                break
            iters += 1
            batch_sum += len(live)
            for s in list(live):
                live[s][1] += 1
                gen += 1
                if live[s][1] >= out_len[live[s][0]]:
                    del live[s]
                    finished += 1
                    completed += 1
    return phases, iters, batch_sum / max(iters, 1), gen


@pytest.mark.parametrize("BD,ND,max_enc", [(4, 3, 4), (3, 1, 2), (8, 16, 3)])
def test_rra_tokens_and_counters(BD, ND, max_enc):
    shape = wl.tiny_shape()
    m, o, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=2048, max_seqs=16, max_batch_tokens=256, max_batch_seqs=8)
    rng = np.random.default_rng(5)
    n = 13
    in_len = wl.uniform_lengths(rng, n, 4, 24)
    out_len = rng.integers(1, 9, size=n).astype(np.int32)
    out_len[3] = 1                                        # finishes at its encoding
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    got, st = m.run_rra(BD, ND, in_len, out_len, toks, max_encode_batch=max_enc)
    off = np.concatenate([[0], np.cumsum(in_len)])
    want = []
    for i in range(n):
        t, _ = o.encode(0, toks[off[i]:off[i + 1]])
        seq = [t]
        for _ in range(out_len[i] - 1):
            t, _ = o.decode(0, t)
            seq.append(t)
        o.release(0)
        want += seq
    assert got.tolist() == want
    phases, iters, mean_b, gen = simulate_rra(in_len, out_len, BD, ND)
    assert st["generated_tokens"] == gen == int(out_len.sum())
    assert st["encoded_tokens"] == int(in_len.sum())
    assert st["encode_phases"] == phases and st["decode_iterations"] == iters
    assert abs(st["mean_decode_batch"] - mean_b) < 1e-9
    assert st["encode_calls"] >= phases
    assert 0 < st["latency_p50_s"] <= st["latency_p99_s"] <= st["latency_max_s"] <= st["wall_s"]
    assert m.kv_stats()["used_bytes"] == 0 and m.kv_stats()["live_seqs"] == 0
    m.close()


def test_rra_workload_adjustment_and_errors():
    shape = wl.tiny_shape()
    m, o, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=2048, max_seqs=16, max_batch_tokens=256, max_batch_seqs=8)
    rng = np.random.default_rng(6)
    n = 20
    in_len = wl.uniform_lengths(rng, n, 4, 30)
    out_len = rng.integers(2, 6, size=n).astype(np.int32)
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    base, st0 = m.run_rra(6, 2, in_len, out_len, toks, max_encode_batch=6)
    adj, st1 = m.run_rra(6, 2, in_len, out_len, toks, max_encode_batch=6, adjust=True, workload_tolerance=0.0)
    assert adj.tolist() == base.tolist()                  # the schedule never changes a sequence's tokens
    assert st1["generated_tokens"] == st0["generated_tokens"]
    assert st1["encode_phases"] >= st0["encode_phases"]   # a capped encoder workload needs at least as many phases
    with pytest.raises(exe.ExeError) as e:
        m.run_rra(9, 2, in_len, out_len, toks, max_encode_batch=4)   # decode batch above max_batch_seqs
    assert e.value.code == -1
    bad = out_len.copy(); bad[0] = 0
    with pytest.raises(exe.ExeError) as e:
        m.run_rra(4, 2, in_len, bad, toks, max_encode_batch=4)
    assert e.value.code == -5
    m.close()


def test_rra_encoder_decoder():
    shape = wl.small_t5_shape(wl.DTYPE_F32)
    m, o, _ = make_pair(shape, 9, "float", pool_tokens=4096, max_seqs=8, max_batch_tokens=512, max_batch_seqs=8)
    rng = np.random.default_rng(7)
    n = 7
    in_len = wl.uniform_lengths(rng, n, 5, 40)
    out_len = rng.integers(1, 7, size=n).astype(np.int32)
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    got, st = m.run_rra(3, 2, in_len, out_len, toks, max_encode_batch=2)
    off = np.concatenate([[0], np.cumsum(in_len)])
    want = []
    for i in range(n):
        o.encode(0, toks[off[i]:off[i + 1]])
        t = 0
        for _ in range(out_len[i]):
            t, _ = o.decode(0, t)
            want.append(t)
        o.release(0)
    assert got.tolist() == want
    assert st["generated_tokens"] == int(out_len.sum())
    m.close()


def test_rra_pool_pressure_defers_admission():
    """A pool that holds only a few sequences: admission is deferred, never failed, and tokens do not change."""
    shape = wl.tiny_shape()
    m, o, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=100, max_seqs=16, max_batch_tokens=256, max_batch_seqs=8)
    rng = np.random.default_rng(8)
    n = 10
    in_len = wl.uniform_lengths(rng, n, 10, 24)
    out_len = rng.integers(2, 7, size=n).astype(np.int32)
    toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
    got, st = m.run_rra(8, 2, in_len, out_len, toks, max_encode_batch=2)
    m2, _, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=4096, max_seqs=16, max_batch_tokens=256, max_batch_seqs=8)
    ref, st2 = m2.run_rra(8, 2, in_len, out_len, toks, max_encode_batch=2)
    assert got.tolist() == ref.tolist()
    assert st["mean_decode_batch"] < st2["mean_decode_batch"]      # fewer sequences fit at once
    assert m.kv_stats()["used_bytes"] == 0
    m.close(); m2.close()
