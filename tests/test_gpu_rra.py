"""exe_run_rra: the RRA schedule (encode once, N_D decode iterations, refill with as many queries as completed)
on one GPU.  Sequences are independent, so every request's tokens must equal the oracle's greedy decoding of
that request alone; the schedule's counters must equal the oracle's request-by-request simulation of the schedule
(oracle/sched_oracle.py, written from Section 4 "RRA Scheduling" and Section 5's dynamic workload adjustment)."""
import numpy as np
import pytest

import paper_2404_07947_amd as exe
import workload as wl
from gpu_util import make_pair
from oracle.sched_oracle import simulate_rra

pytestmark = pytest.mark.gpu


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
    sim = simulate_rra(in_len, out_len, BD, ND)
    assert st["generated_tokens"] == sim["generated_tokens"] == int(out_len.sum())
    assert st["encoded_tokens"] == sim["encoded_tokens"] == int(in_len.sum())
    assert st["encode_phases"] == sim["encode_phases"] and st["decode_iterations"] == sim["decode_iterations"]
    assert abs(st["mean_decode_batch"] - sim["mean_decode_batch"]) < 1e-9
    assert st["encode_calls"] >= sim["encode_phases"]
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
    # counters against the oracle's simulation, with and without the adjustment; an encoding phase that the
    # workload cap cut short leaves its remainder to the next phase, so the decode batch returns to B_D
    for st, kw in ((st0, {}), (st1, {"adjust": True, "tolerance": 0.0})):
        sim = simulate_rra(in_len, out_len, 6, 2, **kw)
        assert st["encode_phases"] == sim["encode_phases"] and st["decode_iterations"] == sim["decode_iterations"], (st, sim)
        assert abs(st["mean_decode_batch"] - sim["mean_decode_batch"]) < 1e-9
    for tol in (0.1, 0.5):
        _, st2 = m.run_rra(6, 3, in_len, out_len, toks, max_encode_batch=3, adjust=True, workload_tolerance=tol)
        sim = simulate_rra(in_len, out_len, 6, 3, adjust=True, tolerance=tol)
        assert st2["encode_phases"] == sim["encode_phases"] and st2["decode_iterations"] == sim["decode_iterations"]
        assert abs(st2["mean_decode_batch"] - sim["mean_decode_batch"]) < 1e-9
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
    sim = simulate_rra(in_len, out_len, 3, 2, decoder_only=False)
    assert st["encode_phases"] == sim["encode_phases"] and st["decode_iterations"] == sim["decode_iterations"]
    assert abs(st["mean_decode_batch"] - sim["mean_decode_batch"]) < 1e-9
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


def test_rra_random_schedules_against_the_simulation():
    """Seeded random schedules (decode batch, N_D, encode-batch cap, workload adjustment and its tolerance, request
    mix): the counters must equal the oracle's simulation each time and the tokens never depend on the schedule."""
    shape = wl.tiny_shape()
    m, o, _ = make_pair(shape, wl.BASE_SEED, "float", pool_tokens=4096, max_seqs=32, max_batch_tokens=512, max_batch_seqs=12)
    rng = np.random.default_rng(31)
    for case in range(14):
        n = int(rng.integers(3, 30))
        in_len = wl.uniform_lengths(rng, n, 1, 30)
        out_len = rng.integers(1, 12, size=n).astype(np.int32)
        toks = wl.random_tokens(rng, int(in_len.sum()), shape.vocab)
        BD, ND = int(rng.integers(1, 13)), int(rng.integers(1, 9))
        max_enc = int(rng.integers(1, 13))
        adjust = bool(rng.integers(0, 2))
        tol = float(rng.choice([0.0, 0.1, 0.25, 1.0]))
        print(f"case {case}: n {n} BD {BD} ND {ND} max_enc {max_enc} adjust {adjust} tol {tol}", flush=True)
        got, st = m.run_rra(BD, ND, in_len, out_len, toks, max_encode_batch=max_enc, adjust=adjust, workload_tolerance=tol)
        sim = simulate_rra(in_len, out_len, BD, ND, adjust=adjust, tolerance=tol)
        assert st["generated_tokens"] == sim["generated_tokens"] == int(out_len.sum())
        assert st["encoded_tokens"] == sim["encoded_tokens"] == int(in_len.sum())
        assert (st["encode_phases"], st["decode_iterations"]) == (sim["encode_phases"], sim["decode_iterations"]), (st, sim)
        assert abs(st["mean_decode_batch"] - sim["mean_decode_batch"]) < 1e-9
        ref, _ = m.run_rra(12, 1, in_len, out_len, toks, max_encode_batch=12)      # another schedule, same tokens
        assert got.tolist() == ref.tolist()
        if case < 3:                                                              # and the oracle's, request by request
            off = np.concatenate([[0], np.cumsum(in_len)])
            want = []
            for i in range(n):
                t, _ = o.encode(0, toks[off[i]:off[i + 1]])
                want.append(t)
                for _ in range(out_len[i] - 1):
                    t, _ = o.decode(0, t)
                    want.append(t)
                o.release(0)
            assert got.tolist() == want
        assert m.kv_stats()["used_bytes"] == 0 and m.kv_stats()["live_seqs"] == 0
    m.close()
