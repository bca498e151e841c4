"""Pins of the scheduling oracle (oracle/sched_oracle.py) against what the paper and the mathematics fix:
the closed forms Section 6 states for P_D(U|S), special cases that reduce to elementary results, Monte-Carlo
simulation of the completion process, hand-computed timelines, and exhaustive search for Algorithm 1."""
import math

import numpy as np
import pytest

from oracle import sched_oracle as so


def normal_dist(mean, std, lo, hi):
    s = np.arange(1, hi + 1, dtype=np.float64)
    p = np.exp(-0.5 * ((s - mean) / std) ** 2)
    p[: lo - 1] = 0.0
    return p / p.sum()


# ---------------------------------------------------------------- P_D(U|S), P_D(U)
@pytest.mark.parametrize("N_D", [1, 2, 3, 7, 16, 40])
def test_conditional_sums_to_the_papers_closed_form(N_D):
    # Section 6: a query of length S <= N_D completes in the phase with certainty; a longer one needs
    # ceil(S / N_D) phases and completes in a given one with probability 1 / ceil(S / N_D)
    for S in range(1, 100):
        total = sum(so.cond_completion(U, S, N_D) for U in range(1, N_D + 1))
        expect = 1.0 if S <= N_D else 1.0 / math.ceil(S / N_D)
        assert total == pytest.approx(expect, abs=1e-15)
        hits = [U for U in range(1, N_D + 1) if so.cond_completion(U, S, N_D) > 0]
        # the completing iteration is the one at which the S-th token is produced: S = (phases - 1) N_D + U
        assert hits == [S - (math.ceil(S / N_D) - 1) * N_D]


def test_completion_dist_special_cases():
    p = normal_dist(20, 6, 3, 40)
    # every output fits in one phase: P_D(U) is P_D(S) itself and every query completes
    pu = so.completion_dist(p, 64)
    assert np.allclose(pu[:40], p, atol=1e-15) and pu[40:].sum() == 0 and pu.sum() == pytest.approx(1.0)
    # one decode iteration per phase: P_D(U=1) = E[1/S]
    pu = so.completion_dist(p, 1)
    assert pu[0] == pytest.approx(float((p / np.arange(1, 41)).sum()), rel=1e-14)
    # a single output length: 1 / ceil(S / N_D) at U = 1 + (S - 1) mod N_D
    for S, N_D in [(9, 4), (8, 4), (5, 7), (100, 16)]:
        q = np.zeros(S); q[S - 1] = 1.0
        pu = so.completion_dist(q, N_D)
        U = 1 + (S - 1) % N_D if S > N_D else S
        assert pu[U - 1] == pytest.approx(1.0 / math.ceil(S / N_D)) and pu.sum() == pytest.approx(pu[U - 1])


@pytest.mark.parametrize("N_D", [4, 16])
def test_completion_dist_against_sampling_of_the_papers_model(N_D):
    # the model behind the formula: a query of length S ~ P_D(S) is, in a given phase, in any of its
    # ceil(S / N_D) phases with equal probability, and completes only in the last one
    p = normal_dist(24, 9, 2, 60)
    rng = np.random.default_rng(7)
    n = 400_000
    S = rng.choice(np.arange(1, 61), size=n, p=p)
    phases = np.ceil(S / N_D).astype(np.int64)
    in_last = rng.integers(0, phases) == phases - 1
    U = S - (phases - 1) * N_D
    emp = np.bincount(U[in_last], minlength=N_D + 1)[1:] / n
    pu = so.completion_dist(p, N_D)
    sigma = np.sqrt(np.maximum(pu * (1 - pu), 1e-12) / n)
    assert np.all(np.abs(emp - pu) < 5 * sigma + 1e-9)


def simulate_rra_occupancy(p_out, B_D, N_D, phases, seed):
    """Direct simulation of the RRA schedule's queue: every phase tops the decode batch up to B_D with new queries
    (S ~ P_D(S)), then runs N_D iterations in which finished queries leave.  Returns mean admitted per phase."""
    rng = np.random.default_rng(seed)
    lens = np.arange(1, len(p_out) + 1)
    remaining = np.zeros(0, dtype=np.int64)
    admitted = []
    for ph in range(phases):
        new = B_D - remaining.size
        remaining = np.concatenate([remaining, rng.choice(lens, size=new, p=p_out)])
        if ph >= phases // 4:
            admitted.append(new)
        remaining = remaining - N_D
        remaining = remaining[remaining > 0]
    return float(np.mean(admitted))


def test_exact_occupancy_is_littles_law():
    # B_D / B_E of the true steady state is E[ceil(S / N_D)] (each admitted query occupies a slot for that many
    # phases); for a single output length it coincides with the paper's 1 / sum_U P_D(U)
    enc = so.Table([1, 512], [8, 64], np.array([[1.0, 2.0], [10.0, 20.0]]))
    dec = so.Table([1, 512], [8, 256], np.array([[1.0, 1.0], [2.0, 3.0]]))
    p_in = normal_dist(32, 8, 8, 64)
    p_out = normal_dist(24, 9, 2, 60)
    r = so.rra_timeline(enc, dec, p_in, p_out, 256.0, 8, 24)
    b_e = simulate_rra_occupancy(p_out, 4096, 8, 400, 3)
    assert 4096 / b_e == pytest.approx(r.occupancy_exact, rel=5e-3)
    q = np.zeros(20); q[19] = 1.0
    r1 = so.rra_timeline(enc, dec, p_in, q, 256.0, 8, 20)
    assert r1.occupancy_exact == pytest.approx(1.0 / r1.completed_fraction) == pytest.approx(3.0)
    # and in general the paper's estimate is the smaller one (Jensen), which is why both are reported
    assert 1.0 / r.completed_fraction <= r.occupancy_exact + 1e-12


def test_context_length_is_the_mean_kv_length_of_the_steady_state_queue():
    """The length at which a decode iteration is priced, pinned by a direct simulation of the RRA queue in Section 6's
    model (a query of S tokens is decoded for S iterations; its t-th iteration attends to its input plus t
    positions): the mean over all (live query, iteration) pairs of the K/V length after the append.  The closed form
    is E[S_E] + E[S (S + 1) / 2] / E[S] = E[S_E] + E[S^2] / (2 E[S]) + 1/2, whatever B_D and N_D are."""
    p_in = normal_dist(32, 8, 8, 64)
    p_out = normal_dist(24, 9, 2, 60)
    enc = so.Table([1, 512], [8, 64], np.array([[1.0, 2.0], [10.0, 20.0]]))
    dec = so.Table([1, 512], [8, 256], np.array([[1.0, 1.0], [2.0, 3.0]]))
    r = so.rra_timeline(enc, dec, p_in, p_out, 256.0, 8, 24)
    rng = np.random.default_rng(11)
    in_lens, out_lens = np.arange(1, 65), np.arange(1, 61)
    B_D, N_D = 512, 8
    live_in = np.zeros(0, dtype=np.int64)
    live_out = np.zeros(0, dtype=np.int64)
    live_done = np.zeros(0, dtype=np.int64)
    total, count = 0.0, 0
    for phase in range(300):
        new = B_D - live_in.size
        live_in = np.concatenate([live_in, rng.choice(in_lens, size=new, p=p_in)])
        live_out = np.concatenate([live_out, rng.choice(out_lens, size=new, p=p_out)])
        live_done = np.concatenate([live_done, np.zeros(new, dtype=np.int64)])
        for it in range(N_D):
            live_done = live_done + 1                      # this iteration appends one position to every live query
            if phase >= 75:
                total += float((live_in + live_done).sum())
                count += live_in.size
            keep = live_done < live_out
            live_in, live_out, live_done = live_in[keep], live_out[keep], live_done[keep]
    assert total / count == pytest.approx(r.context_length, rel=3e-3)
    # a single output length makes it exact: K/V lengths in+1 .. in+S, each as often as the others
    q = np.zeros(7); q[6] = 1.0
    one_in = np.zeros(10); one_in[9] = 1.0
    assert so.rra_timeline(enc, dec, one_in, q, 64.0, 3, 7).context_length == pytest.approx(10 + (1 + 7) / 2)


def test_simulate_rra_by_hand():
    # three requests of 2 output tokens, decode batch 2, one iteration per phase: requests 0 and 1 are encoded (a
    # token each), the one iteration finishes both; request 2 is encoded alone and finished by the next iteration
    r = so.simulate_rra([5, 5, 5], [2, 2, 2], 2, 1)
    assert r == {"encode_phases": 2, "decode_iterations": 2, "mean_decode_batch": 1.5, "generated_tokens": 6, "encoded_tokens": 15}
    # encoder-decoder: no token at the encoding, so 2 iterations per request; B_D = 3 takes all three at once
    r = so.simulate_rra([5, 5, 5], [2, 2, 2], 3, 4, decoder_only=False)
    assert (r["encode_phases"], r["decode_iterations"], r["mean_decode_batch"], r["generated_tokens"]) == (1, 2, 3.0, 6)
    # workload adjustment with no tolerance: 4 free slots and a mean input of 10 give a budget of 40 tokens; the
    # inputs 30, 10 fill it, the third request (10) has to wait for the next phase, which then asks for the two
    # slots still free plus whatever completed
    r = so.simulate_rra([30, 10, 10, 5, 5, 5, 5, 10], [3] * 8, 4, 1, adjust=True, tolerance=0.0)
    plain = so.simulate_rra([30, 10, 10, 5, 5, 5, 5, 10], [3] * 8, 4, 1)
    assert r["generated_tokens"] == plain["generated_tokens"] == 24 and r["encoded_tokens"] == 80
    assert r["encode_phases"] > plain["encode_phases"] and r["mean_decode_batch"] < plain["mean_decode_batch"]
    # a request with a single output token completes at its encoding and never enters the decode batch
    r = so.simulate_rra([4, 4], [1, 3], 2, 2)
    assert (r["decode_iterations"], r["mean_decode_batch"], r["generated_tokens"]) == (2, 1.0, 4)


# ---------------------------------------------------------------- table look-up
def test_table_lookup():
    t = so.Table([1, 4, 16], [10, 20], np.array([[1.0, 2.0], [3.0, 6.0], [9.0, 20.0]]))
    for i, b in enumerate(t.batches):
        for j, l in enumerate(t.lengths):
            assert t.time_ms(b, l) == pytest.approx(t.step_ms[i, j])
    assert t.time_ms(2.5, 15) == pytest.approx(0.25 * (1 + 2 + 3 + 6))                 # cell midpoint
    assert t.time_ms(10, 10) == pytest.approx(3 + (9 - 3) * 0.5)
    assert t.time_ms(32, 20) == pytest.approx(40.0)                                   # beyond the grid: proportional
    assert t.time_ms(4, 5) == t.time_ms(4, 10) and t.time_ms(4, 99) == t.time_ms(4, 20)  # length clamped
    assert t.time_ms(0.5, 10) == pytest.approx(0.5)                                   # below the grid: proportional
    assert t.time_ms(0, 10) == 0.0


def test_table_lookup_reproduces_a_cost_that_is_proportional_to_the_batch():
    # A step whose time is c * batch * (1 + length / 100) (every sequence costs the same, no fixed cost) is bilinear
    # in (batch, length), so interpolation inside the grid is exact; and because it is proportional to the batch,
    # a look-up outside the profiled batches must still return it: the per-sequence cost measured at the nearest
    # profiled batch carries over (no look-up that clamps the batch, or extrapolates the last segment of a table
    # with an intercept, does).  The throughput batch / time is then the same at every batch, profiled or not.
    batches, lengths = [4, 16, 64], [128, 512, 2048]
    cost = lambda b, l: 0.03 * b * (1 + l / 100.0)
    t = so.Table(batches, lengths, np.array([[cost(b, l) for l in lengths] for b in batches]))
    for b in (0.25, 1, 3, 4, 9.5, 64, 65, 200, 1000):
        for l in (128, 300, 512, 1999, 2048):
            assert t.time_ms(b, l) == pytest.approx(cost(b, l), rel=1e-12)
            assert b / t.time_ms(b, l) == pytest.approx(4 / t.time_ms(4, l), rel=1e-12)
    # with a fixed cost per step in the table the look-up below the grid keeps the smallest profiled batch's
    # per-sequence time, i.e. a batch half as large takes half as long and gains no throughput
    u = so.Table([8, 32], [100], np.array([[5.0 + 8], [5.0 + 32]]))
    assert u.time_ms(4, 100) == pytest.approx(0.5 * u.time_ms(8, 100))
    assert u.time_ms(64, 100) == pytest.approx(2.0 * u.time_ms(32, 100))
    assert u.time_ms(8, 100) == pytest.approx(13.0) and u.time_ms(7.999, 100) == pytest.approx(13.0, rel=1e-3)


# ---------------------------------------------------------------- timeline by hand
def test_rra_timeline_by_hand():
    # every input has 10 tokens, every output 4; N_D = 2: a query stays 2 phases and completes at U = 2, so
    # half the batch completes per phase, nobody leaves after iteration 1, and B_E = B_D / 2
    enc = so.Table([1, 100], [10], np.array([[2.0], [101.0]]))        # 1 + batch  ms
    dec = so.Table([1, 100], [1, 100], np.array([[0.5, 0.5], [50.0, 50.0]]))   # 0.5 * batch ms, any context
    p_in = np.zeros(10); p_in[9] = 1.0
    p_out = np.zeros(4); p_out[3] = 1.0
    r = so.rra_timeline(enc, dec, p_in, p_out, 40.0, 2, 4)
    assert r.completed_fraction == pytest.approx(0.5) and r.b_e == pytest.approx(20.0)
    assert r.encode_ms == pytest.approx(21.0)
    assert r.decode_ms == pytest.approx(20.0 + 20.0)
    assert r.tokens_per_cycle == pytest.approx(80.0)
    assert r.cycle_ms == pytest.approx(61.0)
    assert r.throughput_tok_s == pytest.approx(80.0 / 61.0 * 1e3)
    assert r.throughput_seq_s == pytest.approx(20.0 / 61.0 * 1e3)
    assert r.context_length == pytest.approx(10 + 16 / 8 + 0.5)      # K/V lengths 11, 12, 13, 14 with equal weight
    # encoded (21), one whole cycle (61), then both iterations of its last phase (40)
    assert r.latency_ms == pytest.approx(21.0 + 61.0 + 40.0)
    # a 3-token answer: second phase, first iteration only
    assert so.rra_timeline(enc, dec, p_in, p_out, 40.0, 2, 3).latency_ms == pytest.approx(21.0 + 61.0 + 20.0)


def test_rra_live_batch_shrinks_within_a_phase():
    # outputs 1 or 2 with equal probability, N_D = 2: half the batch leaves after the first iteration
    enc = so.Table([1, 100], [10], np.array([[1.0], [1.0]]))
    dec = so.Table([1, 100], [1, 100], np.array([[1.0, 1.0], [100.0, 100.0]]))   # batch ms
    r = so.rra_timeline(enc, dec, [0] * 9 + [1.0], [0.5, 0.5], 10.0, 2, 2)
    assert r.completed_fraction == pytest.approx(1.0)
    assert r.tokens_per_cycle == pytest.approx(10.0 + 5.0) and r.decode_ms == pytest.approx(15.0)


def test_waa_workload():
    enc = so.Table([1, 64], [32], np.array([[1.0], [64.0]]))          # batch ms
    dec = so.Table([1, 4096], [1, 4096], np.array([[0.01, 0.01], [40.96, 40.96]]))   # 0.01 * batch ms
    p_in = np.zeros(32); p_in[31] = 1.0
    p_out = np.zeros(100); p_out[99] = 1.0
    r = so.waa_workload(enc, dec, p_in, p_out, 8.0, 4)
    assert r.b_d == pytest.approx(800.0)                               # B_D = B_E * S_D
    assert r.encode_ms == pytest.approx(8.0) and r.decode_ms == pytest.approx(8.0)
    assert (r.gpus_encode, r.gpus_decode) == (2, 2)
    assert r.throughput_seq_s == pytest.approx(8.0 / 4.0 * 1e3)


# ---------------------------------------------------------------- Algorithm 1 against exhaustive search
def monotone_grid(rng, n1, n2):
    lat = np.cumsum(np.cumsum(rng.uniform(0.0, 1.0, (n1, n2)), axis=0), axis=1)
    thr = np.cumsum(np.cumsum(rng.uniform(0.0, 1.0, (n1, n2)), axis=0), axis=1)
    return lat, thr


@pytest.mark.parametrize("seed", range(12))
def test_branch_and_bound_finds_the_exhaustive_optimum(seed):
    rng = np.random.default_rng(seed)
    n1, n2 = int(rng.integers(1, 40)), int(rng.integers(1, 40))
    lat, thr = monotone_grid(rng, n1, n2)
    perf = lambda x1, x2: (float(lat[x1, x2]), float(thr[x1, x2]))
    for q in (0.0, 0.2, 0.6, 0.95, 1.1):
        L_b = float(lat.min() + q * (lat.max() - lat.min())) + 1e-9
        ref = so.exhaustive_best(perf, (0, n1 - 1), (0, n2 - 1), L_b)
        got, evals = so.branch_and_bound(perf, (0, n1 - 1), (0, n2 - 1), 0.0, 0.0, L_b)
        assert (ref is None) == (got is None)
        if ref is not None:
            assert got[0] == pytest.approx(ref[0]) and lat[got[1], got[2]] < L_b
        assert evals <= n1 * n2


def test_branch_and_bound_examines_a_small_subset():
    rng = np.random.default_rng(5)
    lat, thr = monotone_grid(rng, 128, 64)
    perf = lambda x1, x2: (float(lat[x1, x2]), float(thr[x1, x2]))
    L_b = float(np.quantile(lat, 0.4))
    ref = so.exhaustive_best(perf, (0, 127), (0, 63), L_b)
    got, evals = so.branch_and_bound(perf, (0, 127), (0, 63), 0.0, 0.0, L_b)
    assert got[0] == pytest.approx(ref[0])
    assert evals < 128 * 64 // 4


def test_branch_and_bound_tolerances_cover_small_non_monotonicity():
    rng = np.random.default_rng(9)
    lat, thr = monotone_grid(rng, 24, 24)
    thr = thr + rng.uniform(-0.3, 0.3, thr.shape)          # ripples smaller than eps_T
    lat = lat + rng.uniform(-0.2, 0.2, lat.shape)
    perf = lambda x1, x2: (float(lat[x1, x2]), float(thr[x1, x2]))
    L_b = float(np.quantile(lat, 0.5))
    ref = so.exhaustive_best(perf, (0, 23), (0, 23), L_b)
    got, _ = so.branch_and_bound(perf, (0, 23), (0, 23), 1.5, 1.0, L_b)
    assert got[0] >= ref[0] - 1.5 and lat[got[1], got[2]] < L_b
