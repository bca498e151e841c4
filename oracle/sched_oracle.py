"""Oracle of the schedule simulator and of the scheduling search (Sections 5 and 6).

TEST INFRASTRUCTURE: imported only by tests.  Plain, slow numpy / Python in fp64, one function per passage of the
paper, sharing no code with the library's implementation.

The simulator (Section 6) is an approximation by construction, so the functions below take the paper's steps in the
paper's order and notation:

  completion_dist   Section 6, "Simulating RRA Schedule": P_D(U|S) (the piecewise definition) and
                    P_D(U) = sum_S P_D(U|S) P_D(S)
  rra_timeline      Section 6, same passage: B_E = B_D sum_U P_D(U); expected encoding workload from B_E and P_E(S),
                    expected decoding workload from B_D and P_D(U); execution times from the profile table; timeline,
                    throughput and latency
  waa_workload      Section 6, "Simulating WAA Schedule": B_D = B_E * S_D, workloads B_E * S_E and B_D; Section 4
                    "WAA-C": GPUs in proportion to the estimated encoding / decoding times
  simulate_rra      Section 4, "RRA Scheduling", and Section 5, dynamic workload adjustment: the schedule itself played
                    out request by request (counters only), what the run loop's statistics must equal
  exhaustive_best   Section 5, the optimisation problem itself (arg max throughput subject to latency < L_Bound),
                    by evaluating every configuration point: what the branch-and-bound search must find
  branch_and_bound  Section 5, Algorithm 1, step by step (selecting, splitting with the corner heuristic, bounding,
                    updating T*, pruning)

Readings where the paper leaves the timeline open (the same ones the library documents):
  * a decode iteration's time is read from the profile table at (live batch, mean context length), the context
    length being E[S_E] + E[S_D^2] / (2 E[S_D]) + 1/2: the mean, over the (live query, iteration) pairs of the
    steady state, of the K/V length after the iteration's append, which is what a profile row's length means.  In
    Section 6's model a query of S tokens is decoded for S iterations and its t-th iteration attends to the input
    plus t positions, so the mean is E[S_E] + E[S (S + 1) / 2] / E[S];
  * the live batch of iteration U of a decoding phase is B_D (1 - sum_{u<U} P_D(u)) (completed queries leave at
    once: early termination, Section 7);
  * a query of output length s is encoded once, spends ceil(s / N_D) - 1 whole cycles and then
    1 + ((s - 1) mod N_D) iterations of its last decoding phase;
  * table look-ups interpolate bilinearly in (batch, length) between profiled points, clamp the length to the
    profiled range and scale in proportion to the batch outside the profiled batches (an expected batch of half a
    query costs half a one-query step: the step then runs every other cycle).
"""
from __future__ import annotations

import heapq
import math
from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np


# ------------------------------------------------------------------ Section 6: completion distribution
def cond_completion(U: int, S: int, N_D: int) -> float:
    """P_D(U | S): probability that a query producing S tokens completes at the U-th iteration of a decoding phase."""
    if S <= N_D:
        return 1.0 if U == S else 0.0
    phases = math.ceil(S / N_D)
    return 1.0 / phases if U == 1 + ((S - 1) % N_D) else 0.0


def completion_dist(p_out: Sequence[float], N_D: int) -> np.ndarray:
    """P_D(U), U = 1..N_D (returned at index U-1), from P_D(S), S = 1..len(p_out) (given at index S-1)."""
    p_u = np.zeros(N_D, dtype=np.float64)
    for U in range(1, N_D + 1):
        for S in range(1, len(p_out) + 1):
            p_u[U - 1] += cond_completion(U, S, N_D) * float(p_out[S - 1])
    return p_u


# ------------------------------------------------------------------ profile table look-up
@dataclass
class Table:
    """Per-(batch, length) step times of one phase, in ms: a full rectangular grid."""
    batches: List[int]
    lengths: List[int]
    step_ms: np.ndarray            # [len(batches), len(lengths)]

    def time_ms(self, batch: float, length: float) -> float:
        if batch <= 0:
            return 0.0
        scale = 1.0
        b = batch
        if b > self.batches[-1]:
            scale = b / self.batches[-1]
            b = float(self.batches[-1])
        if b < self.batches[0]:
            scale = b / self.batches[0]
            b = float(self.batches[0])
        l = min(max(length, float(self.lengths[0])), float(self.lengths[-1]))

        def bracket(grid, x):
            if len(grid) == 1:
                return 0, 0, 0.0
            hi = 1
            while hi < len(grid) - 1 and grid[hi] < x:
                hi += 1
            lo = hi - 1
            return lo, hi, (x - grid[lo]) / (grid[hi] - grid[lo])

        i0, i1, fb = bracket(self.batches, b)
        j0, j1, fl = bracket(self.lengths, l)
        t00, t01 = self.step_ms[i0, j0], self.step_ms[i0, j1]
        t10, t11 = self.step_ms[i1, j0], self.step_ms[i1, j1]
        t = (1 - fb) * ((1 - fl) * t00 + fl * t01) + fb * ((1 - fl) * t10 + fl * t11)
        return float(t) * scale


def moments(p: Sequence[float]) -> Tuple[float, float]:
    """Mean and second moment of a length distribution given at index s-1 for s = 1..len(p)."""
    s = np.arange(1, len(p) + 1, dtype=np.float64)
    p = np.asarray(p, dtype=np.float64)
    return float((s * p).sum()), float((s * s * p).sum())


# ------------------------------------------------------------------ Section 6: RRA timeline
@dataclass
class RraResult:
    b_e: float
    b_d: float
    completed_fraction: float
    context_length: float
    encode_ms: float
    decode_ms: float
    cycle_ms: float
    tokens_per_cycle: float
    throughput_tok_s: float
    throughput_seq_s: float
    latency_ms: float
    occupancy_exact: float          # E[ceil(S / N_D)]: B_D / B_E of the exact steady state (Little's law), for reference


def rra_timeline(enc: Table, dec: Table, p_in: Sequence[float], p_out: Sequence[float], b_d: float, N_D: int,
                 latency_len: int) -> RraResult:
    p_u = completion_dist(p_out, N_D)
    frac = float(p_u.sum())
    b_e = b_d * frac
    mean_in, _ = moments(p_in)
    mean_out, second_out = moments(p_out)
    ctx = mean_in + second_out / (2.0 * mean_out) + 0.5
    t_enc = enc.time_ms(b_e, mean_in)
    live = []
    done = 0.0
    for U in range(1, N_D + 1):
        live.append(b_d * (1.0 - done))
        done += float(p_u[U - 1])
    t_iter = [dec.time_ms(b, ctx) for b in live]
    t_dec = float(sum(t_iter))
    cycle = t_enc + t_dec
    tokens = float(sum(live))
    phases = math.ceil(latency_len / N_D)
    last = 1 + ((latency_len - 1) % N_D)
    latency = t_enc + (phases - 1) * cycle + float(sum(t_iter[:last]))
    occ = float(sum(math.ceil(s / N_D) * float(p_out[s - 1]) for s in range(1, len(p_out) + 1)))
    return RraResult(b_e, b_d, frac, ctx, t_enc, t_dec, cycle, tokens, tokens / cycle * 1e3, b_e / cycle * 1e3,
                     latency, occ)


# ------------------------------------------------------------------ Section 4 / Section 5: the RRA schedule, request by request
def simulate_rra(in_len: Sequence[int], out_len: Sequence[int], B_D: int, N_D: int, decoder_only: bool = True,
                 adjust: bool = False, tolerance: float = 0.25) -> Dict[str, float]:
    """Counters of the RRA schedule on a queue of requests served first-come first-served with forced output lengths.

    Encoding and decoding phases alternate: an encoding phase, then N_D decoding iterations (Section 4).  The
    encoding batch is the number of queries completed since the decode batch was last full, i.e. its free slots
    (the first phase fills all B_D); a decoder-only query produces its first token at its encoding, every live
    query one token per decoding iteration, and a query leaves when it has produced its forced output length.
    With `adjust` (Section 5), an encoding phase admits requests only while the sum of their input lengths stays
    within (1 + tolerance) x (encoding batch x mean input length), always at least one; what it leaves out raises
    the next phase's encoding batch, because that is again the number of free slots.
    Returns encode_phases, decode_iterations, mean_decode_batch, generated_tokens, encoded_tokens."""
    n = len(in_len)
    mean_in = sum(int(x) for x in in_len) / n
    nxt = finished = phases = iters = batch_sum = gen = enc = 0
    live: List[List[int]] = []                    # [request, tokens produced]
    while finished < n:
        want = min(B_D - len(live), n - nxt)
        budget = (1.0 + tolerance) * max(1, want) * mean_in if adjust else float("inf")
        taken = 0
        if want > 0:
            phases += 1
        while want > 0:
            L = int(in_len[nxt])
            if taken > 0 and taken + L > budget:
                break
            taken += L
            enc += L
            if decoder_only:
                gen += 1
                if out_len[nxt] == 1:
                    finished += 1
                else:
                    live.append([nxt, 1])
            else:
                live.append([nxt, 0])
            nxt += 1
            want -= 1
        for _ in range(N_D):
            if not live:
                break
            iters += 1
            batch_sum += len(live)
            still = []
            for q in live:
                q[1] += 1
                gen += 1
                if q[1] >= out_len[q[0]]:
                    finished += 1
                else:
                    still.append(q)
            live = still
    return {"encode_phases": phases, "decode_iterations": iters, "mean_decode_batch": batch_sum / max(iters, 1),
            "generated_tokens": gen, "encoded_tokens": enc}


# ------------------------------------------------------------------ Section 6 / Section 4: WAA workload and allocation
@dataclass
class WaaResult:
    b_e: float
    b_d: float
    encode_ms: float               # C_E: one encoding iteration of B_E queries of mean length S_E
    decode_ms: float               # C_D: one decoding iteration of B_D queries
    gpus_encode: int
    gpus_decode: int
    throughput_seq_s: float


def waa_workload(enc: Table, dec: Table, p_in: Sequence[float], p_out: Sequence[float], b_e: float,
                 n_gpus: int) -> WaaResult:
    mean_in, _ = moments(p_in)
    mean_out, second_out = moments(p_out)
    b_d = b_e * mean_out
    ctx = mean_in + second_out / (2.0 * mean_out) + 0.5
    c_e = enc.time_ms(b_e, mean_in)
    c_d = dec.time_ms(b_d, ctx)
    g_e = int(round(n_gpus * c_e / (c_e + c_d)))
    g_e = min(max(g_e, 1), n_gpus - 1) if n_gpus >= 2 else 1
    g_d = n_gpus - g_e if n_gpus >= 2 else 1
    # one encoding iteration admits B_E queries; the slower side of the pipeline sets the rate
    period = max(c_e / g_e, c_d / g_d)
    return WaaResult(b_e, b_d, c_e, c_d, g_e, g_d, b_e / period * 1e3)


# ------------------------------------------------------------------ Section 5: the problem, exhaustively
Perf = Callable[[int, int], Tuple[float, float]]      # (x1, x2) -> (latency, throughput)


def exhaustive_best(perf: Perf, r1: Tuple[int, int], r2: Tuple[int, int], L_b: float) -> Optional[Tuple[float, int, int]]:
    best = None
    for x1 in range(r1[0], r1[1] + 1):
        for x2 in range(r2[0], r2[1] + 1):
            lat, thr = perf(x1, x2)
            if lat < L_b and (best is None or thr > best[0]):
                best = (thr, x1, x2)
    return best


# ------------------------------------------------------------------ Section 5: Algorithm 1
def branch_and_bound(perf: Perf, r1: Tuple[int, int], r2: Tuple[int, int], eps_T: float, eps_L: float,
                     L_b: float) -> Tuple[Optional[Tuple[float, int, int]], int]:
    """Returns ((throughput, x1, x2) of T*, or None when no examined point meets the bound; number of distinct
    configuration points evaluated).  Both functions are taken to be non-decreasing in x1 and in x2, so a block's
    bottom-left corner bounds it from below and its top-right corner from above."""
    cache: Dict[Tuple[int, int], Tuple[float, float]] = {}

    def P(x1, x2):
        if (x1, x2) not in cache:
            cache[(x1, x2)] = perf(x1, x2)
        return cache[(x1, x2)]

    (a1, b1), (a2, b2) = r1, r2
    best = None
    lat, thr = P(a1, a2)
    if lat < L_b:
        best = (thr, a1, a2)
    lat, thr = P(b1, b2)
    if lat < L_b:                                   # the whole range meets the bound: its top-right corner is optimal
        return (thr, b1, b2), len(cache)
    counter = 0
    queue = [(-P(a1, a2)[1], counter, (a1, a2, b1, b2))]          # max-heap on the lower bound's throughput
    upper = {(a1, a2, b1, b2): P(b1, b2)[1]}
    while queue:
        _, _, B = heapq.heappop(queue)
        if B not in upper:                          # pruned
            continue
        del upper[B]
        lo1, lo2, hi1, hi2 = B
        if lo1 == hi1 and lo2 == hi2:
            continue
        p_tl, p_br = P(lo1, hi2), P(hi1, lo2)
        ok_tl, ok_br = p_tl[0] < L_b, p_br[0] < L_b
        if ok_tl and (not ok_br or p_tl[1] >= p_br[1]):
            vertical = True
        elif ok_br:
            vertical = False
        else:
            vertical = (hi1 - lo1) >= (hi2 - lo2)
        if vertical and lo1 == hi1:
            vertical = False
        if not vertical and lo2 == hi2:
            vertical = True
        if vertical:                                # cut the x1 range
            mid = (lo1 + hi1) // 2
            children = [(lo1, lo2, mid, hi2), (mid + 1, lo2, hi1, hi2)]
        else:
            mid = (lo2 + hi2) // 2
            children = [(lo1, lo2, hi1, mid), (lo1, mid + 1, hi1, hi2)]
        cand = None
        for C in children:
            upp, lowr = P(C[2], C[3]), P(C[0], C[1])
            if lowr[0] < L_b + eps_L:
                counter += 1
                heapq.heappush(queue, (-lowr[1], counter, C))
                upper[C] = upp[1]
            if upp[0] < L_b and (cand is None or upp[1] > cand[0]):
                cand = (upp[1], C[2], C[3])
        if cand is not None and (best is None or cand[0] > best[0]):
            best = cand
        if best is not None:
            for Bq in [Bq for Bq, u in upper.items() if u + eps_T < best[0]]:
                del upper[Bq]
    return best, len(cache)
