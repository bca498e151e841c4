/*
 * exe_sched.h -- schedule simulator and constraint-aware scheduling search (host code only: these entry points
 * touch no GPU and may be called on a machine without one).  They consume the latency table that exe_profile
 * (exe.h) emits and produce the (B_E, B_D, N_D) configuration that exe_run_rra executes.
 *
 * Conventions: length distributions are arrays of doubles, entry s-1 = probability of length s, s = 1..n; they
 * must be non-negative and sum to 1 within 1e-6.  Times are milliseconds, throughputs per second.  Every function
 * returns EXE_OK or a negative EXE_ERR_* (exe.h) and leaves a message for exe_last_error(); output arguments are
 * written only on success.  No entry point keeps a pointer after it returns.
 */
#ifndef EXE_SCHED_H
#define EXE_SCHED_H

#include "exe.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Section 6, "Simulating RRA Schedule": P_D(U), the probability that a query completes at the U-th decoding
 * iteration after an encoding phase, U = 1..n_decode, from the output-length distribution P_D(S):
 * P_D(U) = sum_S P_D(U|S) P_D(S) with the piecewise P_D(U|S) of that passage (a query of S <= N_D tokens completes
 * at U = S; a longer one needs ceil(S / N_D) phases and completes in a given phase, at U = 1 + (S-1) mod N_D, with
 * probability 1 / ceil(S / N_D)).
 *  p_out [s_max] host in; p_u [n_decode] host out; completed_fraction (nullable) out: sum_U P_D(U).
 */
int exe_sim_completion(const double* p_out, int32_t s_max, int32_t n_decode, double* p_u, double* completed_fraction);

/* Both phases' rows of one or several exe_profile calls, in any order; each phase's rows must form a full
 * (batch x length) grid.  n_layers_encode / n_layers_decode: layers an encoding / a decoding iteration runs
 * through (decoder-only models: both the model's depth).  The step time of a row is
 * layers * (attn_ms_per_layer + rest_ms_per_layer) + head_ms. */
typedef struct exe_sim_table {
    const exe_profile_row_t* rows;
    int32_t n_rows;
    int32_t n_layers_encode, n_layers_decode;
} exe_sim_table_t;

/* Step time read from the table (Section 3, "XProfiler" tables as the simulator's input): bilinear in (batch, length)
 * between profiled points; the length is clamped to the profiled range; a batch outside the profiled ones scales
 * the nearest profiled row in proportion (an expected batch of half a query costs half a one-query step: the step
 * then runs every other cycle).  batch <= 0 gives 0. */
int exe_sim_step_ms(const exe_sim_table_t* table, int32_t phase, double batch, double length, double* ms);

/*
 * Section 6, "Simulating RRA Schedule": the steady-state timeline of the RRA schedule (Section 4: encode once, then
 * N_D decoding iterations, repeatedly) on one GPU for a decoding batch B_D:
 *   B_E = B_D sum_U P_D(U)               queries admitted per encoding phase
 *   encoding time                        one encoding iteration of B_E queries of the mean input length
 *   decoding time                        sum over U of one iteration of the live batch B_D (1 - sum_{u<U} P_D(u))
 *                                        (completed queries leave at once) at the mean context length
 *                                        E[S_E] + E[S_D^2] / (2 E[S_D])
 *   throughput                           tokens generated per cycle / (encoding + decoding time)
 *   latency of a query of latency_len    encoding time + (ceil(len / N_D) - 1) cycles
 *   output tokens                        + the first 1 + (len-1) mod N_D iterations of a decoding phase
 * occupancy_exact reports E[ceil(S_D / N_D)], the B_D / B_E ratio of the exact steady state, next to the paper's
 * 1 / sum_U P_D(U) (equal for a single output length, smaller otherwise).
 */
typedef struct exe_sim_rra_result {
    double b_e, b_d, completed_fraction, context_length;
    double encode_ms, decode_ms, cycle_ms, tokens_per_cycle;
    double throughput_tok_s, throughput_seq_s, latency_ms, occupancy_exact;
} exe_sim_rra_result_t;
int exe_sim_rra(const exe_sim_table_t* table, const double* p_in, int32_t in_max, const double* p_out, int32_t out_max,
                double decode_batch, int32_t n_decode, int32_t latency_len, exe_sim_rra_result_t* result);

/*
 * Section 6, "Simulating WAA Schedule" with the WAA-C allocation of Section 4: B_D = B_E * S_D; the encoding
 * workload B_E * S_E and the decoding workload B_D give the times C_E and C_D of one encoding / decoding
 * iteration; of n_gpus, round(n_gpus C_E / (C_E + C_D)) go to encoding (at least one to each side when
 * n_gpus >= 2); the slower side sets the rate at which batches of B_E queries are admitted.
 */
typedef struct exe_sim_waa_result {
    double b_e, b_d, encode_ms, decode_ms;
    int32_t gpus_encode, gpus_decode;
    double throughput_seq_s;
} exe_sim_waa_result_t;
int exe_sim_waa(const exe_sim_table_t* table, const double* p_in, int32_t in_max, const double* p_out, int32_t out_max,
                double encode_batch, int32_t n_gpus, exe_sim_waa_result_t* result);

/*
 * Section 5, Algorithm 1 (branch-and-bound scheduling) over two integer control variables x1 in [a1, b1] and
 * x2 in [a2, b2] in which latency and throughput are non-decreasing (within the tolerances): arg max throughput
 * subject to latency < latency_bound.  perf(x1, x2, user, &latency, &throughput) returns 0 on success; it is called
 * at most once per configuration point.
 *  eps_throughput, eps_latency: the tolerances of Algorithm 1 (a block is kept while its lower-left latency is below
 *  the bound + eps_latency, and pruned once its upper-right throughput + eps_throughput is below T*).
 *  found = 0 when no examined point meets the bound (x1, x2, throughput are then not written).
 */
typedef int (*exe_perf_fn)(int32_t x1, int32_t x2, void* user, double* latency, double* throughput);
typedef struct exe_sched_result {
    int32_t found, x1, x2;
    double throughput, latency;
    int32_t evaluations;           /* distinct configuration points evaluated */
    int32_t blocks;                /* blocks taken from the queue */
} exe_sched_result_t;
int exe_sched_search(exe_perf_fn perf, void* user, int32_t a1, int32_t b1, int32_t a2, int32_t b2, double eps_throughput,
                     double eps_latency, double latency_bound, exe_sched_result_t* result);

/*
 * The same search with exe_sim_rra as perf: x1 = B_D in [bd_min, bd_max]; x2 indexes the encoding frequency
 * (Section 4: encoding more often, i.e. a smaller N_D, raises throughput and latency), N_D = nd_max - x2 for
 * x2 in [0, nd_max - nd_min].  The latency is that of a query of latency_len output tokens.
 */
typedef struct exe_sched_rra_result {
    exe_sched_result_t search;
    int32_t decode_batch, n_decode;           /* the configuration for exe_rra_config_t */
    exe_sim_rra_result_t sim;                 /* its simulated timeline */
} exe_sched_rra_result_t;
int exe_sched_rra(const exe_sim_table_t* table, const double* p_in, int32_t in_max, const double* p_out, int32_t out_max,
                  int32_t bd_min, int32_t bd_max, int32_t nd_min, int32_t nd_max, int32_t latency_len,
                  double latency_bound_ms, double eps_throughput, double eps_latency_ms, exe_sched_rra_result_t* result);

#ifdef __cplusplus
}
#endif
#endif
