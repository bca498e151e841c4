/*
 * exe -- batched Transformer execution on one MI355X (gfx950): the per-GPU model execution that an
 * execution-schedule-driven LLM inference engine runs and that its profiler times.
 *
 * The computation is the one the paper's background section describes (Section 2): a batch of
 * variable-length inputs is ENCODED once; then DECODE iterations each produce one token per live
 * sequence, reading that sequence's memoized keys/values (incremental decoding).  Attention runs per
 * sequence, everything else runs on the packed batch (selective batching, Section 2, review of ORCA).
 * Sequences that are finished leave the batch (early termination, Section 3 "XRunner") and sequences
 * from different encode calls may share a decode batch (decoupled batches, Section 6).  exe_profile
 * emits the per-layer attention / rest-of-layer latency table (Section 3 "XProfiler").
 *
 * Conventions
 *  - Every call returns an int: EXE_OK (0) or a negative exe_status.  Nothing throws or aborts on bad
 *    input; exe_last_error() returns a thread-local description of the last failure.
 *  - "host" pointers are ordinary CPU memory read/written before the call returns.  "device" pointers
 *    are HIP device memory on the current device, owned by the caller.
 *  - Calls are synchronous: when they return, host outputs are filled and device outputs are complete
 *    on the model's stream (the stream has been synchronised).
 *  - A model handle is not thread-safe; use one handle per thread.
 *  - Linear weights are [out_features, in_features] row-major in the model's dtype.  The fused QKV
 *    weight's rows are [all query heads | all key heads | all value heads], head-major.
 */
#ifndef EXE_H
#define EXE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct exe_model exe_model_t;

enum exe_status {
    EXE_OK = 0,
    EXE_ERR_ARG = -1,           /* NULL pointer, negative count, bad enum value */
    EXE_ERR_SHAPE = -2,         /* config/shape not supported by the kernels */
    EXE_ERR_OOM_KV = -3,        /* key/value pool or a sequence's reserved capacity exhausted */
    EXE_ERR_BAD_SEQ = -4,       /* unknown, duplicate, already-live or released sequence id */
    EXE_ERR_BAD_LENGTH = -5,    /* a length argument contradicts the library's own bookkeeping */
    EXE_ERR_HIP = -6,           /* a HIP call failed (message carries the HIP error string) */
    EXE_ERR_UNIMPLEMENTED = -7
};

enum { EXE_ARCH_DECODER_ONLY = 0, EXE_ARCH_ENC_DEC = 1 };
enum { EXE_ACT_RELU = 0, EXE_ACT_GELU = 1 };          /* GELU is the erf form */
enum { EXE_NORM_LAYERNORM = 0, EXE_NORM_RMSNORM = 1 };
enum { EXE_POS_LEARNED = 0, EXE_POS_RELBIAS = 1, EXE_POS_NONE = 2 };
enum { EXE_DTYPE_F32 = 0, EXE_DTYPE_BF16 = 1 };
enum { EXE_SCALE_RSQRT_DH = 0, EXE_SCALE_NONE = 1 };

typedef struct exe_config {
    int32_t arch;            /* EXE_ARCH_* */
    int32_t n_layers;        /* decoder-only: layers; enc-dec: encoder layers */
    int32_t n_dec_layers;    /* enc-dec: decoder layers; 0 otherwise */
    int32_t d_model, n_heads, head_dim, d_ff, vocab;
    int32_t max_pos;         /* rows of the learned position table (EXE_POS_LEARNED) */
    int32_t act, norm, pos;
    int32_t rel_buckets, rel_max_dist;   /* EXE_POS_RELBIAS: T5 bucket scheme parameters */
    int32_t cross_rel_bias;  /* enc-dec: 1 = cross-attention adds a bidirectional relative-position bias */
    int32_t dtype;           /* storage type of weights, activations between kernels and the K/V cache */
    int32_t has_embed;       /* 0: callers pass hidden states [tokens, d_model] instead of token ids */
    int32_t has_lm_head;     /* 0: calls return hidden states instead of logits/tokens */
    int32_t scale_mode;      /* EXE_SCALE_* for attention scores */
    float norm_eps;
    uint64_t kv_pool_bytes;  /* size of the key/value pool the model allocates */
    int32_t max_seqs;        /* sequence ids are 0 .. max_seqs-1 */
    int32_t max_batch_tokens;/* largest sum of input lengths in one exe_encode (workspace size) */
    int32_t max_batch_seqs;  /* largest number of sequences in one exe_encode / exe_decode_step call */
    int32_t kv_block_size;   /* 0: every sequence's K/V entries live in one extent of the pool with a reserved capacity.
                              * A power of two in [8, 4096]: paged pool (Section 2: paging applied to the memorization
                              * cache) -- the pool is cut into blocks of that many positions, a sequence takes blocks as
                              * it grows (reserve_lengths are then only validated), none is wasted on capacity not yet
                              * used.  Decoder-only models only (else EXE_ERR_UNIMPLEMENTED). */
} exe_config_t;

/* A weight tensor: device pointer, dtype = config.dtype. */
typedef struct exe_tensor { const void* ptr; } exe_tensor_t;

/*
 * Weight order (paper Section 2 names the pieces; the layout is this library's):
 *  decoder-only: [tok_emb [V,d]] (if has_embed or has_lm_head), [pos_emb [max_pos,d]] (if has_embed and
 *    learned positions), then per layer: ln1_g, ln1_b, w_qkv [3*H*dh, d], b_qkv, w_o [d, H*dh], b_o,
 *    ln2_g, ln2_b, w_1 [d_ff, d], b_1, w_2 [d, d_ff], b_2; then lnf_g, lnf_b (if has_lm_head).
 *    The LM head is tied to tok_emb, no bias.
 *  enc-dec: tok_emb, enc_rel_bias [buckets, H], dec_rel_bias [buckets, H], [cross_rel_bias [buckets, H]],
 *    per encoder layer: rms1_g, w_qkv, w_o, rms2_g, w_1, w_2; enc_final_g;
 *    per decoder layer: rms1_g, w_qkv, w_o, rmsx_g, w_xq [H*dh, d], w_xkv [2*H*dh, d], w_xo, rms3_g, w_1, w_2;
 *    dec_final_g.  No biases; logits = (final-normed hidden * d^-1/2) . tok_emb^T.
 */
int exe_expected_weights(const exe_config_t* cfg);   /* number of tensors, or a negative status */

/* Creates a model.  `weights` (host array of n_weights entries) are device tensors BORROWED until
 * exe_model_free.  `hip_stream` is a hipStream_t (NULL = the default stream) on which all work is
 * enqueued.  Allocates the K/V pool (cfg->kv_pool_bytes) and the activation workspace. */
int exe_model_load(const exe_config_t* cfg, const exe_tensor_t* weights, int32_t n_weights,
                   void* hip_stream, exe_model_t** out);
int exe_model_free(exe_model_t* m);

/*
 * Encode (prefill) n sequences (Section 2: "encoding the input once").
 *  seq_ids [n] host: caller-chosen, unique, not live, in [0, max_seqs).
 *  input_lengths [n] host (>= 1); tokens_packed [sum lengths] host, sequence after sequence
 *    (ignored if !has_embed; then hidden_in [sum lengths, d_model] device is read instead).
 *  reserve_lengths [n] host, nullable: K/V capacity of each sequence in positions (decoder-only: input +
 *    all outputs; enc-dec: decoder positions).  NULL reserves input+256 (decoder-only, capped at max_pos
 *    for learned positions) or 256 (enc-dec).
 *  next_tokens [n] host, nullable: decoder-only with LM head: greedy first generated token (lowest index
 *    on ties).  enc-dec: not written (the encoder generates nothing).
 *  out_device nullable device: decoder-only with LM head: float logits [n, vocab] of the last position;
 *    decoder-only without LM head: hidden states [sum lengths, d_model] in dtype; enc-dec: encoder output
 *    [sum lengths, d_model] in dtype.
 * On any error nothing is admitted (no sequence becomes live).
 */
int exe_encode(exe_model_t* m, int32_t n, const int32_t* seq_ids, const int32_t* input_lengths,
               const int32_t* tokens_packed, const int32_t* reserve_lengths, const void* hidden_in,
               int32_t* next_tokens, void* out_device);

/*
 * One decode iteration for n live sequences (Section 2: "each decoding iteration producing a single
 * output token"; the batch may mix sequences from different encode calls and shrinks as sequences finish).
 *  tokens_in [n] host: the token fed at this step (decoder-only: the previously generated token;
 *    enc-dec: the start token, then the previously generated token).  Ignored if !has_embed: then
 *    hidden_in [n, d_model] device.
 *  kv_lengths [n] host: self-attention K/V length AFTER this token is appended; must equal the library's
 *    own count + 1, else EXE_ERR_BAD_LENGTH and no state changes.
 *  next_tokens [n] host nullable; out_device nullable: float logits [n, vocab] or hidden [n, d_model].
 */
int exe_decode_step(exe_model_t* m, int32_t n, const int32_t* seq_ids, const int32_t* tokens_in,
                    const int32_t* kv_lengths, const void* hidden_in, int32_t* next_tokens, void* out_device);

/* Early termination: the sequences leave; their K/V extents return to the pool. */
int exe_seq_release(exe_model_t* m, int32_t n, const int32_t* seq_ids);

/* Current K/V length of a live sequence (decoder-only: positions memoized; enc-dec: decoder positions),
 * or a negative status. */
int exe_seq_length(exe_model_t* m, int32_t seq_id);

/*
 * K/V hand-over (Section 3 "XRunner": for WAA scheduling the key/value cache entries of a query move from the
 * encoding GPU to the decoding GPU through CPU memory).  exe_seq_export copies a live sequence's entries, without
 * the unused capacity of its extent, into a host buffer: self-attention entries
 * [decoder layer][K|V][head][kv_len][head_dim] in the storage type, then (encoder-decoder models) the cross-attention
 * entries [decoder layer][K|V][head][cross_len][head_dim]; the sequence stays live (release it separately).
 * exe_seq_import admits those entries under a free sequence id of a model of the same shape and type (this or
 * another one, on any GPU), with capacity for reserve_length positions (<= 0: kv_len + 256; clamped to the position
 * table), after which exe_decode_step continues the sequence from the token the caller kept.
 * host_buf: host memory (pinned memory makes the copy faster), buf_bytes >= exe_seq_export_bytes; both calls
 * synchronise the model's stream.  Errors: EXE_ERR_BAD_SEQ (id not live / already live), EXE_ERR_ARG (buffer too
 * small), EXE_ERR_BAD_LENGTH (state inconsistent with the model), EXE_ERR_OOM_KV (pool full; nothing is admitted).
 */
typedef struct exe_seq_state {
    int32_t kv_len;                /* self-attention positions memoized */
    int32_t cross_len;             /* encoder length of an encoder-decoder sequence, else 0 */
} exe_seq_state_t;
int64_t exe_seq_export_bytes(exe_model_t* m, int32_t seq_id);       /* bytes, or a negative status */
int exe_seq_export(exe_model_t* m, int32_t seq_id, void* host_buf, uint64_t buf_bytes, exe_seq_state_t* state);
int exe_seq_import(exe_model_t* m, int32_t seq_id, const void* host_buf, uint64_t buf_bytes,
                   const exe_seq_state_t* state, int32_t reserve_length);

/*
 * Extent relocation and compaction (Section 3 "XRunner": early termination of completed queries comes with the
 * compaction of the key/value cache entries of the terminated ones).  A sequence's entries live in one extent of the
 * pool with room for a reserved number of positions, so terminated sequences leave holes of different sizes.
 *  exe_seq_reserve moves a live sequence's self-attention entries into a new extent with room for reserve_length
 *    positions (>= its current length, rounded up to 8; growing lets a sequence outlive its first reservation,
 *    shrinking returns capacity it will not use).  EXE_ERR_BAD_SEQ, EXE_ERR_BAD_LENGTH (shorter than the current
 *    length, or beyond the position table), EXE_ERR_OOM_KV (no free extent of that size; nothing changes).
 *  exe_kv_compact slides the extents of all live sequences towards the start of the pool, in address order, so
 *    that the free space becomes one piece; *moved_bytes (nullable) receives the bytes copied.  An extent whose
 *    move would overlap itself is copied in pieces no longer than the distance moved; one that would need more
 *    than 64 pieces stays where it is.
 * Both enqueue device-to-device copies on the model's stream, in order with the model's kernels, and return
 * without waiting; sequence ids, lengths and results of later calls are unchanged by them.
 */
int exe_seq_reserve(exe_model_t* m, int32_t seq_id, int32_t reserve_length);
int exe_kv_compact(exe_model_t* m, uint64_t* moved_bytes);

/* Pool accounting (bytes). Any pointer may be NULL. */
int exe_kv_stats(exe_model_t* m, uint64_t* pool_bytes, uint64_t* used_bytes, uint64_t* largest_free_bytes,
                 int32_t* live_seqs);

/*
 * Latency table for a scheduler (Section 3 "XProfiler": for a single layer, the attention kernel is
 * timed separately from the rest of the layer, over batch sizes and sequence lengths).
 *  phase 0: encode -- `batch` sequences of `length` input tokens.
 *  phase 1: decode -- `batch` sequences whose self-attention K/V length (after the append) is `length`;
 *           encoder-decoder models: cross-attention length is `length`, self-attention length max(1, length/12).
 *  dist NULL or kind 0: every sequence has exactly `length`; kind 1: lengths ~ Normal(length, dist->std) rounded
 *  and clipped to [dist->lo, dist->hi], drawn from dist->seed (the row's `ragged` is then 1).
 * One row per (batch, length) pair, batch-major.  A single layer (layer 0's weights) runs n_steps timed
 * repetitions after 3 warm-up ones; only that layer's K/V is allocated (from the model's pool, which must
 * hold no live sequence; it is returned afterwards).  attn_ms_per_layer is the attention kernels' own time
 * (HIP events around each launch); rest_ms_per_layer is the whole layer's latency (events around the layer,
 * launch gaps included) minus it; std_ms is the standard deviation of the whole-layer latency; head_ms is the
 * final norm + LM head + argmax (encoder-decoder encode: final norm + every decoder layer's cross K/V
 * projection); full_step_ms = layers * (attn + rest) + head_ms is an extrapolation to the full depth.
 */
typedef struct exe_profile_row {
    int32_t phase, batch, length, ragged;
    int32_t total_tokens;          /* sum of the row's lengths */
    float attn_ms_per_layer, rest_ms_per_layer, head_ms, full_step_ms, std_ms;
    int32_t n_timed;
} exe_profile_row_t;
typedef struct exe_length_dist {
    int32_t kind;                  /* 0 fixed (= the row's length), 1 normal, rounded, clipped to [lo, hi] */
    float mean, std;
    int32_t lo, hi;
    uint64_t seed;
} exe_length_dist_t;
int exe_profile(exe_model_t* m, int32_t phase, const int32_t* batch_sizes, int32_t n_batch,
                const int32_t* lengths, int32_t n_len, const exe_length_dist_t* dist /* nullable */,
                int32_t n_steps, exe_profile_row_t* rows, int32_t rows_cap, int32_t* n_rows);

/*
 * RRA schedule on one GPU (Section 4 "RRA Scheduling": encode once, then decode for N_D iterations, repeatedly;
 * the encoding batch B_E equals the number of queries completed in the previous N_D decoding iterations, which
 * keeps the decoding batch near B_D; Section 5 "dynamic workload adjustment": the sum of input lengths of an
 * encoding batch is kept within a tolerance of the average encoder workload).
 * All n_requests are queued at time 0 and served first-come first-served with forced output lengths (Section 7:
 * decoding continues for the given length, no end-of-sequence token); finished sequences leave the decode
 * batch at once (early termination).  Needs a model with token embedding and LM head and no live sequence;
 * uses sequence ids 0 .. decode_batch-1.
 *  input_lengths, output_lengths [n_requests] host (output_lengths >= 1); tokens_packed [sum input_lengths] host.
 *  out_tokens [sum output_lengths] host, nullable: the generated tokens, request after request.
 */
typedef struct exe_rra_config {
    int32_t decode_batch;        /* B_D: live sequences the schedule keeps in the decode batch */
    int32_t n_decode;            /* N_D: decode iterations between two encoding phases */
    int32_t max_encode_batch;    /* most sequences per exe_encode call (<= max_batch_seqs) */
    int32_t adjust;              /* 1: dynamic workload adjustment of the encoding batch */
    float workload_tolerance;    /* adjust: an encoding phase takes at most (1 + tol) * B_E * mean input length tokens */
} exe_rra_config_t;
typedef struct exe_rra_stats {
    double wall_s, encode_s, decode_s;
    int64_t encoded_tokens, generated_tokens;
    int32_t encode_phases, encode_calls, decode_iterations;
    double mean_decode_batch;                 /* over decode iterations */
    double latency_mean_s, latency_p50_s, latency_p99_s, latency_max_s;   /* admission (encode start) -> last token */
    double queue_p99_s;                       /* time 0 -> admission */
} exe_rra_stats_t;
int exe_run_rra(exe_model_t* m, const exe_rra_config_t* cfg, int32_t n_requests, const int32_t* input_lengths,
                const int32_t* output_lengths, const int32_t* tokens_packed, int32_t* out_tokens,
                exe_rra_stats_t* stats);

/*
 * Per-kernel-class timing (HIP events on the model's stream around every launch of the class) with the
 * algorithmic bytes and flops of those launches; used to report achieved GB/s or TFLOP/s.
 * Enabling it serialises nothing but adds two event records per launch.
 */
/* EXE_K_GEMM_TILE: GEMM launches with more than 256 rows (MFMA-bound); EXE_K_GEMM_SKINNY: at most 256 rows
 * (the weights are streamed once: HBM-bound). */
enum { EXE_K_GEMM_TILE = 0, EXE_K_GEMM_SKINNY = 1, EXE_K_PREFILL_ATTN = 2, EXE_K_DECODE_ATTN = 3,
       EXE_K_CROSS_ATTN = 4, EXE_K_NORM = 5, EXE_K_OTHER = 6, EXE_K_COUNT = 7 };
typedef struct exe_kernel_time {
    int32_t kind;
    int64_t launches;
    double ms;                     /* summed event time */
    double bytes;                  /* algorithmic HBM bytes of those launches */
    double flops;                  /* algorithmic flops of those launches */
} exe_kernel_time_t;
int exe_kernel_timing(exe_model_t* m, int32_t enable);           /* also resets the accumulators */
int exe_kernel_times(exe_model_t* m, exe_kernel_time_t* rows /* [EXE_K_COUNT] */);

/*
 * Tooling of this library, no part of the paper's method and citing nothing from it: the per-kernel-class timing
 * above (exe_kernel_timing, exe_kernel_times), the single-operation entry points below (exe_op_*: device pointers,
 * enqueued on `hip_stream`, NOT synchronised; they run the same kernels the model calls use, for per-kernel
 * parity tests and micro-benchmarks), exe_probe_peaks and exe_probe_ingest.
 */
/* out = epilogue(alpha * A[M,K] . W[N,K]^T + bias):  out_mode 0: dtype out [M,N] with activation
 * act (-1 none, EXE_ACT_*); 1: float resid [M,N] += result; 2: float out [M,N].
 * workspace: device scratch of workspace_bytes (>= exe_op_gemm_workspace), may be NULL if that is 0. */
int exe_op_gemm(void* hip_stream, int32_t dtype, int32_t M, int32_t N, int32_t K, const void* A,
                const void* W, const void* bias, int32_t act, float alpha, int32_t out_mode, void* out,
                void* workspace, uint64_t workspace_bytes);
uint64_t exe_op_gemm_workspace(int32_t dtype, int32_t M, int32_t N, int32_t K);
/* exe_op_gemm for callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the split-K partial sums live in a static device array
 * inside the library (exe_op_gemm_noalloc_max_workspace() bytes, 64 MiB, held on every GPU the library runs on until
 * the process ends), whose address on the current device is looked up once per device.  The call allocates
 * nothing, on the device or through any library.  Shapes whose partial sums do not fit (exe_op_gemm_workspace(...)
 * above the maximum) are rejected with EXE_ERR_SHAPE.  Nothing in the array needs clearing between calls (a call
 * writes every partial sum it later reads), but all calls on one GPU share it: calls that overlap on one GPU, on
 * different streams or from different threads, race.  Same arithmetic, kernels and results as exe_op_gemm. */
int exe_op_gemm_noalloc(void* hip_stream, int32_t dtype, int32_t M, int32_t N, int32_t K, const void* A, const void* W,
                        const void* bias, int32_t act, float alpha, int32_t out_mode, void* out);
uint64_t exe_op_gemm_noalloc_max_workspace(void);
/* How exe_op_gemm launches a shape (host function; lets a test assert that its cases cover every kernel
 * instantiation): *route 0 = MFMA tile kernel, 2 = plain-FMA kernel; *cfg = tile configuration (0 64x256, 1 128x256,
 * 2 256x256, 3 64x128, 4 128x128, 5 256x128 rows x features); *splits = split-K parts (> 1: float partials in the
 * workspace, summed in split order by a second kernel); *rows_first = rows of the first launch (M, unless the rows
 * beyond whole rounds of 256 x 256 tiles go to a second, separately planned launch: ask again with M - *rows_first). */
int exe_op_gemm_plan(int32_t dtype, int32_t M, int32_t N, int32_t K, int32_t* route, int32_t* cfg, int32_t* splits,
                     int32_t* rows_first);
/* exe_op_gemm for bf16 operands whose rows are lda / ldw elements apart (>= K, multiples of 8; K a multiple of 64;
 * shapes the MFMA tile kernel serves only).  Row strides that are not a multiple of 4 KiB spread a tile's rows
 * over more memory channels. */
int exe_op_gemm_ld(void* hip_stream, int32_t dtype, int32_t M, int32_t N, int32_t K, const void* A, int32_t lda,
                   const void* W, int32_t ldw, const void* bias, int32_t act, float alpha, int32_t out_mode, void* out,
                   void* workspace, uint64_t workspace_bytes);
/* rows of float x [*, d] (row_index nullable selects rows) -> dtype out [rows, d] */
int exe_op_norm(void* hip_stream, int32_t dtype, int32_t rms, const float* x, const int32_t* row_index,
                int32_t rows, int32_t d, const void* gain, const void* shift, float eps, float out_scale,
                void* out);
/* Ragged prefill attention over packed qkv [T, 3*H*dh] (dtype): cu_seqlens [n_seqs+1] host.
 * causal 0/1; bias_by_dist nullable device float [H, 2*bias_radius+1] indexed by clamp(key-query)+radius.
 * out [T, H*dh] dtype. */
int exe_op_prefill_attention(void* hip_stream, int32_t dtype, int32_t n_seqs, const int32_t* cu_seqlens,
                             const void* qkv, int32_t H, int32_t dh, float scale, int32_t causal,
                             const float* bias_by_dist, int32_t bias_radius, void* out, int32_t force_generic);
/* The launch order of the MFMA prefill kernel's query tiles (host function; lets a test check the list without a
 * GPU): for sequences of the given lengths (host, each >= 1), pairs (sequence, first query row) of the 128-row tiles,
 * written to tiles[2 * k], tiles[2 * k + 1].  Sequences go longest first (ties in their given order), a sequence's
 * tiles together, last rows first.  *n_tiles receives the count; cap = capacity of tiles in pairs; a list that does
 * not fit is EXE_ERR_ARG with *n_tiles set to the count needed. */
int exe_op_prefill_tiles(int32_t n_seqs, const int32_t* lengths, int32_t* tiles, int32_t cap, int32_t* n_tiles);
/* Decode attention: q [B, H*dh] dtype; per sequence b the keys are at kv + k_offset[b] (elements) laid out
 * [H][cap[b]][dh] and the values at kv + k_offset[b] + H*cap[b]*dh; len[b] keys are valid; the query's
 * position is qpos[b] (for the bias only: index clamp(j - qpos)+radius).  All arrays device.  out [B, H*dh]. */
int exe_op_decode_attention(void* hip_stream, int32_t dtype, int32_t B, const void* q, int32_t q_stride,
                            const void* kv, const int64_t* k_offset, const int32_t* cap, const int32_t* len,
                            const int32_t* qpos, int32_t H, int32_t dh, float scale,
                            const float* bias_by_dist, int32_t bias_radius, void* out);
/* Decode attention over a paged cache (Section 2: paging applied to the key/value memorization cache; the
 * evaluation notes that paging would further help WAA scheduling): as exe_op_decode_attention, but the entries of one
 * layer live in blocks of block_size positions (a power of two in [8, 4096]).  Block b starts at
 * kv_blocks + b * 2*H*block_size*dh elements and holds [K|V][H][block_size][dh]; block_table [B, max_blocks] (device)
 * lists each sequence's blocks in position order, so position p of sequence b is row p % block_size of block
 * block_table[b][p / block_size].  new_kv_offset > 0: the newest position (len[b] - 1) is not in the cache yet; its
 * key / value rows of (b, head) are read from q + b*q_stride + new_kv_offset + head*dh and
 * q + b*q_stride + 2*new_kv_offset + head*dh and stored into the cache by this call (q then is the packed output of
 * the QKV projection).  The caller guarantees that every table entry a sequence needs names a block inside the pool
 * and that no block is shared between sequences. */
int exe_op_decode_attention_paged(void* hip_stream, int32_t dtype, int32_t B, const void* q, int32_t q_stride,
                                  const void* kv_blocks, const int32_t* block_table, int32_t max_blocks,
                                  int32_t block_size, const int32_t* len, const int32_t* qpos, int32_t H, int32_t dh,
                                  float scale, const float* bias_by_dist, int32_t bias_radius, int32_t new_kv_offset,
                                  void* out);
/* Host-side replay of the row indexing of the paged decode-attention kernel for one sequence of `len` cached rows
 * (the same index functions the kernel calls, for the launch shape of n_waves = 4 or 16 waves): returns 0 when every
 * row read is a cached row inside the block its table look-up names and every cached row is read exactly once, else
 * the number of violations (> 0), or a negative status for bad arguments. */
int exe_op_paged_index_check(int32_t dtype, int32_t dh, int32_t block_size, int32_t n_waves, int32_t len);
/* Measured ceilings of this machine, to set beside the nominal peaks when a kernel is judged against its roofline:
 * *hbm_read_bytes_per_s = rate of a plain streaming read of read_bytes bytes (0 = 4 GiB; allocated and
 * freed by the call), *mfma_bf16_flops_per_s = rate of back-to-back bf16 16x16x32 MFMAs on all compute units at the
 * clock that load sustains.  Either pointer may be NULL.  Synchronises the stream; host pointers. */
int exe_probe_peaks(void* hip_stream, uint64_t read_bytes, double* hbm_read_bytes_per_s, double* mfma_bf16_flops_per_s);
/* Rate at which the compute units take tile data in (tooling, like exe_probe_peaks): one workgroup of `waves` waves
 * (1, 2, 4, 8, 16) per compute unit reads a private region of region_bytes `passes` times, each wave issuing batches
 * of loads_per_batch (2, 4, 8, 16) wave-wide 16-byte loads (1 KB each) with the batch before still in flight, so
 * waves x loads_per_batch (at most 64) to twice that many KB are in flight per compute unit.  mode 0 = loads to
 * registers, 1 = the same nontemporal, 2 = direct global->LDS loads (the tile loader of the GEMM and prefill
 * kernels), 3 = the same nontemporal.  A small region with many passes stays in L2 (the L1 <-> L2 path of a compute
 * unit); a region of megabytes with passes = 1 is a stream from HBM.  row_bytes = 0 reads the region front to back;
 * row_bytes > 0 (modes 2 and 3, waves x loads_per_batch = 16, a multiple of 128) makes the region a panel of 128 rows
 * of row_bytes bytes, walked 128 bytes at a time with 8 rows per wave-load, as the loader of a 128-row operand tile of a
 * row-major matrix does (region_bytes is then 128 x row_bytes).  region_bytes must be a multiple of
 * waves x loads_per_batch KB.  *bytes_per_s = bytes read per second over all compute units.  Allocates and frees its
 * buffer, synchronises the stream; host pointer. */
int exe_probe_ingest(void* hip_stream, int32_t mode, uint64_t region_bytes, int32_t passes, int32_t waves,
                     int32_t loads_per_batch, int32_t row_bytes, double* bytes_per_s);
/* argmax over each row of float logits [rows, n] -> int32 out [rows]; lowest index on ties */
int exe_op_argmax(void* hip_stream, const float* logits, int32_t rows, int32_t n, int32_t* out);
/* T5 bucket of rel = key - query as this library computes it (host function, exact integer arithmetic) */
int exe_rel_bucket(int32_t rel, int32_t bidirectional, int32_t n_buckets, int32_t max_dist);

const char* exe_last_error(void);
const char* exe_version(void);

#ifdef __cplusplus
}
#endif
#endif
