/*
 * CPU oracle for batched Transformer execution (encode once, decode iteratively with a
 * key/value memo cache) -- the computation described in the paper's background section
 * (Section 2: query/key/value, dot product + softmax, context vector, feed-forward network,
 * residual connections; self- vs cross-attention; incremental decoding with memoized keys/values).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, one-sequence-at-a-time definition of the
 * result, used only by tests, by the smoke check and by the benchmark's cpu_baseline leg.  It
 * shares no code, header, table or constant with the GPU library and must never be called from
 * the product path.
 *
 * Arithmetic type: `REAL` (compile-time; the build makes one library with float and one with
 * double).  Weights are always passed as float arrays holding the already-rounded storage values.
 * No intermediate rounding to a narrower type happens anywhere.
 *
 * Pinning status (see tests, "not gpu"):
 *   orc_linear, orc_layernorm, orc_rmsnorm, orc_act, orc_attention_row, orc_argmax
 *        -- pinned against library routines in float64, closed forms and special cases.
 *   orc_bucket -- pinned against exact integer arithmetic and the scheme's stated properties.
 *   model forward (decoder-only and encoder-decoder) -- pinned by: cached decode == full-prefix
 *        recomputation, causality, softmax row sums, identity-layer closed form, an independent
 *        float64 re-derivation of a whole forward pass with library routines, batch independence.
 *   parity unpinned: the conventions the paper does not fix (pre-norm placement, eps values,
 *        erf-GELU, bias placement, tied LM head, T5 d^-1/2 logit scale, cross-attention bias)
 *        are definitions of this build, identical on both sides.
 */
#ifndef EXE_ORACLE_H
#define EXE_ORACLE_H

#include <stdint.h>

#ifndef REAL
#define REAL double
#endif
typedef REAL real;

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t arch;          /* 0 decoder-only, 1 encoder-decoder */
    int32_t n_layers;      /* decoder-only: layers; enc-dec: encoder layers */
    int32_t n_dec_layers;  /* enc-dec: decoder layers */
    int32_t d_model, n_heads, head_dim, d_ff, vocab, max_pos;
    int32_t act;           /* 0 relu, 1 gelu (erf) */
    int32_t norm;          /* 0 layernorm, 1 rmsnorm */
    int32_t pos;           /* 0 learned, 1 relative-position bias, 2 none */
    int32_t rel_buckets, rel_max_dist, cross_rel_bias;
    int32_t has_embed, has_lm_head;
    int32_t scale_mode;    /* 0: 1/sqrt(head_dim), 1: none */
    float norm_eps;
} orc_config;

typedef struct orc_model orc_model;

/* ---- primitives (each is the plain definition of one operation) ---- */

/* y[i][j] = (b ? b[j] : 0) + sum_k x[i][k] * W[j][k];  W is [out][in] row-major. */
void orc_linear(const real* x, int rows, int in, const float* W, const float* b, int out, real* y);
/* y = (x - mean) / sqrt(var + eps) * g + b, biased variance over the row. */
void orc_layernorm(const real* x, int rows, int d, const float* g, const float* b, real eps, real* y);
/* y = x / sqrt(mean(x^2) + eps) * g */
void orc_rmsnorm(const real* x, int rows, int d, const float* g, real eps, real* y);
/* in place: kind 0 relu, 1 gelu(x) = x/2 (1 + erf(x/sqrt 2)) */
void orc_act(real* x, int64_t n, int kind);
/* one query row against nk keys/values: s_j = scale * q.k_j + (bias ? bias[j] : 0);
 * p = softmax(s) with the maximum subtracted; out = sum_j p_j v_j.  probs (nullable) receives p.
 * k_j = K + j*stride_k, v_j = V + j*stride_v.  Returns sum_j p_j. */
real orc_attention_row(const real* q, const real* K, int64_t stride_k, const real* V, int64_t stride_v,
                       int nk, int dh, real scale, const real* bias, real* out, real* probs);
/* index of the largest element, lowest index on ties */
int orc_argmax(const real* x, int n);
/* T5 relative-position bucket of rel = key_pos - query_pos */
int orc_bucket(int rel, int bidirectional, int n_buckets, int max_dist);

/* ---- model ---- */

/* weights: float arrays in the documented order (token embedding, position embedding, per-layer
 * tensors, final norm; for enc-dec: embedding, bias tables, encoder layers, encoder final gain,
 * decoder layers, decoder final gain).  Borrowed until orc_free. Returns NULL on a bad count. */
orc_model* orc_create(const orc_config* cfg, const float* const* weights, int n_weights, int max_seqs);
void orc_free(orc_model* m);
int orc_expected_weights(const orc_config* cfg);
int orc_threads(void);
int orc_real_bytes(void);

/* Encode one sequence into slot `seq` (keys/values are memoized).
 * decoder-only: tokens[n] (or hidden_in [n][d] if !has_embed); logits_last [vocab] (or hidden_out
 *   [n][d] if !has_lm_head) receives the output; returns the greedy next token (or 0).
 * enc-dec: runs the encoder and stores each decoder layer's cross keys/values; returns 0.
 * Returns -1 on a bad argument. */
int orc_encode(orc_model* m, int seq, int n, const int32_t* tokens, const real* hidden_in,
               real* logits_last, real* hidden_out);
/* One decode iteration for slot `seq` with input token `token` (or hidden_in [d]).
 * Writes logits [vocab] (or hidden_out [d]); returns the greedy next token. */
int orc_decode(orc_model* m, int seq, int32_t token, const real* hidden_in, real* logits, real* hidden_out);
void orc_release(orc_model* m, int seq);
int orc_seq_len(const orc_model* m, int seq);

/* Full recomputation without any cache.
 * decoder-only: all n positions; logits_all [n][vocab] (or hidden_all [n][d]).
 * enc-dec: encoder on tokens[n], then decoder teacher-forced on dec_tokens[n_dec]
 *   (dec_tokens[0] is the start token); logits_all [n_dec][vocab]. */
int orc_full(orc_model* m, int n, const int32_t* tokens, const real* hidden_in,
             int n_dec, const int32_t* dec_tokens, real* logits_all, real* hidden_all);

/* largest |sum_j p_j - 1| over every attention row evaluated since the last reset */
real orc_rowsum_dev(orc_model* m, int reset);

#ifdef __cplusplus
}
#endif
#endif
