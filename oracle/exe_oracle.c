/*
 * CPU oracle: plain definition of encode-once / decode-iteratively Transformer inference with a
 * memoized key/value cache (paper, Section 2).  TEST INFRASTRUCTURE -- see exe_oracle.h.
 *
 * One sequence at a time, no packing, no tiling, no fusion.  OpenMP only spreads independent output
 * elements (output features of a linear map, (position, head) pairs of attention) over host threads.
 */
#include "exe_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ primitives */

void orc_linear(const real* x, int rows, int in, const float* W, const float* b, int out, real* y)
{
#pragma omp parallel for schedule(static)
    for (int j = 0; j < out; ++j) {
        const float* w = W + (int64_t)j * in;
        for (int i = 0; i < rows; ++i) {
            const real* xi = x + (int64_t)i * in;
            real acc = 0;
#pragma omp simd reduction(+ : acc)
            for (int k = 0; k < in; ++k) acc += xi[k] * (real)w[k];
            y[(int64_t)i * out + j] = acc + (b ? (real)b[j] : (real)0);
        }
    }
}

void orc_layernorm(const real* x, int rows, int d, const float* g, const float* b, real eps, real* y)
{
    for (int i = 0; i < rows; ++i) {
        const real* xi = x + (int64_t)i * d;
        real* yi = y + (int64_t)i * d;
        real mean = 0;
        for (int k = 0; k < d; ++k) mean += xi[k];
        mean /= d;
        real var = 0;
        for (int k = 0; k < d; ++k) var += (xi[k] - mean) * (xi[k] - mean);
        var /= d;
        real r = 1 / sqrt(var + eps);
        for (int k = 0; k < d; ++k) yi[k] = (xi[k] - mean) * r * (real)g[k] + (real)b[k];
    }
}

void orc_rmsnorm(const real* x, int rows, int d, const float* g, real eps, real* y)
{
    for (int i = 0; i < rows; ++i) {
        const real* xi = x + (int64_t)i * d;
        real* yi = y + (int64_t)i * d;
        real ms = 0;
        for (int k = 0; k < d; ++k) ms += xi[k] * xi[k];
        ms /= d;
        real r = 1 / sqrt(ms + eps);
        for (int k = 0; k < d; ++k) yi[k] = xi[k] * r * (real)g[k];
    }
}

void orc_act(real* x, int64_t n, int kind)
{
    if (kind == 0) {
        for (int64_t i = 0; i < n; ++i) x[i] = x[i] > 0 ? x[i] : 0;
    } else {
        for (int64_t i = 0; i < n; ++i) {
            double v = (double)x[i];
            x[i] = (real)(0.5 * v * (1.0 + erf(v * 0.70710678118654752440)));
        }
    }
}

real orc_attention_row(const real* q, const real* K, int64_t stride_k, const real* V, int64_t stride_v,
                       int nk, int dh, real scale, const real* bias, real* out, real* probs)
{
    real* s = (real*)malloc(sizeof(real) * (size_t)(nk > 0 ? nk : 1));
    real mx = -INFINITY;
    for (int j = 0; j < nk; ++j) {
        const real* kj = K + (int64_t)j * stride_k;
        real dot = 0;
        for (int c = 0; c < dh; ++c) dot += q[c] * kj[c];
        s[j] = dot * scale + (bias ? bias[j] : (real)0);
        if (s[j] > mx) mx = s[j];
    }
    real denom = 0;
    for (int j = 0; j < nk; ++j) {
        s[j] = exp(s[j] - mx);
        denom += s[j];
    }
    real psum = 0;
    for (int c = 0; c < dh; ++c) out[c] = 0;
    for (int j = 0; j < nk; ++j) {
        real p = s[j] / denom;
        psum += p;
        if (probs) probs[j] = p;
        const real* vj = V + (int64_t)j * stride_v;
        for (int c = 0; c < dh; ++c) out[c] += p * vj[c];
    }
    free(s);
    return psum;
}

int orc_argmax(const real* x, int n)
{
    int best = 0;
    for (int i = 1; i < n; ++i)
        if (x[i] > x[best]) best = i;
    return best;
}

/* T5 bucket scheme.  rel = key position - query position.
 * bidirectional: half the buckets per sign (keys after the query get the upper half); within a sign
 *   the first half of those are exact distances, the rest are logarithmically spaced up to max_dist.
 * unidirectional: keys after the query count as distance 0; same exact/log split over all buckets. */
int orc_bucket(int rel, int bidirectional, int n_buckets, int max_dist)
{
    int base = 0, nb = n_buckets, n;
    if (bidirectional) {
        nb = n_buckets / 2;
        if (rel > 0) base = nb;
        n = rel < 0 ? -rel : rel;
    } else {
        n = rel < 0 ? -rel : 0;
    }
    int exact = nb / 2;
    if (n < exact) return base + n;
    double t = log((double)n / (double)exact) / log((double)max_dist / (double)exact);
    int b = exact + (int)floor(t * (double)(nb - exact) + 1e-9);
    if (b > nb - 1) b = nb - 1;
    return base + b;
}

/* ------------------------------------------------------------------ model */

typedef struct {
    int live;
    int len;        /* decoder-only: memoized positions; enc-dec: decoder positions so far */
    int cap;
    int n_in;       /* enc-dec: encoder length */
    real** K;       /* [layers][cap*inner] self-attention keys */
    real** V;
    real** XK;      /* enc-dec: [dec layers][n_in*inner] cross keys */
    real** XV;
} orc_seq;

struct orc_model {
    orc_config c;
    const float* const* w;
    int n_w;
    int max_seqs;
    orc_seq* seqs;
    real rowsum_dev;
};

int orc_expected_weights(const orc_config* c)
{
    if (c->arch == 0) {
        int n = 0;
        if (c->has_embed || c->has_lm_head) n += 1;
        if (c->has_embed && c->pos == 0) n += 1;
        n += 12 * c->n_layers;
        if (c->has_lm_head) n += 2;
        return n;
    }
    return 1 + 2 + (c->cross_rel_bias ? 1 : 0) + 6 * c->n_layers + 1 + 10 * c->n_dec_layers + 1;
}

int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int orc_real_bytes(void) { return (int)sizeof(real); }

orc_model* orc_create(const orc_config* cfg, const float* const* weights, int n_weights, int max_seqs)
{
    if (!cfg || !weights || n_weights != orc_expected_weights(cfg) || max_seqs <= 0) return NULL;
    orc_model* m = (orc_model*)calloc(1, sizeof(orc_model));
    m->c = *cfg;
    const float** w = (const float**)malloc(sizeof(float*) * (size_t)n_weights);
    memcpy(w, weights, sizeof(float*) * (size_t)n_weights);
    m->w = w;
    m->n_w = n_weights;
    m->max_seqs = max_seqs;
    m->seqs = (orc_seq*)calloc((size_t)max_seqs, sizeof(orc_seq));
    return m;
}

static void seq_clear(orc_model* m, orc_seq* s)
{
    int nl = m->c.arch == 0 ? m->c.n_layers : m->c.n_dec_layers;
    for (int l = 0; l < nl; ++l) {
        if (s->K) free(s->K[l]);
        if (s->V) free(s->V[l]);
        if (s->XK) free(s->XK[l]);
        if (s->XV) free(s->XV[l]);
    }
    free(s->K); free(s->V); free(s->XK); free(s->XV);
    memset(s, 0, sizeof(*s));
}

void orc_release(orc_model* m, int seq)
{
    if (!m || seq < 0 || seq >= m->max_seqs) return;
    seq_clear(m, &m->seqs[seq]);
}

void orc_free(orc_model* m)
{
    if (!m) return;
    for (int i = 0; i < m->max_seqs; ++i) seq_clear(m, &m->seqs[i]);
    free(m->seqs);
    free((void*)m->w);
    free(m);
}

int orc_seq_len(const orc_model* m, int seq)
{
    if (!m || seq < 0 || seq >= m->max_seqs || !m->seqs[seq].live) return -1;
    return m->seqs[seq].len;
}

real orc_rowsum_dev(orc_model* m, int reset)
{
    real r = m->rowsum_dev;
    if (reset) m->rowsum_dev = 0;
    return r;
}

static void note_rowsum(orc_model* m, real psum)
{
    real dev = fabs(psum - 1);
#pragma omp critical(orc_rowsum)
    if (dev > m->rowsum_dev) m->rowsum_dev = dev;
}

static void seq_reserve(orc_model* m, orc_seq* s, int need)
{
    int nl = m->c.arch == 0 ? m->c.n_layers : m->c.n_dec_layers;
    int64_t inner = (int64_t)m->c.n_heads * m->c.head_dim;
    if (!s->K) {
        s->K = (real**)calloc((size_t)nl, sizeof(real*));
        s->V = (real**)calloc((size_t)nl, sizeof(real*));
    }
    if (need <= s->cap) return;
    int cap = s->cap ? s->cap : 16;
    while (cap < need) cap *= 2;
    for (int l = 0; l < nl; ++l) {
        s->K[l] = (real*)realloc(s->K[l], sizeof(real) * (size_t)(cap * inner));
        s->V[l] = (real*)realloc(s->V[l], sizeof(real) * (size_t)(cap * inner));
    }
    s->cap = cap;
}

static void norm_rows(const orc_model* m, const real* x, int rows, const float* g, const float* b, real* y)
{
    if (m->c.norm == 0) orc_layernorm(x, rows, m->c.d_model, g, b, (real)m->c.norm_eps, y);
    else orc_rmsnorm(x, rows, m->c.d_model, g, (real)m->c.norm_eps, y);
}

static real score_scale(const orc_model* m)
{
    return m->c.scale_mode == 0 ? (real)(1.0 / sqrt((double)m->c.head_dim)) : (real)1;
}

/* position-wise feed-forward with residual: h += act(a W1^T + b1) W2^T + b2, a = norm(h) */
static void ffn_block(const orc_model* m, real* h, int rows, const float* ng, const float* nb,
                      const float* W1, const float* b1, const float* W2, const float* b2)
{
    int d = m->c.d_model, f = m->c.d_ff;
    real* a = (real*)malloc(sizeof(real) * (size_t)rows * d);
    real* u = (real*)malloc(sizeof(real) * (size_t)rows * f);
    real* o = (real*)malloc(sizeof(real) * (size_t)rows * d);
    norm_rows(m, h, rows, ng, nb, a);
    orc_linear(a, rows, d, W1, b1, f, u);
    orc_act(u, (int64_t)rows * f, m->c.act);
    orc_linear(u, rows, f, W2, b2, d, o);
    for (int64_t i = 0; i < (int64_t)rows * d; ++i) h[i] += o[i];
    free(a); free(u); free(o);
}

/* ---------------- decoder-only ---------------- */

typedef struct {
    const float *tok, *pos, *lnf_g, *lnf_b;
    int layer0;
} dec_only_w;

static dec_only_w dec_only_weights(const orc_model* m)
{
    dec_only_w r;
    memset(&r, 0, sizeof(r));
    int i = 0;
    if (m->c.has_embed || m->c.has_lm_head) r.tok = m->w[i++];
    if (m->c.has_embed && m->c.pos == 0) r.pos = m->w[i++];
    r.layer0 = i;
    i += 12 * m->c.n_layers;
    if (m->c.has_lm_head) { r.lnf_g = m->w[i++]; r.lnf_b = m->w[i++]; }
    return r;
}

static void embed_rows(const orc_model* m, const dec_only_w* W, int n, int pos0, const int32_t* tokens,
                       const real* hidden_in, real* h)
{
    int d = m->c.d_model;
    for (int i = 0; i < n; ++i)
        for (int k = 0; k < d; ++k) {
            if (m->c.has_embed) {
                real v = (real)W->tok[(int64_t)tokens[i] * d + k];
                if (W->pos) v += (real)W->pos[(int64_t)(pos0 + i) * d + k];
                h[(int64_t)i * d + k] = v;
            } else {
                h[(int64_t)i * d + k] = hidden_in[(int64_t)i * d + k];
            }
        }
}

/* All n positions of one sequence through the decoder-only stack, causal self-attention computed
 * from scratch.  If s != NULL the keys/values are memoized into it. */
static void dec_only_prefix(orc_model* m, int n, const int32_t* tokens, const real* hidden_in, orc_seq* s,
                            real* h /* [n][d] out */)
{
    const orc_config* c = &m->c;
    int d = c->d_model, H = c->n_heads, dh = c->head_dim, inner = H * dh;
    dec_only_w W = dec_only_weights(m);
    embed_rows(m, &W, n, 0, tokens, hidden_in, h);
    real* a = (real*)malloc(sizeof(real) * (size_t)n * d);
    real* qkv = (real*)malloc(sizeof(real) * (size_t)n * 3 * inner);
    real* ctx = (real*)malloc(sizeof(real) * (size_t)n * inner);
    real* o = (real*)malloc(sizeof(real) * (size_t)n * d);
    real scale = score_scale(m);
    if (s) seq_reserve(m, s, n);
    for (int l = 0; l < c->n_layers; ++l) {
        const float* const* lw = m->w + W.layer0 + 12 * l;
        norm_rows(m, h, n, lw[0], lw[1], a);
        orc_linear(a, n, d, lw[2], lw[3], 3 * inner, qkv);
#pragma omp parallel for collapse(2) schedule(dynamic)
        for (int i = 0; i < n; ++i)
            for (int hd = 0; hd < H; ++hd) {
                const real* q = qkv + (int64_t)i * 3 * inner + hd * dh;
                const real* K = qkv + inner + hd * dh;
                const real* V = qkv + 2 * inner + hd * dh;
                /* causal mask: position i attends to keys 0..i only */
                real ps = orc_attention_row(q, K, 3 * inner, V, 3 * inner, i + 1, dh, scale, NULL,
                                            ctx + (int64_t)i * inner + hd * dh, NULL);
                note_rowsum(m, ps);
            }
        if (s)
            for (int i = 0; i < n; ++i) {
                memcpy(s->K[l] + (int64_t)i * inner, qkv + (int64_t)i * 3 * inner + inner, sizeof(real) * inner);
                memcpy(s->V[l] + (int64_t)i * inner, qkv + (int64_t)i * 3 * inner + 2 * inner, sizeof(real) * inner);
            }
        orc_linear(ctx, n, inner, lw[4], lw[5], d, o);
        for (int64_t i = 0; i < (int64_t)n * d; ++i) h[i] += o[i];
        ffn_block(m, h, n, lw[6], lw[7], lw[8], lw[9], lw[10], lw[11]);
    }
    if (s) s->len = n;
    free(a); free(qkv); free(ctx); free(o);
}

static void dec_only_head(const orc_model* m, const real* h_row, real* logits)
{
    dec_only_w W = dec_only_weights(m);
    int d = m->c.d_model;
    real* a = (real*)malloc(sizeof(real) * (size_t)d);
    norm_rows(m, h_row, 1, W.lnf_g, W.lnf_b, a);
    orc_linear(a, 1, d, W.tok, NULL, m->c.vocab, logits);
    free(a);
}

/* One new position for a sequence whose earlier keys/values are memoized. */
static void dec_only_step(orc_model* m, orc_seq* s, int32_t token, const real* hidden_in, real* h /*[d]*/)
{
    const orc_config* c = &m->c;
    int d = c->d_model, H = c->n_heads, dh = c->head_dim, inner = H * dh;
    dec_only_w W = dec_only_weights(m);
    int i = s->len; /* position of the new token */
    seq_reserve(m, s, i + 1);
    embed_rows(m, &W, 1, i, &token, hidden_in, h);
    real* a = (real*)malloc(sizeof(real) * (size_t)d);
    real* qkv = (real*)malloc(sizeof(real) * (size_t)3 * inner);
    real* ctx = (real*)malloc(sizeof(real) * (size_t)inner);
    real* o = (real*)malloc(sizeof(real) * (size_t)d);
    real scale = score_scale(m);
    for (int l = 0; l < c->n_layers; ++l) {
        const float* const* lw = m->w + W.layer0 + 12 * l;
        norm_rows(m, h, 1, lw[0], lw[1], a);
        orc_linear(a, 1, d, lw[2], lw[3], 3 * inner, qkv);
        memcpy(s->K[l] + (int64_t)i * inner, qkv + inner, sizeof(real) * inner);
        memcpy(s->V[l] + (int64_t)i * inner, qkv + 2 * inner, sizeof(real) * inner);
#pragma omp parallel for schedule(static)
        for (int hd = 0; hd < H; ++hd) {
            real ps = orc_attention_row(qkv + hd * dh, s->K[l] + hd * dh, inner, s->V[l] + hd * dh, inner,
                                        i + 1, dh, scale, NULL, ctx + hd * dh, NULL);
            note_rowsum(m, ps);
        }
        orc_linear(ctx, 1, inner, lw[4], lw[5], d, o);
        for (int k = 0; k < d; ++k) h[k] += o[k];
        ffn_block(m, h, 1, lw[6], lw[7], lw[8], lw[9], lw[10], lw[11]);
    }
    s->len = i + 1;
    free(a); free(qkv); free(ctx); free(o);
}

/* ---------------- encoder-decoder (T5 style) ---------------- */

typedef struct {
    const float *tok, *enc_bias, *dec_bias, *x_bias, *enc_final, *dec_final;
    int enc0, dec0;
} encdec_w;

static encdec_w encdec_weights(const orc_model* m)
{
    encdec_w r;
    memset(&r, 0, sizeof(r));
    int i = 0;
    r.tok = m->w[i++];
    r.enc_bias = m->w[i++];
    r.dec_bias = m->w[i++];
    if (m->c.cross_rel_bias) r.x_bias = m->w[i++];
    r.enc0 = i;
    i += 6 * m->c.n_layers;
    r.enc_final = m->w[i++];
    r.dec0 = i;
    i += 10 * m->c.n_dec_layers;
    r.dec_final = m->w[i++];
    return r;
}

/* bias[j] for query position qi, head hd, keys 0..nk-1, from a [buckets][heads] table */
static void rel_bias_row(const orc_model* m, const float* table, int bidirectional, int qi, int hd, int nk,
                         real* bias)
{
    for (int j = 0; j < nk; ++j) {
        int b = orc_bucket(j - qi, bidirectional, m->c.rel_buckets, m->c.rel_max_dist);
        bias[j] = (real)table[(int64_t)b * m->c.n_heads + hd];
    }
}

/* encoder stack over one input sequence: enc_out [n][d] (after the final norm) */
static void encoder_forward(orc_model* m, int n, const int32_t* tokens, real* enc_out)
{
    const orc_config* c = &m->c;
    int d = c->d_model, H = c->n_heads, dh = c->head_dim, inner = H * dh;
    encdec_w W = encdec_weights(m);
    real* h = (real*)malloc(sizeof(real) * (size_t)n * d);
    for (int i = 0; i < n; ++i)
        for (int k = 0; k < d; ++k) h[(int64_t)i * d + k] = (real)W.tok[(int64_t)tokens[i] * d + k];
    real* a = (real*)malloc(sizeof(real) * (size_t)n * d);
    real* qkv = (real*)malloc(sizeof(real) * (size_t)n * 3 * inner);
    real* ctx = (real*)malloc(sizeof(real) * (size_t)n * inner);
    real* o = (real*)malloc(sizeof(real) * (size_t)n * d);
    real scale = score_scale(m);
    for (int l = 0; l < c->n_layers; ++l) {
        const float* const* lw = m->w + W.enc0 + 6 * l;
        norm_rows(m, h, n, lw[0], NULL, a);
        orc_linear(a, n, d, lw[1], NULL, 3 * inner, qkv);
#pragma omp parallel for collapse(2) schedule(dynamic)
        for (int i = 0; i < n; ++i)
            for (int hd = 0; hd < H; ++hd) {
                real* bias = (real*)malloc(sizeof(real) * (size_t)n);
                rel_bias_row(m, W.enc_bias, 1, i, hd, n, bias);
                /* bidirectional: every position attends to every position of its own sequence */
                real ps = orc_attention_row(qkv + (int64_t)i * 3 * inner + hd * dh, qkv + inner + hd * dh,
                                            3 * inner, qkv + 2 * inner + hd * dh, 3 * inner, n, dh, scale, bias,
                                            ctx + (int64_t)i * inner + hd * dh, NULL);
                note_rowsum(m, ps);
                free(bias);
            }
        orc_linear(ctx, n, inner, lw[2], NULL, d, o);
        for (int64_t i = 0; i < (int64_t)n * d; ++i) h[i] += o[i];
        ffn_block(m, h, n, lw[3], NULL, lw[4], NULL, lw[5], NULL);
    }
    norm_rows(m, h, n, W.enc_final, NULL, enc_out);
    free(h); free(a); free(qkv); free(ctx); free(o);
}

/* decoder position i (token y_i) given self keys/values 0..i-1 in (K,V) and cross keys/values.
 * Appends this position's self key/value at row i of K[l], V[l]. */
static void decoder_position(orc_model* m, int i, int32_t token, real** K, real** V, real** XK, real** XV,
                             int n_in, real* logits)
{
    const orc_config* c = &m->c;
    int d = c->d_model, H = c->n_heads, dh = c->head_dim, inner = H * dh;
    encdec_w W = encdec_weights(m);
    real* h = (real*)malloc(sizeof(real) * (size_t)d);
    for (int k = 0; k < d; ++k) h[k] = (real)W.tok[(int64_t)token * d + k];
    real* a = (real*)malloc(sizeof(real) * (size_t)d);
    real* qkv = (real*)malloc(sizeof(real) * (size_t)3 * inner);
    real* ctx = (real*)malloc(sizeof(real) * (size_t)inner);
    real* o = (real*)malloc(sizeof(real) * (size_t)d);
    real scale = score_scale(m);
    for (int l = 0; l < c->n_dec_layers; ++l) {
        const float* const* lw = m->w + W.dec0 + 10 * l;
        /* causal self-attention with the unidirectional relative-position bias */
        norm_rows(m, h, 1, lw[0], NULL, a);
        orc_linear(a, 1, d, lw[1], NULL, 3 * inner, qkv);
        memcpy(K[l] + (int64_t)i * inner, qkv + inner, sizeof(real) * inner);
        memcpy(V[l] + (int64_t)i * inner, qkv + 2 * inner, sizeof(real) * inner);
#pragma omp parallel for schedule(static)
        for (int hd = 0; hd < H; ++hd) {
            real* bias = (real*)malloc(sizeof(real) * (size_t)(i + 1));
            rel_bias_row(m, W.dec_bias, 0, i, hd, i + 1, bias);
            real ps = orc_attention_row(qkv + hd * dh, K[l] + hd * dh, inner, V[l] + hd * dh, inner, i + 1, dh,
                                        scale, bias, ctx + hd * dh, NULL);
            note_rowsum(m, ps);
            free(bias);
        }
        orc_linear(ctx, 1, inner, lw[2], NULL, d, o);
        for (int k = 0; k < d; ++k) h[k] += o[k];
        /* cross-attention over the encoder output's keys/values */
        norm_rows(m, h, 1, lw[3], NULL, a);
        orc_linear(a, 1, d, lw[4], NULL, inner, qkv);
#pragma omp parallel for schedule(static)
        for (int hd = 0; hd < H; ++hd) {
            real* bias = NULL;
            if (W.x_bias) {
                bias = (real*)malloc(sizeof(real) * (size_t)n_in);
                rel_bias_row(m, W.x_bias, 1, i, hd, n_in, bias);
            }
            real ps = orc_attention_row(qkv + hd * dh, XK[l] + hd * dh, inner, XV[l] + hd * dh, inner, n_in, dh,
                                        scale, bias, ctx + hd * dh, NULL);
            note_rowsum(m, ps);
            free(bias);
        }
        orc_linear(ctx, 1, inner, lw[6], NULL, d, o);
        for (int k = 0; k < d; ++k) h[k] += o[k];
        ffn_block(m, h, 1, lw[7], NULL, lw[8], NULL, lw[9], NULL);
    }
    norm_rows(m, h, 1, W.dec_final, NULL, a);
    real sc = (real)(1.0 / sqrt((double)d));
    for (int k = 0; k < d; ++k) a[k] *= sc;
    orc_linear(a, 1, d, W.tok, NULL, c->vocab, logits);
    free(h); free(a); free(qkv); free(ctx); free(o);
}

/* cross keys/values of every decoder layer from the encoder output */
static void cross_kv(orc_model* m, const real* enc_out, int n_in, real** XK, real** XV)
{
    const orc_config* c = &m->c;
    int d = c->d_model, inner = c->n_heads * c->head_dim;
    encdec_w W = encdec_weights(m);
    real* kv = (real*)malloc(sizeof(real) * (size_t)n_in * 2 * inner);
    for (int l = 0; l < c->n_dec_layers; ++l) {
        const float* const* lw = m->w + W.dec0 + 10 * l;
        orc_linear(enc_out, n_in, d, lw[5], NULL, 2 * inner, kv);
        XK[l] = (real*)malloc(sizeof(real) * (size_t)n_in * inner);
        XV[l] = (real*)malloc(sizeof(real) * (size_t)n_in * inner);
        for (int j = 0; j < n_in; ++j) {
            memcpy(XK[l] + (int64_t)j * inner, kv + (int64_t)j * 2 * inner, sizeof(real) * inner);
            memcpy(XV[l] + (int64_t)j * inner, kv + (int64_t)j * 2 * inner + inner, sizeof(real) * inner);
        }
    }
    free(kv);
}

/* Teacher-forced decoder over all n_dec target positions at once, layer by layer, with nothing
 * memoized: causal self-attention is computed from the layer's full key/value matrix. */
static void decoder_prefix(orc_model* m, int n_dec, const int32_t* dec_tokens, real** XK, real** XV, int n_in,
                           real* logits_all)
{
    const orc_config* c = &m->c;
    int d = c->d_model, H = c->n_heads, dh = c->head_dim, inner = H * dh;
    encdec_w W = encdec_weights(m);
    real* h = (real*)malloc(sizeof(real) * (size_t)n_dec * d);
    for (int i = 0; i < n_dec; ++i)
        for (int k = 0; k < d; ++k) h[(int64_t)i * d + k] = (real)W.tok[(int64_t)dec_tokens[i] * d + k];
    real* a = (real*)malloc(sizeof(real) * (size_t)n_dec * d);
    real* qkv = (real*)malloc(sizeof(real) * (size_t)n_dec * 3 * inner);
    real* ctx = (real*)malloc(sizeof(real) * (size_t)n_dec * inner);
    real* o = (real*)malloc(sizeof(real) * (size_t)n_dec * d);
    real scale = score_scale(m);
    for (int l = 0; l < c->n_dec_layers; ++l) {
        const float* const* lw = m->w + W.dec0 + 10 * l;
        norm_rows(m, h, n_dec, lw[0], NULL, a);
        orc_linear(a, n_dec, d, lw[1], NULL, 3 * inner, qkv);
        for (int i = 0; i < n_dec; ++i)
            for (int hd = 0; hd < H; ++hd) {
                real* bias = (real*)malloc(sizeof(real) * (size_t)(i + 1));
                rel_bias_row(m, W.dec_bias, 0, i, hd, i + 1, bias);
                real ps = orc_attention_row(qkv + (int64_t)i * 3 * inner + hd * dh, qkv + inner + hd * dh,
                                            3 * inner, qkv + 2 * inner + hd * dh, 3 * inner, i + 1, dh, scale,
                                            bias, ctx + (int64_t)i * inner + hd * dh, NULL);
                note_rowsum(m, ps);
                free(bias);
            }
        orc_linear(ctx, n_dec, inner, lw[2], NULL, d, o);
        for (int64_t i = 0; i < (int64_t)n_dec * d; ++i) h[i] += o[i];
        norm_rows(m, h, n_dec, lw[3], NULL, a);
        orc_linear(a, n_dec, d, lw[4], NULL, inner, qkv); /* queries only: [n_dec][inner] */
        for (int i = 0; i < n_dec; ++i)
            for (int hd = 0; hd < H; ++hd) {
                real* bias = NULL;
                if (W.x_bias) {
                    bias = (real*)malloc(sizeof(real) * (size_t)n_in);
                    rel_bias_row(m, W.x_bias, 1, i, hd, n_in, bias);
                }
                real ps = orc_attention_row(qkv + (int64_t)i * inner + hd * dh, XK[l] + hd * dh, inner,
                                            XV[l] + hd * dh, inner, n_in, dh, scale, bias,
                                            ctx + (int64_t)i * inner + hd * dh, NULL);
                note_rowsum(m, ps);
                free(bias);
            }
        orc_linear(ctx, n_dec, inner, lw[6], NULL, d, o);
        for (int64_t i = 0; i < (int64_t)n_dec * d; ++i) h[i] += o[i];
        ffn_block(m, h, n_dec, lw[7], NULL, lw[8], NULL, lw[9], NULL);
    }
    norm_rows(m, h, n_dec, W.dec_final, NULL, a);
    real sc = (real)(1.0 / sqrt((double)d));
    for (int64_t i = 0; i < (int64_t)n_dec * d; ++i) a[i] *= sc;
    orc_linear(a, n_dec, d, W.tok, NULL, c->vocab, logits_all);
    free(h); free(a); free(qkv); free(ctx); free(o);
}

/* ------------------------------------------------------------------ public model calls */

static int check_tokens(const orc_model* m, int n, const int32_t* tokens)
{
    if (!tokens) return 0;
    for (int i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= m->c.vocab) return 0;
    return 1;
}

int orc_encode(orc_model* m, int seq, int n, const int32_t* tokens, const real* hidden_in,
               real* logits_last, real* hidden_out)
{
    if (!m || seq < 0 || seq >= m->max_seqs || n <= 0 || m->seqs[seq].live) return -1;
    const orc_config* c = &m->c;
    orc_seq* s = &m->seqs[seq];
    if (c->arch == 0) {
        if (c->has_embed ? !check_tokens(m, n, tokens) : !hidden_in) return -1;
        if (c->has_embed && c->pos == 0 && n > c->max_pos) return -1;
        int d = c->d_model;
        real* h = (real*)malloc(sizeof(real) * (size_t)n * d);
        s->live = 1;
        dec_only_prefix(m, n, tokens, hidden_in, s, h);
        int next = 0;
        if (c->has_lm_head) {
            real* lg = logits_last ? logits_last : (real*)malloc(sizeof(real) * (size_t)c->vocab);
            dec_only_head(m, h + (int64_t)(n - 1) * d, lg);
            next = orc_argmax(lg, c->vocab);
            if (!logits_last) free(lg);
        } else if (hidden_out) {
            memcpy(hidden_out, h, sizeof(real) * (size_t)n * d);
        }
        free(h);
        return next;
    }
    if (!check_tokens(m, n, tokens)) return -1;
    real* enc_out = (real*)malloc(sizeof(real) * (size_t)n * c->d_model);
    encoder_forward(m, n, tokens, enc_out);
    s->live = 1;
    s->n_in = n;
    s->len = 0;
    s->XK = (real**)calloc((size_t)c->n_dec_layers, sizeof(real*));
    s->XV = (real**)calloc((size_t)c->n_dec_layers, sizeof(real*));
    cross_kv(m, enc_out, n, s->XK, s->XV);
    if (hidden_out) memcpy(hidden_out, enc_out, sizeof(real) * (size_t)n * c->d_model);
    free(enc_out);
    return 0;
}

int orc_decode(orc_model* m, int seq, int32_t token, const real* hidden_in, real* logits, real* hidden_out)
{
    if (!m || seq < 0 || seq >= m->max_seqs || !m->seqs[seq].live) return -1;
    const orc_config* c = &m->c;
    orc_seq* s = &m->seqs[seq];
    if (c->arch == 0) {
        if (c->has_embed ? (token < 0 || token >= c->vocab) : !hidden_in) return -1;
        if (c->has_embed && c->pos == 0 && s->len + 1 > c->max_pos) return -1;
        real* h = (real*)malloc(sizeof(real) * (size_t)c->d_model);
        dec_only_step(m, s, token, hidden_in, h);
        int next = 0;
        if (c->has_lm_head) {
            real* lg = logits ? logits : (real*)malloc(sizeof(real) * (size_t)c->vocab);
            dec_only_head(m, h, lg);
            next = orc_argmax(lg, c->vocab);
            if (!logits) free(lg);
        } else if (hidden_out) {
            memcpy(hidden_out, h, sizeof(real) * (size_t)c->d_model);
        }
        free(h);
        return next;
    }
    if (token < 0 || token >= c->vocab) return -1;
    int i = s->len;
    seq_reserve(m, s, i + 1);
    real* lg = logits ? logits : (real*)malloc(sizeof(real) * (size_t)c->vocab);
    decoder_position(m, i, token, s->K, s->V, s->XK, s->XV, s->n_in, lg);
    s->len = i + 1;
    int next = orc_argmax(lg, c->vocab);
    if (!logits) free(lg);
    return next;
}

int orc_full(orc_model* m, int n, const int32_t* tokens, const real* hidden_in,
             int n_dec, const int32_t* dec_tokens, real* logits_all, real* hidden_all)
{
    if (!m || n <= 0) return -1;
    const orc_config* c = &m->c;
    int d = c->d_model;
    if (c->arch == 0) {
        if (c->has_embed ? !check_tokens(m, n, tokens) : !hidden_in) return -1;
        real* h = (real*)malloc(sizeof(real) * (size_t)n * d);
        dec_only_prefix(m, n, tokens, hidden_in, NULL, h);
        if (c->has_lm_head && logits_all)
            for (int i = 0; i < n; ++i) dec_only_head(m, h + (int64_t)i * d, logits_all + (int64_t)i * c->vocab);
        if (hidden_all) memcpy(hidden_all, h, sizeof(real) * (size_t)n * d);
        free(h);
        return 0;
    }
    if (!check_tokens(m, n, tokens) || n_dec <= 0 || !check_tokens(m, n_dec, dec_tokens) || !logits_all) return -1;
    int nl = c->n_dec_layers;
    real* enc_out = (real*)malloc(sizeof(real) * (size_t)n * d);
    encoder_forward(m, n, tokens, enc_out);
    if (hidden_all) memcpy(hidden_all, enc_out, sizeof(real) * (size_t)n * d);
    real** XK = (real**)calloc((size_t)nl, sizeof(real*));
    real** XV = (real**)calloc((size_t)nl, sizeof(real*));
    cross_kv(m, enc_out, n, XK, XV);
    decoder_prefix(m, n_dec, dec_tokens, XK, XV, n, logits_all);
    for (int l = 0; l < nl; ++l) { free(XK[l]); free(XV[l]); }
    free(XK); free(XV); free(enc_out);
    return 0;
}
