// Model object, ragged K/V pool, launch sequencing and the C ABI of include/exe.h.
#include "../../include/exe.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <map>
#include <string>
#include <vector>

#include "common.h"
#include "kernels.h"

using namespace exe;

// ---------------------------------------------------------------- errors
static thread_local char g_err[512] = "";

static int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
#define HIP_TRY(expr)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess) return fail(EXE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

extern "C" const char* exe_last_error(void) { return g_err; }
extern "C" const char* exe_version(void) { return "exe 0.1 (gfx950)"; }

// ---------------------------------------------------------------- T5 relative-position buckets (exact)
// Largest b in [0, span] with (max_dist/exact)^b <= (n/exact)^span, evaluated in integers:
// max_dist^b * exact^(span-b) <= n^span.  Only called for exact <= n < max_dist, so both sides stay
// below max_dist^span, which exe_model_load checks fits 127 bits.
static int log_bucket(int n, int exact, int span, int max_dist)
{
    unsigned __int128 rhs = 1;
    for (int i = 0; i < span; ++i) rhs *= (unsigned)n;
    int b = 0;
    for (;;) {
        if (b + 1 > span) break;
        unsigned __int128 lhs = 1;
        for (int i = 0; i < b + 1; ++i) lhs *= (unsigned)max_dist;
        for (int i = 0; i < span - b - 1; ++i) lhs *= (unsigned)exact;
        if (lhs <= rhs) ++b; else break;
    }
    return b;
}

extern "C" int exe_rel_bucket(int32_t rel, int32_t bidirectional, int32_t n_buckets, int32_t max_dist)
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
    if (exact < 1 || max_dist <= exact) return -1;
    if (n < exact) return base + n;
    if (n >= max_dist) return base + nb - 1;
    int b = exact + log_bucket(n, exact, nb - exact, max_dist);
    return base + (b < nb - 1 ? b : nb - 1);
}

// ---------------------------------------------------------------- K/V pool: first-fit free list of extents
struct Pool {
    void* ptr = nullptr;
    int64_t elems = 0;
    std::map<int64_t, int64_t> free_;      // offset -> size (elements), non-adjacent
    int64_t used = 0;

    void reset(int64_t n) { free_.clear(); if (n > 0) free_[0] = n; elems = n; used = 0; }
    int64_t alloc(int64_t n)
    {
        for (auto it = free_.begin(); it != free_.end(); ++it) {
            if (it->second < n) continue;
            int64_t off = it->first, sz = it->second;
            free_.erase(it);
            if (sz > n) free_[off + n] = sz - n;
            used += n;
            return off;
        }
        return -1;
    }
    void release(int64_t off, int64_t n)
    {
        used -= n;
        auto nx = free_.lower_bound(off);
        if (nx != free_.end() && off + n == nx->first) { n += nx->second; nx = free_.erase(nx); }
        if (nx != free_.begin()) {
            auto pv = std::prev(nx);
            if (pv->first + pv->second == off) { pv->second += n; return; }
        }
        free_[off] = n;
    }
    int64_t largest() const
    {
        int64_t m = 0;
        for (auto& kv : free_) m = std::max(m, kv.second);
        return m;
    }
};

struct Seq {
    bool live = false;
    int len = 0;             // self-attention K/V length
    int cap = 0;
    int64_t base = -1, elems = 0;
    int n_in = 0;            // enc-dec: encoder length = cross K/V length
    int64_t xbase = -1, xelems = 0;
};

struct DecLayerW {   // decoder-only layer, or the shared part of T5 layers
    const void *n1_g = nullptr, *n1_b = nullptr, *w_qkv = nullptr, *b_qkv = nullptr, *w_o = nullptr, *b_o = nullptr;
    const void *n2_g = nullptr, *n2_b = nullptr, *w_1 = nullptr, *b_1 = nullptr, *w_2 = nullptr, *b_2 = nullptr;
    const void *nx_g = nullptr, *w_xq = nullptr, *w_xkv = nullptr, *w_xo = nullptr;   // T5 decoder cross-attention
};

struct KTimer {
    bool on = false;
    struct Rec { int kind; hipEvent_t a, b; double bytes, flops; };
    std::vector<Rec> recs;
    std::vector<hipEvent_t> pool;
    size_t used = 0;
    hipEvent_t get()
    {
        if (used == pool.size()) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return nullptr;
            pool.push_back(e);
        }
        return pool[used++];
    }
};

struct exe_model {
    exe_config_t c;
    hipStream_t stream;
    int esz;                              // bytes per element of dtype
    int inner;
    const void *tok_emb = nullptr, *pos_emb = nullptr, *fin_g = nullptr, *fin_b = nullptr, *enc_fin_g = nullptr;
    std::vector<DecLayerW> enc, dec;      // decoder-only models use `dec`
    float *bias_enc = nullptr, *bias_dec = nullptr, *bias_x = nullptr;   // [H, 2R+1] device
    int radius = 0;

    Pool pool;
    std::vector<Seq> seqs;
    int live = 0;

    // activation workspace
    int rows_cap = 0;
    float* h = nullptr;
    void *a = nullptr, *qkv = nullptr, *ctx = nullptr, *u = nullptr, *a_last = nullptr;
    float* logits = nullptr;
    int32_t* d_next = nullptr;
    float* gemm_ws = nullptr;
    size_t gemm_ws_bytes = 0;
    // descriptor staging
    unsigned char *stage_h = nullptr, *stage_d = nullptr;
    size_t stage_bytes = 0;
    int32_t* h_next = nullptr;            // pinned
    std::vector<int32_t> mark;            // duplicate detection
    int32_t mark_gen = 0;
    KTimer timer;
};

// ---------------------------------------------------------------- timing helpers
static void t_begin(exe_model* m, int kind, double bytes, double flops)
{
    if (!m->timer.on) return;
    KTimer::Rec r{kind, m->timer.get(), m->timer.get(), bytes, flops};
    if (!r.a || !r.b) return;
    (void)hipEventRecord(r.a, m->stream);
    m->timer.recs.push_back(r);
}
static void t_end(exe_model* m)
{
    if (!m->timer.on || m->timer.recs.empty()) return;
    (void)hipEventRecord(m->timer.recs.back().b, m->stream);
}
#define LAUNCH(m, kind, bytes, flops, expr)                                                       \
    do {                                                                                          \
        t_begin(m, kind, bytes, flops);                                                           \
        hipError_t e_ = (expr);                                                                   \
        t_end(m);                                                                                 \
        if (e_ != hipSuccess) return fail(EXE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));   \
    } while (0)

extern "C" int exe_kernel_timing(exe_model_t* m, int32_t enable)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    (void)hipStreamSynchronize(m->stream);
    m->timer.on = enable != 0;
    m->timer.recs.clear();
    m->timer.used = 0;
    return EXE_OK;
}

extern "C" int exe_kernel_times(exe_model_t* m, exe_kernel_time_t* rows)
{
    if (!m || !rows) return fail(EXE_ERR_ARG, "null argument");
    HIP_TRY(hipStreamSynchronize(m->stream));
    for (int k = 0; k < EXE_K_COUNT; ++k) rows[k] = exe_kernel_time_t{k, 0, 0.0, 0.0, 0.0};
    for (auto& r : m->timer.recs) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) continue;
        rows[r.kind].launches += 1;
        rows[r.kind].ms += ms;
        rows[r.kind].bytes += r.bytes;
        rows[r.kind].flops += r.flops;
    }
    m->timer.recs.clear();
    m->timer.used = 0;
    return EXE_OK;
}

// ---------------------------------------------------------------- config checks and weights
static int n_dec_layers(const exe_config_t& c) { return c.arch == EXE_ARCH_DECODER_ONLY ? c.n_layers : c.n_dec_layers; }

static int check_config(const exe_config_t* c)
{
    if (!c) return fail(EXE_ERR_ARG, "null config");
    if (c->arch != EXE_ARCH_DECODER_ONLY && c->arch != EXE_ARCH_ENC_DEC) return fail(EXE_ERR_ARG, "bad arch");
    if (c->dtype != EXE_DTYPE_F32 && c->dtype != EXE_DTYPE_BF16) return fail(EXE_ERR_ARG, "bad dtype");
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_ff < 1) return fail(EXE_ERR_ARG, "bad sizes");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(EXE_ERR_SHAPE, "head_dim must be 64 or 128");
    if (c->d_model % 8 || c->d_ff % 8 || c->d_model > 16384) return fail(EXE_ERR_SHAPE, "d_model/d_ff must be multiples of 8, d_model <= 16384");
    if (c->act != EXE_ACT_RELU && c->act != EXE_ACT_GELU) return fail(EXE_ERR_ARG, "bad act");
    if (c->norm != EXE_NORM_LAYERNORM && c->norm != EXE_NORM_RMSNORM) return fail(EXE_ERR_ARG, "bad norm");
    if (c->max_seqs < 1 || c->max_batch_tokens < 1 || c->max_batch_seqs < 1) return fail(EXE_ERR_ARG, "bad limits");
    if (c->arch == EXE_ARCH_DECODER_ONLY) {
        if (c->pos != EXE_POS_LEARNED && c->pos != EXE_POS_NONE) return fail(EXE_ERR_SHAPE, "decoder-only supports learned or no positions");
        if (c->norm != EXE_NORM_LAYERNORM) return fail(EXE_ERR_SHAPE, "decoder-only uses LayerNorm");
        if ((c->has_embed || c->has_lm_head) && c->vocab < 1) return fail(EXE_ERR_ARG, "vocab");
        if (c->has_embed && c->pos == EXE_POS_LEARNED && c->max_pos < 1) return fail(EXE_ERR_ARG, "max_pos");
        if (c->has_lm_head && c->vocab % 4) return fail(EXE_ERR_SHAPE, "vocab must be a multiple of 4");
    } else {
        if (c->n_dec_layers < 1 || c->vocab < 1 || !c->has_embed || !c->has_lm_head) return fail(EXE_ERR_ARG, "enc-dec needs decoder layers, embedding and LM head");
        if (c->pos != EXE_POS_RELBIAS || c->norm != EXE_NORM_RMSNORM) return fail(EXE_ERR_SHAPE, "enc-dec uses relative-position bias and RMSNorm");
        if (c->rel_buckets < 4 || c->rel_buckets % 4 || c->rel_max_dist <= c->rel_buckets / 2 || c->rel_max_dist > 511)
            return fail(EXE_ERR_SHAPE, "bad bucket parameters");
        if (std::log2((double)c->rel_max_dist) * (c->rel_buckets / 2) >= 126.0) return fail(EXE_ERR_SHAPE, "bucket parameters too large for exact arithmetic");
        if (c->vocab % 4) return fail(EXE_ERR_SHAPE, "vocab must be a multiple of 4");
    }
    return EXE_OK;
}

extern "C" int exe_expected_weights(const exe_config_t* c)
{
    int r = check_config(c);
    if (r) return r;
    if (c->arch == EXE_ARCH_DECODER_ONLY) {
        int n = 12 * c->n_layers;
        if (c->has_embed || c->has_lm_head) n += 1;
        if (c->has_embed && c->pos == EXE_POS_LEARNED) n += 1;
        if (c->has_lm_head) n += 2;
        return n;
    }
    return 3 + (c->cross_rel_bias ? 1 : 0) + 6 * c->n_layers + 1 + 10 * c->n_dec_layers + 1;
}

static float host_to_f32(const void* p, int dtype, size_t i)
{
    if (dtype == EXE_DTYPE_F32) return ((const float*)p)[i];
    uint32_t u = (uint32_t)((const uint16_t*)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

// bias_by_dist[h][rel + R] = table[bucket(rel)][h] for rel in [-R, R]; beyond +-R the bucket no longer changes.
static int build_bias(exe_model* m, const void* table_dev, int bidirectional, float** out)
{
    const exe_config_t& c = m->c;
    int R = m->radius, H = c.n_heads, nb = c.rel_buckets;
    std::vector<unsigned char> raw((size_t)nb * H * m->esz);
    HIP_TRY(hipMemcpy(raw.data(), table_dev, raw.size(), hipMemcpyDeviceToHost));
    std::vector<float> tab((size_t)H * (2 * R + 1));
    for (int rel = -R; rel <= R; ++rel) {
        int b = exe_rel_bucket(rel, bidirectional, nb, c.rel_max_dist);
        if (b < 0 || b >= nb) return fail(EXE_ERR_SHAPE, "bucket out of range");
        for (int hh = 0; hh < H; ++hh) tab[(size_t)hh * (2 * R + 1) + rel + R] = host_to_f32(raw.data(), c.dtype, (size_t)b * H + hh);
    }
    HIP_TRY(hipMalloc((void**)out, tab.size() * sizeof(float)));
    HIP_TRY(hipMemcpy(*out, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice));
    return EXE_OK;
}

static void free_model(exe_model* m)
{
    if (!m) return;
    (void)hipStreamSynchronize(m->stream);
    void* ptrs[] = {m->pool.ptr, m->h, m->a, m->qkv, m->ctx, m->u, m->a_last, m->logits, m->d_next, m->gemm_ws,
                    m->stage_d, m->bias_enc, m->bias_dec, m->bias_x};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    if (m->stage_h) (void)hipHostFree(m->stage_h);
    if (m->h_next) (void)hipHostFree(m->h_next);
    for (auto e : m->timer.pool) (void)hipEventDestroy(e);
    delete m;
}

extern "C" int exe_model_free(exe_model_t* m)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    free_model(m);
    return EXE_OK;
}

static size_t gemm_ws_need(const exe_model* m, int N, int K)
{
    size_t need = 0;
    int lim = std::min(m->rows_cap, 4096);
    for (int M = 1; M <= lim; ++M) need = std::max(need, gemm_workspace_bytes(m->c.dtype, M, N, K));
    return need;
}

extern "C" int exe_model_load(const exe_config_t* cfg, const exe_tensor_t* weights, int32_t n_weights,
                              void* hip_stream, exe_model_t** out)
{
    if (!out) return fail(EXE_ERR_ARG, "null out");
    *out = nullptr;
    int expect = exe_expected_weights(cfg);
    if (expect < 0) return expect;
    if (!weights || n_weights != expect) return fail(EXE_ERR_ARG, "expected %d weight tensors, got %d", expect, n_weights);
    for (int i = 0; i < n_weights; ++i)
        if (!weights[i].ptr) return fail(EXE_ERR_ARG, "weight %d is NULL", i);

    exe_model* m = new exe_model();
    m->c = *cfg;
    m->stream = (hipStream_t)hip_stream;
    m->esz = cfg->dtype == EXE_DTYPE_F32 ? 4 : 2;
    m->inner = cfg->n_heads * cfg->head_dim;
    const exe_config_t& c = m->c;
    int i = 0;
    auto next = [&]() { return weights[i++].ptr; };
    if (c.arch == EXE_ARCH_DECODER_ONLY) {
        if (c.has_embed || c.has_lm_head) m->tok_emb = next();
        if (c.has_embed && c.pos == EXE_POS_LEARNED) m->pos_emb = next();
        m->dec.resize(c.n_layers);
        for (auto& L : m->dec) {
            L.n1_g = next(); L.n1_b = next(); L.w_qkv = next(); L.b_qkv = next(); L.w_o = next(); L.b_o = next();
            L.n2_g = next(); L.n2_b = next(); L.w_1 = next(); L.b_1 = next(); L.w_2 = next(); L.b_2 = next();
        }
        if (c.has_lm_head) { m->fin_g = next(); m->fin_b = next(); }
    } else {
        m->tok_emb = next();
        const void* t_enc = next();
        const void* t_dec = next();
        const void* t_x = c.cross_rel_bias ? next() : nullptr;
        m->enc.resize(c.n_layers);
        for (auto& L : m->enc) { L.n1_g = next(); L.w_qkv = next(); L.w_o = next(); L.n2_g = next(); L.w_1 = next(); L.w_2 = next(); }
        m->enc_fin_g = next();
        m->dec.resize(c.n_dec_layers);
        for (auto& L : m->dec) {
            L.n1_g = next(); L.w_qkv = next(); L.w_o = next(); L.nx_g = next(); L.w_xq = next(); L.w_xkv = next();
            L.w_xo = next(); L.n2_g = next(); L.w_1 = next(); L.w_2 = next();
        }
        m->fin_g = next();
        m->radius = c.rel_max_dist;
        int r;
        if ((r = build_bias(m, t_enc, 1, &m->bias_enc)) || (r = build_bias(m, t_dec, 0, &m->bias_dec)) ||
            (t_x && (r = build_bias(m, t_x, 1, &m->bias_x)))) { free_model(m); return r; }
    }

#define LOAD_TRY(expr)                                                                                   \
    do {                                                                                                 \
        hipError_t e_ = (expr);                                                                          \
        if (e_ != hipSuccess) { free_model(m); return fail(EXE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); } \
    } while (0)

    m->pool.elems = (int64_t)(c.kv_pool_bytes / m->esz);
    if (m->pool.elems > 0) LOAD_TRY(hipMalloc(&m->pool.ptr, (size_t)m->pool.elems * m->esz));
    m->pool.reset(m->pool.elems);
    m->seqs.resize(c.max_seqs);
    m->mark.assign(c.max_seqs, 0);

    int rows = std::max(c.max_batch_tokens, c.max_batch_seqs);
    m->rows_cap = rows;
    size_t d = c.d_model, f = c.d_ff, inner = m->inner, e = m->esz;
    LOAD_TRY(hipMalloc((void**)&m->h, rows * d * sizeof(float)));
    LOAD_TRY(hipMalloc(&m->a, rows * d * e));
    LOAD_TRY(hipMalloc(&m->qkv, rows * 3 * inner * e));
    LOAD_TRY(hipMalloc(&m->ctx, rows * inner * e));
    LOAD_TRY(hipMalloc(&m->u, rows * f * e));
    if (c.has_lm_head) {
        LOAD_TRY(hipMalloc(&m->a_last, (size_t)c.max_batch_seqs * d * e));
        LOAD_TRY(hipMalloc((void**)&m->logits, (size_t)c.max_batch_seqs * c.vocab * sizeof(float)));
        LOAD_TRY(hipMalloc((void**)&m->d_next, (size_t)c.max_batch_seqs * sizeof(int32_t)));
        LOAD_TRY(hipHostMalloc((void**)&m->h_next, (size_t)c.max_batch_seqs * sizeof(int32_t), hipHostMallocDefault));
    }
    size_t ws = 0;
    ws = std::max(ws, gemm_ws_need(m, 3 * m->inner, c.d_model));
    ws = std::max(ws, gemm_ws_need(m, c.d_model, m->inner));
    ws = std::max(ws, gemm_ws_need(m, c.d_ff, c.d_model));
    ws = std::max(ws, gemm_ws_need(m, c.d_model, c.d_ff));
    if (c.has_lm_head) ws = std::max(ws, gemm_ws_need(m, c.vocab, c.d_model));
    if (c.arch == EXE_ARCH_ENC_DEC) {
        ws = std::max(ws, gemm_ws_need(m, m->inner, c.d_model));
        ws = std::max(ws, gemm_ws_need(m, 2 * m->inner, c.d_model));
    }
    m->gemm_ws_bytes = ws;
    if (ws) LOAD_TRY(hipMalloc((void**)&m->gemm_ws, ws));

    // descriptor staging: token-sized int arrays (3), tile list (2 ints per 128 query rows + one per sequence),
    // and per-sequence arrays (int64 x2, int32 x6)
    size_t tiles_max = (size_t)c.max_batch_tokens / PREFILL_TILE_Q + c.max_batch_seqs + 1;
    m->stage_bytes = 3 * (size_t)rows * 4 + tiles_max * 8 + (size_t)(c.max_batch_seqs + 1) * (2 * 8 + 6 * 4) + 256;
    LOAD_TRY(hipHostMalloc((void**)&m->stage_h, m->stage_bytes, hipHostMallocDefault));
    LOAD_TRY(hipMalloc((void**)&m->stage_d, m->stage_bytes));
#undef LOAD_TRY
    *out = m;
    return EXE_OK;
}

// ---------------------------------------------------------------- staging of per-call descriptor arrays
struct Stager {
    exe_model* m;
    size_t off = 0;
    template <typename T> T* take(size_t n, T** dev)
    {
        off = (off + 15) & ~(size_t)15;
        T* hp = (T*)(m->stage_h + off);
        *dev = (T*)(m->stage_d + off);
        off += n * sizeof(T);
        return hp;
    }
};

// ---------------------------------------------------------------- shared pieces of a forward pass
static double esz_of(const exe_model* m) { return (double)m->esz; }

static int run_gemm(exe_model* m, int M, int N, int K, const void* A, const void* W, const void* bias, int act,
                    float alpha, int out_mode, void* out)
{
    GemmArgs g{m->c.dtype, M, N, K, A, W, bias, act, alpha, out_mode, out, m->gemm_ws, m->gemm_ws_bytes};
    double e = esz_of(m);
    double bytes = ((double)M * K + (double)N * K) * e +
                   (double)M * N * (out_mode == OUT_T ? e : (out_mode == OUT_RESID ? 8.0 : 4.0));
    int kind = M <= 256 ? EXE_K_GEMM_SKINNY : EXE_K_GEMM_TILE;   // weight streaming (HBM) vs MFMA regime
    LAUNCH(m, kind, bytes, 2.0 * M * N * K, launch_gemm(g, m->stream));
    return EXE_OK;
}

static int run_norm(exe_model* m, const int32_t* row_index, int rows, const void* g, const void* b, float out_scale,
                    void* out)
{
    LAUNCH(m, EXE_K_NORM, (double)rows * m->c.d_model * (4.0 + esz_of(m)), 0.0,
           launch_norm(m->c.dtype, m->c.norm == EXE_NORM_RMSNORM, m->h, row_index, rows, m->c.d_model, g, b,
                       m->c.norm_eps, out_scale, out, m->stream));
    return EXE_OK;
}

// h += FFN(norm(h)) for `rows` rows
static int run_ffn(exe_model* m, int rows, const DecLayerW& L)
{
    int r;
    if ((r = run_norm(m, nullptr, rows, L.n2_g, L.n2_b, 1.f, m->a))) return r;
    if ((r = run_gemm(m, rows, m->c.d_ff, m->c.d_model, m->a, L.w_1, L.b_1, m->c.act, 1.f, OUT_T, m->u))) return r;
    return run_gemm(m, rows, m->c.d_model, m->c.d_ff, m->u, L.w_2, L.b_2, -1, 1.f, OUT_RESID, m->h);
}

static float attn_scale(const exe_model* m)
{
    return m->c.scale_mode == EXE_SCALE_RSQRT_DH ? 1.f / sqrtf((float)m->c.head_dim) : 1.f;
}

// final norm of selected rows, LM head, argmax; copies tokens to host and logits to out_device
static int run_head(exe_model* m, const int32_t* row_index_dev, int n, int32_t* next_tokens, void* out_device)
{
    const exe_config_t& c = m->c;
    int r;
    float out_scale = c.arch == EXE_ARCH_ENC_DEC ? 1.f / sqrtf((float)c.d_model) : 1.f;
    if ((r = run_norm(m, row_index_dev, n, m->fin_g, m->fin_b, out_scale, m->a_last))) return r;
    if ((r = run_gemm(m, n, c.vocab, c.d_model, m->a_last, m->tok_emb, nullptr, -1, 1.f, OUT_F32, m->logits))) return r;
    LAUNCH(m, EXE_K_OTHER, (double)n * c.vocab * 4.0, 0.0, launch_argmax(m->logits, n, c.vocab, m->d_next, m->stream));
    if (next_tokens) HIP_TRY(hipMemcpyAsync(m->h_next, m->d_next, (size_t)n * 4, hipMemcpyDeviceToHost, m->stream));
    if (out_device)
        HIP_TRY(hipMemcpyAsync(out_device, m->logits, (size_t)n * c.vocab * 4, hipMemcpyDeviceToDevice, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (next_tokens) memcpy(next_tokens, m->h_next, (size_t)n * 4);
    return EXE_OK;
}

static void release_seq(exe_model* m, Seq& s)
{
    if (s.base >= 0) m->pool.release(s.base, s.elems);
    if (s.xbase >= 0) m->pool.release(s.xbase, s.xelems);
    if (s.live) m->live--;
    s = Seq();
}

static int round8(int x) { return (x + 7) & ~7; }

// ---------------------------------------------------------------- encode
struct EncodeDesc {
    int32_t *tok, *tok_b, *tok_pos, *cu, *cap, *last, *tiles, *xcap;
    int64_t *base, *xbase;
    int n_tiles;
};

static int encode_layers(exe_model* m, int n, int T, const EncodeDesc& d, const std::vector<int>& lens)
{
    const exe_config_t& c = m->c;
    bool encdec = c.arch == EXE_ARCH_ENC_DEC;
    std::vector<DecLayerW>& layers = encdec ? m->enc : m->dec;
    double attn_flops = 0;
    for (int L : lens) attn_flops += encdec ? 4.0 * m->inner * (double)L * L : 2.0 * m->inner * (double)L * (L + 1);
    double attn_bytes = 4.0 * T * m->inner * esz_of(m);
    int r;
    for (size_t l = 0; l < layers.size(); ++l) {
        const DecLayerW& L = layers[l];
        if ((r = run_norm(m, nullptr, T, L.n1_g, L.n1_b, 1.f, m->a))) return r;
        if ((r = run_gemm(m, T, 3 * m->inner, c.d_model, m->a, L.w_qkv, L.b_qkv, -1, 1.f, OUT_T, m->qkv))) return r;
        if (!encdec)
            LAUNCH(m, EXE_K_OTHER, 4.0 * T * m->inner * esz_of(m), 0.0,
                   launch_kv_append(c.dtype, m->qkv, 3 * m->inner, m->inner, 2 * m->inner, T, d.tok_b, d.tok_pos, d.base,
                                    d.cap, (int)l, c.n_heads, c.head_dim, m->pool.ptr, m->stream));
        AttnPackedArgs a{c.dtype, T, c.n_heads, c.head_dim, n, m->qkv, d.tok_b, d.tok_pos, d.cu, encdec ? 0 : 1,
                         attn_scale(m), encdec ? m->bias_enc : nullptr, m->radius, m->ctx, d.tiles, d.n_tiles, 0};
        LAUNCH(m, EXE_K_PREFILL_ATTN, attn_bytes, attn_flops, launch_attn_packed(a, m->stream));
        if ((r = run_gemm(m, T, c.d_model, m->inner, m->ctx, L.w_o, L.b_o, -1, 1.f, OUT_RESID, m->h))) return r;
        if ((r = run_ffn(m, T, L))) return r;
    }
    return EXE_OK;
}

extern "C" int exe_encode(exe_model_t* m, int32_t n, const int32_t* seq_ids, const int32_t* input_lengths,
                          const int32_t* tokens_packed, const int32_t* reserve_lengths, const void* hidden_in,
                          int32_t* next_tokens, void* out_device)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    const exe_config_t& c = m->c;
    if (n < 1 || !seq_ids || !input_lengths) return fail(EXE_ERR_ARG, "n < 1 or null seq_ids/input_lengths");
    if (n > c.max_batch_seqs) return fail(EXE_ERR_ARG, "n = %d exceeds max_batch_seqs = %d", n, c.max_batch_seqs);
    if (c.has_embed ? !tokens_packed : !hidden_in) return fail(EXE_ERR_ARG, "missing tokens / hidden_in");
    bool encdec = c.arch == EXE_ARCH_ENC_DEC;
    bool learned = c.has_embed && c.pos == EXE_POS_LEARNED;
    int64_t T64 = 0;
    ++m->mark_gen;
    std::vector<int> lens(n), caps(n);
    for (int i = 0; i < n; ++i) {
        int id = seq_ids[i];
        if (id < 0 || id >= c.max_seqs) return fail(EXE_ERR_BAD_SEQ, "seq id %d out of range", id);
        if (m->mark[id] == m->mark_gen) return fail(EXE_ERR_BAD_SEQ, "seq id %d appears twice", id);
        m->mark[id] = m->mark_gen;
        if (m->seqs[id].live) return fail(EXE_ERR_BAD_SEQ, "seq id %d is still live", id);
        int L = input_lengths[i];
        if (L < 1) return fail(EXE_ERR_BAD_LENGTH, "input length %d", L);
        if (learned && L > c.max_pos) return fail(EXE_ERR_BAD_LENGTH, "input length %d exceeds max_pos %d", L, c.max_pos);
        int cap;
        if (reserve_lengths) {
            cap = reserve_lengths[i];
            if (cap < (encdec ? 1 : L)) return fail(EXE_ERR_BAD_LENGTH, "reserve length %d too small", cap);
        } else {
            cap = encdec ? 256 : L + 256;
        }
        if (learned && !encdec && cap > c.max_pos) cap = c.max_pos;
        lens[i] = L;
        caps[i] = round8(cap);
        T64 += L;
    }
    if (T64 > c.max_batch_tokens) return fail(EXE_ERR_ARG, "%lld tokens exceed max_batch_tokens = %d", (long long)T64, c.max_batch_tokens);
    int T = (int)T64;
    if (c.has_embed)
        for (int t = 0; t < T; ++t)
            if (tokens_packed[t] < 0 || tokens_packed[t] >= c.vocab) return fail(EXE_ERR_ARG, "token %d out of range", tokens_packed[t]);

    // admit: allocate every extent or none
    int ndl = n_dec_layers(c);
    std::vector<Seq> fresh(n);
    bool ok = true;
    for (int i = 0; i < n && ok; ++i) {
        Seq& s = fresh[i];
        s.cap = caps[i];
        s.elems = (int64_t)ndl * 2 * m->inner * s.cap;
        s.base = m->pool.alloc(s.elems);
        if (s.base < 0) { ok = false; break; }
        if (encdec) {
            s.n_in = lens[i];
            s.xelems = (int64_t)ndl * 2 * m->inner * round8(lens[i]);
            s.xbase = m->pool.alloc(s.xelems);
            if (s.xbase < 0) ok = false;
        }
    }
    auto rollback = [&]() {
        for (auto& s : fresh) {
            if (s.base >= 0) m->pool.release(s.base, s.elems);
            if (s.xbase >= 0) m->pool.release(s.xbase, s.xelems);
        }
    };
    if (!ok) { rollback(); return fail(EXE_ERR_OOM_KV, "K/V pool exhausted (%lld of %lld elements in use)", (long long)m->pool.used, (long long)m->pool.elems); }

    // descriptors
    Stager st{m};
    EncodeDesc d{};
    int32_t* h_tok = st.take<int32_t>(T, &d.tok);
    int32_t* h_tb = st.take<int32_t>(T, &d.tok_b);
    int32_t* h_tp = st.take<int32_t>(T, &d.tok_pos);
    int32_t* h_cu = st.take<int32_t>(n + 1, &d.cu);
    int32_t* h_cap = st.take<int32_t>(n, &d.cap);
    int32_t* h_last = st.take<int32_t>(n, &d.last);
    int32_t* h_xcap = st.take<int32_t>(n, &d.xcap);
    int64_t* h_base = st.take<int64_t>(n, &d.base);
    int64_t* h_xbase = st.take<int64_t>(n, &d.xbase);
    std::vector<std::pair<int, std::pair<int, int>>> tl;   // (work, (seq, q0))
    int t = 0;
    for (int i = 0; i < n; ++i) {
        h_cu[i] = t;
        for (int p = 0; p < lens[i]; ++p, ++t) {
            h_tok[t] = c.has_embed ? tokens_packed[t] : 0;
            h_tb[t] = i;
            h_tp[t] = p;
        }
        h_cap[i] = encdec ? 0 : fresh[i].cap;
        h_base[i] = encdec ? 0 : fresh[i].base;
        h_xcap[i] = encdec ? round8(lens[i]) : 0;
        h_xbase[i] = encdec ? fresh[i].xbase : 0;
        h_last[i] = t - 1;
        for (int q0 = 0; q0 < lens[i]; q0 += PREFILL_TILE_Q)
            tl.push_back({encdec ? lens[i] : std::min(lens[i], q0 + PREFILL_TILE_Q), {i, q0}});
    }
    h_cu[n] = t;
    std::stable_sort(tl.begin(), tl.end(), [](const auto& x, const auto& y) { return x.first > y.first; });
    int32_t* h_tiles = st.take<int32_t>(2 * tl.size(), &d.tiles);
    d.n_tiles = (int)tl.size();
    for (size_t k = 0; k < tl.size(); ++k) { h_tiles[2 * k] = tl[k].second.first; h_tiles[2 * k + 1] = tl[k].second.second; }
    if (st.off > m->stage_bytes) { rollback(); return fail(EXE_ERR_ARG, "descriptor staging overflow"); }

    auto body = [&]() -> int {
        HIP_TRY(hipMemcpyAsync(m->stage_d, m->stage_h, st.off, hipMemcpyHostToDevice, m->stream));
        if (c.has_embed)
            LAUNCH(m, EXE_K_OTHER, (double)T * c.d_model * (esz_of(m) + 4.0), 0.0,
                   launch_embed(c.dtype, d.tok, d.tok_pos, T, c.d_model, m->tok_emb, m->pos_emb, m->h, m->stream));
        else
            LAUNCH(m, EXE_K_OTHER, (double)T * c.d_model * (esz_of(m) + 4.0), 0.0,
                   launch_load_hidden(c.dtype, hidden_in, (int64_t)T * c.d_model, m->h, m->stream));
        int r = encode_layers(m, n, T, d, lens);
        if (r) return r;
        if (encdec) {
            // encoder output (after the final norm) -> every decoder layer's cross keys/values
            if ((r = run_norm(m, nullptr, T, m->enc_fin_g, nullptr, 1.f, m->a))) return r;
            for (size_t l = 0; l < m->dec.size(); ++l) {
                if ((r = run_gemm(m, T, 2 * m->inner, c.d_model, m->a, m->dec[l].w_xkv, nullptr, -1, 1.f, OUT_T, m->qkv))) return r;
                LAUNCH(m, EXE_K_OTHER, 4.0 * T * m->inner * esz_of(m), 0.0,
                       launch_kv_append(c.dtype, m->qkv, 2 * m->inner, 0, m->inner, T, d.tok_b, d.tok_pos, d.xbase, d.xcap,
                                        (int)l, c.n_heads, c.head_dim, m->pool.ptr, m->stream));
            }
            if (out_device)
                HIP_TRY(hipMemcpyAsync(out_device, m->a, (size_t)T * c.d_model * m->esz, hipMemcpyDeviceToDevice, m->stream));
            HIP_TRY(hipStreamSynchronize(m->stream));
            return EXE_OK;
        }
        if (c.has_lm_head) return run_head(m, d.last, n, next_tokens, out_device);
        if (out_device)
            LAUNCH(m, EXE_K_OTHER, (double)T * c.d_model * (esz_of(m) + 4.0), 0.0,
                   launch_store_hidden(c.dtype, m->h, (int64_t)T * c.d_model, out_device, m->stream));
        HIP_TRY(hipStreamSynchronize(m->stream));
        return EXE_OK;
    };
    int r = body();
    if (r) { (void)hipStreamSynchronize(m->stream); rollback(); return r; }
    for (int i = 0; i < n; ++i) {
        Seq& s = m->seqs[seq_ids[i]];
        s = fresh[i];
        s.live = true;
        s.len = encdec ? 0 : lens[i];
        m->live++;
    }
    return EXE_OK;
}

// ---------------------------------------------------------------- decode step
extern "C" int exe_decode_step(exe_model_t* m, int32_t n, const int32_t* seq_ids, const int32_t* tokens_in,
                               const int32_t* kv_lengths, const void* hidden_in, int32_t* next_tokens, void* out_device)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    const exe_config_t& c = m->c;
    if (n < 1 || !seq_ids || !kv_lengths) return fail(EXE_ERR_ARG, "n < 1 or null seq_ids/kv_lengths");
    if (n > c.max_batch_seqs) return fail(EXE_ERR_ARG, "n = %d exceeds max_batch_seqs = %d", n, c.max_batch_seqs);
    if (c.has_embed ? !tokens_in : !hidden_in) return fail(EXE_ERR_ARG, "missing tokens_in / hidden_in");
    bool encdec = c.arch == EXE_ARCH_ENC_DEC;
    bool learned = c.has_embed && c.pos == EXE_POS_LEARNED;
    ++m->mark_gen;
    double sum_len = 0, sum_x = 0;
    for (int i = 0; i < n; ++i) {
        int id = seq_ids[i];
        if (id < 0 || id >= c.max_seqs || !m->seqs[id].live) return fail(EXE_ERR_BAD_SEQ, "seq id %d is not live", id);
        if (m->mark[id] == m->mark_gen) return fail(EXE_ERR_BAD_SEQ, "seq id %d appears twice", id);
        m->mark[id] = m->mark_gen;
        const Seq& s = m->seqs[id];
        if (kv_lengths[i] != s.len + 1) return fail(EXE_ERR_BAD_LENGTH, "seq %d: kv_length %d, expected %d", id, kv_lengths[i], s.len + 1);
        if (s.len + 1 > s.cap) return fail(EXE_ERR_OOM_KV, "seq %d: reserved capacity %d exhausted", id, s.cap);
        if (learned && s.len + 1 > c.max_pos) return fail(EXE_ERR_BAD_LENGTH, "seq %d: position %d exceeds max_pos", id, s.len);
        if (c.has_embed && (tokens_in[i] < 0 || tokens_in[i] >= c.vocab)) return fail(EXE_ERR_ARG, "token %d out of range", tokens_in[i]);
        sum_len += s.len + 1;
        sum_x += s.n_in;
    }
    Stager st{m};
    int32_t *d_tok, *d_pos, *d_len, *d_cap, *d_xcap, *d_xlen;
    int64_t *d_base, *d_xbase;
    int32_t* h_tok = st.take<int32_t>(n, &d_tok);
    int32_t* h_pos = st.take<int32_t>(n, &d_pos);
    int32_t* h_len = st.take<int32_t>(n, &d_len);
    int32_t* h_cap = st.take<int32_t>(n, &d_cap);
    int32_t* h_xcap = st.take<int32_t>(n, &d_xcap);
    int32_t* h_xlen = st.take<int32_t>(n, &d_xlen);
    int64_t* h_base = st.take<int64_t>(n, &d_base);
    int64_t* h_xbase = st.take<int64_t>(n, &d_xbase);
    for (int i = 0; i < n; ++i) {
        const Seq& s = m->seqs[seq_ids[i]];
        h_tok[i] = c.has_embed ? tokens_in[i] : 0;
        h_pos[i] = s.len;
        h_len[i] = s.len + 1;
        h_cap[i] = s.cap;
        h_base[i] = s.base;
        h_xcap[i] = round8(s.n_in);
        h_xlen[i] = s.n_in;
        h_xbase[i] = s.xbase < 0 ? 0 : s.xbase;
    }
    HIP_TRY(hipMemcpyAsync(m->stage_d, m->stage_h, st.off, hipMemcpyHostToDevice, m->stream));
    if (c.has_embed)
        LAUNCH(m, EXE_K_OTHER, (double)n * c.d_model * (esz_of(m) + 4.0), 0.0,
               launch_embed(c.dtype, d_tok, d_pos, n, c.d_model, m->tok_emb, m->pos_emb, m->h, m->stream));
    else
        LAUNCH(m, EXE_K_OTHER, (double)n * c.d_model * (esz_of(m) + 4.0), 0.0,
               launch_load_hidden(c.dtype, hidden_in, (int64_t)n * c.d_model, m->h, m->stream));
    int r;
    double e = esz_of(m);
    double self_bytes = (2.0 * sum_len + 2.0 * n) * m->inner * e, self_flops = 4.0 * sum_len * m->inner;
    double x_bytes = (2.0 * sum_x + 2.0 * n) * m->inner * e, x_flops = 4.0 * sum_x * m->inner;
    for (size_t l = 0; l < m->dec.size(); ++l) {
        const DecLayerW& L = m->dec[l];
        if ((r = run_norm(m, nullptr, n, L.n1_g, L.n1_b, 1.f, m->a))) return r;
        if ((r = run_gemm(m, n, 3 * m->inner, c.d_model, m->a, L.w_qkv, L.b_qkv, -1, 1.f, OUT_T, m->qkv))) return r;
        LAUNCH(m, EXE_K_OTHER, 4.0 * n * m->inner * e, 0.0,
               launch_kv_append(c.dtype, m->qkv, 3 * m->inner, m->inner, 2 * m->inner, n, nullptr, d_pos, d_base, d_cap,
                                (int)l, c.n_heads, c.head_dim, m->pool.ptr, m->stream));
        AttnCacheArgs a{c.dtype, n, c.n_heads, c.head_dim, m->qkv, 3 * m->inner, m->pool.ptr, d_base, d_cap, d_len, d_pos,
                        (int)l, attn_scale(m), encdec ? m->bias_dec : nullptr, m->radius, m->ctx};
        LAUNCH(m, EXE_K_DECODE_ATTN, self_bytes, self_flops, launch_attn_cache(a, m->stream));
        if ((r = run_gemm(m, n, c.d_model, m->inner, m->ctx, L.w_o, L.b_o, -1, 1.f, OUT_RESID, m->h))) return r;
        if (encdec) {
            if ((r = run_norm(m, nullptr, n, L.nx_g, nullptr, 1.f, m->a))) return r;
            if ((r = run_gemm(m, n, m->inner, c.d_model, m->a, L.w_xq, nullptr, -1, 1.f, OUT_T, m->qkv))) return r;
            AttnCacheArgs x{c.dtype, n, c.n_heads, c.head_dim, m->qkv, m->inner, m->pool.ptr, d_xbase, d_xcap, d_xlen, d_pos,
                            (int)l, attn_scale(m), m->bias_x, m->radius, m->ctx};
            LAUNCH(m, EXE_K_CROSS_ATTN, x_bytes, x_flops, launch_attn_cache(x, m->stream));
            if ((r = run_gemm(m, n, c.d_model, m->inner, m->ctx, L.w_xo, nullptr, -1, 1.f, OUT_RESID, m->h))) return r;
        }
        if ((r = run_ffn(m, n, L))) return r;
    }
    if (c.has_lm_head) {
        if ((r = run_head(m, nullptr, n, next_tokens, out_device))) return r;
    } else {
        if (out_device)
            LAUNCH(m, EXE_K_OTHER, (double)n * c.d_model * (e + 4.0), 0.0,
                   launch_store_hidden(c.dtype, m->h, (int64_t)n * c.d_model, out_device, m->stream));
        HIP_TRY(hipStreamSynchronize(m->stream));
    }
    for (int i = 0; i < n; ++i) m->seqs[seq_ids[i]].len += 1;
    return EXE_OK;
}

// ---------------------------------------------------------------- bookkeeping calls
extern "C" int exe_seq_release(exe_model_t* m, int32_t n, const int32_t* seq_ids)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    if (n < 0 || (n > 0 && !seq_ids)) return fail(EXE_ERR_ARG, "bad arguments");
    ++m->mark_gen;
    for (int i = 0; i < n; ++i) {
        int id = seq_ids[i];
        if (id < 0 || id >= m->c.max_seqs || !m->seqs[id].live) return fail(EXE_ERR_BAD_SEQ, "seq id %d is not live", id);
        if (m->mark[id] == m->mark_gen) return fail(EXE_ERR_BAD_SEQ, "seq id %d appears twice", id);
        m->mark[id] = m->mark_gen;
    }
    for (int i = 0; i < n; ++i) release_seq(m, m->seqs[seq_ids[i]]);
    return EXE_OK;
}

extern "C" int exe_seq_length(exe_model_t* m, int32_t seq_id)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    if (seq_id < 0 || seq_id >= m->c.max_seqs || !m->seqs[seq_id].live) return fail(EXE_ERR_BAD_SEQ, "seq id %d is not live", seq_id);
    return m->seqs[seq_id].len;
}

extern "C" int exe_kv_stats(exe_model_t* m, uint64_t* pool_bytes, uint64_t* used_bytes, uint64_t* largest_free_bytes,
                            int32_t* live_seqs)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    if (pool_bytes) *pool_bytes = (uint64_t)m->pool.elems * m->esz;
    if (used_bytes) *used_bytes = (uint64_t)m->pool.used * m->esz;
    if (largest_free_bytes) *largest_free_bytes = (uint64_t)m->pool.largest() * m->esz;
    if (live_seqs) *live_seqs = m->live;
    return EXE_OK;
}

extern "C" int exe_profile(exe_model_t* m, int32_t phase, const int32_t* batch_sizes, int32_t n_batch,
                           const int32_t* lengths, int32_t n_len, const exe_length_dist_t* dist, int32_t n_steps,
                           exe_profile_row_t* rows, int32_t rows_cap, int32_t* n_rows)
{
    (void)m; (void)phase; (void)batch_sizes; (void)n_batch; (void)lengths; (void)n_len; (void)dist; (void)n_steps;
    (void)rows; (void)rows_cap; (void)n_rows;
    return fail(EXE_ERR_UNIMPLEMENTED, "exe_profile is not implemented yet");
}

// ---------------------------------------------------------------- single-operation entry points
extern "C" uint64_t exe_op_gemm_workspace(int32_t dtype, int32_t M, int32_t N, int32_t K)
{
    return gemm_workspace_bytes(dtype, M, N, K);
}

extern "C" int exe_op_gemm(void* hip_stream, int32_t dtype, int32_t M, int32_t N, int32_t K, const void* A,
                           const void* W, const void* bias, int32_t act, float alpha, int32_t out_mode, void* out,
                           void* workspace, uint64_t workspace_bytes)
{
    if (M < 0 || N < 1 || K < 1 || !A || !W || !out) return fail(EXE_ERR_ARG, "bad gemm arguments");
    if (dtype != DT_F32 && dtype != DT_BF16) return fail(EXE_ERR_ARG, "bad dtype");
    if (out_mode < 0 || out_mode > 2) return fail(EXE_ERR_ARG, "bad out_mode");
    if (K % 8 || N % 4) return fail(EXE_ERR_SHAPE, "K must be a multiple of 8 and N of 4");
    if (gemm_workspace_bytes(dtype, M, N, K) > workspace_bytes) return fail(EXE_ERR_ARG, "workspace too small");
    GemmArgs g{dtype, M, N, K, A, W, bias, act, alpha, out_mode, out, (float*)workspace, (size_t)workspace_bytes};
    HIP_TRY(launch_gemm(g, (hipStream_t)hip_stream));
    return EXE_OK;
}

extern "C" int exe_op_norm(void* hip_stream, int32_t dtype, int32_t rms, const float* x, const int32_t* row_index,
                           int32_t rows, int32_t d, const void* gain, const void* shift, float eps, float out_scale,
                           void* out)
{
    if (!x || !gain || !out || rows < 0 || d < 1 || (!rms && !shift)) return fail(EXE_ERR_ARG, "bad norm arguments");
    HIP_TRY(launch_norm(dtype, rms, x, row_index, rows, d, gain, shift, eps, out_scale, out, (hipStream_t)hip_stream));
    return EXE_OK;
}

extern "C" int exe_op_prefill_attention(void* hip_stream, int32_t dtype, int32_t n_seqs, const int32_t* cu_seqlens,
                                        const void* qkv, int32_t H, int32_t dh, float scale, int32_t causal,
                                        const float* bias_by_dist, int32_t bias_radius, void* out, int32_t force_generic)
{
    if (n_seqs < 1 || !cu_seqlens || !qkv || !out || H < 1) return fail(EXE_ERR_ARG, "bad prefill arguments");
    if (dh != 64 && dh != 128) return fail(EXE_ERR_SHAPE, "head_dim must be 64 or 128");
    hipStream_t s = (hipStream_t)hip_stream;
    int T = cu_seqlens[n_seqs];
    std::vector<int32_t> host;
    std::vector<std::pair<int, std::pair<int, int>>> tl;
    host.resize((size_t)2 * T + n_seqs + 1);
    for (int i = 0; i < n_seqs; ++i) {
        int L = cu_seqlens[i + 1] - cu_seqlens[i];
        if (L < 1) return fail(EXE_ERR_BAD_LENGTH, "empty sequence");
        for (int p = 0; p < L; ++p) { host[cu_seqlens[i] + p] = i; host[T + cu_seqlens[i] + p] = p; }
        for (int q0 = 0; q0 < L; q0 += PREFILL_TILE_Q) tl.push_back({causal ? std::min(L, q0 + PREFILL_TILE_Q) : L, {i, q0}});
    }
    for (int i = 0; i <= n_seqs; ++i) host[2 * T + i] = cu_seqlens[i];
    std::stable_sort(tl.begin(), tl.end(), [](const auto& x, const auto& y) { return x.first > y.first; });
    for (auto& t : tl) { host.push_back(t.second.first); host.push_back(t.second.second); }
    int32_t* dev = nullptr;
    HIP_TRY(hipMalloc((void**)&dev, host.size() * 4));
    hipError_t e = hipMemcpyAsync(dev, host.data(), host.size() * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) {
        AttnPackedArgs a{dtype, T, H, dh, n_seqs, qkv, dev, dev + T, dev + 2 * T, causal, scale, bias_by_dist, bias_radius,
                         out, dev + 2 * T + n_seqs + 1, (int)tl.size(), force_generic};
        e = launch_attn_packed(a, s);
    }
    hipError_t e2 = hipStreamSynchronize(s);
    (void)hipFree(dev);
    if (e != hipSuccess) return fail(EXE_ERR_HIP, "prefill attention: %s", hipGetErrorString(e));
    if (e2 != hipSuccess) return fail(EXE_ERR_HIP, "prefill attention: %s", hipGetErrorString(e2));
    return EXE_OK;
}

extern "C" int exe_op_decode_attention(void* hip_stream, int32_t dtype, int32_t B, const void* q, int32_t q_stride,
                                       const void* kv, const int64_t* k_offset, const int32_t* cap, const int32_t* len,
                                       const int32_t* qpos, int32_t H, int32_t dh, float scale,
                                       const float* bias_by_dist, int32_t bias_radius, void* out)
{
    if (B < 0 || !q || !kv || !k_offset || !cap || !len || !qpos || !out || H < 1) return fail(EXE_ERR_ARG, "bad decode attention arguments");
    if (dh != 64 && dh != 128) return fail(EXE_ERR_SHAPE, "head_dim must be 64 or 128");
    AttnCacheArgs a{dtype, B, H, dh, q, q_stride, kv, k_offset, cap, len, qpos, 0, scale, bias_by_dist, bias_radius, out};
    HIP_TRY(launch_attn_cache(a, (hipStream_t)hip_stream));
    return EXE_OK;
}

extern "C" int exe_op_argmax(void* hip_stream, const float* logits, int32_t rows, int32_t n, int32_t* out)
{
    if (!logits || !out || rows < 0 || n < 1) return fail(EXE_ERR_ARG, "bad argmax arguments");
    HIP_TRY(launch_argmax(logits, rows, n, out, (hipStream_t)hip_stream));
    return EXE_OK;
}
