// Model object, ragged K/V pool, launch sequencing and the C ABI of include/exe.h.
#include "../../include/exe.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <map>
#include <mutex>
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
namespace exe {
// for the library's other translation units: records the message exe_last_error() returns, passes the code through
int set_error(int code, const char* msg)
{
    snprintf(g_err, sizeof(g_err), "%s", msg);
    return code;
}
}  // namespace exe
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
    std::vector<int32_t> blocks;   // paged pool: the sequence's blocks in position order (cap = blocks * block rows)
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
    // paged pool (cfg.kv_block_size > 0): per decoder layer a slab of n_blocks blocks, block b of layer l at element
    // (l * n_blocks + b) * blk_elems, each [K|V][head][blk_rows][head_dim]; a sequence owns the same block ids in
    // every layer.  The extent allocator above then serves exe_profile only (which needs an empty pool).
    int blk_rows = 0, blk_shift = 0, n_blocks = 0;
    int64_t blk_elems = 0;
    std::vector<int32_t> free_blocks;      // stack; the back is handed out next

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
    size_t table_max = 0;                  // ints of the widest block table one call can stage
    if (c.kv_block_size != 0) {
        int sh = 0;
        while ((1 << sh) < c.kv_block_size) ++sh;
        if (c.kv_block_size < 8 || c.kv_block_size > 4096 || (1 << sh) != c.kv_block_size) {
            free_model(m);
            return fail(EXE_ERR_ARG, "kv_block_size %d is not a power of two in [8, 4096]", c.kv_block_size);
        }
        if (c.arch != EXE_ARCH_DECODER_ONLY) {
            free_model(m);
            return fail(EXE_ERR_UNIMPLEMENTED, "the paged K/V pool serves decoder-only models");
        }
        m->blk_rows = c.kv_block_size;
        m->blk_shift = sh;
        m->blk_elems = (int64_t)2 * m->inner * m->blk_rows;
        int64_t nb = m->pool.elems / ((int64_t)n_dec_layers(c) * m->blk_elems);
        m->n_blocks = (int)std::min<int64_t>(nb, 1 << 24);
        m->free_blocks.resize(m->n_blocks);
        for (int b = 0; b < m->n_blocks; ++b) m->free_blocks[b] = m->n_blocks - 1 - b;     // block 0 goes out first
        bool learned = c.has_embed && c.pos == EXE_POS_LEARNED;
        size_t width = learned ? (size_t)((c.max_pos + m->blk_rows - 1) >> sh) : (size_t)m->n_blocks;
        table_max = (size_t)c.max_batch_seqs * std::max<size_t>(width, 1);
    }

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
    m->stage_bytes = 3 * (size_t)rows * 4 + tiles_max * 8 + (size_t)(c.max_batch_seqs + 1) * (2 * 8 + 6 * 4) + 256 +
                     table_max * 4 + 16;
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

// final norm of selected rows, LM head, argmax (launches only)
static int head_launches(exe_model* m, const int32_t* row_index_dev, int n)
{
    const exe_config_t& c = m->c;
    int r;
    float out_scale = c.arch == EXE_ARCH_ENC_DEC ? 1.f / sqrtf((float)c.d_model) : 1.f;
    if ((r = run_norm(m, row_index_dev, n, m->fin_g, m->fin_b, out_scale, m->a_last))) return r;
    if ((r = run_gemm(m, n, c.vocab, c.d_model, m->a_last, m->tok_emb, nullptr, -1, 1.f, OUT_F32, m->logits))) return r;
    LAUNCH(m, EXE_K_OTHER, (double)n * c.vocab * 4.0, 0.0, launch_argmax(m->logits, n, c.vocab, m->d_next, m->stream));
    return EXE_OK;
}

// head, then tokens to the host and logits to out_device; synchronises the stream
static int run_head(exe_model* m, const int32_t* row_index_dev, int n, int32_t* next_tokens, void* out_device)
{
    const exe_config_t& c = m->c;
    int r = head_launches(m, row_index_dev, n);
    if (r) return r;
    if (next_tokens) HIP_TRY(hipMemcpyAsync(m->h_next, m->d_next, (size_t)n * 4, hipMemcpyDeviceToHost, m->stream));
    if (out_device)
        HIP_TRY(hipMemcpyAsync(out_device, m->logits, (size_t)n * c.vocab * 4, hipMemcpyDeviceToDevice, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    if (next_tokens) memcpy(next_tokens, m->h_next, (size_t)n * 4);
    return EXE_OK;
}

static void release_seq(exe_model* m, Seq& s)
{
    for (auto it = s.blocks.rbegin(); it != s.blocks.rend(); ++it) m->free_blocks.push_back(*it);
    if (s.base >= 0) m->pool.release(s.base, s.elems);
    if (s.xbase >= 0) m->pool.release(s.xbase, s.xelems);
    if (s.live) m->live--;
    s = Seq();
}

static int round8(int x) { return (x + 7) & ~7; }
static bool paged(const exe_model* m) { return m->blk_rows > 0; }
static int blocks_for(const exe_model* m, int positions) { return (positions + m->blk_rows - 1) >> m->blk_shift; }
static void* layer_blocks(const exe_model* m, int layer)
{
    return (char*)m->pool.ptr + (size_t)layer * m->n_blocks * m->blk_elems * m->esz;
}
// takes `count` blocks for `s` (the caller has checked that they are free)
static void take_blocks(exe_model* m, Seq& s, int count)
{
    for (int i = 0; i < count; ++i) {
        s.blocks.push_back(m->free_blocks.back());
        m->free_blocks.pop_back();
    }
    s.cap = (int)s.blocks.size() * m->blk_rows;
}
// widest block list among `seqs`, and the table [n][width] staged for the device
static int stage_block_table(exe_model* m, Stager& st, const std::vector<const Seq*>& seqs, int32_t** dev)
{
    size_t w = 1;
    for (const Seq* s : seqs) w = std::max(w, s->blocks.size());
    int32_t* h = st.take<int32_t>(seqs.size() * w, dev);
    if (st.off > m->stage_bytes) return (int)w;       // the caller reports the overflow; nothing is written
    for (size_t i = 0; i < seqs.size(); ++i)
        for (size_t j = 0; j < w; ++j) h[i * w + j] = j < seqs[i]->blocks.size() ? seqs[i]->blocks[j] : 0;
    return (int)w;
}

// ---------------------------------------------------------------- encode
struct EncodeDesc {
    int32_t *tok, *tok_b, *tok_pos, *cu, *cap, *last, *tiles, *xcap;
    int64_t *base, *xbase;
    int n_tiles;
    int32_t* table = nullptr;   // paged pool: block table [n][table_w]
    int table_w = 0;
    int max_len = 0;            // longest sequence of the batch
};

// One encode (prefill) layer over T packed tokens of n sequences.  parts: bit 0 = everything but the
// attention kernel, bit 1 = the attention kernel (the profiler times them separately).
static int encode_layer(exe_model* m, const DecLayerW& L, int layer, int n, int T, const EncodeDesc& d,
                        double attn_bytes, double attn_flops, int parts)
{
    const exe_config_t& c = m->c;
    bool encdec = c.arch == EXE_ARCH_ENC_DEC;
    int r;
    if (parts & 1) {
        if ((r = run_norm(m, nullptr, T, L.n1_g, L.n1_b, 1.f, m->a))) return r;
        if ((r = run_gemm(m, T, 3 * m->inner, c.d_model, m->a, L.w_qkv, L.b_qkv, -1, 1.f, OUT_T, m->qkv))) return r;
        if (!encdec && d.table)
            LAUNCH(m, EXE_K_OTHER, 4.0 * T * m->inner * esz_of(m), 0.0,
                   launch_kv_append_paged(c.dtype, m->qkv, 3 * m->inner, m->inner, 2 * m->inner, T, d.tok_b, d.tok_pos,
                                          d.table, d.table_w, m->blk_shift, c.n_heads, c.head_dim, layer_blocks(m, layer),
                                          m->stream));
        else if (!encdec)
            LAUNCH(m, EXE_K_OTHER, 4.0 * T * m->inner * esz_of(m), 0.0,
                   launch_kv_append(c.dtype, m->qkv, 3 * m->inner, m->inner, 2 * m->inner, T, d.tok_b, d.tok_pos, d.base,
                                    d.cap, layer, c.n_heads, c.head_dim, m->pool.ptr, m->stream));
    }
    if (parts & 2) {
        AttnPackedArgs a{c.dtype, T, c.n_heads, c.head_dim, n, m->qkv, d.tok_b, d.tok_pos, d.cu, encdec ? 0 : 1,
                         attn_scale(m), encdec ? m->bias_enc : nullptr, m->radius, m->ctx, d.tiles, d.n_tiles, 0};
        a.max_len = d.max_len;
        LAUNCH(m, EXE_K_PREFILL_ATTN, attn_bytes, attn_flops, launch_attn_packed(a, m->stream));
    }
    if (parts & 1) {
        if ((r = run_gemm(m, T, c.d_model, m->inner, m->ctx, L.w_o, L.b_o, -1, 1.f, OUT_RESID, m->h))) return r;
        if ((r = run_ffn(m, T, L))) return r;
    }
    return EXE_OK;
}

static void prefill_attn_work(const exe_model* m, const std::vector<int>& lens, int T, double* bytes, double* flops)
{
    bool encdec = m->c.arch == EXE_ARCH_ENC_DEC;
    double f = 0;
    for (int L : lens) f += encdec ? 4.0 * m->inner * (double)L * L : 2.0 * m->inner * (double)L * (L + 1);
    *flops = f;
    *bytes = 4.0 * T * m->inner * esz_of(m);
}

static int encode_layers(exe_model* m, int n, int T, const EncodeDesc& d, const std::vector<int>& lens)
{
    std::vector<DecLayerW>& layers = m->c.arch == EXE_ARCH_ENC_DEC ? m->enc : m->dec;
    double attn_bytes, attn_flops;
    prefill_attn_work(m, lens, T, &attn_bytes, &attn_flops);
    for (size_t l = 0; l < layers.size(); ++l) {
        int r = encode_layer(m, layers[l], (int)l, n, T, d, attn_bytes, attn_flops, 3);
        if (r) return r;
    }
    return EXE_OK;
}

// fills the per-token and per-sequence descriptor arrays of an encode batch (host side) and the tile list
static void fill_encode_desc(exe_model* m, Stager& st, EncodeDesc& d, int n, const std::vector<int>& lens,
                             const int32_t* tokens, const std::vector<Seq>& fresh)
{
    bool encdec = m->c.arch == EXE_ARCH_ENC_DEC;
    int T = 0;
    for (int L : lens) { T += L; d.max_len = std::max(d.max_len, L); }
    int32_t* h_tok = st.take<int32_t>(T, &d.tok);
    int32_t* h_tb = st.take<int32_t>(T, &d.tok_b);
    int32_t* h_tp = st.take<int32_t>(T, &d.tok_pos);
    int32_t* h_cu = st.take<int32_t>(n + 1, &d.cu);
    int32_t* h_cap = st.take<int32_t>(n, &d.cap);
    int32_t* h_last = st.take<int32_t>(n, &d.last);
    int32_t* h_xcap = st.take<int32_t>(n, &d.xcap);
    int64_t* h_base = st.take<int64_t>(n, &d.base);
    int64_t* h_xbase = st.take<int64_t>(n, &d.xbase);
    int t = 0;
    for (int i = 0; i < n; ++i) {
        h_cu[i] = t;
        for (int p = 0; p < lens[i]; ++p, ++t) {
            h_tok[t] = tokens ? tokens[t] : 0;
            h_tb[t] = i;
            h_tp[t] = p;
        }
        h_cap[i] = encdec ? 0 : fresh[i].cap;
        h_base[i] = encdec ? 0 : fresh[i].base;
        h_xcap[i] = encdec ? round8(lens[i]) : 0;
        h_xbase[i] = encdec ? fresh[i].xbase : 0;
        h_last[i] = t - 1;
    }
    h_cu[n] = t;
    std::vector<int32_t> tl;
    prefill_tile_order(lens.data(), n, tl);
    int32_t* h_tiles = st.take<int32_t>(tl.size(), &d.tiles);
    d.n_tiles = (int)(tl.size() / 2);
    std::copy(tl.begin(), tl.end(), h_tiles);
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

    // admit: allocate every extent (paged pool: every block) or none
    int ndl = n_dec_layers(c);
    std::vector<Seq> fresh(n);
    bool ok = true;
    if (paged(m)) {
        // blocks for the input positions only; decode steps take further blocks as the sequences grow
        int64_t need = 0;
        for (int i = 0; i < n; ++i) need += blocks_for(m, lens[i]);
        if (need > (int64_t)m->free_blocks.size())
            return fail(EXE_ERR_OOM_KV, "K/V pool exhausted (%lld blocks needed, %lld of %d free)", (long long)need,
                        (long long)m->free_blocks.size(), m->n_blocks);
        for (int i = 0; i < n; ++i) take_blocks(m, fresh[i], blocks_for(m, lens[i]));
    }
    for (int i = 0; i < n && ok && !paged(m); ++i) {
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
            for (auto it = s.blocks.rbegin(); it != s.blocks.rend(); ++it) m->free_blocks.push_back(*it);
            s.blocks.clear();
            if (s.base >= 0) m->pool.release(s.base, s.elems);
            if (s.xbase >= 0) m->pool.release(s.xbase, s.xelems);
        }
    };
    if (!ok) { rollback(); return fail(EXE_ERR_OOM_KV, "K/V pool exhausted (%lld of %lld elements in use)", (long long)m->pool.used, (long long)m->pool.elems); }

    // descriptors
    Stager st{m};
    EncodeDesc d{};
    fill_encode_desc(m, st, d, n, lens, c.has_embed ? tokens_packed : nullptr, fresh);
    if (paged(m)) {
        std::vector<const Seq*> sp(n);
        for (int i = 0; i < n; ++i) sp[i] = &fresh[i];
        d.table_w = stage_block_table(m, st, sp, &d.table);
    }
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
struct DecodeSeq { int32_t token; int len_before; int cap; int64_t base; int n_in; int64_t xbase; };
struct DecodeDesc {
    int32_t *tok, *pos, *len, *cap, *xcap, *xlen;
    int64_t *base, *xbase;
    double self_bytes, self_flops, x_bytes, x_flops;
    int mean_len, mean_xlen;      // average self / cross rows per sequence
    int32_t* table = nullptr;     // paged pool: block table [n][table_w]
    int table_w = 0;
};

static void fill_decode_desc(exe_model* m, Stager& st, DecodeDesc& d, const std::vector<DecodeSeq>& ds)
{
    int n = (int)ds.size();
    int32_t* h_tok = st.take<int32_t>(n, &d.tok);
    int32_t* h_pos = st.take<int32_t>(n, &d.pos);
    int32_t* h_len = st.take<int32_t>(n, &d.len);
    int32_t* h_cap = st.take<int32_t>(n, &d.cap);
    int32_t* h_xcap = st.take<int32_t>(n, &d.xcap);
    int32_t* h_xlen = st.take<int32_t>(n, &d.xlen);
    int64_t* h_base = st.take<int64_t>(n, &d.base);
    int64_t* h_xbase = st.take<int64_t>(n, &d.xbase);
    double sum_len = 0, sum_x = 0;
    for (int i = 0; i < n; ++i) {
        h_tok[i] = ds[i].token;
        h_pos[i] = ds[i].len_before;
        h_len[i] = ds[i].len_before + 1;
        h_cap[i] = ds[i].cap;
        h_base[i] = ds[i].base;
        h_xcap[i] = round8(ds[i].n_in);
        h_xlen[i] = ds[i].n_in;
        h_xbase[i] = ds[i].xbase;
        sum_len += ds[i].len_before + 1;
        sum_x += ds[i].n_in;
    }
    double e = esz_of(m);
    d.mean_len = n > 0 ? (int)(sum_len / n + 0.5) : 0;
    d.mean_xlen = n > 0 ? (int)(sum_x / n + 0.5) : 0;
    d.self_bytes = (2.0 * sum_len + 2.0 * n) * m->inner * e;
    d.self_flops = 4.0 * sum_len * m->inner;
    d.x_bytes = (2.0 * sum_x + 2.0 * n) * m->inner * e;
    d.x_flops = 4.0 * sum_x * m->inner;
}

// residual stream of the step's n rows from the token (+position) embedding, or from caller hidden states
static int decode_input(exe_model* m, const DecodeDesc& d, int n, const void* hidden_in)
{
    const exe_config_t& c = m->c;
    if (c.has_embed)
        LAUNCH(m, EXE_K_OTHER, (double)n * c.d_model * (esz_of(m) + 4.0), 0.0,
               launch_embed(c.dtype, d.tok, d.pos, n, c.d_model, m->tok_emb, m->pos_emb, m->h, m->stream));
    else
        LAUNCH(m, EXE_K_OTHER, (double)n * c.d_model * (esz_of(m) + 4.0), 0.0,
               launch_load_hidden(c.dtype, hidden_in, (int64_t)n * c.d_model, m->h, m->stream));
    return EXE_OK;
}

// One decode layer for n rows.  parts: bit 0 = everything but the attention kernels, bit 1 = the attention
// kernels (self, and cross for encoder-decoder models).
static int decode_layer(exe_model* m, const DecLayerW& L, int layer, int n, const DecodeDesc& d, int parts)
{
    const exe_config_t& c = m->c;
    bool encdec = c.arch == EXE_ARCH_ENC_DEC;
    double e = esz_of(m);
    int r;
    if (parts & 1) {
        if ((r = run_norm(m, nullptr, n, L.n1_g, L.n1_b, 1.f, m->a))) return r;
        if ((r = run_gemm(m, n, 3 * m->inner, c.d_model, m->a, L.w_qkv, L.b_qkv, -1, 1.f, OUT_T, m->qkv))) return r;
        if (!(parts & 2))      // the attention kernel appends the new key/value rows itself when it runs
            LAUNCH(m, EXE_K_OTHER, 4.0 * n * m->inner * e, 0.0,
                   launch_kv_append(c.dtype, m->qkv, 3 * m->inner, m->inner, 2 * m->inner, n, nullptr, d.pos, d.base, d.cap,
                                    layer, c.n_heads, c.head_dim, m->pool.ptr, m->stream));
    }
    if ((parts & 2) && d.table) {
        AttnPagedArgs a{c.dtype, n, c.n_heads, c.head_dim, m->qkv, 3 * m->inner, layer_blocks(m, layer), d.table, d.table_w,
                        m->blk_shift, d.len, d.pos, attn_scale(m), nullptr, 0, m->ctx};
        a.new_k_off = m->inner;
        a.new_v_off = 2 * m->inner;
        a.mean_len = d.mean_len;
        LAUNCH(m, EXE_K_DECODE_ATTN, d.self_bytes, d.self_flops, launch_attn_paged(a, m->stream));
    } else if (parts & 2) {
        AttnCacheArgs a{c.dtype, n, c.n_heads, c.head_dim, m->qkv, 3 * m->inner, m->pool.ptr, d.base, d.cap, d.len, d.pos,
                        layer, attn_scale(m), encdec ? m->bias_dec : nullptr, m->radius, m->ctx};
        a.new_k_off = m->inner;
        a.new_v_off = 2 * m->inner;
        a.mean_len = d.mean_len;
        LAUNCH(m, EXE_K_DECODE_ATTN, d.self_bytes, d.self_flops, launch_attn_cache(a, m->stream));
    }
    if (parts & 1)
        if ((r = run_gemm(m, n, c.d_model, m->inner, m->ctx, L.w_o, L.b_o, -1, 1.f, OUT_RESID, m->h))) return r;
    if (encdec) {
        if (parts & 1) {
            if ((r = run_norm(m, nullptr, n, L.nx_g, nullptr, 1.f, m->a))) return r;
            if ((r = run_gemm(m, n, m->inner, c.d_model, m->a, L.w_xq, nullptr, -1, 1.f, OUT_T, m->qkv))) return r;
        }
        if (parts & 2) {
            AttnCacheArgs x{c.dtype, n, c.n_heads, c.head_dim, m->qkv, m->inner, m->pool.ptr, d.xbase, d.xcap, d.xlen, d.pos,
                            layer, attn_scale(m), m->bias_x, m->radius, m->ctx};
            x.mean_len = d.mean_xlen;
            LAUNCH(m, EXE_K_CROSS_ATTN, d.x_bytes, d.x_flops, launch_attn_cache(x, m->stream));
        }
        if (parts & 1)
            if ((r = run_gemm(m, n, c.d_model, m->inner, m->ctx, L.w_xo, nullptr, -1, 1.f, OUT_RESID, m->h))) return r;
    }
    if (parts & 1)
        if ((r = run_ffn(m, n, L))) return r;
    return EXE_OK;
}

extern "C" int exe_decode_step(exe_model_t* m, int32_t n, const int32_t* seq_ids, const int32_t* tokens_in,
                               const int32_t* kv_lengths, const void* hidden_in, int32_t* next_tokens, void* out_device)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    const exe_config_t& c = m->c;
    if (n < 1 || !seq_ids || !kv_lengths) return fail(EXE_ERR_ARG, "n < 1 or null seq_ids/kv_lengths");
    if (n > c.max_batch_seqs) return fail(EXE_ERR_ARG, "n = %d exceeds max_batch_seqs = %d", n, c.max_batch_seqs);
    if (c.has_embed ? !tokens_in : !hidden_in) return fail(EXE_ERR_ARG, "missing tokens_in / hidden_in");
    bool learned = c.has_embed && c.pos == EXE_POS_LEARNED;
    int64_t blocks_needed = 0;
    ++m->mark_gen;
    for (int i = 0; i < n; ++i) {
        int id = seq_ids[i];
        if (id < 0 || id >= c.max_seqs || !m->seqs[id].live) return fail(EXE_ERR_BAD_SEQ, "seq id %d is not live", id);
        if (m->mark[id] == m->mark_gen) return fail(EXE_ERR_BAD_SEQ, "seq id %d appears twice", id);
        m->mark[id] = m->mark_gen;
        const Seq& s = m->seqs[id];
        if (kv_lengths[i] != s.len + 1) return fail(EXE_ERR_BAD_LENGTH, "seq %d: kv_length %d, expected %d", id, kv_lengths[i], s.len + 1);
        if (paged(m)) {
            if (s.len + 1 > s.cap && ++blocks_needed > (int64_t)m->free_blocks.size())
                return fail(EXE_ERR_OOM_KV, "K/V pool exhausted: no free block for seq %d (%d blocks in all)", id, m->n_blocks);
        } else if (s.len + 1 > s.cap) {
            return fail(EXE_ERR_OOM_KV, "seq %d: reserved capacity %d exhausted", id, s.cap);
        }
        if (learned && s.len + 1 > c.max_pos) return fail(EXE_ERR_BAD_LENGTH, "seq %d: position %d exceeds max_pos", id, s.len);
        if (c.has_embed && (tokens_in[i] < 0 || tokens_in[i] >= c.vocab)) return fail(EXE_ERR_ARG, "token %d out of range", tokens_in[i]);
    }
    Stager st{m};
    DecodeDesc dd{};
    std::vector<DecodeSeq> ds(n);
    for (int i = 0; i < n; ++i) {
        Seq& s = m->seqs[seq_ids[i]];
        if (paged(m) && s.len + 1 > s.cap) take_blocks(m, s, 1);          // checked above: the blocks are there
        ds[i] = DecodeSeq{c.has_embed ? tokens_in[i] : 0, s.len, s.cap, s.base, s.n_in, s.xbase < 0 ? 0 : s.xbase};
    }
    fill_decode_desc(m, st, dd, ds);
    if (paged(m)) {
        std::vector<const Seq*> sp(n);
        for (int i = 0; i < n; ++i) sp[i] = &m->seqs[seq_ids[i]];
        dd.table_w = stage_block_table(m, st, sp, &dd.table);
        if (st.off > m->stage_bytes) return fail(EXE_ERR_ARG, "descriptor staging overflow");
    }
    HIP_TRY(hipMemcpyAsync(m->stage_d, m->stage_h, st.off, hipMemcpyHostToDevice, m->stream));
    int r;
    if ((r = decode_input(m, dd, n, hidden_in))) return r;
    for (size_t l = 0; l < m->dec.size(); ++l)
        if ((r = decode_layer(m, m->dec[l], (int)l, n, dd, 3))) return r;
    double e = esz_of(m);
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

// ---------------------------------------------------------------- K/V hand-over (Section 3 "XRunner", WAA scheduling)
// Exported layout: the self-attention entries [decoder layer][K|V][head][kv_len][head_dim] in the storage type,
// then (encoder-decoder models) the cross-attention entries [decoder layer][K|V][head][cross_len][head_dim]:
// the extent without its unused capacity.  Either side of the copy is one strided 2-D transfer.
// paged pool: the self-attention entries of `s` between its blocks and a host buffer in the exported layout, one
// strided copy per (layer, block)
static hipError_t copy_blocks(exe_model* m, const Seq& s, char* host, bool to_host)
{
    size_t rowb = (size_t)m->c.head_dim * m->esz, layer_rows = (size_t)2 * m->c.n_heads;
    for (int l = 0; l < n_dec_layers(m->c); ++l) {
        char* hl = host + (size_t)l * layer_rows * s.len * rowb;
        for (int i = 0; i * m->blk_rows < s.len; ++i) {
            int rows_in = std::min(m->blk_rows, s.len - i * m->blk_rows);
            char* dev = (char*)layer_blocks(m, l) + (size_t)s.blocks[i] * m->blk_elems * m->esz;
            char* hp = hl + (size_t)i * m->blk_rows * rowb;
            hipError_t e = to_host ? hipMemcpy2DAsync(hp, s.len * rowb, dev, m->blk_rows * rowb, rows_in * rowb, layer_rows,
                                                      hipMemcpyDeviceToHost, m->stream)
                                   : hipMemcpy2DAsync(dev, m->blk_rows * rowb, hp, s.len * rowb, rows_in * rowb, layer_rows,
                                                      hipMemcpyHostToDevice, m->stream);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

static uint64_t export_bytes_of(const exe_model* m, const Seq& s)
{
    uint64_t rows = (uint64_t)n_dec_layers(m->c) * 2 * m->c.n_heads;
    return rows * ((uint64_t)s.len + (uint64_t)s.n_in) * m->c.head_dim * m->esz;
}

extern "C" int64_t exe_seq_export_bytes(exe_model_t* m, int32_t seq_id)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    if (seq_id < 0 || seq_id >= m->c.max_seqs || !m->seqs[seq_id].live) return fail(EXE_ERR_BAD_SEQ, "seq id %d is not live", seq_id);
    return (int64_t)export_bytes_of(m, m->seqs[seq_id]);
}

extern "C" int exe_seq_export(exe_model_t* m, int32_t seq_id, void* host_buf, uint64_t buf_bytes, exe_seq_state_t* state)
{
    if (!m || !host_buf || !state) return fail(EXE_ERR_ARG, "null argument");
    if (seq_id < 0 || seq_id >= m->c.max_seqs || !m->seqs[seq_id].live) return fail(EXE_ERR_BAD_SEQ, "seq id %d is not live", seq_id);
    const Seq& s = m->seqs[seq_id];
    uint64_t need = export_bytes_of(m, s);
    if (buf_bytes < need) return fail(EXE_ERR_ARG, "buffer of %llu bytes, %llu needed", (unsigned long long)buf_bytes, (unsigned long long)need);
    size_t rows = (size_t)n_dec_layers(m->c) * 2 * m->c.n_heads, rowb = (size_t)m->c.head_dim * m->esz;
    char* dst = (char*)host_buf;
    if (s.len > 0 && paged(m)) {
        HIP_TRY(copy_blocks(m, s, dst, true));
        dst += rows * s.len * rowb;
    } else if (s.len > 0) {
        HIP_TRY(hipMemcpy2DAsync(dst, s.len * rowb, (const char*)m->pool.ptr + s.base * m->esz, s.cap * rowb, s.len * rowb, rows,
                                 hipMemcpyDeviceToHost, m->stream));
        dst += rows * s.len * rowb;
    }
    if (s.n_in > 0)
        HIP_TRY(hipMemcpy2DAsync(dst, s.n_in * rowb, (const char*)m->pool.ptr + s.xbase * m->esz, round8(s.n_in) * rowb,
                                 s.n_in * rowb, rows, hipMemcpyDeviceToHost, m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    state->kv_len = s.len;
    state->cross_len = s.n_in;
    return EXE_OK;
}

extern "C" int exe_seq_import(exe_model_t* m, int32_t seq_id, const void* host_buf, uint64_t buf_bytes,
                              const exe_seq_state_t* state, int32_t reserve_length)
{
    if (!m || !host_buf || !state) return fail(EXE_ERR_ARG, "null argument");
    const exe_config_t& c = m->c;
    if (seq_id < 0 || seq_id >= c.max_seqs) return fail(EXE_ERR_BAD_SEQ, "seq id %d out of range", seq_id);
    if (m->seqs[seq_id].live) return fail(EXE_ERR_BAD_SEQ, "seq id %d is live", seq_id);
    bool encdec = c.arch == EXE_ARCH_ENC_DEC;
    bool learned = c.has_embed && c.pos == EXE_POS_LEARNED;
    if (state->kv_len < 0 || state->cross_len < 0 || (encdec ? state->cross_len < 1 : (state->kv_len < 1 || state->cross_len != 0)))
        return fail(EXE_ERR_BAD_LENGTH, "bad state: kv_len %d, cross_len %d", state->kv_len, state->cross_len);
    if (learned && !encdec && state->kv_len > c.max_pos) return fail(EXE_ERR_BAD_LENGTH, "kv_len %d exceeds max_pos", state->kv_len);
    Seq s;
    s.len = state->kv_len;
    s.n_in = state->cross_len;
    if (buf_bytes < export_bytes_of(m, s)) return fail(EXE_ERR_ARG, "buffer of %llu bytes is too small for the state", (unsigned long long)buf_bytes);
    int cap = reserve_length > 0 ? reserve_length : s.len + 256;
    if (cap < std::max(s.len, 1)) return fail(EXE_ERR_BAD_LENGTH, "reserve length %d too small", cap);
    if (learned && !encdec && cap > c.max_pos) cap = c.max_pos;
    s.cap = round8(cap);
    int ndl = n_dec_layers(c);
    if (paged(m)) {
        int need = blocks_for(m, std::max(s.len, 1));
        if (need > (int)m->free_blocks.size())
            return fail(EXE_ERR_OOM_KV, "K/V pool exhausted (%d blocks needed, %d of %d free)", need, (int)m->free_blocks.size(), m->n_blocks);
        take_blocks(m, s, need);
        hipError_t e = copy_blocks(m, s, (char*)const_cast<void*>(host_buf), false);
        if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
        if (e != hipSuccess) {
            for (auto it = s.blocks.rbegin(); it != s.blocks.rend(); ++it) m->free_blocks.push_back(*it);
            return fail(EXE_ERR_HIP, "K/V import copy: %s", hipGetErrorString(e));
        }
        s.live = true;
        m->seqs[seq_id] = s;
        m->live++;
        return EXE_OK;
    }
    s.elems = (int64_t)ndl * 2 * m->inner * s.cap;
    s.base = m->pool.alloc(s.elems);
    if (s.base >= 0 && encdec) {
        s.xelems = (int64_t)ndl * 2 * m->inner * round8(s.n_in);
        s.xbase = m->pool.alloc(s.xelems);
    }
    if (s.base < 0 || (encdec && s.xbase < 0)) {
        if (s.base >= 0) m->pool.release(s.base, s.elems);
        return fail(EXE_ERR_OOM_KV, "K/V pool exhausted (%lld of %lld elements in use)", (long long)m->pool.used, (long long)m->pool.elems);
    }
    size_t rows = (size_t)ndl * 2 * c.n_heads, rowb = (size_t)c.head_dim * m->esz;
    const char* src = (const char*)host_buf;
    hipError_t e = hipSuccess;
    if (s.len > 0) {
        e = hipMemcpy2DAsync((char*)m->pool.ptr + s.base * m->esz, s.cap * rowb, src, s.len * rowb, s.len * rowb, rows,
                             hipMemcpyHostToDevice, m->stream);
        src += rows * s.len * rowb;
    }
    if (e == hipSuccess && s.n_in > 0)
        e = hipMemcpy2DAsync((char*)m->pool.ptr + s.xbase * m->esz, round8(s.n_in) * rowb, src, s.n_in * rowb, s.n_in * rowb, rows,
                             hipMemcpyHostToDevice, m->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
    if (e != hipSuccess) {
        m->pool.release(s.base, s.elems);
        if (s.xbase >= 0) m->pool.release(s.xbase, s.xelems);
        return fail(EXE_ERR_HIP, "K/V import copy: %s", hipGetErrorString(e));
    }
    s.live = true;
    m->seqs[seq_id] = s;
    m->live++;
    return EXE_OK;
}

// ---------------------------------------------------------------- extent relocation and compaction
extern "C" int exe_seq_reserve(exe_model_t* m, int32_t seq_id, int32_t reserve_length)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    const exe_config_t& c = m->c;
    if (seq_id < 0 || seq_id >= c.max_seqs || !m->seqs[seq_id].live) return fail(EXE_ERR_BAD_SEQ, "seq id %d is not live", seq_id);
    Seq& s = m->seqs[seq_id];
    bool learned = c.has_embed && c.pos == EXE_POS_LEARNED;
    if (reserve_length < std::max(s.len, 1)) return fail(EXE_ERR_BAD_LENGTH, "reserve length %d below the current length %d", reserve_length, s.len);
    if (learned && c.arch != EXE_ARCH_ENC_DEC && reserve_length > c.max_pos)
        return fail(EXE_ERR_BAD_LENGTH, "reserve length %d exceeds max_pos %d", reserve_length, c.max_pos);
    if (paged(m)) {
        // blocks ahead of need, or surplus blocks back to the pool
        int want = blocks_for(m, reserve_length), have = (int)s.blocks.size();
        if (want - have > (int)m->free_blocks.size())
            return fail(EXE_ERR_OOM_KV, "K/V pool exhausted (%d blocks needed, %d of %d free)", want - have, (int)m->free_blocks.size(), m->n_blocks);
        if (want > have) take_blocks(m, s, want - have);
        while ((int)s.blocks.size() > want) {
            m->free_blocks.push_back(s.blocks.back());
            s.blocks.pop_back();
        }
        s.cap = (int)s.blocks.size() * m->blk_rows;
        return EXE_OK;
    }
    int cap = round8(reserve_length);
    if (cap == s.cap) return EXE_OK;
    int64_t elems = (int64_t)n_dec_layers(c) * 2 * m->inner * cap;
    int64_t base = m->pool.alloc(elems);
    if (base < 0) return fail(EXE_ERR_OOM_KV, "no free extent of %lld elements (largest %lld)", (long long)elems, (long long)m->pool.largest());
    size_t rows = (size_t)n_dec_layers(c) * 2 * c.n_heads, rowb = (size_t)c.head_dim * m->esz;
    if (s.len > 0) {
        hipError_t e = hipMemcpy2DAsync((char*)m->pool.ptr + base * m->esz, cap * rowb, (const char*)m->pool.ptr + s.base * m->esz,
                                        s.cap * rowb, s.len * rowb, rows, hipMemcpyDeviceToDevice, m->stream);
        if (e != hipSuccess) {
            m->pool.release(base, elems);
            return fail(EXE_ERR_HIP, "K/V relocation copy: %s", hipGetErrorString(e));
        }
    }
    m->pool.release(s.base, s.elems);
    s.base = base;
    s.elems = elems;
    s.cap = cap;
    return EXE_OK;
}

extern "C" int exe_kv_compact(exe_model_t* m, uint64_t* moved_bytes)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    if (moved_bytes) *moved_bytes = 0;
    if (paged(m)) return EXE_OK;           // blocks are interchangeable: nothing to compact
    struct Ext { int64_t base, elems; int seq; bool cross; };
    std::vector<Ext> ex;
    for (int i = 0; i < m->c.max_seqs; ++i) {
        const Seq& s = m->seqs[i];
        if (!s.live) continue;
        if (s.base >= 0 && s.elems > 0) ex.push_back({s.base, s.elems, i, false});
        if (s.xbase >= 0 && s.xelems > 0) ex.push_back({s.xbase, s.xelems, i, true});
    }
    std::sort(ex.begin(), ex.end(), [](const Ext& a, const Ext& b) { return a.base < b.base; });
    // the free list is what lies between the extents
    auto rebuild_free = [&]() {
        m->pool.free_.clear();
        int64_t at = 0;
        for (const Ext& e : ex) {
            if (e.base > at) m->pool.free_[at] = e.base - at;
            at = e.base + e.elems;
        }
        if (m->pool.elems > at) m->pool.free_[at] = m->pool.elems - at;
    };
    int64_t end = 0;           // first element not occupied by the extents placed so far
    uint64_t moved = 0;
    for (Ext& e : ex) {
        int64_t shift = e.base - end;
        if (shift > 0 && (e.elems + shift - 1) / shift <= 64) {
            // forward move in pieces that do not overlap their own source
            for (int64_t o = 0; o < e.elems; o += shift) {
                int64_t n = std::min(shift, e.elems - o);
                hipError_t h = hipMemcpyAsync((char*)m->pool.ptr + (end + o) * m->esz, (const char*)m->pool.ptr + (e.base + o) * m->esz,
                                              (size_t)n * m->esz, hipMemcpyDeviceToDevice, m->stream);
                if (h != hipSuccess) {
                    // a device error: this extent stays registered where it was (its entries may be damaged where
                    // the pieces already enqueued overlap it); the extents moved before it keep their new places
                    (void)hipStreamSynchronize(m->stream);
                    rebuild_free();
                    return fail(EXE_ERR_HIP, "K/V compaction copy: %s", hipGetErrorString(h));
                }
            }
            moved += (uint64_t)e.elems * m->esz;
            Seq& s = m->seqs[e.seq];
            if (e.cross) s.xbase = end; else s.base = end;
            e.base = end;
        }
        end = e.base + e.elems;
    }
    rebuild_free();
    if (moved_bytes) *moved_bytes = moved;
    return EXE_OK;
}

extern "C" int exe_kv_stats(exe_model_t* m, uint64_t* pool_bytes, uint64_t* used_bytes, uint64_t* largest_free_bytes,
                            int32_t* live_seqs)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    if (paged(m)) {
        uint64_t blk = (uint64_t)n_dec_layers(m->c) * m->blk_elems * m->esz;      // one block id across all layers
        if (pool_bytes) *pool_bytes = blk * m->n_blocks;
        if (used_bytes) *used_bytes = blk * (m->n_blocks - m->free_blocks.size());
        if (largest_free_bytes) *largest_free_bytes = blk * m->free_blocks.size();
        if (live_seqs) *live_seqs = m->live;
        return EXE_OK;
    }
    if (pool_bytes) *pool_bytes = (uint64_t)m->pool.elems * m->esz;
    if (used_bytes) *used_bytes = (uint64_t)m->pool.used * m->esz;
    if (largest_free_bytes) *largest_free_bytes = (uint64_t)m->pool.largest() * m->esz;
    if (live_seqs) *live_seqs = m->live;
    return EXE_OK;
}

// ---------------------------------------------------------------- profile sweep
// splitmix64 + Box-Muller: the same lengths on every platform
struct Rng {
    uint64_t s;
    uint64_t next() { uint64_t z = (s += 0x9E3779B97F4A7C15ull); z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull; z = (z ^ (z >> 27)) * 0x94D049BB133111EBull; return z ^ (z >> 31); }
    double uniform() { return ((next() >> 11) + 0.5) * (1.0 / 9007199254740992.0); }
    double normal() { return std::sqrt(-2.0 * std::log(uniform())) * std::cos(6.283185307179586 * uniform()); }
};

struct EventTimer {
    hipEvent_t a = nullptr, b = nullptr;
    ~EventTimer() { if (a) (void)hipEventDestroy(a); if (b) (void)hipEventDestroy(b); }
    hipError_t init() { hipError_t e = hipEventCreate(&a); return e != hipSuccess ? e : hipEventCreate(&b); }
};

static double attn_ms_of(exe_model* m)
{
    exe_kernel_time_t rows[EXE_K_COUNT];
    if (exe_kernel_times(m, rows)) return 0.0;
    return rows[EXE_K_PREFILL_ATTN].ms + rows[EXE_K_DECODE_ATTN].ms + rows[EXE_K_CROSS_ATTN].ms;
}

// One row of the table: a single layer (layer 0's weights) on `lens`, K/V of one layer only.
static int profile_row(exe_model* m, int phase, const std::vector<int>& lens, int n_steps, exe_profile_row_t* row)
{
    const exe_config_t& c = m->c;
    bool encdec = c.arch == EXE_ARCH_ENC_DEC;
    int n = (int)lens.size();
    int64_t total = 0;
    for (int L : lens) total += L;
    row->total_tokens = (int32_t)std::min<int64_t>(total, 0x7fffffff);
    if (n > c.max_batch_seqs) return fail(EXE_ERR_ARG, "profile batch %d exceeds max_batch_seqs %d", n, c.max_batch_seqs);
    if (phase == 0 && total > c.max_batch_tokens) return fail(EXE_ERR_ARG, "profile batch of %lld tokens exceeds max_batch_tokens %d", (long long)total, c.max_batch_tokens);

    // single-layer extents
    std::vector<Seq> fresh(n);
    auto rollback = [&]() {
        for (auto& s : fresh) {
            if (s.base >= 0) m->pool.release(s.base, s.elems);
            if (s.xbase >= 0) m->pool.release(s.xbase, s.xelems);
        }
    };
    for (int i = 0; i < n; ++i) {
        Seq& s = fresh[i];
        int self_len = encdec ? (phase == 0 ? 1 : std::max(1, lens[i] / 12)) : lens[i];
        s.len = self_len;
        s.cap = round8(self_len + 1);
        s.elems = (int64_t)2 * m->inner * s.cap;
        s.base = m->pool.alloc(s.elems);
        bool ok = s.base >= 0;
        if (ok && encdec) {
            s.n_in = lens[i];
            s.xelems = (int64_t)2 * m->inner * round8(lens[i]);
            s.xbase = m->pool.alloc(s.xelems);
            ok = s.xbase >= 0;
        }
        if (!ok) { rollback(); return fail(EXE_ERR_OOM_KV, "K/V pool too small for one layer of this profile row"); }
    }
    // K/V that is read without having been written by this run must be finite: 0x3c3c is 0.0115 in bf16,
    // 0x3c3c3c3c is 0.0115 in float
    hipError_t he = hipSuccess;
    for (int i = 0; i < n && he == hipSuccess; ++i) {
        he = hipMemsetAsync((char*)m->pool.ptr + fresh[i].base * m->esz, 0x3c, (size_t)fresh[i].elems * m->esz, m->stream);
        if (he == hipSuccess && encdec)
            he = hipMemsetAsync((char*)m->pool.ptr + fresh[i].xbase * m->esz, 0x3c, (size_t)fresh[i].xelems * m->esz, m->stream);
    }
    if (he == hipSuccess) he = hipMemsetAsync(m->h, 0, (size_t)m->rows_cap * c.d_model * sizeof(float), m->stream);
    if (he != hipSuccess) { rollback(); return fail(EXE_ERR_HIP, "profile memset: %s", hipGetErrorString(he)); }

    Stager st{m};
    EncodeDesc ed{};
    DecodeDesc dd{};
    int rows_n;
    const DecLayerW* L;
    double ab = 0, af = 0;
    if (phase == 0) {
        fill_encode_desc(m, st, ed, n, lens, nullptr, fresh);
        prefill_attn_work(m, lens, (int)total, &ab, &af);
        rows_n = (int)total;
        L = encdec ? &m->enc[0] : &m->dec[0];
    } else {
        std::vector<DecodeSeq> ds(n);
        for (int i = 0; i < n; ++i)
            ds[i] = DecodeSeq{0, fresh[i].len - 1 > 0 ? fresh[i].len - 1 : 0, fresh[i].cap, fresh[i].base, fresh[i].n_in,
                              fresh[i].xbase < 0 ? 0 : fresh[i].xbase};
        fill_decode_desc(m, st, dd, ds);
        rows_n = n;
        L = &m->dec[0];
    }
    auto layer = [&](int parts) -> int {
        return phase == 0 ? encode_layer(m, *L, 0, n, rows_n, ed, ab, af, parts) : decode_layer(m, *L, 0, n, dd, parts);
    };
    auto body = [&]() -> int {
        if (st.off > m->stage_bytes) return fail(EXE_ERR_ARG, "descriptor staging overflow");
        HIP_TRY(hipMemcpyAsync(m->stage_d, m->stage_h, st.off, hipMemcpyHostToDevice, m->stream));
        EventTimer t;
        HIP_TRY(t.init());
        int r;
        for (int w = 0; w < 3; ++w)
            if ((r = layer(3))) return r;
        // pass A: whole-layer latency per repetition (launch gaps included), no per-kernel events
        std::vector<double> layer_ms(n_steps);
        for (int i = 0; i < n_steps; ++i) {
            HIP_TRY(hipEventRecord(t.a, m->stream));
            if ((r = layer(3))) return r;
            HIP_TRY(hipEventRecord(t.b, m->stream));
            HIP_TRY(hipEventSynchronize(t.b));
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, t.a, t.b));
            layer_ms[i] = ms;
        }
        // pass B: the attention kernels alone, from events around each launch
        bool was_on = m->timer.on;
        exe_kernel_timing(m, 1);
        double attn = 0;
        for (int i = 0; i < n_steps; ++i) {
            if ((r = layer(2))) { exe_kernel_timing(m, was_on); return r; }
            attn += attn_ms_of(m);
        }
        exe_kernel_timing(m, was_on);
        attn /= n_steps;
        double mean = 0, var = 0;
        for (double x : layer_ms) mean += x;
        mean /= n_steps;
        for (double x : layer_ms) var += (x - mean) * (x - mean);
        row->attn_ms_per_layer = (float)attn;
        row->rest_ms_per_layer = (float)std::max(0.0, mean - attn);
        row->std_ms = (float)std::sqrt(var / n_steps);
        // head: final norm + LM head + argmax (decode: n rows; encode: the last row of each sequence);
        // encoder-decoder encode: final norm + one decoder layer's cross K/V projection and store
        double head = 0;
        if (phase == 0 && encdec) {
            HIP_TRY(hipEventRecord(t.a, m->stream));
            for (int i = 0; i < n_steps; ++i) {
                if ((r = run_norm(m, nullptr, rows_n, m->enc_fin_g, nullptr, 1.f, m->a))) return r;
                if ((r = run_gemm(m, rows_n, 2 * m->inner, c.d_model, m->a, m->dec[0].w_xkv, nullptr, -1, 1.f, OUT_T, m->qkv))) return r;
                LAUNCH(m, EXE_K_OTHER, 0.0, 0.0,
                       launch_kv_append(c.dtype, m->qkv, 2 * m->inner, 0, m->inner, rows_n, ed.tok_b, ed.tok_pos, ed.xbase,
                                        ed.xcap, 0, c.n_heads, c.head_dim, m->pool.ptr, m->stream));
            }
            HIP_TRY(hipEventRecord(t.b, m->stream));
            HIP_TRY(hipEventSynchronize(t.b));
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, t.a, t.b));
            head = ms / n_steps * c.n_dec_layers;
        } else if (c.has_lm_head) {
            HIP_TRY(hipEventRecord(t.a, m->stream));
            for (int i = 0; i < n_steps; ++i)
                if ((r = head_launches(m, phase == 0 ? ed.last : nullptr, n))) return r;
            HIP_TRY(hipEventRecord(t.b, m->stream));
            HIP_TRY(hipEventSynchronize(t.b));
            float ms = 0.f;
            HIP_TRY(hipEventElapsedTime(&ms, t.a, t.b));
            head = ms / n_steps;
        }
        row->head_ms = (float)head;
        int layers = phase == 0 ? c.n_layers : n_dec_layers(c);
        row->full_step_ms = (float)(layers * mean + head);
        row->n_timed = n_steps;
        return EXE_OK;
    };
    int r = body();
    (void)hipStreamSynchronize(m->stream);
    rollback();
    return r;
}

extern "C" int exe_profile(exe_model_t* m, int32_t phase, const int32_t* batch_sizes, int32_t n_batch,
                           const int32_t* lengths, int32_t n_len, const exe_length_dist_t* dist, int32_t n_steps,
                           exe_profile_row_t* rows, int32_t rows_cap, int32_t* n_rows)
{
    if (!m) return fail(EXE_ERR_ARG, "null model");
    if (n_rows) *n_rows = 0;
    if ((phase != 0 && phase != 1) || !batch_sizes || !lengths || n_batch < 1 || n_len < 1 || n_steps < 1 || !rows || !n_rows)
        return fail(EXE_ERR_ARG, "bad profile arguments");
    if (rows_cap < n_batch * n_len) return fail(EXE_ERR_ARG, "rows_cap %d < %d rows", rows_cap, n_batch * n_len);
    if (m->live > 0) return fail(EXE_ERR_BAD_SEQ, "exe_profile needs a model with no live sequence (%d live)", m->live);
    if (dist && dist->kind != 0 && dist->kind != 1) return fail(EXE_ERR_ARG, "bad length distribution kind");
    bool ragged = dist && dist->kind == 1;
    bool learned = m->c.has_embed && m->c.pos == EXE_POS_LEARNED;
    for (int bi = 0; bi < n_batch; ++bi)
        for (int li = 0; li < n_len; ++li) {
            int B = batch_sizes[bi], Lm = lengths[li];
            if (B < 1 || Lm < 1) return fail(EXE_ERR_ARG, "batch and length must be positive");
            std::vector<int> lens(B, Lm);
            if (ragged) {
                Rng rng{dist->seed + (uint64_t)bi * 1000003ull + (uint64_t)li};
                for (int i = 0; i < B; ++i) {
                    double x = std::nearbyint((double)Lm + (double)dist->std * rng.normal());
                    lens[i] = (int)std::min<double>(std::max<double>(x, dist->lo), dist->hi);
                    if (lens[i] < 1) lens[i] = 1;
                }
            }
            // a learned position table has max_pos rows: an input of max_pos tokens, and a decode step whose K/V
            // length after the append is max_pos, are its longest valid cases; ragged draws are clipped to that,
            // a uniform length beyond it is an error (the row would otherwise carry a length that did not run)
            if (learned && Lm > m->c.max_pos)
                return fail(EXE_ERR_BAD_LENGTH, "profile length %d exceeds max_pos %d", Lm, m->c.max_pos);
            if (learned)
                for (int& L : lens) L = std::min(L, m->c.max_pos);
            exe_profile_row_t* row = &rows[*n_rows];
            memset(row, 0, sizeof(*row));
            row->phase = phase; row->batch = B; row->length = Lm; row->ragged = ragged ? 1 : 0;
            int r = profile_row(m, phase, lens, n_steps, row);
            if (r) return r;
            ++*n_rows;
        }
    return EXE_OK;
}

// ---------------------------------------------------------------- RRA schedule (single GPU)
static double now_s()
{
    return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

extern "C" int exe_run_rra(exe_model_t* m, const exe_rra_config_t* cfg, int32_t n_requests, const int32_t* input_lengths,
                           const int32_t* output_lengths, const int32_t* tokens_packed, int32_t* out_tokens,
                           exe_rra_stats_t* stats)
{
    if (!m || !cfg || !input_lengths || !output_lengths || !tokens_packed || !stats) return fail(EXE_ERR_ARG, "null argument");
    const exe_config_t& c = m->c;
    if (!c.has_embed || !c.has_lm_head) return fail(EXE_ERR_SHAPE, "exe_run_rra needs token embedding and LM head");
    if (m->live > 0) return fail(EXE_ERR_BAD_SEQ, "exe_run_rra needs a model with no live sequence");
    if (n_requests < 1 || cfg->decode_batch < 1 || cfg->n_decode < 1 || cfg->max_encode_batch < 1)
        return fail(EXE_ERR_ARG, "bad schedule parameters");
    if (cfg->decode_batch > c.max_batch_seqs || cfg->decode_batch > c.max_seqs || cfg->max_encode_batch > c.max_batch_seqs)
        return fail(EXE_ERR_ARG, "decode_batch / max_encode_batch exceed the model's limits");
    bool dec_only = c.arch == EXE_ARCH_DECODER_ONLY;
    std::vector<int64_t> tok_off(n_requests + 1, 0), out_off(n_requests + 1, 0);
    double mean_in = 0;
    for (int i = 0; i < n_requests; ++i) {
        if (input_lengths[i] < 1 || output_lengths[i] < 1) return fail(EXE_ERR_BAD_LENGTH, "request %d has an empty input or output", i);
        tok_off[i + 1] = tok_off[i] + input_lengths[i];
        out_off[i + 1] = out_off[i] + output_lengths[i];
        mean_in += input_lengths[i];
    }
    mean_in /= n_requests;

    const int BD = cfg->decode_batch;
    std::vector<int> slot_req(BD, -1), slot_done(BD, 0), slot_tok(BD, 0);   // request in a slot, tokens produced, last token
    std::vector<int> free_slots;
    for (int s = BD - 1; s >= 0; --s) free_slots.push_back(s);
    std::vector<double> t_admit(n_requests, 0.0), t_finish(n_requests, 0.0);
    memset(stats, 0, sizeof(*stats));
    int next_req = 0, finished = 0, live = 0;
    double batch_sum = 0;
    double t0 = now_s();

    auto emit = [&](int slot, int token, double t) -> bool {   // records a generated token; true if the request is done
        int r = slot_req[slot];
        if (out_tokens) out_tokens[out_off[r] + slot_done[slot]] = token;
        slot_tok[slot] = token;
        slot_done[slot] += 1;
        stats->generated_tokens += 1;
        if (slot_done[slot] < output_lengths[r]) return false;
        t_finish[r] = t;
        return true;
    };
    auto retire = [&](const std::vector<int>& slots) -> int {
        if (slots.empty()) return EXE_OK;
        int r = exe_seq_release(m, (int)slots.size(), slots.data());
        if (r) return r;
        for (int s : slots) { slot_req[s] = -1; free_slots.push_back(s); --live; ++finished; }
        return EXE_OK;
    };

    std::vector<int32_t> ids, lens, res, toks, kv, nxt;
    while (finished < n_requests) {
        // ---- encoding phase: B_E = the queries completed since the decode batch was last full, i.e. its free
        // slots.  When every phase admits all it asks for, that is the number completed during the previous decoding
        // phase (Section 4); a phase cut short (workload adjustment below, or a full K/V pool) leaves its remainder
        // to the next phase, whose B_E is raised accordingly, so the decode batch returns to B_D (Section 5).
        int want = std::min(BD - live, n_requests - next_req);
        double budget = cfg->adjust ? (1.0 + cfg->workload_tolerance) * std::max(1, want) * mean_in : 1e300;
        double taken = 0;
        if (want > 0) stats->encode_phases += 1;
        while (want > 0) {
            ids.clear(); lens.clear(); res.clear();
            int64_t first_tok = tok_off[next_req], T = 0;
            int first_req = next_req;
            while (want > 0 && (int)ids.size() < cfg->max_encode_batch && next_req < n_requests) {
                int L = input_lengths[next_req];
                if (T + L > c.max_batch_tokens) break;
                if (!ids.empty() || taken > 0) if (taken + L > budget) { want = 0; break; }   // workload adjustment
                int s = free_slots.back();
                free_slots.pop_back();
                ids.push_back(s); lens.push_back(L);
                res.push_back(dec_only ? L + output_lengths[next_req] : output_lengths[next_req]);
                slot_req[s] = next_req; slot_done[s] = 0;
                T += L; taken += L;
                ++next_req; --want;
            }
            if (ids.empty()) {
                if (next_req < n_requests && input_lengths[next_req] > c.max_batch_tokens)
                    return fail(EXE_ERR_ARG, "request %d is longer than max_batch_tokens", next_req);
                break;
            }
            nxt.assign(ids.size(), 0);
            double ta = now_s();
            int r = exe_encode(m, (int)ids.size(), ids.data(), lens.data(), tokens_packed + first_tok, res.data(), nullptr,
                               dec_only ? nxt.data() : nullptr, nullptr);
            if (r == EXE_ERR_OOM_KV && live > 0) {
                // the pool cannot take this batch yet: put the requests back and decode on; sequences that
                // finish will free their extents before the next encoding phase
                for (int s : ids) { slot_req[s] = -1; free_slots.push_back(s); }
                next_req = first_req;
                break;
            }
            if (r) return r;
            double tb = now_s();
            stats->encode_s += tb - ta;
            stats->encode_calls += 1;
            stats->encoded_tokens += T;
            live += (int)ids.size();
            std::vector<int> done;
            for (size_t k = 0; k < ids.size(); ++k) {
                t_admit[first_req + k] = ta - t0;
                if (dec_only) { if (emit(ids[k], nxt[k], tb - t0)) done.push_back(ids[k]); }
                else slot_tok[ids[k]] = 0;                    // encoder-decoder: decoding starts from token id 0
            }
            if ((r = retire(done))) return r;
        }
        if (live == 0) {
            if (next_req >= n_requests) break;
            continue;                                         // nothing to decode: go straight to the next encoding phase
        }
        // ---- decoding phase: N_D iterations over the live batch
        for (int it = 0; it < cfg->n_decode && live > 0; ++it) {
            ids.clear(); toks.clear(); kv.clear();
            for (int s = 0; s < BD; ++s) {
                if (slot_req[s] < 0) continue;
                ids.push_back(s);
                toks.push_back(slot_tok[s]);
                int r = slot_req[s];
                kv.push_back(dec_only ? input_lengths[r] + slot_done[s] : slot_done[s] + 1);
            }
            nxt.assign(ids.size(), 0);
            double ta = now_s();
            int r = exe_decode_step(m, (int)ids.size(), ids.data(), toks.data(), kv.data(), nullptr, nxt.data(), nullptr);
            if (r) return r;
            double tb = now_s();
            stats->decode_s += tb - ta;
            stats->decode_iterations += 1;
            batch_sum += (double)ids.size();
            std::vector<int> done;
            for (size_t k = 0; k < ids.size(); ++k)
                if (emit(ids[k], nxt[k], tb - t0)) done.push_back(ids[k]);
            if ((r = retire(done))) return r;
        }
    }
    stats->wall_s = now_s() - t0;
    stats->mean_decode_batch = stats->decode_iterations ? batch_sum / stats->decode_iterations : 0.0;
    std::vector<double> lat(n_requests), q(n_requests);
    for (int i = 0; i < n_requests; ++i) { lat[i] = t_finish[i] - t_admit[i]; q[i] = t_admit[i]; stats->latency_mean_s += lat[i] / n_requests; }
    std::sort(lat.begin(), lat.end());
    std::sort(q.begin(), q.end());
    auto pct = [&](const std::vector<double>& v, double p) { return v[std::min<size_t>(v.size() - 1, (size_t)(p * v.size()))]; };
    stats->latency_p50_s = pct(lat, 0.50);
    stats->latency_p99_s = pct(lat, 0.99);
    stats->latency_max_s = lat.back();
    stats->queue_p99_s = pct(q, 0.99);
    return EXE_OK;
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

// ---------------------------------------------------------------- GEMM without allocations
// The split-K partial sums of exe_op_gemm_noalloc live in this array instead of a caller workspace.  Every GPU the
// library runs on holds its own copy until the process ends.  In host code the array's name is only a stand-in for
// the symbol, never a device address: the address on the current device comes from hipGetSymbolAddress, once per
// device, and only that pointer is handed to kernels.
#define EXE_NOALLOC_SCRATCH_BYTES (64ull << 20)
static __device__ __align__(256) unsigned char scratch[EXE_NOALLOC_SCRATCH_BYTES];

static int noalloc_scratch(void** out)
{
    constexpr int MAXDEV = 64;
    static std::once_flag once[MAXDEV];
    static void* ptr[MAXDEV];
    static hipError_t err[MAXDEV];
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAXDEV) return fail(EXE_ERR_ARG, "device %d is beyond the %d this entry point serves", dev, MAXDEV);
    std::call_once(once[dev], [&]() {
        void* p = nullptr;
        err[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        ptr[dev] = err[dev] == hipSuccess ? p : nullptr;
    });
    if (err[dev] != hipSuccess || !ptr[dev]) return fail(EXE_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(err[dev]));
    *out = ptr[dev];
    return EXE_OK;
}

extern "C" uint64_t exe_op_gemm_noalloc_max_workspace(void) { return EXE_NOALLOC_SCRATCH_BYTES; }

extern "C" int exe_op_gemm_noalloc(void* hip_stream, int32_t dtype, int32_t M, int32_t N, int32_t K, const void* A,
                                   const void* W, const void* bias, int32_t act, float alpha, int32_t out_mode, void* out)
{
    if (M < 0 || N < 1 || K < 1 || !A || !W || !out) return fail(EXE_ERR_ARG, "bad gemm arguments");
    if (dtype != DT_F32 && dtype != DT_BF16) return fail(EXE_ERR_ARG, "bad dtype");
    if (out_mode < 0 || out_mode > 2) return fail(EXE_ERR_ARG, "bad out_mode");
    if (K % 8 || N % 4) return fail(EXE_ERR_SHAPE, "K must be a multiple of 8 and N of 4");
    size_t need = gemm_workspace_bytes(dtype, M, N, K);
    if (need > EXE_NOALLOC_SCRATCH_BYTES)
        return fail(EXE_ERR_SHAPE, "this shape's split-K partial sums take %llu bytes, the static scratch holds %llu",
                    (unsigned long long)need, (unsigned long long)EXE_NOALLOC_SCRATCH_BYTES);
    void* ws = nullptr;
    int r = noalloc_scratch(&ws);
    if (r) return r;
    // every partial sum that the reduction reads is written by the GEMM launch before it, so nothing left in the
    // array by an earlier call is ever read and nothing needs clearing
    GemmArgs g{dtype, M, N, K, A, W, bias, act, alpha, out_mode, out, (float*)ws, (size_t)EXE_NOALLOC_SCRATCH_BYTES};
    HIP_TRY(launch_gemm(g, (hipStream_t)hip_stream));
    return EXE_OK;
}

extern "C" int exe_op_gemm_plan(int32_t dtype, int32_t M, int32_t N, int32_t K, int32_t* route, int32_t* cfg, int32_t* splits,
                                int32_t* rows_first)
{
    if (M < 1 || N < 1 || K < 1 || !route || !cfg || !splits || !rows_first) return fail(EXE_ERR_ARG, "bad gemm plan arguments");
    gemm_plan_info(dtype, M, N, K, route, cfg, splits, rows_first);
    return EXE_OK;
}

extern "C" int exe_op_paged_index_check(int32_t dtype, int32_t dh, int32_t block_size, int32_t n_waves, int32_t len)
{
    int shift = 0;
    while ((1 << shift) < block_size) ++shift;
    if ((dtype != DT_F32 && dtype != DT_BF16) || (dh != 64 && dh != 128) || block_size < 8 || block_size > 4096 ||
        (1 << shift) != block_size || (n_waves != 4 && n_waves != 16) || len < 1)
        return fail(EXE_ERR_ARG, "bad paged index check arguments");
    return paged_index_check(dtype, dh, shift, n_waves, len);
}

extern "C" int exe_op_gemm_ld(void* hip_stream, int32_t dtype, int32_t M, int32_t N, int32_t K, const void* A, int32_t lda,
                              const void* W, int32_t ldw, const void* bias, int32_t act, float alpha, int32_t out_mode,
                              void* out, void* workspace, uint64_t workspace_bytes)
{
    if (M < 0 || N < 1 || K < 1 || !A || !W || !out) return fail(EXE_ERR_ARG, "bad gemm arguments");
    if (dtype != DT_BF16) return fail(EXE_ERR_ARG, "strided rows are a bf16 feature");
    if (out_mode < 0 || out_mode > 2) return fail(EXE_ERR_ARG, "bad out_mode");
    if (K % 64 || N % 4 || lda < K || ldw < K || lda % 8 || ldw % 8) return fail(EXE_ERR_SHAPE, "K must be a multiple of 64, N of 4, strides of 8 and >= K");
    if (gemm_route(dtype, M, N, K) != 0) return fail(EXE_ERR_SHAPE, "shape not served by the tile kernel");
    if (gemm_workspace_bytes(dtype, M, N, K) > workspace_bytes) return fail(EXE_ERR_ARG, "workspace too small");
    GemmArgs g{dtype, M, N, K, A, W, bias, act, alpha, out_mode, out, (float*)workspace, (size_t)workspace_bytes};
    g.lda = lda;
    g.ldw = ldw;
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
    std::vector<int32_t> host, lens(n_seqs);
    host.resize((size_t)2 * T + n_seqs + 1);
    int max_len = 0;
    for (int i = 0; i < n_seqs; ++i) {
        int L = cu_seqlens[i + 1] - cu_seqlens[i];
        if (L < 1) return fail(EXE_ERR_BAD_LENGTH, "empty sequence");
        max_len = std::max(max_len, L);
        for (int p = 0; p < L; ++p) { host[cu_seqlens[i] + p] = i; host[T + cu_seqlens[i] + p] = p; }
        lens[i] = L;
    }
    for (int i = 0; i <= n_seqs; ++i) host[2 * T + i] = cu_seqlens[i];
    size_t tiles_at = host.size();
    prefill_tile_order(lens.data(), n_seqs, host);
    int n_tiles = (int)((host.size() - tiles_at) / 2);
    int32_t* dev = nullptr;
    HIP_TRY(hipMalloc((void**)&dev, host.size() * 4));
    hipError_t e = hipMemcpyAsync(dev, host.data(), host.size() * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) {
        AttnPackedArgs a{dtype, T, H, dh, n_seqs, qkv, dev, dev + T, dev + 2 * T, causal, scale, bias_by_dist, bias_radius,
                         out, dev + 2 * T + n_seqs + 1, n_tiles, force_generic};
        a.max_len = max_len;
        e = launch_attn_packed(a, s);
    }
    hipError_t e2 = hipStreamSynchronize(s);
    (void)hipFree(dev);
    if (e != hipSuccess) return fail(EXE_ERR_HIP, "prefill attention: %s", hipGetErrorString(e));
    if (e2 != hipSuccess) return fail(EXE_ERR_HIP, "prefill attention: %s", hipGetErrorString(e2));
    return EXE_OK;
}

extern "C" int exe_op_prefill_tiles(int32_t n_seqs, const int32_t* lengths, int32_t* tiles, int32_t cap, int32_t* n_tiles)
{
    if (n_seqs < 0 || (n_seqs > 0 && !lengths) || !n_tiles || cap < 0 || (cap > 0 && !tiles)) return fail(EXE_ERR_ARG, "bad tile list arguments");
    for (int i = 0; i < n_seqs; ++i)
        if (lengths[i] < 1) return fail(EXE_ERR_BAD_LENGTH, "empty sequence");
    std::vector<int32_t> tl;
    prefill_tile_order(lengths, n_seqs, tl);
    *n_tiles = (int32_t)(tl.size() / 2);
    if (*n_tiles > cap) return fail(EXE_ERR_ARG, "tile list needs %d pairs, capacity %d", *n_tiles, cap);
    std::copy(tl.begin(), tl.end(), tiles);
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

extern "C" int exe_op_decode_attention_paged(void* hip_stream, int32_t dtype, int32_t B, const void* q, int32_t q_stride,
                                             const void* kv_blocks, const int32_t* block_table, int32_t max_blocks,
                                             int32_t block_size, const int32_t* len, const int32_t* qpos, int32_t H,
                                             int32_t dh, float scale, const float* bias_by_dist, int32_t bias_radius,
                                             int32_t new_kv_offset, void* out)
{
    if (B < 0 || !q || !kv_blocks || !block_table || !len || !qpos || !out || H < 1 || max_blocks < 1)
        return fail(EXE_ERR_ARG, "bad paged decode attention arguments");
    if (dh != 64 && dh != 128) return fail(EXE_ERR_SHAPE, "head_dim must be 64 or 128");
    int shift = 0;
    while ((1 << shift) < block_size) ++shift;
    if (block_size < 8 || block_size > 4096 || (1 << shift) != block_size)
        return fail(EXE_ERR_ARG, "block_size %d is not a power of two in [8, 4096]", block_size);
    AttnPagedArgs a{dtype, B, H, dh, q, q_stride, kv_blocks, block_table, max_blocks, shift, len, qpos, scale, bias_by_dist,
                    bias_radius, out};
    if (new_kv_offset > 0) {
        a.new_k_off = new_kv_offset;
        a.new_v_off = 2 * new_kv_offset;
    }
    HIP_TRY(launch_attn_paged(a, (hipStream_t)hip_stream));
    return EXE_OK;
}

extern "C" int exe_op_argmax(void* hip_stream, const float* logits, int32_t rows, int32_t n, int32_t* out)
{
    if (!logits || !out || rows < 0 || n < 1) return fail(EXE_ERR_ARG, "bad argmax arguments");
    HIP_TRY(launch_argmax(logits, rows, n, out, (hipStream_t)hip_stream));
    return EXE_OK;
}
