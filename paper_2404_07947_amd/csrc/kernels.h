// Launchers of the gfx950 kernels.  All pointers are device pointers unless a comment says host.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace exe {

struct GemmArgs {
    int dtype;            // DT_F32 / DT_BF16: type of A, W, bias and (for OUT_T) out
    int M, N, K;
    const void* A;        // [M, K] row-major
    const void* W;        // [N, K] row-major
    const void* bias;     // [N] or nullptr
    int act;              // -1 none, 0 relu, 1 gelu(erf); applied in OUT_T mode
    float alpha;          // result = alpha * (A.W^T) + bias
    int out_mode;         // OUT_T, OUT_RESID (float out += result), OUT_F32
    void* out;            // [M, N]
    float* workspace;     // split-K partial sums
    size_t workspace_bytes;
    int lda = 0, ldw = 0; // row strides of A and W in elements (0 = K); the generic kernel takes dense rows only
};
size_t gemm_workspace_bytes(int dtype, int M, int N, int K);
// which kernel family a shape runs on: 0 tile (MFMA), 2 generic (plain FMA)
int gemm_route(int dtype, int M, int N, int K);
// how a shape is launched: route (as gemm_route), tile configuration (0 64x256, 1 128x256, 2 256x256, 3 64x128,
// 4 128x128, 5 256x128), split-K parts, and the leading rows that the first launch takes (M unless the rows beyond
// whole rounds of tiles go to a second launch)
void gemm_plan_info(int dtype, int M, int N, int K, int* route, int* cfg, int* splits, int* rows_first);
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);

hipError_t launch_embed(int dtype, const int32_t* tokens, const int32_t* pos, int T, int d, const void* tok_emb,
                        const void* pos_emb, float* h, hipStream_t s);
hipError_t launch_load_hidden(int dtype, const void* x, int64_t n, float* h, hipStream_t s);
hipError_t launch_store_hidden(int dtype, const float* h, int64_t n, void* out, hipStream_t s);
hipError_t launch_norm(int dtype, int rms, const float* x, const int32_t* row_index, int rows, int d,
                       const void* gain, const void* shift, float eps, float out_scale, void* out, hipStream_t s);
// copies K and V rows of `src` (row stride ld, K at column k_off, V at v_off) into the cache:
// token t belongs to batch entry tok_b[t] (t itself if nullptr) at position tok_pos[t];
// K of (b, head, pos) lives at pool + base[b] + ((layer*2+0)*H + head)*cap[b]*dh + pos*dh, V at kv index 1.
hipError_t launch_kv_append(int dtype, const void* src, int ld, int k_off, int v_off, int T, const int32_t* tok_b,
                            const int32_t* tok_pos, const int64_t* base, const int32_t* cap, int layer, int H, int dh,
                            void* pool, hipStream_t s);
hipError_t launch_kv_append_paged(int dtype, const void* src, int ld, int k_off, int v_off, int T, const int32_t* tok_b,
                                  const int32_t* tok_pos, const int32_t* table, int table_w, int shift, int H, int dh,
                                  void* layer_pool, hipStream_t s);
hipError_t launch_argmax(const float* logits, int rows, int n, int32_t* out, hipStream_t s);

struct AttnCacheArgs {       // one query row per batch entry against that sequence's cached K/V
    int dtype, B, H, dh;
    const void* q; int q_stride;          // q of (b, head) at q + b*q_stride + head*dh
    const void* pool;
    const int64_t* base; const int32_t* cap; const int32_t* len; const int32_t* qpos;
    int layer;                             // K at base + ((layer*2)*H + head)*cap*dh
    float scale;
    const float* bias_by_dist; int bias_radius;   // [H, 2r+1] or nullptr
    void* out;                             // [B, H*dh]
    // fused append (optional): the new position's key / value rows of (b, head) are at
    // q + b*q_stride + new_k_off + head*dh and ... + new_v_off; the kernel stores them at position len-1 of the
    // cache and attends to them straight from there (new_k_off = 0 disables)
    int new_k_off = 0, new_v_off = 0;
    int mean_len = 0;                      // average of len over the batch (0 = unknown): picks the launch shape
};
hipError_t launch_attn_cache(const AttnCacheArgs& a, hipStream_t s);

struct AttnPagedArgs {       // as AttnCacheArgs, with the cache of one layer held in blocks of 2^block_shift positions
    int dtype, B, H, dh;
    const void* q; int q_stride;
    const void* pool;                      // block b at pool + b * 2*H*2^block_shift*dh elements: [K|V][head][row][dh]
    const int32_t* block_table; int max_blocks; int block_shift;    // [B, max_blocks]
    const int32_t* len; const int32_t* qpos;
    float scale;
    const float* bias_by_dist; int bias_radius;
    void* out;
    int new_k_off = 0, new_v_off = 0;      // fused append, as in AttnCacheArgs
    int mean_len = 0;
};
hipError_t launch_attn_paged(const AttnPagedArgs& a, hipStream_t s);
// host-side replay of the paged kernel's row indexing (0 = every row read lies in its block and is read once)
int paged_index_check(int dtype, int dh, int block_shift, int nwv, int len);

struct AttnPackedArgs {      // ragged prefill over packed qkv [T, 3*H*dh]
    int dtype, T, H, dh, n_seqs;
    const void* qkv;
    const int32_t* tok_b;    // [T] sequence index of each token
    const int32_t* tok_pos;  // [T] position in its sequence
    const int32_t* cu;       // [n_seqs+1] first token of each sequence
    int causal;
    float scale;
    const float* bias_by_dist; int bias_radius;
    void* out;               // [T, H*dh]
    // tile list for the MFMA kernel: (seq, first query row) pairs in the order prefill_tile_order gives
    const int32_t* tiles; int n_tiles;
    int force_generic;
    int max_len = 0;         // longest sequence of the batch (0 = unknown: T is taken)
};
bool prefill_mfma_supported(int dtype, int dh);
constexpr int PREFILL_TILE_Q = 128;
// Appends the (seq, first query row) pairs of a batch's 128-row query tiles to `tiles`: sequences longest first, the
// tiles of one sequence together, last rows (causal: most keys) first.  The tiles of a sequence read the same keys
// and values, and the kernel's workgroup numbering puts neighbours of this list (for one head) on one XCD at about
// the same time, so that they arrive in that XCD's L2 once; longest first keeps the short work for the end of the
// launch.  (Measured against most-work-first over the whole batch and over groups of 8 to 40 tiles: this order is
// the fastest or within 1 % of it on ragged and uniform batches, and halves the kernel's HBM reads.)
void prefill_tile_order(const int32_t* lens, int n_seqs, std::vector<int32_t>& tiles);
hipError_t launch_attn_packed(const AttnPackedArgs& a, hipStream_t s);

}  // namespace exe
