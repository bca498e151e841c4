// Attention kernels.
//
//  * attn_row_kernel<T, DH, PACKED>: one workgroup per (query row, head) streams that row's keys and values
//    with 16-byte loads, float dot products reduced over the lanes that share a key row, and an online
//    softmax whose partial results are merged across the workgroup at the end.
//      PACKED = false: decode / cross attention -- keys and values come from a sequence's cache extent
//                      ([head][capacity][dh] per layer, keys then values).  HBM-bandwidth bound.
//      PACKED = true : ragged prefill straight from the packed qkv activations (float configs, unusual
//                      head sizes); the MFMA kernel below replaces it for bf16 with head size 128.
//  * prefill_mfma_kernel<CAUSAL, BIAS>: flash-style ragged prefill for bf16, head size 128.  A workgroup
//    owns 128 query rows of one (sequence, head); keys/values go through LDS in tiles of 64.
//    S^T = K.Q^T and O^T = V^T.P^T are both computed with MFMA 16x16x32 so that softmax statistics of a
//    query live in the lanes of one accumulator column and P feeds the second MFMA straight from the first
//    one's accumulators.
#include <stdio.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "common.h"
#include "kernels.h"

namespace exe {

constexpr float LOG2E = 1.44269504088896340736f;
constexpr int ATTN_BIAS_LDS = 1024;       // entries of a head's bias table that the row kernel keeps in LDS
constexpr int ATTN_SHORT_LEN = 320;      // decode attention: mean rows per sequence up to which 4 waves serve a row

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename T, int EPL> struct Chunk;
template <> struct Chunk<float, 4> {
    static __device__ __forceinline__ void unpack(uint4 u, float* f)
    {
        f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y); f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
    }
};
template <> struct Chunk<bf16_t, 8> {
    static __device__ __forceinline__ void unpack(uint4 u, float* f)
    {
        f[0] = bf16lo(u.x); f[1] = bf16hi(u.x); f[2] = bf16lo(u.y); f[3] = bf16hi(u.y);
        f[4] = bf16lo(u.z); f[5] = bf16hi(u.z); f[6] = bf16lo(u.w); f[7] = bf16hi(u.w);
    }
};

// 16 bytes from global memory.  STREAM marks data that is read once (a sequence's cached keys and values during
// decode): a nontemporal load keeps it from displacing other lines in L2, measured 6.3 -> 6.9 .. 7.1 TB/s.
template <bool STREAM, typename T> __device__ __forceinline__ uint4 load_chunk(const T* p)
{
    if (STREAM) {
        typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
        v4u_t t = __builtin_nontemporal_load((const v4u_t*)p);
        return uint4{t.x, t.y, t.z, t.w};
    }
    return *(const uint4*)p;
}

// Paged cache indexing, shared by the kernel and by the host-side check paged_index_check below.
// paged_lookup_row: the row whose block look-up x of the step starting at row j names (nc rows are cached);
// paged_lane_row: the row that the lane group rg of load u of that step reads.
__host__ __device__ __forceinline__ int paged_lookup_row(int j, int x, int rpw, int nc)
{
    int row = j + x * rpw;
    return row < nc ? row : nc - 1;
}
__host__ __device__ __forceinline__ int paged_lane_row(int j, int u, int rg, int rpw, int nc)
{
    int row = j + u * rpw + rg;
    return row < nc ? row : nc - 1;
}

// PAGED (with PACKED = false): the cache of a sequence is a list of blocks of 2^block_shift positions instead of
// one extent.  Block b of the pool holds [K|V][head][position in block][DH]; block_table[r * max_blocks + i] is the
// block with positions i * 2^block_shift .. of sequence r.  The rows of one load of a wave (RPW <= 8 consecutive
// rows starting at a multiple of RPW) never straddle a block (block_shift >= 3).  The RPW * U rows of a whole step
// do not either when RPW * U <= 8: then one table look-up per wave and step suffices; otherwise (bf16, head size
// 64: 16 rows per step) every load of the step has a look-up of its own.
template <typename T, int DH, bool PACKED, int NWV = 4, int U = 4, bool PAGED = false>
__global__ __launch_bounds__(NWV * 64) void attn_row_kernel(
    const T* __restrict__ q, int q_stride, const T* kvbuf, const int64_t* __restrict__ base,
    const int32_t* __restrict__ cap, const int32_t* __restrict__ len, const int32_t* __restrict__ qpos_arr,
    const int32_t* __restrict__ tok_b, const int32_t* __restrict__ cu, int layer, int H, int causal, float scale,
    const float* __restrict__ bias_by_dist, int radius, T* __restrict__ out, int new_k_off, int new_v_off,
    const int32_t* __restrict__ block_table = nullptr, int max_blocks = 0, int block_shift = 0)
{
    static_assert(!(PAGED && PACKED), "paged mode is a cache mode");
    constexpr int EPL = 16 / sizeof(T);      // elements per 16-byte chunk
    constexpr int LPR = DH / EPL;            // lanes that share one key/value row
    constexpr int RPW = 64 / LPR;            // rows per wave per load
    constexpr int G = NWV * RPW;             // partial softmax states per workgroup (U row blocks in flight per wave)
    constexpr int NL = (PAGED && RPW * U > 8) ? U : 1;   // PAGED: table look-ups per step
    static_assert(RPW <= 8, "the rows of one load must fit the smallest block");
    __shared__ float s_m[G], s_l[G];
    __shared__ float s_acc[G][DH];

    int h = blockIdx.x, r = blockIdx.y;
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int rg = lane / LPR, cl = lane % LPR;
    int inner = H * DH;

    const T *kp, *vp, *qp;
    int64_t row_stride;
    int nk, qpos;
    if (PACKED) {
        int sb = tok_b[r];
        int t0 = cu[sb];
        qpos = qpos_arr[r];
        nk = causal ? qpos + 1 : cu[sb + 1] - t0;
        row_stride = 3 * (int64_t)inner;
        kp = kvbuf + (int64_t)t0 * row_stride + inner + h * DH;
        vp = kp + inner;
        qp = kvbuf + (int64_t)r * row_stride + h * DH;
    } else if (PAGED) {
        nk = len[r];
        qpos = qpos_arr[r];
        row_stride = DH;
        kp = vp = kvbuf;                    // set per block below
        qp = q + (int64_t)r * q_stride + h * DH;
    } else {
        int64_t c = cap[r];
        nk = len[r];
        qpos = qpos_arr[r];
        row_stride = DH;
        kp = kvbuf + base[r] + ((int64_t)(layer * 2) * H + h) * c * DH;
        vp = kp + (int64_t)H * c * DH;
        qp = q + (int64_t)r * q_stride + h * DH;
    }
    // PAGED: keys of block b for this head start at block_k(b), its values H * block_rows * DH elements further on
    const int block_rows = 1 << block_shift;
    const int32_t* tbl = PAGED ? block_table + (int64_t)r * max_blocks : nullptr;
    auto block_k = [&](int b) { return kvbuf + ((int64_t)b * 2 * H + h) * block_rows * DH; };
    // Fused append: the newest position's key/value rows come from the projection output; one 16-lane group
    // stores them into the cache, and every lane that meets row nk-1 reads it from the source instead of the
    // cache, so no ordering between that store and the loads is needed.
    const T *knew = nullptr, *vnew = nullptr;
    if (!PACKED && new_k_off) {
        knew = qp + new_k_off;
        vnew = qp + new_v_off;
        if (wave == 0 && rg == 0) {
            const T *kd = kp, *vd = vp;
            int row = nk - 1;
            if (PAGED) {
                kd = block_k(tbl[row >> block_shift]);
                vd = kd + (int64_t)H * block_rows * DH;
                row &= block_rows - 1;
            }
            *(uint4*)(const_cast<T*>(kd) + (int64_t)row * DH + cl * EPL) = *(const uint4*)(knew + cl * EPL);
            *(uint4*)(const_cast<T*>(vd) + (int64_t)row * DH + cl * EPL) = *(const uint4*)(vnew + cl * EPL);
        }
    }

    float qf[EPL];
    {
        float t[EPL];
        Chunk<T, EPL>::unpack(*(const uint4*)(qp + cl * EPL), t);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qf[e] = t[e] * scale * LOG2E;
    }
    const float* bias = bias_by_dist ? bias_by_dist + (int64_t)h * (2 * radius + 1) + radius : nullptr;
    // The head's bias table goes to LDS first (scaled for exp2): a look-up in global memory shares the wave's
    // in-order load counter with the K/V stream and cost 12 % of the kernel's bandwidth.
    __shared__ float s_bias[ATTN_BIAS_LDS];
    const bool bias_lds = bias && 2 * radius + 1 <= ATTN_BIAS_LDS;
    if (bias_lds) {
        for (int i = threadIdx.x; i < 2 * radius + 1; i += NWV * 64) s_bias[i] = bias[i - radius] * LOG2E;
        __syncthreads();
    }
    auto bias_at = [&](int rel) {
        rel = rel < -radius ? -radius : (rel > radius ? radius : rel);
        return bias_lds ? s_bias[rel + radius] : bias[rel] * LOG2E;
    };

    float m_run = -INFINITY, l_run = 0.f, acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

    // with a fused append the cached rows are 0 .. nk-2; the new row is folded in after the loop
    const int nc = (!PACKED && knew) ? nk - 1 : nk;
    // PAGED: the blocks of a step are looked up one step ahead, so that the step's loads do not wait for the table.
    // Look-up x of the step starting at row j serves the rows of loads x, x + NL, ...; it names the block of row
    // min(j + x * RPW, nc - 1), which is also the block of every row those loads touch: rows past the end are
    // clamped to row nc - 1.
    int blk[NL];
    auto lookup = [&](int j) {
#pragma unroll
        for (int x = 0; x < NL; ++x) blk[x] = tbl[paged_lookup_row(j, x, RPW, nc) >> block_shift];
    };
    if (PAGED && wave * RPW * U < nc) lookup(wave * RPW * U);
    const int64_t v_off = PAGED ? (int64_t)H * block_rows * DH : vp - kp;        // values behind the keys
    for (int j0 = wave * RPW * U; j0 < nc; j0 += NWV * RPW * U) {
        uint4 kc[U], vc[U];
        float s[U];
        const T* kpb[NL];                     // PAGED: keys of this head in the block of look-up x
        int jb[NL];                           // PAGED: first row of that block
        kpb[0] = kp;
        jb[0] = 0;
        if (PAGED) {
#pragma unroll
            for (int x = 0; x < NL; ++x) {
                kpb[x] = block_k(blk[x]);
                jb[x] = paged_lookup_row(j0, x, RPW, nc) & ~(block_rows - 1);
            }
            int jn = j0 + NWV * RPW * U;
            if (jn < nc) lookup(jn);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int x = NL == 1 ? 0 : u;
            int jj = paged_lane_row(j0, u, rg, RPW, nc) - jb[x];
            const T* kr = kpb[x] + (int64_t)jj * row_stride + cl * EPL;
            kc[u] = load_chunk<!PACKED>(kr);
            vc[u] = load_chunk<!PACKED>(kr + v_off);
        }
        float mx = m_run;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float kf[EPL];
            Chunk<T, EPL>::unpack(kc[u], kf);
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) d = fmaf(qf[e], kf[e], d);
#pragma unroll
            for (int o = LPR / 2; o > 0; o >>= 1) d += __shfl_xor(d, o, WAVE);
            int j = j0 + u * RPW + rg;
            if (bias) d += bias_at(j - qpos);
            s[u] = j < nc ? d : -INFINITY;
            mx = fmaxf(mx, s[u]);
        }
        float mref = mx == -INFINITY ? 0.f : mx;
        float alpha = fast_exp2(m_run - mref);
        l_run *= alpha;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float p = fast_exp2(s[u] - mref);
            l_run += p;
            float vf[EPL];
            Chunk<T, EPL>::unpack(vc[u], vf);
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
        }
        m_run = mx;
    }

    // the appended position (its key and value come from the projection output): folded into the state of the
    // first row group of wave 0
    if (!PACKED && knew && wave == 0 && rg == 0) {
        float kf[EPL], vf[EPL];
        Chunk<T, EPL>::unpack(*(const uint4*)(knew + cl * EPL), kf);
        Chunk<T, EPL>::unpack(*(const uint4*)(vnew + cl * EPL), vf);
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) d = fmaf(qf[e], kf[e], d);
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) d += __shfl_xor(d, o, WAVE);
        if (bias) d += bias_at(nk - 1 - qpos);
        float mx = fmaxf(m_run, d);
        float alpha = fast_exp2(m_run - mx), p = fast_exp2(d - mx);
        l_run = l_run * alpha + p;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e] * alpha);
        m_run = mx;
    }

    // merge the G partial states (wave, row group) of this workgroup
    int gi = wave * RPW + rg;
    if (cl == 0) { s_m[gi] = m_run; s_l[gi] = l_run; }
#pragma unroll
    for (int e = 0; e < EPL; ++e) s_acc[gi][cl * EPL + e] = acc[e];
    __syncthreads();
    for (int c = threadIdx.x; c < DH; c += NWV * 64) {
        float M = -INFINITY;
        for (int g = 0; g < G; ++g) M = fmaxf(M, s_m[g]);
        float L = 0.f, o = 0.f;
        for (int g = 0; g < G; ++g) {
            float w = fast_exp2(s_m[g] - M);      // 0 for groups that saw no key
            L += s_l[g] * w;
            o += s_acc[g][c] * w;
        }
        out[(int64_t)r * inner + h * DH + c] = from_f32<T>(o / L);
    }
}

hipError_t launch_attn_cache(const AttnCacheArgs& a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    dim3 grid(a.H, a.B);
    // 16 waves per (sequence, head), 2 row blocks in flight per wave: measured best of a sweep over
    // {1,2,4,8,16} waves x {1,2,3,4,8} blocks (6.4 TB/s at batch 256, 6.0 at batch 32; 4 waves x 4: 6.0 / 5.3).
    // Short sequences (mean_len rows on average, 0 = unknown) leave most of 16 waves without a row: 4 waves serve
    // them better (32 rows: 6.3 against 2.2 TB/s, cache-assisted; even at about 300 rows).
    int nwv = a.mean_len > 0 && a.mean_len <= ATTN_SHORT_LEN ? 4 : 16;
#define EXE_ROW_N(T, DH, NWV)                                                                                   \
    attn_row_kernel<T, DH, false, NWV, 2><<<grid, NWV * 64, 0, s>>>((const T*)a.q, a.q_stride, (const T*)a.pool, \
                                                               a.base, a.cap, a.len, a.qpos, nullptr, nullptr,  \
                                                               a.layer, a.H, 0, a.scale, a.bias_by_dist,        \
                                                               a.bias_radius, (T*)a.out, a.new_k_off, a.new_v_off)
#define EXE_ROW(T, DH)                                                                                          \
    do {                                                                                                        \
        if (nwv == 4) EXE_ROW_N(T, DH, 4);                                                                      \
        else EXE_ROW_N(T, DH, 16);                                                                              \
    } while (0)
    if (a.dtype == DT_F32 && a.dh == 64) EXE_ROW(float, 64);
    else if (a.dtype == DT_F32 && a.dh == 128) EXE_ROW(float, 128);
    else if (a.dtype == DT_BF16 && a.dh == 64) EXE_ROW(bf16_t, 64);
    else if (a.dtype == DT_BF16 && a.dh == 128) EXE_ROW(bf16_t, 128);
    else return hipErrorInvalidValue;
#undef EXE_ROW
#undef EXE_ROW_N
    return hipGetLastError();
}

// Host-side replay of the paged kernel's row indexing for one sequence of `len` cached rows (the rows a launch with
// these parameters reads, through the same index functions): every row read must be a cached row, lie inside the
// block its look-up names, and every cached row must be read exactly once by an unclamped lane.  Returns 0, or the
// number of violations.
int paged_index_check(int dtype, int dh, int block_shift, int nwv, int len)
{
    int epl = dtype == DT_F32 ? 4 : 8, lpr = dh / epl, rpw = 64 / lpr;
    constexpr int U = 2;                       // as launched below
    int nl = rpw * U > 8 ? U : 1, block_rows = 1 << block_shift, bad = 0;
    if (len < 1 || rpw > 8) return -1;
    int n_blocks = (len + block_rows - 1) >> block_shift;
    std::vector<int> seen(len, 0);
    for (int wave = 0; wave < nwv; ++wave)
        for (int j0 = wave * rpw * U; j0 < len; j0 += nwv * rpw * U)
            for (int u = 0; u < U; ++u) {
                int x = nl == 1 ? 0 : u;
                int lrow = paged_lookup_row(j0, x, rpw, len);
                int entry = lrow >> block_shift, first = lrow & ~(block_rows - 1);
                if (entry < 0 || entry >= n_blocks) ++bad;
                for (int rg = 0; rg < rpw; ++rg) {
                    int row = paged_lane_row(j0, u, rg, rpw, len), in_block = row - first;
                    if (row < 0 || row >= len || in_block < 0 || in_block >= block_rows) ++bad;
                    if (j0 + u * rpw + rg < len) seen[row] += 1;
                }
            }
    for (int r = 0; r < len; ++r)
        if (seen[r] != 1) ++bad;
    return bad;
}

hipError_t launch_attn_paged(const AttnPagedArgs& a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    if (a.block_shift < 3 || a.block_shift > 12 || a.max_blocks < 1) return hipErrorInvalidValue;
    dim3 grid(a.H, a.B);
    int nwv = a.mean_len > 0 && a.mean_len <= ATTN_SHORT_LEN ? 4 : 16;
#define EXE_ROW_N(T, DH, NWV)                                                                                       \
    attn_row_kernel<T, DH, false, NWV, 2, true><<<grid, NWV * 64, 0, s>>>(                                          \
        (const T*)a.q, a.q_stride, (const T*)a.pool, nullptr, nullptr, a.len, a.qpos, nullptr, nullptr, 0, a.H, 0,  \
        a.scale, a.bias_by_dist, a.bias_radius, (T*)a.out, a.new_k_off, a.new_v_off, a.block_table, a.max_blocks,   \
        a.block_shift)
#define EXE_ROW(T, DH)                                                                                              \
    do {                                                                                                            \
        if (nwv == 4) EXE_ROW_N(T, DH, 4);                                                                          \
        else EXE_ROW_N(T, DH, 16);                                                                                  \
    } while (0)
    if (a.dtype == DT_F32 && a.dh == 64) EXE_ROW(float, 64);
    else if (a.dtype == DT_F32 && a.dh == 128) EXE_ROW(float, 128);
    else if (a.dtype == DT_BF16 && a.dh == 64) EXE_ROW(bf16_t, 64);
    else if (a.dtype == DT_BF16 && a.dh == 128) EXE_ROW(bf16_t, 128);
    else return hipErrorInvalidValue;
#undef EXE_ROW
#undef EXE_ROW_N
    return hipGetLastError();
}

// ---------------------------------------------------------------- MFMA prefill (bf16, head size 128)
// A workgroup of 4 waves owns PREFILL_TILE_Q = 128 query rows of one (sequence, head), 32 per wave as two 16-row
// blocks; three workgroups fit a CU (48 KB of LDS each, at most 168 registers; the variants with a bias table need
// more registers than that without spilling, and a spill in the tile loop waits for the tile loads in flight, so
// they run two per CU).  Keys and values pass through LDS in tiles of 64 rows (two
// key tiles, double buffered, and one value tile), both by direct global->LDS loads in the same row-major swizzled
// layout.  Per tile a wave computes
//   S^T[key][query] = K . Q^T      (MFMA 16x16x32: A = key rows from LDS, B = the wave's query fragments)
//   O^T[d][query]  += V^T . P^T    (A = values through the transposing LDS read, B = P straight from the
//                                   accumulators of S^T)
// so a query's softmax statistics live in the four lanes that share its column, and the probabilities never leave
// registers.  Two barriers per tile (the value tile is loaded behind the scores).  The workgroups of a CU drift
// apart, so one wave's softmax (vector ALU) overlaps another's MFMAs on the same SIMD.
constexpr int PF_NW = 4, PF_DH = 128, PF_KT = 64, PF_THREADS = PF_NW * 64, PF_QT = PF_NW * 32;
constexpr int PF_LPT = 16 / PF_NW;                                // direct-to-LDS loads per wave and tile
constexpr int PF_TILE = 16384, PF_LDS = 3 * PF_TILE;              // key tiles 0 and 1, then the value tile
static_assert(PF_QT == PREFILL_TILE_Q, "the tile list is built for PREFILL_TILE_Q query rows per workgroup");

// A key or value tile [64 rows][128] in LDS: 256-byte rows of 16 chunks, chunk c of row r stored at slot c ^ (r & 15).
__device__ __forceinline__ int pf_off(int row, int chunk) { return row * 256 + ((chunk ^ (row & 15)) << 4); }

typedef __attribute__((ext_vector_type(4))) short pf_v4s;
// Transposing LDS read (ds_read_b64_tr_b16).  Within each block of 16 lanes, lane L points at 4 consecutive 16-bit
// elements M[L][0..3]; lane i receives M[4*j + i/4][i%4], j = 0..3.  With lane L = 4*j + q pointing at columns
// d0 + 4*q .. +3 of row j, lane i ends up with column d0 + i of rows 0..3: four values along the row index for one
// column, which is how an MFMA operand wants a row-major tile whose rows are the contraction index.
__device__ __forceinline__ uint2 pf_read_tr(const unsigned char* p)
{
    pf_v4s r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) pf_v4s*)p);
    return __builtin_bit_cast(uint2, r);
}

// Reductions over the four 16-lane rows of a wave (the lanes that share a column of a 16x16 accumulator tile),
// with the row-swap instructions of gfx950: v_permlane16_swap exchanges rows 1 and 3 of its first operand with
// rows 0 and 2 of its second, v_permlane32_swap the upper half of the first with the lower half of the second.
__device__ __forceinline__ float rows_max(float x)
{
    unsigned u = __float_as_uint(x);
    auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    u = __float_as_uint(fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1])));
    auto b = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_sum(float x)
{
    unsigned u = __float_as_uint(x);
    auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    u = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

template <bool CAUSAL, bool BIAS>
__global__ __launch_bounds__(PF_THREADS, BIAS ? 2 : 3) void prefill_mfma_kernel(const bf16_t* __restrict__ qkv,
                                                                  const int32_t* __restrict__ cu,
                                                                  const int32_t* __restrict__ tiles, int H,
                                                                  float scale, const float* __restrict__ bias_by_dist,
                                                                  int radius, bf16_t* __restrict__ out)
{
    extern __shared__ __align__(16) unsigned char pf_smem[];      // 2 key tiles, then 1 value tile
    __shared__ float sbias[BIAS ? 1024 : 1];

    // Workgroup -> (tile, head).  Workgroups go to the 8 XCDs round-robin in launch order.  With a multiple of 8 heads,
    // XCD x takes heads x, x + 8, ...: its j-th workgroup is tile j / (H/8) for its head number j % (H/8), so the
    // tiles of one sequence and head (neighbours in the list, readers of the same keys and values) share an L2 and
    // run side by side.  Otherwise heads vary fastest.
    int tile, h;
    if ((H & 7) == 0) {
        int hpx = H >> 3, j = blockIdx.x >> 3;
        tile = j / hpx;
        h = (blockIdx.x & 7) + 8 * (j - tile * hpx);
    } else {
        tile = blockIdx.x / H;
        h = blockIdx.x - tile * H;
    }
    int sb = tiles[tile * 2], q0 = tiles[tile * 2 + 1];
    int t0 = cu[sb], n = cu[sb + 1] - t0;
    int inner = H * PF_DH;
    int64_t ld = 3 * (int64_t)inner;
    int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int qi = lane & 15, g = lane >> 4;
    int wq0 = q0 + wave * 32;                                     // this wave's first query row
    const bf16_t* seq = qkv + (int64_t)t0 * ld + h * PF_DH;

    if (BIAS) {
        for (int i = tid; i < 2 * radius + 1; i += PF_THREADS)
            sbias[i] = bias_by_dist[(int64_t)h * (2 * radius + 1) + i] * LOG2E;
    }

    // query fragments (B operand): lane (query qi, lane group g) holds features 32*ds + 8*g .. +7
    bf16x8 qf[2][4];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        int qr = wq0 + qb * 16 + qi;
        qr = qr < n ? qr : n - 1;
        const bf16_t* qp = seq + (int64_t)qr * ld + g * 8;
#pragma unroll
        for (int ds = 0; ds < 4; ++ds) qf[qb][ds] = *(const bf16x8*)(qp + ds * 32);
    }
    int kend = n;
    if (CAUSAL) kend = q0 + PF_QT < n ? q0 + PF_QT : n;
    int n_tiles = (kend + PF_KT - 1) / PF_KT;

    // ---- loaders.  Per tile of keys and of values a wave issues two 1 KB direct-to-LDS loads of 4 rows each; a
    // lane fills slot lane%16 of its row with the chunk that the swizzle puts there.  Written as inline assembly
    // so that the compiler does not order every later LDS read behind them.
    unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)pf_smem;
    const char* kbase = (const char*)(seq + inner);
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
    auto load_to_lds = [&](const char* src, unsigned voff, unsigned dst) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff), "s"(src) : "memory", "m0");
    };
#pragma clang diagnostic pop
    const char* vbase = (const char*)(seq + 2 * inner);
    auto load_tile = [&](const char* base, int kt, unsigned dst) {
#pragma unroll
        for (int p = 0; p < 16 / PF_NW; ++p) {
            int row = (p * PF_NW + wave) * 4;                       // first of the 4 tile rows of this load
            int key = row + (lane >> 4);
            int kg = kt * PF_KT + key;
            kg = kg < n ? kg : n - 1;
            unsigned voff = (unsigned)kg * (unsigned)(ld * 2) + (((lane & 15) ^ (key & 15)) << 4);
            load_to_lds(base, voff, dst + row * 256);
        }
    };
    auto load_k = [&](int kt) { load_tile(kbase, kt, lds_base + (kt & 1) * PF_TILE); };
    auto load_v = [&](int kt) { load_tile(vbase, kt, lds_base + 2 * PF_TILE); };

    f32x4 o_acc[2][8];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o_acc[qb][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
    float sc = scale * LOG2E;
    f32x4 s_acc[2][4];

    // a wave whose queries all lie before a tile's first key (causal) or past the sequence end has nothing to
    // compute for that tile; it still moves its share of the tiles
    auto active = [&](int kt) { return wq0 < n && (!CAUSAL || kt * PF_KT <= wq0 + 31); };

    // ---- the three phases of a tile
    auto phase_s = [&](int kt) {
        const unsigned char* sK = pf_smem + (kt & 1) * PF_TILE;
        // The four swizzled chunk offsets of a lane ((4 ds + g) ^ qi for ds = 0..3) are recomputed per tile from one
        // register: held across the tile loop they cost four, and a register spilled in this loop puts a full wait
        // for the tile loads in flight in front of its reload (scratch reloads count with them).
        int qx = qi;
        asm volatile("" : "+v"(qx));
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            s_acc[0][kb] = f32x4{0.f, 0.f, 0.f, 0.f};
            s_acc[1][kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ds = 0; ds < 4; ++ds) {
                bf16x8 fk = *(const bf16x8*)(sK + (kb * 16 + qi) * 256 + (((ds * 4 + g) ^ qx) << 4));
                s_acc[0][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fk, qf[0][ds], s_acc[0][kb], 0, 0, 0);
                s_acc[1][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fk, qf[1][ds], s_acc[1][kb], 0, 0, 0);
            }
        }
    };
    // element r of lane (qi, g) in s_acc[qb][kb]: key = kt*64 + kb*16 + 4*g + r, query wq0 + qb*16 + qi.
    // Only tiles that straddle the sequence end or (causal) this wave's diagonal need the per-element mask.
    auto phase_softmax = [&](int kt) {
        // With a bias, a tile whose keys all lie at least `radius` before (or after) every query of this wave adds one
        // constant, the table's first (last) entry, to all of its scores: it takes the path without look-ups with that
        // constant folded into the exponent.  (The bias table is indexed by the clamped distance.)
        bool edge = kt * PF_KT + PF_KT > n || (CAUSAL && kt * PF_KT + PF_KT - 1 > wq0);
        bool masked = BIAS || edge;
        float cbias = 0.f;
        if (BIAS && !edge) {
            if (kt * PF_KT + PF_KT - 1 - wq0 <= -radius) {
                masked = false;
                cbias = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, sbias[0])));
            } else if (kt * PF_KT - (wq0 + 31) >= radius) {
                masked = false;
                cbias = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, sbias[2 * radius])));
            }
        }
        float alpha[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            int qpos = wq0 + qb * 16 + qi;
            float mx = -INFINITY;
            if (masked) {
                int key0 = kt * PF_KT + 4 * g;
                asm volatile("" : "+v"(key0));      // keeps the mask arithmetic inside this branch
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        int key = key0 + kb * 16 + r;
                        float v = s_acc[qb][kb][r] * sc;
                        if (BIAS) {
                            int rel = key - qpos;
                            rel = rel < -radius ? -radius : (rel > radius ? radius : rel);
                            v += sbias[rel + radius];
                        }
                        if (edge) {
                            bool ok = key < n && (!CAUSAL || key <= qpos);
                            v = ok ? v : -INFINITY;
                        }
                        s_acc[qb][kb][r] = v;
                        mx = fmaxf(mx, v);
                    }
            } else {
                // the scale is positive: take the maximum of the raw scores and fold the scale into the exponent
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int r = 0; r < 4; ++r) mx = fmaxf(mx, s_acc[qb][kb][r]);
                mx = fmaf(mx, sc, cbias);
            }
            mx = rows_max(mx);
            float m_new = fmaxf(m_run[qb], mx);
            float mref = m_new == -INFINITY ? 0.f : m_new;
            alpha[qb] = fast_exp2(m_run[qb] - mref);
            float mul = masked ? 1.f : sc;
            float shift = cbias - mref;             // cbias is 0 on the path with look-ups
            float rs = 0.f;
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float p = fast_exp2(fmaf(s_acc[qb][kb][r], mul, shift));
                    s_acc[qb][kb][r] = p;
                    rs += p;
                }
            rs = rows_sum(rs);
            l_run[qb] = l_run[qb] * alpha[qb] + rs;
            m_run[qb] = m_new;
        }
        // the running maximum of a query stops moving after the first tiles: rescale only when some lane needs it
        if (__builtin_amdgcn_ballot_w64(alpha[0] != 1.f || alpha[1] != 1.f) != 0) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int dt = 0; dt < 8; ++dt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) o_acc[qb][dt][r] *= alpha[qb];
        }
    };
    // O^T += V^T . P^T.  MFMA k-step ks covers keys 32*ks .. +31 of the tile; lane group g supplies keys
    // 4*g .. +3 of key blocks 2*ks and 2*ks+1.  The value tile lies row-major (one key per row); the transposing
    // read hands lane (qi, g) the column 16*dt + qi of those four keys: within the 16 lanes of a group, lane
    // L = 4*j + q points at columns 16*dt + 4*q .. +3 of key 4*g + j.
    int v_row = 4 * g + (qi >> 2), v_q = qi & 3;
    auto phase_pv = [&](int kt) {
        const unsigned char* sV = pf_smem + 2 * PF_TILE + v_row * 256 + (v_q & 1) * 8;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 pf[2];
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[qb][e] = (bf16_t)s_acc[qb][2 * ks + (e >> 2)][e & 3];
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                int slot = ((2 * dt + (v_q >> 1)) ^ v_row) << 4;     // rows v_row, +16, +32, +48 share their low 4 bits
                uint2 lo = pf_read_tr(sV + ks * 32 * 256 + slot);
                uint2 hi = pf_read_tr(sV + (ks * 32 + 16) * 256 + slot);
                uint4 both = {lo.x, lo.y, hi.x, hi.y};
                bf16x8 fv = __builtin_bit_cast(bf16x8, both);
                o_acc[0][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fv, pf[0], o_acc[0][dt], 0, 0, 0);
                o_acc[1][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fv, pf[1], o_acc[1][dt], 0, 0, 0);
            }
        }
    };

    // Key tiles are double buffered; the single value tile is loaded at the start of its own iteration, behind
    // the scores and the softmax, which costs a second barrier per tile but lets three workgroups share a CU.
    load_k(0);
    __builtin_amdgcn_s_waitcnt(0x0070 | (15 << 8));               // vmcnt(0)
    __syncthreads();

    for (int kt = 0; kt < n_tiles; ++kt) {
        load_v(kt);                                               // PF_LPT loads
        bool more = kt + 1 < n_tiles;
        if (more) load_k(kt + 1);                                 // PF_LPT loads, into the buffer tile kt-1 has left
        bool act = active(kt);
        if (act) {
            phase_s(kt);
            phase_softmax(kt);
        }
        if (more) __builtin_amdgcn_s_waitcnt(0x0070 | PF_LPT | (15 << 8));   // the value tile: all but the key loads
        else __builtin_amdgcn_s_waitcnt(0x0070 | (15 << 8));
        __syncthreads();
        if (act) phase_pv(kt);
        __builtin_amdgcn_s_waitcnt(0x0070 | (15 << 8));           // this wave's part of the next key tile has landed
        __syncthreads();
    }

    // lane (qi, g) holds features 16*dt + 4*g .. +3 of its query
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        int qpos = wq0 + qb * 16 + qi;
        if (qpos < n) {
            float inv = 1.f / l_run[qb];
            bf16_t* op = out + (int64_t)(t0 + qpos) * inner + h * PF_DH + 4 * g;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                bf16x4 w;
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = (bf16_t)(o_acc[qb][dt][j] * inv);
                *(bf16x4*)(op + dt * 16) = w;
            }
        }
    }
}

bool prefill_mfma_supported(int dtype, int dh) { return dtype == DT_BF16 && dh == PF_DH; }

void prefill_tile_order(const int32_t* lens, int n_seqs, std::vector<int32_t>& tiles)
{
    std::vector<int> order(n_seqs);
    for (int i = 0; i < n_seqs; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return lens[x] > lens[y]; });
    for (int i : order)
        for (int q0 = (lens[i] - 1) / PREFILL_TILE_Q * PREFILL_TILE_Q; q0 >= 0; q0 -= PREFILL_TILE_Q) {
            tiles.push_back(i);
            tiles.push_back(q0);
        }
}

hipError_t launch_attn_packed(const AttnPackedArgs& a, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    // The key loader addresses the rows of one sequence with 32-bit byte offsets, and a head's bias table must fit
    // the kernel's LDS copy; a batch outside these limits runs on the row kernel, which is correct but far slower,
    // so say so (once).
    const bool mfma_shape = !a.force_generic && prefill_mfma_supported(a.dtype, a.dh) && a.n_tiles > 0;
    const int64_t longest = a.max_len > 0 ? a.max_len : a.T;
    const bool mfma_fits = longest * 3 * a.H * a.dh * 2 < ((int64_t)1 << 32) && (!a.bias_by_dist || 2 * a.bias_radius + 1 <= 1024);
    if (mfma_shape && !mfma_fits) {
        static std::once_flag warned;
        std::call_once(warned, [&]() {
            fprintf(stderr, "exe: prefill attention falls back to the row kernel (longest sequence %lld rows of %d bytes, bias "
                            "radius %d): expect it to be much slower\n", (long long)longest, 3 * a.H * a.dh * 2, a.bias_radius);
        });
    }
    if (mfma_shape && mfma_fits) {
        if ((int64_t)a.n_tiles * a.H > 0x7fffffff) return hipErrorInvalidValue;
        dim3 grid((unsigned)(a.n_tiles * a.H));
        const bf16_t* qkv = (const bf16_t*)a.qkv;
        bf16_t* out = (bf16_t*)a.out;
        constexpr int lds = PF_LDS;
        // the kernels' dynamic LDS limit is raised once per device
        static std::once_flag attr_once[64];
        static hipError_t attr_err[64];
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
        std::call_once(attr_once[dev], [&]() {
            const void* kerns[4] = {(const void*)prefill_mfma_kernel<true, true>, (const void*)prefill_mfma_kernel<true, false>,
                                    (const void*)prefill_mfma_kernel<false, true>, (const void*)prefill_mfma_kernel<false, false>};
            attr_err[dev] = hipSuccess;
            for (const void* k : kerns) {
                hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
                if (e != hipSuccess) attr_err[dev] = e;
            }
        });
        if (attr_err[dev] != hipSuccess) return attr_err[dev];
        auto launch = [&](auto kern, const float* bias, int radius) -> hipError_t {
            kern<<<grid, PF_THREADS, lds, s>>>(qkv, a.cu, a.tiles, a.H, a.scale, bias, radius, out);
            return hipGetLastError();
        };
        if (a.causal) {
            if (a.bias_by_dist) return launch(prefill_mfma_kernel<true, true>, a.bias_by_dist, a.bias_radius);
            return launch(prefill_mfma_kernel<true, false>, nullptr, 0);
        }
        if (a.bias_by_dist) return launch(prefill_mfma_kernel<false, true>, a.bias_by_dist, a.bias_radius);
        return launch(prefill_mfma_kernel<false, false>, nullptr, 0);
    }
    dim3 grid(a.H, a.T);
#define EXE_ROW(T, DH)                                                                                           \
    attn_row_kernel<T, DH, true><<<grid, 256, 0, s>>>(nullptr, 0, (const T*)a.qkv, nullptr, nullptr, nullptr,    \
                                                      a.tok_pos, a.tok_b, a.cu, 0, a.H, a.causal, a.scale,       \
                                                      a.bias_by_dist, a.bias_radius, (T*)a.out, 0, 0)
    if (a.dtype == DT_F32 && a.dh == 64) EXE_ROW(float, 64);
    else if (a.dtype == DT_F32 && a.dh == 128) EXE_ROW(float, 128);
    else if (a.dtype == DT_BF16 && a.dh == 64) EXE_ROW(bf16_t, 64);
    else if (a.dtype == DT_BF16 && a.dh == 128) EXE_ROW(bf16_t, 128);
    else return hipErrorInvalidValue;
#undef EXE_ROW
    return hipGetLastError();
}

}  // namespace exe
