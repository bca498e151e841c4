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
//    S^T = K.Q^T and O^T = V^T.P^T are both computed with MFMA 32x32x16 so that softmax statistics of a
//    query live in one lane and P feeds the second MFMA straight from the first one's accumulators.
#include "common.h"
#include "kernels.h"

namespace exe {

constexpr float LOG2E = 1.44269504088896340736f;

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

template <typename T, int DH, bool PACKED, int NWV = 4, int U = 4>
__global__ __launch_bounds__(NWV * 64) void attn_row_kernel(
    const T* __restrict__ q, int q_stride, const T* kvbuf, const int64_t* __restrict__ base,
    const int32_t* __restrict__ cap, const int32_t* __restrict__ len, const int32_t* __restrict__ qpos_arr,
    const int32_t* __restrict__ tok_b, const int32_t* __restrict__ cu, int layer, int H, int causal, float scale,
    const float* __restrict__ bias_by_dist, int radius, T* __restrict__ out, int new_k_off, int new_v_off)
{
    constexpr int EPL = 16 / sizeof(T);      // elements per 16-byte chunk
    constexpr int LPR = DH / EPL;            // lanes that share one key/value row
    constexpr int RPW = 64 / LPR;            // rows per wave per load
    constexpr int G = NWV * RPW;             // partial softmax states per workgroup (U row blocks in flight per wave)
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
    } else {
        int64_t c = cap[r];
        nk = len[r];
        qpos = qpos_arr[r];
        row_stride = DH;
        kp = kvbuf + base[r] + ((int64_t)(layer * 2) * H + h) * c * DH;
        vp = kp + (int64_t)H * c * DH;
        qp = q + (int64_t)r * q_stride + h * DH;
    }
    // Fused append: the newest position's key/value rows come from the projection output; one 16-lane group
    // stores them into the cache, and every lane that meets row nk-1 reads it from the source instead of the
    // cache, so no ordering between that store and the loads is needed.
    const T *knew = nullptr, *vnew = nullptr;
    if (!PACKED && new_k_off) {
        knew = qp + new_k_off;
        vnew = qp + new_v_off;
        if (wave == 0 && rg == 0) {
            *(uint4*)(const_cast<T*>(kp) + (int64_t)(nk - 1) * DH + cl * EPL) = *(const uint4*)(knew + cl * EPL);
            *(uint4*)(const_cast<T*>(vp) + (int64_t)(nk - 1) * DH + cl * EPL) = *(const uint4*)(vnew + cl * EPL);
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

    float m_run = -INFINITY, l_run = 0.f, acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

    // with a fused append the cached rows are 0 .. nk-2; the new row is folded in after the loop
    const int nc = (!PACKED && knew) ? nk - 1 : nk;
    for (int j0 = wave * RPW * U; j0 < nc; j0 += NWV * RPW * U) {
        uint4 kc[U], vc[U];
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int j = j0 + u * RPW + rg;
            int jj = j < nc ? j : nc - 1;
            kc[u] = *(const uint4*)(kp + (int64_t)jj * row_stride + cl * EPL);
            vc[u] = *(const uint4*)(vp + (int64_t)jj * row_stride + cl * EPL);
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
            if (bias) {
                int rel = j - qpos;
                rel = rel < -radius ? -radius : (rel > radius ? radius : rel);
                d += bias[rel] * LOG2E;
            }
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
        if (bias) {
            int rel = nk - 1 - qpos;
            rel = rel < -radius ? -radius : (rel > radius ? radius : rel);
            d += bias[rel] * LOG2E;
        }
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
    // {1,2,4,8,16} waves x {1,2,3,4,8} blocks (6.4 TB/s at batch 256, 6.0 at batch 32; 4 waves x 4: 6.0 / 5.3)
#define EXE_ROW(T, DH)                                                                                          \
    attn_row_kernel<T, DH, false, 16, 2><<<grid, 1024, 0, s>>>((const T*)a.q, a.q_stride, (const T*)a.pool,     \
                                                               a.base, a.cap, a.len, a.qpos, nullptr, nullptr,  \
                                                               a.layer, a.H, 0, a.scale, a.bias_by_dist,        \
                                                               a.bias_radius, (T*)a.out, a.new_k_off, a.new_v_off)
    if (a.dtype == DT_F32 && a.dh == 64) EXE_ROW(float, 64);
    else if (a.dtype == DT_F32 && a.dh == 128) EXE_ROW(float, 128);
    else if (a.dtype == DT_BF16 && a.dh == 64) EXE_ROW(bf16_t, 64);
    else if (a.dtype == DT_BF16 && a.dh == 128) EXE_ROW(bf16_t, 128);
    else return hipErrorInvalidValue;
#undef EXE_ROW
    return hipGetLastError();
}

// ---------------------------------------------------------------- MFMA prefill (bf16, head size 128)
constexpr int PF_DH = 128, PF_KT = 64;

// K tile [64 keys][128] in LDS: 256-byte rows of 16 chunks, chunk c of key r stored at slot c ^ (r & 15).
__device__ __forceinline__ int pf_k_off(int key, int chunk) { return key * 256 + ((chunk ^ (key & 15)) << 4); }
// V tile transposed [128 cols][64 keys]: 128-byte rows of 16 four-key groups (8 bytes each); group kq of
// column c is stored at slot kq ^ swz(c).  swz makes both the 2-byte transposing writes (16 columns 8 apart,
// one key) and the 8-byte operand reads (32 consecutive columns, one key group) spread over all banks.
__device__ __forceinline__ int pf_swz(int c) { return ((c >> 1) & 15) ^ ((c >> 5) & 3); }
__device__ __forceinline__ int pf_v_off(int c, int kq) { return c * 128 + ((kq ^ pf_swz(c)) << 3); }

template <bool CAUSAL, bool BIAS>
__global__ __launch_bounds__(256) void prefill_mfma_kernel(const bf16_t* __restrict__ qkv,
                                                           const int32_t* __restrict__ cu,
                                                           const int32_t* __restrict__ tiles, int H, float scale,
                                                           const float* __restrict__ bias_by_dist, int radius,
                                                           bf16_t* __restrict__ out)
{
    __shared__ __align__(16) unsigned char sK[PF_KT * 256];
    __shared__ __align__(16) unsigned char sV[PF_DH * 128];
    __shared__ float sbias[BIAS ? 1024 : 1];

    int sb = tiles[blockIdx.x * 2], q0 = tiles[blockIdx.x * 2 + 1];
    int h = blockIdx.y;
    int t0 = cu[sb], n = cu[sb + 1] - t0;
    int inner = H * PF_DH;
    int64_t ld = 3 * (int64_t)inner;
    int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int qi = lane & 31, g = lane >> 5;
    int qpos = q0 + wave * 32 + qi;
    const bf16_t* seq = qkv + (int64_t)t0 * ld + h * PF_DH;

    if (BIAS) {
        for (int i = tid; i < 2 * radius + 1; i += 256)
            sbias[i] = bias_by_dist[(int64_t)h * (2 * radius + 1) + i] * LOG2E;
    }

    bf16x8 qf[8];
    {
        int qr = qpos < n ? qpos : n - 1;
        const bf16_t* qp = seq + (int64_t)qr * ld + g * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = *(const bf16x8*)(qp + kk * 16);
    }
    int kend = n;
    if (CAUSAL) kend = q0 + PREFILL_TILE_Q < n ? q0 + PREFILL_TILE_Q : n;
    int n_tiles = (kend + PF_KT - 1) / PF_KT;

    int ld_key = tid >> 4, ld_ch = tid & 15;
    uint4 rk[4], rv[4];
    auto load_global = [&](int kt) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            int key = kt * PF_KT + p * 16 + ld_key;
            key = key < n ? key : n - 1;
            const bf16_t* kp = seq + (int64_t)key * ld + inner + ld_ch * 8;
            rk[p] = *(const uint4*)kp;
            rv[p] = *(const uint4*)(kp + inner);
        }
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            int key = p * 16 + ld_key;
            *(uint4*)(sK + pf_k_off(key, ld_ch)) = rk[p];
            uint32_t w[4] = {rv[p].x, rv[p].y, rv[p].z, rv[p].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                int c = ld_ch * 8 + e;
                uint16_t val = (uint16_t)(e & 1 ? w[e >> 1] >> 16 : w[e >> 1] & 0xffff);
                *(uint16_t*)(sV + pf_v_off(c, key >> 2) + (key & 3) * 2) = val;
            }
        }
    };

    f32x16 o_acc[4];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[ct][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    float sc = scale * LOG2E;

    load_global(0);
    for (int kt = 0; kt < n_tiles; ++kt) {
        __syncthreads();            // everyone is done reading the previous tile
        store_lds();
        __syncthreads();
        if (kt + 1 < n_tiles) load_global(kt + 1);

        f32x16 s_acc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s_acc[t][r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                bf16x8 fk = *(const bf16x8*)(sK + pf_k_off(t * 32 + qi, kk * 2 + g));
                s_acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk, qf[kk], s_acc[t], 0, 0, 0);
            }
        }
        // element r of lane (qi, g) in s_acc[t]: key = kt*64 + t*32 + 8*(r/4) + 4*g + r%4, query qpos.
        // Only tiles that straddle the sequence end or (causal) this wave's diagonal need the per-element mask.
        bool edge = kt * PF_KT + PF_KT > n || (CAUSAL && kt * PF_KT + PF_KT - 1 > q0 + wave * 32);
        float mx = -INFINITY;
        if (BIAS || edge) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int key = kt * PF_KT + t * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    float v = s_acc[t][r] * sc;
                    if (BIAS) {
                        int rel = key - qpos;
                        rel = rel < -radius ? -radius : (rel > radius ? radius : rel);
                        v += sbias[rel + radius];
                    }
                    bool ok = key < n && (!CAUSAL || key <= qpos);
                    v = ok ? v : -INFINITY;
                    s_acc[t][r] = v;
                    mx = fmaxf(mx, v);
                }
        } else {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = s_acc[t][r] * sc;
                    s_acc[t][r] = v;
                    mx = fmaxf(mx, v);
                }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
        float m_new = fmaxf(m_run, mx);
        float mref = m_new == -INFINITY ? 0.f : m_new;
        float alpha = fast_exp2(m_run - mref);
        float rs = 0.f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p = fast_exp2(s_acc[t][r] - mref);
                s_acc[t][r] = p;
                rs += p;
            }
        rs += __shfl_xor(rs, 32, WAVE);
        l_run = l_run * alpha + rs;
        m_run = m_new;
        // the running maximum of a query stops moving after the first tiles: rescale only when some lane needs it
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                for (int r = 0; r < 16; ++r) o_acc[ct][r] *= alpha;
        }

        // O^T += V^T . P^T.  MFMA k-step ks covers, in lane group g, the 8 keys held in accumulator
        // elements 8*(ks%2) .. +7 of s_acc[ks/2]: key groups kq = (ks/2)*8 + (ks%2)*4 + g and kq + 2.
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 pf;
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[e] = (bf16_t)s_acc[ks >> 1][(ks & 1) * 8 + e];
            int kq = (ks >> 1) * 8 + (ks & 1) * 4 + g;
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) {
                int c = ct * 32 + qi;
                uint2 lo = *(const uint2*)(sV + pf_v_off(c, kq));
                uint2 hi = *(const uint2*)(sV + pf_v_off(c, kq + 2));
                uint4 both = {lo.x, lo.y, hi.x, hi.y};
                o_acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf, o_acc[ct], 0, 0, 0);
            }
        }
    }

    if (qpos < n) {
        float inv = 1.f / l_run;
        bf16_t* op = out + (int64_t)(t0 + qpos) * inner + h * PF_DH;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                bf16x4 w;
#pragma unroll
                for (int j = 0; j < 4; ++j) w[j] = (bf16_t)(o_acc[ct][q4 * 4 + j] * inv);
                *(bf16x4*)(op + ct * 32 + q4 * 8 + g * 4) = w;
            }
    }
}

bool prefill_mfma_supported(int dtype, int dh) { return dtype == DT_BF16 && dh == PF_DH; }

hipError_t launch_attn_packed(const AttnPackedArgs& a, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    if (!a.force_generic && prefill_mfma_supported(a.dtype, a.dh) && a.n_tiles > 0 &&
        (!a.bias_by_dist || 2 * a.bias_radius + 1 <= 1024)) {
        dim3 grid(a.n_tiles, a.H);
        const bf16_t* qkv = (const bf16_t*)a.qkv;
        bf16_t* out = (bf16_t*)a.out;
        if (a.causal) {
            if (a.bias_by_dist) prefill_mfma_kernel<true, true><<<grid, 256, 0, s>>>(qkv, a.cu, a.tiles, a.H, a.scale, a.bias_by_dist, a.bias_radius, out);
            else prefill_mfma_kernel<true, false><<<grid, 256, 0, s>>>(qkv, a.cu, a.tiles, a.H, a.scale, nullptr, 0, out);
        } else {
            if (a.bias_by_dist) prefill_mfma_kernel<false, true><<<grid, 256, 0, s>>>(qkv, a.cu, a.tiles, a.H, a.scale, a.bias_by_dist, a.bias_radius, out);
            else prefill_mfma_kernel<false, false><<<grid, 256, 0, s>>>(qkv, a.cu, a.tiles, a.H, a.scale, nullptr, 0, out);
        }
        return hipGetLastError();
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
