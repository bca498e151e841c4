// GEMM kernels for the projections of a Transformer layer: out = epilogue(alpha * A[M,K] . W[N,K]^T + bias).
//
//  * gemm_tile_kernel   bf16, MFMA 32x32x16, LDS double-buffered macro tiles (256x256 or 128x128, BK = 64),
//                       optional split-K into float partial sums.  The encode (prefill) workhorse.
//  * gemm_skinny_kernel bf16, MFMA 16x16x32, M <= 64: every wave streams its own 16 weight rows straight
//                       from HBM into MFMA operand registers; activations are staged through LDS; split-K
//                       over the grid.  The decode (weight-streaming) workhorse.
//  * gemm_generic_kernel float or bf16 inputs, plain FMA in float, any shape (tiny fp32 config, odd shapes).
//  * splitk_reduce_kernel sums the partials in a fixed order (deterministic) and applies the epilogue.
//
// Both A and W are K-contiguous, so both MFMA operands are 16-byte vectors along K.  The MFMA "A" operand
// is fed with weight rows and the "B" operand with activation rows: the accumulator then holds 4
// consecutive output features per lane, which makes the epilogue's loads and stores 8/16-byte vectors.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"

namespace exe {

// ---------------------------------------------------------------- shared epilogue
// Stores 4 consecutive output features n..n+3 of row m.  v = raw accumulators.
template <typename T>
__device__ __forceinline__ void epilogue_store4(f32x4 v, int m, int n, int N, const T* __restrict__ bias, int act,
                                                float alpha, int out_mode, void* __restrict__ out)
{
    f32x4 r;
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = v[j] * alpha + (bias ? to_f32(bias[n + j]) : 0.f);
    int64_t o = (int64_t)m * N + n;
    if (out_mode == OUT_T) {
        T* p = (T*)out + o;
        if constexpr (sizeof(T) == 2) {
            bf16x4 w;
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = (bf16_t)act_apply(r[j], act);
            *(bf16x4*)p = w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = act_apply(r[j], act);
            *(f32x4*)p = r;
        }
    } else if (out_mode == OUT_RESID) {
        f32x4* p = (f32x4*)((float*)out + o);
        f32x4 h = *p;
        *p = h + r;
    } else {
        *(f32x4*)((float*)out + o) = r;
    }
}

// ---------------------------------------------------------------- tile kernel (bf16, MFMA 32x32x16)
// LDS tile layout for a stage of TBK bf16 along K: row r is TBK*2 bytes = CPR chunks of 16 bytes; chunk c is
// stored at slot c ^ swz(r) with swz chosen so that 16 consecutive rows read at the same chunk index touch
// 16 distinct 16-byte bank groups (256 bytes of banks): TBK = 64 -> (r>>1)&7, TBK = 32 -> (r>>2)&3.
template <int TBK> __device__ __forceinline__ int lds_swz(int row)
{
    return TBK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}
template <int TBK> __device__ __forceinline__ int lds_off(int row, int chunk)
{
    return row * (TBK * 2) + ((chunk ^ lds_swz<TBK>(row)) << 4);
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* gbl_ptr_t;

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    // s_waitcnt with expcnt/lgkmcnt left at their maxima; vmcnt is split over bits [3:0] and [15:14]
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Tiles are filled with direct global->LDS loads (no staging registers): one wave-wide 16-byte load
// writes 1 KB of consecutive tile rows, lane l landing at byte 16*l.  The swizzle is therefore applied on
// the global side: lane l fetches chunk (l % 8) ^ swz(row) of row l / 8.
//
// Two LDS stages of 64 k.  Inside a tile the loop is software-pipelined: the operand fragments of k-step
// ks+1 are fetched from LDS while the MFMAs of step ks run.  The one barrier per tile sits after the last
// fragment fetch of the tile (before its last MFMA group): behind it every wave has finished reading the
// current stage and the next tile's data has landed, so the loads of tile kt+2 are issued into the stage
// just vacated and the first fragments of tile kt+1 are fetched while the last MFMAs of tile kt execute.
// Measured limits on MI355X (256x256 tile, 16384x15360x5120): MFMA loop alone 1.84 PFLOP/s, the
// global->LDS path alone 2.2 PFLOP/s-equivalent, both with a per-tile drain 1.5; this kernel 1.25.
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_tile_kernel(
    int M, int N, int K, const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const bf16_t* __restrict__ bias,
    int act, float alpha, int out_mode, void* __restrict__ out, float* __restrict__ partial, int tiles_m, int tiles_n,
    int k_per_split)
{
    constexpr int TBK = 64;
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_PASSES = BM / 8 / NW, B_PASSES = BN / 8 / NW;   // 1 KB wave-loads per wave per stage
    static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "tile/waves mismatch");
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int STAGE = (BM + BN) * TBK * 2;     // bytes per LDS stage: A tile then W tile

    // workgroup -> tile: consecutive ids on one XCD (dispatch is round-robin over 8 XCDs) get a
    // GM x (32/GM) patch of tiles so that the XCD's L2 sees each A and W tile a few times only.
    int total = tiles_m * tiles_n;
    int pid = blockIdx.x;
    int chunk = total / 8;
    if (pid < chunk * 8) pid = (pid % 8) * chunk + pid / 8;
    constexpr int GM = 8;
    int group = pid / (GM * tiles_n);
    int first_m = group * GM;
    int gsz = tiles_m - first_m < GM ? tiles_m - first_m : GM;
    int within = pid - group * GM * tiles_n;
    int tile_m = first_m + within % gsz;
    int tile_n = within / gsz;
    int m0 = tile_m * BM, n0 = tile_n * BN;
    int kbeg = blockIdx.z * k_per_split;
    int kend = kbeg + k_per_split < K ? kbeg + k_per_split : K;
    int nk = (kend - kbeg) / TBK;

    int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int wm = wave % (BM / WM), wn = wave / (BM / WM);

    // per-lane global source of each wave-load (row clamped into the matrix; rows past the edge are never stored)
    const bf16_t* src_a[A_PASSES];
    const bf16_t* src_w[B_PASSES];
#pragma unroll
    for (int p = 0; p < A_PASSES; ++p) {
        int rl = (p * NW + wave) * 8 + (lane >> 3);
        int r = m0 + rl;
        r = r < M ? r : M - 1;
        src_a[p] = A + (int64_t)r * K + kbeg + (((lane & 7) ^ lds_swz<TBK>(rl)) << 3);
    }
#pragma unroll
    for (int p = 0; p < B_PASSES; ++p) {
        int rl = (p * NW + wave) * 8 + (lane >> 3);
        int r = n0 + rl;
        r = r < N ? r : N - 1;
        src_w[p] = W + (int64_t)r * K + kbeg + (((lane & 7) ^ lds_swz<TBK>(rl)) << 3);
    }
    auto issue_loads = [&](int kt, int stage) {
        unsigned char* base = lds + stage * STAGE;
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(src_a[p] + kt * TBK), (lds_ptr_t)(base + (p * NW + wave) * 1024), 16, 0, 0);
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(src_w[p] + kt * TBK), (lds_ptr_t)(base + BM * TBK * 2 + (p * NW + wave) * 1024), 16, 0, 0);
    };

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    int frow = lane & 31, fk = lane >> 5;
    bf16x8 fa[2][TM], fw[2][TN];
    auto fetch = [&](int stage, int ks, int b) {
        const unsigned char* sa = lds + stage * STAGE;
        const unsigned char* sw = sa + BM * TBK * 2;
#pragma unroll
        for (int j = 0; j < TM; ++j) fa[b][j] = *(const bf16x8*)(sa + lds_off<TBK>(wm * WM + j * 32 + frow, ks * 2 + fk));
#pragma unroll
        for (int i = 0; i < TN; ++i) fw[b][i] = *(const bf16x8*)(sw + lds_off<TBK>(wn * WN + i * 32 + frow, ks * 2 + fk));
    };
    auto mma = [&](int b) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[b][i], fa[b][j], acc[i][j], 0, 0, 0);
    };

    issue_loads(0, 0);
    wait_vmcnt<0>();
    __syncthreads();
    if (nk > 1) issue_loads(1, 1);
    fetch(0, 0, 0);
    for (int kt = 0; kt < nk; ++kt) {
        int st = kt & 1;
        fetch(st, 1, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(0);
        __builtin_amdgcn_sched_barrier(0);
        fetch(st, 2, 0);
        __builtin_amdgcn_sched_barrier(0);
        mma(1);
        __builtin_amdgcn_sched_barrier(0);
        fetch(st, 3, 1);
        __builtin_amdgcn_sched_barrier(0);
        mma(0);
        __builtin_amdgcn_sched_barrier(0);
        // every read of this stage has been issued: wait for them (lgkmcnt) and for the next tile's data
        // (vmcnt), then synchronise
        __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        if (kt + 2 < nk) issue_loads(kt + 2, st);
        if (kt + 1 < nk) fetch(st ^ 1, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        mma(1);
        __builtin_amdgcn_sched_barrier(0);
    }

    // accumulator layout: element r of lane l is (n = 8*(r/4) + 4*(l/32) + r%4, m = l%32) of its 32x32 tile
    bool split = gridDim.z > 1;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        int m = m0 + wm * WM + j * 32 + (lane & 31);
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int n = n0 + wn * WN + i * 32 + q * 8 + (lane >> 5) * 4;
                if (n >= N) continue;
                f32x4 v = {acc[i][j][q * 4], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
                if (split) *(f32x4*)(partial + ((int64_t)blockIdx.z * M + m) * N + n) = v;
                else epilogue_store4<bf16_t>(v, m, n, N, bias, act, alpha, out_mode, out);
            }
    }
}

// ---------------------------------------------------------------- skinny kernel (bf16, M <= 64)
// Workgroup = 4 waves; wave w owns weight rows n0 + 16w .. +15 for the whole k-range of this split.
// Per 128-wide k block a lane loads 64 contiguous bytes of its weight row (lane group g = lane/16 takes
// bytes [64g, 64g+64) of the row's 256-byte block), so every weight cache line is consumed whole by four
// lanes.  MFMA step j of the block uses chunk j of every lane: k = kblock + 32g + 8j + e.  The activation
// operand is read from LDS with the same k mapping.
constexpr int SK_KC = 256;   // k elements per LDS stage
__device__ __forceinline__ int sk_lds_off(int row, int chunk)   // row = 512 bytes = 32 chunks of 16 bytes
{
    return row * 512 + ((chunk ^ (row & 15)) << 4);
}

template <int MT>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(int M, int N, int K, const bf16_t* __restrict__ A,
                                                          const bf16_t* __restrict__ W,
                                                          const bf16_t* __restrict__ bias, int act, float alpha,
                                                          int out_mode, void* __restrict__ out,
                                                          float* __restrict__ partial, int k_per_split)
{
    constexpr int ROWS = MT * 16;
    constexpr int A_PASSES = ROWS * 32 / 256;   // 16-byte chunks per thread per stage
    __shared__ __align__(16) unsigned char sA[2][ROWS * 512];
    int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int n_row = blockIdx.x * 64 + wave * 16 + (lane & 15);
    n_row = n_row < N ? n_row : N - 1;
    int g = lane >> 4;
    int kbeg = blockIdx.y * k_per_split;
    int nchunks = k_per_split / SK_KC;
    const bf16_t* wrow = W + (int64_t)n_row * K + kbeg + g * 32;

    uint4 rw[8], ra[A_PASSES];
    auto load_global = [&](int c) {
        const bf16_t* p = wrow + c * SK_KC;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j) rw[b * 4 + j] = *(const uint4*)(p + b * 128 + j * 8);
#pragma unroll
        for (int q = 0; q < A_PASSES; ++q) {
            int idx = tid + q * 256;
            int r = idx >> 5, ch = idx & 31;
            int rr = r < M ? r : M - 1;
            ra[q] = *(const uint4*)(A + (int64_t)rr * K + kbeg + c * SK_KC + ch * 8);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int q = 0; q < A_PASSES; ++q) {
            int idx = tid + q * 256;
            *(uint4*)(sA[buf] + sk_lds_off(idx >> 5, idx & 31)) = ra[q];
        }
    };

    f32x4 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        int buf = c & 1;
        uint4 cw[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) cw[i] = rw[i];
        if (c + 1 < nchunks) load_global(c + 1);
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bf16x8 fw = __builtin_bit_cast(bf16x8, cw[b * 4 + j]);
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    bf16x8 fa = *(const bf16x8*)(sA[buf] + sk_lds_off(t * 16 + (lane & 15), b * 16 + g * 4 + j));
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw, fa, acc[t], 0, 0, 0);
                }
            }
        if (c + 1 < nchunks) store_lds(buf ^ 1);
        __syncthreads();
    }
    // accumulator: element r of lane l is (n = 4*(l/16) + r, m = l%16) of the 16x16 tile
    int n = blockIdx.x * 64 + wave * 16 + g * 4;
    if (n >= N) return;
    bool split = gridDim.y > 1;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        int m = t * 16 + (lane & 15);
        if (m >= M) continue;
        if (split) *(f32x4*)(partial + ((int64_t)blockIdx.y * M + m) * N + n) = acc[t];
        else epilogue_store4<bf16_t>(acc[t], m, n, N, bias, act, alpha, out_mode, out);
    }
}

template <typename T>
__global__ void splitk_reduce_kernel(int M, int N, int S, const float* __restrict__ partial,
                                     const T* __restrict__ bias, int act, float alpha, int out_mode,
                                     void* __restrict__ out)
{
    int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= (int64_t)M * N) return;
    int m = (int)(i / N), n = (int)(i - (int64_t)m * N);
    f32x4 v = *(const f32x4*)(partial + i);
    for (int s = 1; s < S; ++s) v += *(const f32x4*)(partial + (int64_t)s * M * N + i);
    epilogue_store4<T>(v, m, n, N, bias, act, alpha, out_mode, out);
}

// ---------------------------------------------------------------- generic kernel (float math, any shape)
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(int M, int N, int K, const T* __restrict__ A,
                                                           const T* __restrict__ W, const T* __restrict__ bias,
                                                           int act, float alpha, int out_mode, void* __restrict__ out)
{
    constexpr int TS = 64, KS = 16;
    __shared__ float sa[KS][TS + 1], sw[KS][TS + 1];
    int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += KS) {
        for (int i = threadIdx.x; i < TS * KS; i += 256) {
            int r = i / KS, k = i % KS;
            sa[k][r] = (m0 + r < M && k0 + k < K) ? to_f32(A[(int64_t)(m0 + r) * K + k0 + k]) : 0.f;
            sw[k][r] = (n0 + r < N && k0 + k < K) ? to_f32(W[(int64_t)(n0 + r) * K + k0 + k]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < KS; ++k) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sa[k][ty * 4 + i]; w[i] = sw[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        int m = m0 + ty * 4 + i;
        if (m >= M) continue;
        for (int j = 0; j < 4; ++j) {
            int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float r = acc[i][j] * alpha + (bias ? to_f32(bias[n]) : 0.f);
            int64_t o = (int64_t)m * N + n;
            if (out_mode == OUT_T) ((T*)out)[o] = from_f32<T>(act_apply(r, act));
            else if (out_mode == OUT_RESID) ((float*)out)[o] += r;
            else ((float*)out)[o] = r;
        }
    }
}

// ---------------------------------------------------------------- host-side routing
constexpr int BK = 64;   // granularity of K the tile kernels accept
struct Plan { int route; int bm; int splits; int k_per_split; int mt; };

static int pick_split(int base_wgs, int k_units, int target, int max_split)
{
    int best = 1;
    for (int s = 1; s <= max_split && s <= k_units; ++s) {
        if (k_units % s) continue;
        best = s;
        if ((int64_t)base_wgs * s >= target) break;
    }
    return best;
}

static Plan make_plan(int dtype, int M, int N, int K)
{
    Plan p{2, 0, 1, K, 0};
    if (dtype != DT_BF16 || N % 4 != 0 || K % BK != 0 || M < 1) return p;
    if (M <= 64 && K % SK_KC == 0) {
        p.route = 1;
        p.mt = (M + 15) / 16;
        int wgs = (N + 63) / 64;
        p.splits = pick_split(wgs, K / SK_KC, 512, 16);
        p.k_per_split = K / p.splits;
        return p;
    }
    p.route = 0;
    int t256 = ((M + 255) / 256) * ((N + 255) / 256);
    if (t256 >= 192) {
        p.bm = 256;
    } else {
        p.bm = 128;
        int t128 = ((M + 127) / 128) * ((N + 127) / 128);
        if (t128 < 256) {
            p.splits = pick_split(t128, K / 256 > 0 ? K / 256 : 1, 512, 8);
            if (K % (p.splits * BK) != 0) p.splits = 1;
        }
    }
    p.k_per_split = K / p.splits;
    return p;
}

int gemm_route(int dtype, int M, int N, int K) { return make_plan(dtype, M, N, K).route; }

size_t gemm_workspace_bytes(int dtype, int M, int N, int K)
{
    Plan p = make_plan(dtype, M, N, K);
    return p.splits > 1 ? (size_t)p.splits * M * N * sizeof(float) : 0;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    Plan p = make_plan(a.dtype, a.M, a.N, a.K);
    if (p.splits > 1 && (!a.workspace || a.workspace_bytes < (size_t)p.splits * a.M * a.N * sizeof(float)))
        return hipErrorInvalidValue;
    if (p.route == 2) {
        dim3 grid((a.N + 63) / 64, (a.M + 63) / 64);
        if (a.dtype == DT_F32)
            gemm_generic_kernel<float><<<grid, 256, 0, s>>>(a.M, a.N, a.K, (const float*)a.A, (const float*)a.W,
                                                            (const float*)a.bias, a.act, a.alpha, a.out_mode, a.out);
        else
            gemm_generic_kernel<bf16_t><<<grid, 256, 0, s>>>(a.M, a.N, a.K, (const bf16_t*)a.A, (const bf16_t*)a.W,
                                                             (const bf16_t*)a.bias, a.act, a.alpha, a.out_mode, a.out);
        return hipGetLastError();
    }
    const bf16_t* A = (const bf16_t*)a.A;
    const bf16_t* W = (const bf16_t*)a.W;
    const bf16_t* bias = (const bf16_t*)a.bias;
    if (p.route == 1) {
        dim3 grid((a.N + 63) / 64, p.splits);
#define EXE_SK(MT)                                                                                               \
    gemm_skinny_kernel<MT><<<grid, 256, 0, s>>>(a.M, a.N, a.K, A, W, bias, a.act, a.alpha, a.out_mode, a.out,    \
                                                a.workspace, p.k_per_split)
        switch (p.mt) {
            case 1: EXE_SK(1); break;
            case 2: EXE_SK(2); break;
            case 3: EXE_SK(3); break;
            default: EXE_SK(4); break;
        }
#undef EXE_SK
    } else if (p.bm == 256) {
        int tm = (a.M + 255) / 256, tn = (a.N + 255) / 256;
        size_t lds = 2 * (256 + 256) * 128;
        auto kern = gemm_tile_kernel<256, 256, 128, 64>;
        static bool attr_set = false;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        kern<<<dim3(tm * tn, 1, p.splits), 512, lds, s>>>(a.M, a.N, a.K, A, W, bias, a.act, a.alpha, a.out_mode, a.out,
                                                         a.workspace, tm, tn, p.k_per_split);
    } else {
        int tm = (a.M + 127) / 128, tn = (a.N + 127) / 128;
        size_t lds = 2 * (128 + 128) * 128;
        gemm_tile_kernel<128, 128, 64, 64><<<dim3(tm * tn, 1, p.splits), 256, lds, s>>>(
            a.M, a.N, a.K, A, W, bias, a.act, a.alpha, a.out_mode, a.out, a.workspace, tm, tn, p.k_per_split);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.splits > 1) {
        int64_t quads = ((int64_t)a.M * a.N) / 4;
        splitk_reduce_kernel<bf16_t><<<(unsigned)((quads + 255) / 256), 256, 0, s>>>(
            a.M, a.N, p.splits, a.workspace, bias, a.act, a.alpha, a.out_mode, a.out);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace exe
