// GEMM kernels for the projections of a Transformer layer: out = epilogue(alpha * A[M,K] . W[N,K]^T + bias).
//
//  * gemm_tile_kernel    bf16, MFMA 32x32x16.  Macro tiles (BM x 256 or BM x 128, 64 k per LDS stage) filled by
//                        direct global->LDS loads into a ring of stages; software-pipelined fragment fetch;
//                        optional split-K into float partials, finished by splitk_reduce_kernel.
//                        Large M (encode) is MFMA / LDS-fill bound; small M (decode) streams the weights.
//  * gemm_generic_kernel float or bf16 inputs, plain FMA in float, any shape (tiny fp32 config, odd shapes).
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
// LDS tile layout for a stage of 64 bf16 along K: row r is 128 bytes = 8 chunks of 16 bytes; chunk c is
// stored at slot c ^ ((r>>1)&7), so that 16 consecutive rows read at the same chunk index touch 16 distinct
// 16-byte bank groups (256 bytes of banks; measured: zero LDS bank conflicts).
constexpr int TBK = 64;
__device__ __forceinline__ int lds_swz(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * 128 + ((chunk ^ lds_swz(row)) << 4); }

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* gbl_ptr_t;

// s_waitcnt vmcnt(N) lgkmcnt(L) with expcnt at its maximum; vmcnt is split over bits [3:0] and [15:14],
// lgkmcnt is bits [11:8]
template <int N, int L> __device__ __forceinline__ void wait_cnt()
{
    __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14) | (L << 8));
}

// Tiles are filled with direct global->LDS loads (no staging registers): one wave-wide 16-byte load
// writes 1 KB of consecutive tile rows, lane l landing at byte 16*l.  The swizzle is therefore applied on
// the global side: lane l fetches chunk (l % 8) ^ swz(row) of row l / 8.
//
// ST LDS stages of 64 k form a ring: while tile kt is multiplied, tiles kt+1 .. kt+ST-1 are in flight.
// Inside a tile the loop is software-pipelined: the operand fragments of k-step ks+1 are fetched from LDS
// while the MFMAs of step ks run.  The one barrier per tile sits after the last fragment fetch of the tile
// (before its last MFMA group): behind it every wave has finished reading the current stage and tile kt+1
// has landed, so the loads of tile kt+ST are issued into the stage just vacated and the first fragments of
// tile kt+1 are fetched while the last MFMAs of tile kt execute.
//
// Split-K (gridDim.z > 1): every workgroup writes its float partial tile; splitk_reduce_kernel finishes.
//
// Measured limits on MI355X (256x256 tile, 16384x15360x5120): MFMA loop alone 1.84 PFLOP/s, the
// global->LDS path alone 2.2 PFLOP/s-equivalent (1.5 with a drain per tile); this kernel about 1.1-1.25.
template <int BM, int BN, int WM, int WN, int ST>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_tile_kernel(
    int M, int N, int K, const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const bf16_t* __restrict__ bias,
    int act, float alpha, int out_mode, void* __restrict__ out, float* __restrict__ partial, int tiles_m, int tiles_n,
    int k_per_split)
{
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_PASSES = BM / 8 / NW, B_PASSES = BN / 8 / NW;   // 1 KB wave-loads per wave per stage
    constexpr int LPT = A_PASSES + B_PASSES;
    static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "tile/waves mismatch");
    static_assert(LPT * (ST - 1) <= 63, "vmcnt range");
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
        src_a[p] = A + (int64_t)r * K + kbeg + (((lane & 7) ^ lds_swz(rl)) << 3);
    }
#pragma unroll
    for (int p = 0; p < B_PASSES; ++p) {
        int rl = (p * NW + wave) * 8 + (lane >> 3);
        int r = n0 + rl;
        r = r < N ? r : N - 1;
        src_w[p] = W + (int64_t)r * K + kbeg + (((lane & 7) ^ lds_swz(rl)) << 3);
    }
    // tile `kt` (clamped to the last one, which keeps the number of loads in flight uniform) -> stage
    auto issue_loads = [&](int kt, int stage) {
        kt = kt < nk ? kt : nk - 1;
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
        for (int j = 0; j < TM; ++j) fa[b][j] = *(const bf16x8*)(sa + lds_off(wm * WM + j * 32 + frow, ks * 2 + fk));
#pragma unroll
        for (int i = 0; i < TN; ++i) fw[b][i] = *(const bf16x8*)(sw + lds_off(wn * WN + i * 32 + frow, ks * 2 + fk));
    };
    // the MFMAs of one k-step in two halves, so that the next step's fragment fetch can be issued between them
    auto mma = [&](int b, int half) {
        constexpr int NM = TN * TM;
#pragma unroll
        for (int x = 0; x < NM; ++x) {
            if ((x < NM / 2) != (half == 0) && NM > 1) continue;
            if (NM == 1 && half == 1) continue;
            int i = x / TM, j = x % TM;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[b][i], fa[b][j], acc[i][j], 0, 0, 0);
        }
    };
    // one k-step: first half of the MFMAs, then the fetch of the following step, then the second half.  The
    // fragments a step needs were requested half a step earlier, so the wait in front of its MFMAs covers
    // only loads that have had time to return.
#define EXE_STEP(b, fetch_stmt)                  \
    __builtin_amdgcn_sched_barrier(0);           \
    mma(b, 0);                                   \
    __builtin_amdgcn_sched_barrier(0);           \
    fetch_stmt;                                  \
    __builtin_amdgcn_sched_barrier(0);           \
    mma(b, 1);                                   \
    __builtin_amdgcn_sched_barrier(0);

    // prologue: tiles 0 .. ST-1 go to stages 0 .. ST-1; wait for tile 0 only
#pragma unroll
    for (int t = 0; t < ST; ++t) issue_loads(t, t);
    wait_cnt<LPT*(ST - 1), 15>();
    __syncthreads();
    fetch(0, 0, 0);
    int st = 0;
    for (int kt = 0; kt < nk; ++kt) {
        int nst = st + 1 == ST ? 0 : st + 1;
        EXE_STEP(0, fetch(st, 1, 1))
        EXE_STEP(1, fetch(st, 2, 0))
        EXE_STEP(0, fetch(st, 3, 1))
        // last step of the tile.  After its first half every read of this stage has been issued and has
        // returned (lgkmcnt 0); wait for tile kt+1 as well (all but the ST-2 most recent tiles' loads),
        // synchronise, refill the stage just vacated and fetch the first fragments of tile kt+1.
        __builtin_amdgcn_sched_barrier(0);
        mma(1, 0);
        __builtin_amdgcn_sched_barrier(0);
        wait_cnt<LPT*(ST - 2), 0>();
        __syncthreads();
        issue_loads(kt + ST, st);
        if (kt + 1 < nk) fetch(nst, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        mma(1, 1);
        __builtin_amdgcn_sched_barrier(0);
        st = nst;
    }
#undef EXE_STEP
    wait_cnt<0, 15>();     // drain the tail loads before the workgroup's LDS is released

    // accumulator layout: element r of lane l is (n = 8*(r/4) + 4*(l/32) + r%4, m = l%32) of its 32x32 tile
    int S = gridDim.z;
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
                if (S > 1) *(f32x4*)(partial + ((int64_t)blockIdx.z * M + m) * N + n) = v;
                else epilogue_store4<bf16_t>(v, m, n, N, bias, act, alpha, out_mode, out);
            }
    }
}

// Sums the split-K partials in split order (deterministic) and applies the epilogue.  (A reduction fused
// into the GEMM through arrival counters was measured 3x slower: the device-scope fences it needs write
// back and invalidate the L2 for every workgroup.)
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
// Tile configurations.  The first three have BN = 256 (the weight share of the LDS fill traffic is
// BN / (BM + BN), which is what a weight-streaming decode GEMM wants large); the last three halve BN for
// matrices with few output features, where more tiles beat deeper split-K.
enum Cfg { C64x256 = 0, C128x256, C256x256, C64x128, C128x128, C256x128, N_CFG };
struct CfgInfo { int bm, bn; };
static const CfgInfo CFG[N_CFG] = {{64, 256}, {128, 256}, {256, 256}, {64, 128}, {128, 128}, {256, 128}};

struct Plan { int route; int cfg; int splits; int k_per_split; int tiles; };

static int env_int(const char* name, int dflt)
{
    const char* v = getenv(name);
    return v ? atoi(v) : dflt;
}

// Cost model behind the choice of tile shape and split count (fitted to a sweep of the six shapes x split
// counts on MI355X for 16 <= M <= 512): a workgroup's time is the larger of its LDS-fill traffic at the rate one
// CU sustains through its vector L1 (about 45 GB/s) and its MFMA work at the rate the tile loop reaches
// (about 4.5 TFLOP/s per CU); workgroups run in rounds of one per CU; the whole launch cannot beat
// streaming W once from HBM; split-K adds the float partials' round trip and a second launch.
static double plan_cost(int cfg, int splits, int M, int N, int K)
{
    int bm = CFG[cfg].bm, bn = CFG[cfg].bn;
    int64_t tiles = (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    int64_t wgs = tiles * splits;
    double rounds = (double)((wgs + 255) / 256);
    double ktiles = (double)(K / TBK) / splits;
    double fill = ktiles * (bm + bn) * TBK * 2 / 45e9;
    double mfma = ktiles * 2.0 * bm * bn * TBK / 4.5e12;
    double t = rounds * (fill > mfma ? fill : mfma);
    double hbm = (double)N * K * 2 / 6e12;
    if (t < hbm) t = hbm;
    t += 4e-6;
    if (splits > 1) t += 2.0 * splits * M * N * 4 / 5e12 + 4e-6;
    return t;
}

static Plan make_plan(int dtype, int M, int N, int K)
{
    Plan p{2, 0, 1, K, 0};
    if (dtype != DT_BF16 || N % 4 != 0 || K % TBK != 0 || M < 1) return p;
    p.route = 0;
    p.cfg = C256x256;
    if (M <= 1024) {
        static const int split_options[] = {1, 2, 4, 5, 8, 10, 16};
        double best = 1e30;
        for (int cfg = 0; cfg < N_CFG; ++cfg) {
            if (CFG[cfg].bm >= 2 * M && CFG[cfg].bm > 64) continue;     // more than half the rows would be padding
            for (int s : split_options) {
                if ((K / TBK) % s || K / TBK / s < 4) continue;
                double c = plan_cost(cfg, s, M, N, K);
                if (c < best) { best = c; p.cfg = cfg; p.splits = s; }
            }
        }
    }
    // tuning knobs (debugging / sweeps): EXE_GEMM_CFG forces a configuration, EXE_GEMM_SPLIT a split count
    int force_cfg = env_int("EXE_GEMM_CFG", -1), force_split = env_int("EXE_GEMM_SPLIT", 0);
    if (force_cfg >= 0 && force_cfg < N_CFG) p.cfg = force_cfg;
    if (force_split > 0 && (K / TBK) % force_split == 0) p.splits = force_split;
    p.tiles = ((M + CFG[p.cfg].bm - 1) / CFG[p.cfg].bm) * ((N + CFG[p.cfg].bn - 1) / CFG[p.cfg].bn);
    p.k_per_split = K / p.splits;
    return p;
}

int gemm_route(int dtype, int M, int N, int K) { return make_plan(dtype, M, N, K).route; }

size_t gemm_workspace_bytes(int dtype, int M, int N, int K)
{
    Plan p = make_plan(dtype, M, N, K);
    return p.splits > 1 ? (size_t)p.splits * M * N * sizeof(float) : 0;
}

template <int BM, int BN, int WM, int WN, int ST>
static hipError_t launch_tile(const GemmArgs& a, const Plan& p, hipStream_t s)
{
    auto kern = gemm_tile_kernel<BM, BN, WM, WN, ST>;
    constexpr int threads = (BM / WM) * (BN / WN) * 64;
    size_t lds = (size_t)ST * (BM + BN) * TBK * 2;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    int tm = (a.M + BM - 1) / BM, tn = (a.N + BN - 1) / BN;
    kern<<<dim3(tm * tn, 1, p.splits), threads, lds, s>>>(a.M, a.N, a.K, (const bf16_t*)a.A, (const bf16_t*)a.W,
                                                         (const bf16_t*)a.bias, a.act, a.alpha, a.out_mode, a.out,
                                                         a.workspace, tm, tn, p.k_per_split);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.splits == 1) return e;
    int64_t quads = ((int64_t)a.M * a.N) / 4;
    splitk_reduce_kernel<bf16_t><<<(unsigned)((quads + 255) / 256), 256, 0, s>>>(
        a.M, a.N, p.splits, a.workspace, (const bf16_t*)a.bias, a.act, a.alpha, a.out_mode, a.out);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    Plan p = make_plan(a.dtype, a.M, a.N, a.K);
    if (p.splits > 1 && (!a.workspace || a.workspace_bytes < gemm_workspace_bytes(a.dtype, a.M, a.N, a.K)))
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
    switch (p.cfg) {
        case C64x256: return launch_tile<64, 256, 32, 64, 3>(a, p, s);
        case C128x256: return launch_tile<128, 256, 64, 64, 3>(a, p, s);
        case C256x256: return launch_tile<256, 256, 128, 64, 2>(a, p, s);
        case C64x128: return launch_tile<64, 128, 32, 64, 4>(a, p, s);
        case C128x128: return launch_tile<128, 128, 64, 64, 3>(a, p, s);
        default: return launch_tile<256, 128, 64, 64, 3>(a, p, s);
    }
}

}  // namespace exe
