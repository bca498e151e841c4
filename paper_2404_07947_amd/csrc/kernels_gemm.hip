// GEMM kernels for the projections of a Transformer layer: out = epilogue(alpha * A[M,K] . W[N,K]^T + bias).
//
//  * gemm_tile_kernel    bf16, MFMA 16x16x32.  Macro tiles (BM x 256 or BM x 128, 64 k per LDS stage) filled by
//                        direct global->LDS loads into a ring of stages; software-pipelined fragment fetch;
//                        optional split-K into float partials, finished by splitk_reduce_kernel.
//                        Large M (encode) is MFMA / LDS-fill bound; small M (decode) streams the weights.
//  * gemm_generic_kernel float or bf16 inputs, plain FMA in float, any shape (tiny fp32 config, odd shapes).
//
// Both A and W are K-contiguous, so both MFMA operands are 16-byte vectors along K.  The MFMA "A" operand
// is fed with weight rows and the "B" operand with activation rows: the accumulator then holds 4
// consecutive output features per lane, which makes the epilogue's loads and stores 8/16-byte vectors.
//
// EXE_GEMM_ABLATE (a compile-time bit mask, 0 in the library proper) builds measurement variants of the tile kernel
// whose results are meaningless and whose timing isolates a part: bit 0 drops the MFMAs (the fragment reads from
// LDS go with them), bit 1 drops the loads of the activation tiles, bit 2 the loads of the weight tiles, bit 5 the
// epilogue (no output is written; a split-K reduction still runs, on whatever the workspace holds).  What
// remains keeps its waits, barriers, epilogue and split-K reduction.  `python -m paper_2404_07947_amd.build
// --variant ablate1 -DEXE_GEMM_ABLATE=1` builds libexe_ablate1.so beside the library.
#include <stdlib.h>

#include <mutex>
#include <type_traits>
#include <unordered_map>

#include "common.h"
#include "kernels.h"

#ifndef EXE_GEMM_ABLATE
#define EXE_GEMM_ABLATE 0
#endif
// Sub-step of a k-tile (8 MFMAs each) at which the second of the four parts of the next stage's loads is issued;
// the third and fourth follow one sub-step apart.  0 in the library; other values build measurement variants
// (-1 issues the second part with the first, behind the barrier).
#ifndef EXE_GEMM_ISSUE_AT
#define EXE_GEMM_ISSUE_AT 0
#endif

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

// ---------------------------------------------------------------- tile kernel (bf16, MFMA 16x16x32): LDS layout
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

// ---------------------------------------------------------------- tile epilogue
// A lane of a 16x16 accumulator tile holds 4 consecutive output features n = 4*(l/16) .. +3 of one row m = l%16:
// stored as it lies, a wave-wide store would scatter 16-byte pieces over 16 output rows.  Each wave therefore
// turns its tiles through a private LDS buffer, a "group" of 32 rows x EN columns (2 x EN/16 tiles) at a time,
// with the 16-byte slots XOR-swizzled by row so that neither side has bank conflicts, and then stores whole
// row segments.
//
// The LDS accesses are written as inline assembly on purpose: the compiler assumes that a DS read may alias the
// destination of the direct global->LDS loads still in flight for the next item and would put a vmcnt(0) in
// front of every one of them, which also waits for the stores of the previous group.  The buffer is private to
// the wave and is never a destination of those loads; DS operations of one wave execute in order, and the
// lgkmcnt(0) after the reads completes them before the next group's writes.
enum EpiMode { EPI_PARTIAL = 0, EPI_F32, EPI_RESID, EPI_T, EPI_T_RELU, EPI_T_GELU };

template <int QW> struct LdsTurn;
template <> struct LdsTurn<4> {
    static __device__ __forceinline__ void read(f32x4 (&v)[4], const unsigned (&a)[4])
    {
        asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %5\n\tds_read_b128 %2, %6\n\tds_read_b128 %3, %7\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
                     : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3])
                     : "memory");
    }
};
template <> struct LdsTurn<2> {
    static __device__ __forceinline__ void read(f32x4 (&v)[2], const unsigned (&a)[2])
    {
        asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %3\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(v[0]), "=&v"(v[1])
                     : "v"(a[0]), "v"(a[1])
                     : "memory");
    }
};

// acc[i][j]: the wave's accumulator tiles (i: 16 output features, j: 16 rows); stg: LDS byte address of the wave's
// buffer (EN * 128 bytes); (row0, col0): output coordinates of the wave's first element; fout: float destination
// of EPI_PARTIAL / EPI_F32 / EPI_RESID; tout: bf16 destination of EPI_T*.
template <int TM, int TN, int EN, int MODE>
__device__ __forceinline__ void epilogue_tiles(const f32x4 (&acc)[TN][TM], unsigned stg, int lane, int row0, int col0,
                                               int M, int N, const bf16_t* __restrict__ bias, float alpha,
                                               float* __restrict__ fout, bf16_t* __restrict__ tout)
{
    static_assert(TM % 2 == 0 && TN % 2 == 0, "groups are 2 tiles high");
    constexpr int QW = EN / 8;                  // 16-byte slots a lane writes, and reads, per group
    constexpr int IW = EN / 16;                 // tiles side by side in a group
    constexpr int NG = TN / IW;                 // groups per 32 rows
    constexpr int G = (TM / 2) * NG;
    constexpr int RPP = EN == 32 ? 8 : 16;      // output rows covered by one wave-wide read
    constexpr int D = G < 2 ? G : 2;            // residual prefetch depth in groups (registers: D * QW * 4)
    int lm = lane & 15, lq = lane >> 4;
    int rc = EN == 32 ? (lane & 7) : (lane & 3);
    int rr = EN == 32 ? (lane >> 3) : (lane >> 2);
    // slot of (row m, 16-byte column c) in the buffer
    auto slot = [](int m, int c) { return EN == 32 ? m * 8 + (c ^ ((m >> 1) & 7)) : m * 4 + (c ^ ((m >> 2) & 3)); };
    unsigned waddr[QW], raddr[QW];
#pragma unroll
    for (int x = 0; x < QW; ++x) {
        int jj = x / IW, ii = x % IW;           // tile (ii, jj) of the group
        waddr[x] = stg + slot(jj * 16 + lm, ii * 4 + lq) * 16;
        raddr[x] = stg + slot(x * RPP + rr, rc) * 16;
    }
    // group g = jp * NG + ig covers rows row0 + 32 jp .. +31 and columns col0 + EN ig .. + EN - 1
    auto g_row = [&](int g, int p) { return row0 + (g / NG) * 32 + p * RPP + rr; };
    auto g_col = [&](int g) { return col0 + (g % NG) * EN + rc * 4; };
    f32x4 bv[NG];
    if (MODE != EPI_PARTIAL) {
#pragma unroll
        for (int x = 0; x < NG; ++x) {
            int n = g_col(x);
            bv[x] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (bias && n < N) {
                bf16x4 b = *(const bf16x4*)(bias + n);
#pragma unroll
                for (int e = 0; e < 4; ++e) bv[x][e] = (float)b[e];
            }
        }
    }
    f32x4 res[D][QW];
    auto load_res = [&](int g) {
        int n = g_col(g);
#pragma unroll
        for (int p = 0; p < QW; ++p) {
            int m = g_row(g, p);
            res[g % D][p] = (m < M && n < N) ? *(const f32x4*)(fout + (int64_t)m * N + n) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };
    if (MODE == EPI_RESID) {
#pragma unroll
        for (int g = 0; g < D; ++g) load_res(g);
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        int jp = g / NG, ig = g % NG;
#pragma unroll
        for (int x = 0; x < QW; ++x) {
            f32x4 vv = acc[ig * IW + x % IW][jp * 2 + x / IW];
            asm volatile("ds_write_b128 %0, %1" ::"v"(waddr[x]), "v"(vv) : "memory");
        }
        f32x4 v[QW];
        LdsTurn<QW>::read(v, raddr);
        int n = g_col(g);
#pragma unroll
        for (int p = 0; p < QW; ++p) {
            int m = g_row(g, p);
            if (m >= M || n >= N) continue;
            int64_t o = (int64_t)m * N + n;
            if (MODE == EPI_PARTIAL) {
                *(f32x4*)(fout + o) = v[p];
            } else {
                f32x4 r = v[p] * alpha + bv[ig];
                if (MODE == EPI_F32) *(f32x4*)(fout + o) = r;
                else if (MODE == EPI_RESID) *(f32x4*)(fout + o) = res[g % D][p] + r;
                else {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        w[e] = (bf16_t)(MODE == EPI_T_RELU ? act_apply(r[e], 0) : MODE == EPI_T_GELU ? act_apply(r[e], 1) : r[e]);
                    *(bf16x4*)(tout + o) = w;
                }
            }
        }
        if (MODE == EPI_RESID && g + D < G) load_res(g + D);
        __builtin_amdgcn_sched_barrier(0);      // keeps the groups in order: hoisted loads would cost registers
    }
}

// Columns that a wave turns through LDS at a time in the epilogue: 32 (4 KB per wave) where the stages leave
// room within the 160 KB of a CU, else 16 (2 KB per wave).
constexpr int epilogue_cols(int BM, int BN, int WM, int WN, int ST)
{
    return ST * (BM + BN) * TBK * 2 + (BM / WM) * (BN / WN) * 4096 <= 160 * 1024 ? 32 : 16;
}

// ---------------------------------------------------------------- tile kernel
// Tiles are filled with direct global->LDS loads (no staging registers): one wave-wide 16-byte load
// writes 1 KB of consecutive tile rows, lane l landing at byte 16*l.  The swizzle is therefore applied on
// the global side: lane l fetches chunk (l % 8) ^ swz(row) of row l / 8.
//
// ST LDS stages of 64 k form a ring: while k-tile kt is multiplied, k-tiles kt+1 .. kt+ST-1 are in flight.
// Inside a k-tile the loop is software-pipelined over sub-steps (32 k x 32 rows of the wave's tile): the operand
// fragments of sub-step s+1 are fetched from LDS before the MFMAs of sub-step s are issued.  The one barrier per
// k-tile sits in front of the MFMAs of its last sub-step: behind it every wave has finished reading the current
// stage and k-tile kt+1 has landed, so the loads of k-tile kt+ST go into the stage just vacated and the first
// fragments of k-tile kt+1 are fetched while the last MFMAs of k-tile kt execute.
//
// The MFMA is the 16x16x32 one (4 passes).  Measured on MI355X: while a SIMD executes 32x32x16 MFMAs (8 passes)
// back to back, vector memory instructions of the waves on it are hardly issued at all (a loader wave beside an
// MFMA wave ran 20x slower), so the tile loads and the MFMAs of a k-tile ran one after the other; beside
// back-to-back 16x16x32 MFMAs the same loads run at 92 % of their stand-alone rate, at an equal MFMA rate.
//
// Workgroups are persistent (one per CU) and the loader runs ahead across items, so that a tile's epilogue and
// the first loads of the next tile overlap.  Split-K (n_split > 1): every item writes its float partial tile;
// splitk_reduce_kernel finishes.
template <int BM, int BN, int WM, int WN, int ST>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_tile_kernel(
    int M, int N, int K, const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const bf16_t* __restrict__ bias,
    int act, float alpha, int out_mode, void* __restrict__ out, float* __restrict__ partial, int tiles_m, int tiles_n,
    int k_per_split, int n_split, int flags, int lda, int ldw)
{
    // flags: bit 0 = spread the loads of a k-tile over the MFMAs (see below); bit 1 = the weights are read once
    // (a single row of output tiles): their loads are marked nontemporal so that they do not displace A in L2
    const int spread = flags & 1;
    const bool w_once = (flags & 2) != 0;
    constexpr int NW = (BM / WM) * (BN / WN);
    constexpr int TM = WM / 16, TN = WN / 16;       // 16x16 accumulator tiles of a wave: TM along rows, TN along features
    constexpr int MH = TM > 2 ? TM / 2 : 1;         // row parts of the wave's tile, one per sub-step
    constexpr int TMH = TM / MH;
    constexpr int NS = 2 * MH;                      // sub-steps per k-tile
    constexpr int A_PASSES = BM / 8 / NW, B_PASSES = BN / 8 / NW;   // 1 KB wave-loads per wave per stage
    // wave-loads a wave issues per k-tile (all of them, unless a measurement variant drops an operand's)
    constexpr int LPT = ((EXE_GEMM_ABLATE & 2) ? 0 : A_PASSES) + ((EXE_GEMM_ABLATE & 4) ? 0 : B_PASSES);
    constexpr int LPX = A_PASSES + B_PASSES;      // positions of the issue sequence: A passes, then W passes
    static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "tile/waves mismatch");
    static_assert(LPT * (ST - 1) <= 63, "vmcnt range");
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int STAGE = (BM + BN) * TBK * 2;     // bytes per LDS stage: A tile then W tile
    constexpr int EN = epilogue_cols(BM, BN, WM, WN, ST);

    // Work items are (split, output tile) pairs, numbered split-major.  The workgroups are persistent: workgroup b
    // takes items b, b + gridDim.x, ...  Item -> tile: consecutive item numbers on one XCD (workgroups are
    // dispatched round-robin over 8 XCDs and gridDim.x is a multiple of 8 whenever a workgroup takes more than
    // one item) get a GM x (32/GM) patch of tiles so that the XCD's L2 sees each A and W tile a few times only.
    int total = tiles_m * tiles_n;
    int items = total * n_split;
    auto locate = [&](int v, int& m0, int& n0, int& z) {
        z = v / total;
        int pid = v - z * total;
        int chunk = total / 8;
        if (pid < chunk * 8) pid = (pid % 8) * chunk + pid / 8;
        constexpr int GM = 8;
        int group = pid / (GM * tiles_n);
        int first_m = group * GM;
        int gsz = tiles_m - first_m < GM ? tiles_m - first_m : GM;
        int within = pid - group * GM * tiles_n;
        m0 = (first_m + within % gsz) * BM;
        n0 = (within / gsz) * BN;
    };
    auto k_tiles = [&](int z) {
        int kbeg = z * k_per_split;
        int kend = kbeg + k_per_split < K ? kbeg + k_per_split : K;
        return (kend - kbeg) / TBK;
    };

    int tid = threadIdx.x, lane = tid & 63;
    int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: keeps what derives from it in SGPRs
    int wm = wave % (BM / WM), wn = wave / (BM / WM);

    // ---- loader: runs ST k-tiles ahead of the MFMA loop, across item boundaries.  The source of a wave-load is a
    // uniform tile origin plus a per-lane byte offset (row clamped into the matrix; rows past the edge are never
    // stored), which keeps the addresses in 8 registers.
    unsigned off_a[A_PASSES], off_w[B_PASSES];
    const char *base_a, *base_w;
    int ld_v = blockIdx.x, ld_kt = 0, ld_nk = 1;
    auto set_src = [&](int v) {
        int m0, n0, z;
        locate(v, m0, n0, z);
        int kbeg = z * k_per_split;
        ld_nk = k_tiles(z);
        base_a = (const char*)(A + (int64_t)m0 * lda + kbeg);
        base_w = (const char*)(W + (int64_t)n0 * ldw + kbeg);
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            int rl = (p * NW + wave) * 8 + (lane >> 3);
            int r = m0 + rl < M ? rl : M - 1 - m0;
            off_a[p] = (unsigned)r * (unsigned)(lda * 2) + (((lane & 7) ^ lds_swz(rl)) << 4);
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            int rl = (p * NW + wave) * 8 + (lane >> 3);
            int r = n0 + rl < N ? rl : N - 1 - n0;
            off_w[p] = (unsigned)r * (unsigned)(ldw * 2) + (((lane & 7) ^ lds_swz(rl)) << 4);
        }
    };
    set_src(ld_v);
    // issues wave-loads X0 .. X1-1 (A passes first, then W passes) of the loader's current k-tile into `stage`.
    // The load is written as inline assembly on purpose: the compiler assumes that any later DS read may alias
    // the destination of a direct-to-LDS load it knows of, and puts a vmcnt(0) in front of the fragment reads,
    // which empties the ring of stages at every k-tile.  Completion is tracked by the explicit waits below.
    unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
    // (m0, the LDS destination, is a reserved register: naming it as clobbered draws a warning, but keeps the
    // compiler from merging its own m0 set-ups across the statement)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
    auto load_to_lds = [&](const char* src, unsigned voff, unsigned dst) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff), "s"(src) : "memory", "m0");
    };
    auto load_to_lds_nt = [&](const char* src, unsigned voff, unsigned dst) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(dst), "v"(voff), "s"(src) : "memory", "m0");
    };
#pragma clang diagnostic pop
    auto issue_range = [&](int stage, auto x0, auto x1) {
        unsigned base = lds_base + stage * STAGE + wave * 1024;
        const char* ka = base_a + ld_kt * (TBK * 2);
        const char* kw = base_w + ld_kt * (TBK * 2);
#pragma unroll
        for (int x = decltype(x0)::value; x < decltype(x1)::value; ++x) {
            if ((EXE_GEMM_ABLATE & 2) && x < A_PASSES) continue;
            if ((EXE_GEMM_ABLATE & 4) && x >= A_PASSES) continue;
            if (x < A_PASSES) load_to_lds(ka, off_a[x], base + x * NW * 1024);
            else if (w_once) load_to_lds_nt(kw, off_w[x - A_PASSES], base + BM * TBK * 2 + (x - A_PASSES) * NW * 1024);
            else load_to_lds(kw, off_w[x - A_PASSES], base + BM * TBK * 2 + (x - A_PASSES) * NW * 1024);
        }
    };
    // moves the loader to the next k-tile; past the last item the last k-tile is loaded again, which keeps the
    // number of loads in flight uniform
    auto advance = [&]() {
        if (ld_kt + 1 < ld_nk) ++ld_kt;
        else if (ld_v + (int)gridDim.x < items) {
            ld_v += gridDim.x;
            ld_kt = 0;
            set_src(ld_v);
        }
    };
    // A k-tile's loads are issued in four parts spread over 24 MFMAs: a burst of all of them fills the queue of
    // the CU's address unit, and a wave waiting to issue a load issues no MFMA either.
    // (`spread` = 0 issues them all at once behind the barrier.)
    constexpr int IA = EXE_GEMM_ISSUE_AT > NS - 4 ? NS - 4 : EXE_GEMM_ISSUE_AT;     // all four parts go out inside the k-tile
    constexpr int Q1 = LPX / 4, Q2 = LPX / 2, Q3 = LPX * 3 / 4;
    using X0 = std::integral_constant<int, 0>;
    using X1 = std::integral_constant<int, Q1>;
    using X2 = std::integral_constant<int, Q2>;
    using X3 = std::integral_constant<int, Q3>;
    using X4 = std::integral_constant<int, LPX>;

    // MFMA operands (16x16x32): lane l holds row l%16 and the 8 k-values 8*(l/16) .. +7 of a 32-k step, i.e.
    // 16-byte chunk 4*ks + l/16 of the stage row.  The W fragments of a 32-k step are kept for all its row parts.
    f32x4 acc[TN][TM];
    int frow = lane & 15, fk = lane >> 4;
    bf16x8 fa[2][TMH], fw[2][TN];
    // fragments of sub-step s of the k-tile in `stage`: activation rows of its row part, and (first row part of a
    // 32-k step only) the weight rows
    auto fetch = [&](int stage, int s) {
        const unsigned char* sa = lds + stage * STAGE;
        const unsigned char* sw = sa + BM * TBK * 2;
        int ks = s / MH, mh = s % MH;
#pragma unroll
        for (int j = 0; j < TMH; ++j)
            fa[s & 1][j] = *(const bf16x8*)(sa + lds_off(wm * WM + (mh * TMH + j) * 16 + frow, ks * 4 + fk));
        if (mh == 0) {
#pragma unroll
            for (int i = 0; i < TN; ++i) fw[ks & 1][i] = *(const bf16x8*)(sw + lds_off(wn * WN + i * 16 + frow, ks * 4 + fk));
        }
    };
    // the MFMAs of sub-step s in two halves, so that the next sub-step's fragment fetch can be issued between them
    auto mma = [&](int s, int half) {
        constexpr int NM = TN * TMH;
        int ks = s / MH, mh = s % MH;
        if (EXE_GEMM_ABLATE & 1) return;
#pragma unroll
        for (int x = 0; x < NM; ++x) {
            if ((x < NM / 2) != (half == 0)) continue;
            int i = x / TMH, j = x % TMH;
            acc[i][mh * TMH + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[ks & 1][i], fa[s & 1][j], acc[i][mh * TMH + j], 0, 0, 0);
        }
    };
#define EXE_SB __builtin_amdgcn_sched_barrier(0)

    // prologue: the first ST k-tiles go to stages 0 .. ST-1; wait for the first only
#pragma unroll
    for (int t = 0; t < ST; ++t) {
        issue_range(t, X0{}, X4{});
        advance();
    }
    wait_cnt<LPT*(ST - 1), 15>();
    __syncthreads();
    fetch(0, 0);
    int st = 0, fill_st = 0;
    bool pend = false;        // parts 2 .. 4 of the k-tile going into stage fill_st are still to be issued
    for (int v = blockIdx.x; v < items; v += gridDim.x) {
        int m0, n0, z;
        locate(v, m0, n0, z);
        int nk = k_tiles(z);
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int kt = 0; kt < nk; ++kt) {
            int nst = st + 1 == ST ? 0 : st + 1;
            // Every sub-step but the last: the fetch of the following sub-step's fragments, then the MFMAs (a full
            // sub-step of MFMAs between a fetch and its use).  The first three also issue the rest of the loads
            // whose first part went out behind the previous barrier.
            if constexpr (NS >= 4) {
#pragma unroll
                for (int s = 0; s < NS - 1; ++s) {
                    fetch(st, s + 1);
                    if (s == IA && pend) issue_range(fill_st, X1{}, X2{});
                    if (s == IA + 1 && pend) issue_range(fill_st, X2{}, X3{});
                    if (s == IA + 2 && pend) {
                        issue_range(fill_st, X3{}, X4{});
                        advance();
                    }
                    EXE_SB; mma(s, 0); mma(s, 1); EXE_SB;
                }
            } else {
                fetch(st, 1);
                if (pend) issue_range(fill_st, X1{}, X2{});
                EXE_SB; mma(0, 0); EXE_SB;
                if (pend) issue_range(fill_st, X2{}, X3{});
                EXE_SB; mma(0, 1); EXE_SB;
                if (pend) {
                    issue_range(fill_st, X3{}, X4{});
                    advance();
                }
            }
            // last sub-step of the k-tile.  Its fragments were the last reads of this stage: once they have
            // returned (lgkmcnt 0) and the following k-tile has landed (all but the ST-2 most recent k-tiles'
            // loads), synchronise, start refilling the stage just vacated and fetch the first fragments of the
            // following k-tile of this item behind the barrier, a full sub-step ahead of their use.
            wait_cnt<LPT*(ST - 2), 0>();
            __syncthreads();
            issue_range(st, X0{}, X1{});
            if (IA < 0 && NS >= 4 && spread) issue_range(st, X1{}, X2{});
            if (spread) {
                fill_st = st;
                pend = true;
            } else {
                issue_range(st, X1{}, X4{});
                advance();
            }
            if (kt + 1 < nk) fetch(nst, 0);
            EXE_SB; mma(NS - 1, 0); mma(NS - 1, 1); EXE_SB;
            st = nst;
        }
        // Epilogue; its stores drain while the next item's first k-tiles are multiplied.
        {
            unsigned stg = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)lds + ST * STAGE + wave * (EN * 128);
            int row0 = m0 + wm * WM, col0 = n0 + wn * WN;
            if (EXE_GEMM_ABLATE & 32) {            // measurement variant: no epilogue, the accumulators are only kept alive
#pragma unroll
                for (int i = 0; i < TN; ++i)
#pragma unroll
                    for (int j = 0; j < TM; ++j) asm volatile("" ::"v"(acc[i][j]));
            } else if (n_split > 1)
                epilogue_tiles<TM, TN, EN, EPI_PARTIAL>(acc, stg, lane, row0, col0, M, N, nullptr, 1.f, partial + (int64_t)z * M * N, nullptr);
            else if (out_mode == OUT_RESID)
                epilogue_tiles<TM, TN, EN, EPI_RESID>(acc, stg, lane, row0, col0, M, N, bias, alpha, (float*)out, nullptr);
            else if (out_mode == OUT_F32)
                epilogue_tiles<TM, TN, EN, EPI_F32>(acc, stg, lane, row0, col0, M, N, bias, alpha, (float*)out, nullptr);
            else if (act == 0)
                epilogue_tiles<TM, TN, EN, EPI_T_RELU>(acc, stg, lane, row0, col0, M, N, bias, alpha, nullptr, (bf16_t*)out);
            else if (act == 1)
                epilogue_tiles<TM, TN, EN, EPI_T_GELU>(acc, stg, lane, row0, col0, M, N, bias, alpha, nullptr, (bf16_t*)out);
            else
                epilogue_tiles<TM, TN, EN, EPI_T>(acc, stg, lane, row0, col0, M, N, bias, alpha, nullptr, (bf16_t*)out);
        }
        // first fragments of the next item (not held across the epilogue: it needs the registers)
        if (v + (int)gridDim.x < items) fetch(st, 0);
    }
#undef EXE_SB
    wait_cnt<0, 15>();     // drain the tail loads before the workgroup's LDS is released
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

struct Plan { int route; int cfg; int splits; int k_per_split; int tiles; int spread; double cost; };

static int env_int(const char* name, int dflt)
{
    const char* v = getenv(name);
    return v ? atoi(v) : dflt;
}

// Tuning knobs for sweeps and debugging, read from the environment once per process: EXE_GEMM_CFG forces a tile
// configuration, EXE_GEMM_SPLIT a split count, EXE_GEMM_SPREAD the load issue pattern, EXE_GEMM_NT the
// nontemporal weight loads, EXE_GEMM_GRID the number of persistent workgroups.
struct Knobs { int cfg, split, spread, nt, grid; };
static const Knobs& knobs()
{
    static const Knobs k{env_int("EXE_GEMM_CFG", -1), env_int("EXE_GEMM_SPLIT", 0), env_int("EXE_GEMM_SPREAD", -1),
                         env_int("EXE_GEMM_NT", -1), env_int("EXE_GEMM_GRID", 0)};
    return k;
}

// Cost model behind the choice of tile shape and split count, fitted to sweeps of the six shapes x 1..16 splits on
// MI355X with the weights coming from HBM (the GEMM shapes of three models, 16 <= M <= 1024; the time of its picks
// is within 1 % of the time of the best picks in total, 13 % at worst): a workgroup's time is the larger of its
// LDS-fill traffic at the rate one CU sustains through its vector L1 (about 35 GB/s) and its MFMA work at the rate
// the tile loop reaches on such short runs (about 3.5 TFLOP/s per CU; the 128 x 256 shape 0.8 of that); workgroups
// run in rounds of one per CU; the whole launch cannot beat streaming W once from HBM; split-K adds the float
// partials' round trip and a second launch.
static double plan_cost(int cfg, int splits, int M, int N, int K)
{
    int bm = CFG[cfg].bm, bn = CFG[cfg].bn;
    int64_t tiles = (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    int64_t wgs = tiles * splits;
    double rounds = (double)((wgs + 255) / 256);
    double ktiles = (double)((K / TBK + splits - 1) / splits);
    double fill = ktiles * (bm + bn) * TBK * 2 / 35e9;
    double mfma = ktiles * 2.0 * bm * bn * TBK / (cfg == C128x256 ? 2.8e12 : 3.5e12);
    double t = rounds * (fill > mfma ? fill : mfma);
    double hbm = (double)N * K * 2 / 5.5e12;
    if (t < hbm) t = hbm;
    t += 4e-6;
    if (splits > 1) t += 2.0 * splits * M * N * 4 / 3e12 + 1e-6;
    return t;
}

// Split-K over `s` parts: every part but the last takes ceil(k-tiles / s) k-tiles, the last one the rest, which must
// be at least 4 k-tiles.
static int split_k_tiles(int K, int s) { return (K / TBK + s - 1) / s; }
static bool split_ok(int K, int s)
{
    if (s == 1) return true;
    int per = split_k_tiles(K, s), last = K / TBK - per * (s - 1);
    return per >= 4 && last >= 4;
}

static Plan make_plan(int dtype, int M, int N, int K)
{
    Plan p{2, 0, 1, K, 0, 0, 0.0};
    if (dtype != DT_BF16 || N % 4 != 0 || K % TBK != 0 || M < 1) return p;
    p.route = 0;
    p.cfg = C256x256;
    // the model's choice per shape is remembered (a decode iteration asks for the same few shapes 4 times per layer)
    struct Choice { int cfg, splits; double cost; };
    thread_local std::unordered_map<uint64_t, Choice> memo;
    uint64_t key = ((uint64_t)M << 44) ^ ((uint64_t)N << 22) ^ (uint64_t)K;
    auto hit = memo.find(key);
    if (hit != memo.end()) {
        p.cfg = hit->second.cfg;
        p.splits = hit->second.splits;
        p.cost = hit->second.cost;
    } else if (M > 1024) {
        p.cost = plan_cost(C256x256, 1, M, N, K);
    } else {
        double best = 1e30;
        for (int cfg = 0; cfg < N_CFG; ++cfg) {
            if (CFG[cfg].bm >= 2 * M && CFG[cfg].bm > 64) continue;     // more than half the rows would be padding
            for (int s = 1; s <= 16; ++s) {
                if (!split_ok(K, s)) continue;
                double c = plan_cost(cfg, s, M, N, K);
                if (c < best) { best = c; p.cfg = cfg; p.splits = s; }
            }
        }
        p.cost = best;
        if (memo.size() > 4096) memo.clear();
        memo[key] = Choice{p.cfg, p.splits, p.cost};
    }
    const Knobs& kn = knobs();
    if (kn.cfg >= 0 && kn.cfg < N_CFG) p.cfg = kn.cfg;
    if (kn.split > 0 && split_ok(K, kn.split)) p.splits = kn.split;
    p.spread = 1;     // never slower than issuing a k-tile's loads at once in that sweep, up to 15 % faster from M = 128 on
    if (kn.spread >= 0) p.spread = kn.spread != 0;
    p.tiles = ((M + CFG[p.cfg].bm - 1) / CFG[p.cfg].bm) * ((N + CFG[p.cfg].bn - 1) / CFG[p.cfg].bn);
    p.k_per_split = split_k_tiles(K, p.splits) * TBK;
    return p;
}

int gemm_route(int dtype, int M, int N, int K) { return make_plan(dtype, M, N, K).route; }


// Per-device launch state: the number of persistent workgroups of a tile GEMM (one per compute unit: every
// configuration takes more than half of a CU's LDS, so one workgroup is resident per CU; rounded down to a
// multiple of 8 for the XCD mapping) and, per tile configuration, whether the kernel's dynamic LDS limit has been
// raised on that device.
constexpr int MAX_DEVICES = 64;
struct DeviceState { std::once_flag grid_once; int grid = 0; std::once_flag attr_once[8]; hipError_t attr_err[8]; };
static DeviceState& device_state()
{
    static DeviceState st[MAX_DEVICES];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) dev = 0;
    return st[dev];
}
static int persistent_grid()
{
    DeviceState& d = device_state();
    std::call_once(d.grid_once, [&]() {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
            cus = 256;
        d.grid = cus / 8 * 8;
        if (knobs().grid >= 8) d.grid = knobs().grid / 8 * 8;
    });
    return d.grid;
}

// A launch of many 256 x 256 tiles runs in rounds of one tile per CU, and a last round that fills few CUs costs as
// much as a full one.  split_rows returns the number of leading rows whose tiles fill whole rounds when handing the
// remaining rows (a few hundred) to a second, separately planned launch is cheaper by the cost model, else M.
static int split_rows(int dtype, int M, int N, int K)
{
    if (M <= 1024 || make_plan(dtype, M, N, K).route != 0) return M;
    int G = persistent_grid();
    int tn = (N + 255) / 256, tm = (M + 255) / 256, total = tm * tn;
    int rounds = total / G;
    if (rounds < 1 || total == rounds * G) return M;
    double whole = plan_cost(C256x256, 1, M, N, K);
    // Candidates for the first launch: the most row tiles that fill whole rounds, and the largest multiple of 64 row
    // tiles.  With a multiple of 64 every XCD keeps one group of 8 row tiles for the whole launch and all eight walk
    // the weight columns in step; measured, a round of such a launch takes 3-6 % less (16 384 rows against 17 120 -
    // 17 352 at the OPT-13B shape: 1826 us + 127 us for the rest against 2049 us in one launch of 16 rounds).
    int best = M;
    double best_cost = whole;
    int cand[2] = {rounds * G / tn, tm / 64 * 64};
    for (int tm1 : cand) {
        if (tm1 < 1 || tm1 >= tm) continue;
        int M1 = tm1 * 256;
        double first = plan_cost(C256x256, 1, M1, N, K);
        if (tm1 % 64 == 0) first *= 0.95;
        double parts = first + make_plan(dtype, M - M1, N, K).cost;
        if (parts < best_cost) { best_cost = parts; best = M1; }
    }
    return best;
}

void gemm_plan_info(int dtype, int M, int N, int K, int* route, int* cfg, int* splits, int* rows_first)
{
    int M1 = split_rows(dtype, M, N, K);
    Plan p = make_plan(dtype, M1, N, K);
    *route = p.route;
    *cfg = p.cfg;
    *splits = p.splits;
    *rows_first = M1;
}

size_t gemm_workspace_bytes(int dtype, int M, int N, int K)
{
    int M1 = split_rows(dtype, M, N, K);
    if (M1 < M) return gemm_workspace_bytes(dtype, M - M1, N, K);
    Plan p = make_plan(dtype, M, N, K);
    return p.splits > 1 ? (size_t)p.splits * M * N * sizeof(float) : 0;
}

template <int BM, int BN, int WM, int WN, int ST>
static hipError_t launch_tile(const GemmArgs& a, const Plan& p, int cfg_index, hipStream_t s)
{
    auto kern = gemm_tile_kernel<BM, BN, WM, WN, ST>;
    constexpr int threads = (BM / WM) * (BN / WN) * 64;
    size_t lds = (size_t)ST * (BM + BN) * TBK * 2 + (size_t)(threads / 64) * epilogue_cols(BM, BN, WM, WN, ST) * 128;
    static_assert(ST * (BM + BN) * TBK * 2 + (BM / WM) * (BN / WN) * epilogue_cols(BM, BN, WM, WN, ST) * 128 <= 160 * 1024, "LDS budget");
    DeviceState& d = device_state();
    std::call_once(d.attr_once[cfg_index], [&]() {
        d.attr_err[cfg_index] = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    if (d.attr_err[cfg_index] != hipSuccess) return d.attr_err[cfg_index];
    int tm = (a.M + BM - 1) / BM, tn = (a.N + BN - 1) / BN;
    int items = tm * tn * p.splits;
    int grid = items < persistent_grid() ? items : persistent_grid();
    int w_once = tm == 1 && a.M <= 64;      // measured: 7-10 % faster up to 32 rows, even from 96 rows on
    if (knobs().nt >= 0) w_once = knobs().nt != 0;
    kern<<<grid, threads, lds, s>>>(a.M, a.N, a.K, (const bf16_t*)a.A, (const bf16_t*)a.W, (const bf16_t*)a.bias, a.act,
                                    a.alpha, a.out_mode, a.out, a.workspace, tm, tn, p.k_per_split, p.splits,
                                    (p.spread ? 1 : 0) | (w_once ? 2 : 0), a.lda ? a.lda : a.K, a.ldw ? a.ldw : a.K);
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
    int M1 = split_rows(a.dtype, a.M, a.N, a.K);
    if (M1 < a.M) {
        GemmArgs head = a, tail = a;
        head.M = M1;
        tail.M = a.M - M1;
        size_t esz = a.dtype == DT_BF16 ? 2 : 4, osz = a.out_mode == OUT_T ? esz : 4;
        tail.A = (const char*)a.A + (size_t)M1 * (a.lda ? a.lda : a.K) * esz;
        tail.out = (char*)a.out + (size_t)M1 * a.N * osz;
        hipError_t e = launch_gemm(head, s);
        return e != hipSuccess ? e : launch_gemm(tail, s);
    }
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
        case C64x256: return launch_tile<64, 256, 32, 64, 3>(a, p, C64x256, s);
        case C128x256: return launch_tile<128, 256, 64, 64, 3>(a, p, C128x256, s);
        case C256x256: return launch_tile<256, 256, 128, 64, 2>(a, p, C256x256, s);
        case C64x128: return launch_tile<64, 128, 32, 64, 4>(a, p, C64x128, s);
        case C128x128: return launch_tile<128, 128, 64, 64, 3>(a, p, C128x128, s);
        default: return launch_tile<256, 128, 64, 64, 3>(a, p, C256x128, s);
    }
}

}  // namespace exe
