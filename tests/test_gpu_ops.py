"""Per-kernel parity: each HIP kernel, called through the C ABI's exe_op_* entry points, against the
oracle's primitive of the same operation on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_07947_amd as exe
import workload as wl
from gpu_util import DEV, relerr, row_relerr

pytestmark = pytest.mark.gpu
BF16, F32 = wl.DTYPE_BF16, wl.DTYPE_F32
P = None


def prim():
    global P
    if P is None:
        P = oracle.Primitives("double")
    return P


def rnd(shape, seed, scale=1.0, dtype=torch.bfloat16):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(dtype)


# ------------------------------------------------------------------ GEMM
# (M, N, K): the shapes cover every tile configuration (64/128/256 rows x 128/256 columns), with and without
# split-K, ragged M and N edges, a launch split into whole rounds and a remainder, and the generic kernel.
GEMM_CASES = [
    (1, 512, 512), (16, 5120, 5120), (17, 1024, 2560), (33, 2048, 512), (64, 15360, 5120), (50, 50272, 512),
    (65, 512, 1024), (200, 1024, 512), (300, 640, 2048), (1000, 2048, 512),
    (4099, 3072, 256), (2049, 6144, 128),
    (2100, 8192, 2048),      # 9 x 32 tiles of 256 x 256: one whole round plus a 52-row remainder launch
    (100, 15360, 1024), (200, 8192, 512), (256, 5120, 5120), (128, 5120, 2048), (64, 8192, 256),
    (16, 512, 64), (70, 768, 128), (250, 8448, 192), (130, 260, 64),
    (37, 100, 72), (5, 52, 8),
]
# Every output row is compared for these: one case per tile configuration with split-K (several k-tiles per part),
# the 256 x 256 configuration without split, the 64 x 128 one without, and a launch split into whole rounds of
# tiles plus a remainder launch.  The M index of an output element is spread over wave rows, 16-row MFMA blocks,
# lanes and the groups of the LDS-turned epilogue, so sampled rows would leave most of that mapping unchecked.
GEMM_EVERY_ROW = [
    (16, 12288, 2048), (65, 20480, 2048), (130, 12288, 5120), (16, 2048, 512), (65, 8192, 2048), (130, 5120, 5120),
    (1100, 1024, 512), (4099, 3072, 256), (300, 8192, 64), (16, 512, 128), (2070, 8192, 256),
]
# configs[3] (GPT-3-175B share: d 12288, FFN 49152, QKV 36864): its K and N
GEMM_GPT3 = [(20, 36864, 12288), (20, 12288, 12288), (20, 49152, 12288), (20, 12288, 49152), (300, 49152, 12288)]
_ref_cache = {}


def gemm_inputs(M, N, K):
    return rnd((M, K), 1, 1.0), rnd((N, K), 2, 0.05), rnd((N,), 3, 0.5)


def gemm_reference(M, N, K, rows):
    """A[rows] . W^T in double by the oracle's linear primitive, without bias (cached: the four epilogue modes share it)."""
    key = (M, N, K, tuple(rows))
    if key not in _ref_cache:
        _ref_cache.clear()                                # one shape at a time: the matrices are large
        A, W, _ = gemm_inputs(M, N, K)
        _ref_cache[key] = prim().linear(A.float().numpy()[rows], W.float().numpy(), None)
    return _ref_cache[key]


def check_gemm(M, N, K, mode, rows):
    A, W, b = gemm_inputs(M, N, K)
    Ad, Wd, bd = A.to(DEV), W.to(DEV), b.to(DEV)
    ws_bytes = exe.exe_op_gemm_workspace(BF16, M, N, K)
    ws = torch.zeros(max(ws_bytes // 4, 1), dtype=torch.float32, device=DEV)
    raw = gemm_reference(M, N, K, rows)
    bias = b.float().numpy().astype(np.float64)
    alpha = 1.0
    if mode == "act_relu" or mode == "act_gelu":
        act = 0 if mode == "act_relu" else 1
        out = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        exe.exe_op_gemm(BF16, M, N, K, Ad, Wd, bd, act, alpha, 0, out, ws)
        ref = prim().act(raw + bias, act)
        tol = 2.0 ** -8
    elif mode == "resid":
        h0 = rnd((M, N), 4, 1.0, torch.float32)
        out = h0.to(DEV).clone()
        exe.exe_op_gemm(BF16, M, N, K, Ad, Wd, bd, -1, alpha, 1, out, ws)
        ref = raw + bias + h0.numpy()[rows].astype(np.float64)
        tol = 1e-5
    else:
        alpha = 0.37
        ref = raw * np.float64(np.float32(alpha)) + bias
        out = torch.zeros((M, N), dtype=torch.float32, device=DEV)
        exe.exe_op_gemm(BF16, M, N, K, Ad, Wd, bd, -1, alpha, 2, out, ws)
        tol = 1e-5
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()[rows]
    # float accumulation of K products of magnitude <= ~|a||w|: error << tol * max|ref|; compared row by row so
    # that a wrong row cannot hide behind a larger one
    assert got.shape == ref.shape
    err = np.max(np.abs(got - ref), axis=1) / np.max(np.abs(ref))
    assert float(err.max()) < tol, (M, N, K, mode, int(err.argmax()), float(err.max()))


def sample_rows(M):
    return np.unique(np.concatenate([[0, M - 1, min(M - 1, 2047), min(M - 1, 2048)],
                                     np.random.default_rng(M).integers(0, M, 6)]))


@pytest.mark.parametrize("M,N,K", GEMM_CASES)
@pytest.mark.parametrize("mode", ["act_relu", "act_gelu", "resid", "f32"])
def test_gemm_bf16(M, N, K, mode):
    print(f"gemm bf16 M={M} N={N} K={K} mode={mode} plan={exe.exe_op_gemm_plan(BF16, M, N, K)}", flush=True)
    check_gemm(M, N, K, mode, sample_rows(M))


def test_gemm_every_row_cases_cover_every_instantiation():
    """The every-row cases below reach all six tile configurations, split-K on each of them, and a launch split into
    whole rounds plus a remainder (asked of the library's own planner, so a retuned planner cannot silently
    leave a kernel instantiation unchecked)."""
    plain, split, remainder = set(), set(), False
    for (M, N, K) in GEMM_EVERY_ROW:
        p = exe.exe_op_gemm_plan(BF16, M, N, K)
        assert p["route"] == 0
        (split if p["splits"] > 1 else plain).add(p["cfg"])
        if p["rows_first"] < M:
            remainder = True
            q = exe.exe_op_gemm_plan(BF16, M - p["rows_first"], N, K)
            (split if q["splits"] > 1 else plain).add(q["cfg"])
    assert split == set(range(6)), split
    assert {2, 3} <= plain and remainder


@pytest.mark.parametrize("M,N,K", GEMM_EVERY_ROW)
@pytest.mark.parametrize("mode", ["act_relu", "act_gelu", "resid", "f32"])
def test_gemm_bf16_every_row(M, N, K, mode):
    print(f"gemm bf16 every row M={M} N={N} K={K} mode={mode} plan={exe.exe_op_gemm_plan(BF16, M, N, K)}", flush=True)
    check_gemm(M, N, K, mode, np.arange(M))


def random_gemm_shapes():
    """Seeded random shapes around the planner's decision boundaries: row counts up to a few tiles, feature counts
    that leave ragged tile columns, depths from one k-tile to many."""
    rng = np.random.default_rng(77)
    shapes = []
    for _ in range(48):
        M = int(rng.choice([rng.integers(1, 70), rng.integers(60, 270), rng.integers(250, 1300)]))
        N = 4 * int(rng.choice([rng.integers(8, 200), rng.integers(200, 1400), rng.integers(1400, 5200)]))
        K = 64 * int(rng.choice([rng.integers(1, 9), rng.integers(8, 40), rng.integers(40, 90)]))
        if M * N > 3_000_000:
            N = max(64, (3_000_000 // M) // 4 * 4)
        if M * N * K > 6_000_000_000:                    # keeps the oracle's double-precision product to a second or two
            K = max(64, 6_000_000_000 // (M * N) // 64 * 64)
        shapes.append((M, N, K, ["act_relu", "act_gelu", "resid", "f32"][int(rng.integers(0, 4))]))
    return shapes


@pytest.mark.parametrize("M,N,K,mode", random_gemm_shapes())
def test_gemm_bf16_random_shapes_every_row(M, N, K, mode):
    print(f"gemm bf16 random M={M} N={N} K={K} mode={mode} plan={exe.exe_op_gemm_plan(BF16, M, N, K)}", flush=True)
    check_gemm(M, N, K, mode, np.arange(M))


@pytest.mark.parametrize("M,N,K", GEMM_GPT3)
@pytest.mark.parametrize("mode", ["act_gelu", "resid"])
def test_gemm_bf16_gpt3_share_shapes(M, N, K, mode):
    """The projections of configs[3] at their own K and N (paper Table 1: GPT-3 175B, hidden 12288)."""
    print(f"gemm bf16 gpt3 M={M} N={N} K={K} mode={mode} plan={exe.exe_op_gemm_plan(BF16, M, N, K)}", flush=True)
    check_gemm(M, N, K, mode, np.arange(M) if M <= 20 else sample_rows(M))


@pytest.mark.parametrize("M,N,K,lda,ldw", [(130, 5120, 5120, 5184, 5248), (1100, 1024, 512, 576, 520), (16, 2048, 512, 512, 640)])
def test_gemm_bf16_padded_rows(M, N, K, lda, ldw):
    """exe_op_gemm_ld: operands whose rows are lda / ldw elements apart (every row compared; the padding holds
    large values that must never be read)."""
    A = torch.full((M, lda), 1000.0, dtype=torch.bfloat16)
    W = torch.full((N, ldw), 1000.0, dtype=torch.bfloat16)
    A[:, :K] = rnd((M, K), 1, 1.0)
    W[:, :K] = rnd((N, K), 2, 0.05)
    b = rnd((N,), 3, 0.5)
    need = exe.exe_op_gemm_workspace(BF16, M, N, K)
    ws = torch.zeros(max(need // 4, 1), dtype=torch.float32, device=DEV)
    out = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    exe.exe_op_gemm_ld(BF16, M, N, K, A.to(DEV), lda, W.to(DEV), ldw, b.to(DEV), -1, 1.0, 2, out, ws)
    torch.cuda.synchronize()
    ref = prim().linear(A[:, :K].float().numpy(), W[:, :K].float().numpy(), b.float().numpy())
    assert relerr(out.cpu().numpy(), ref) < 1e-5
    with pytest.raises(exe.ExeError):
        exe.exe_op_gemm_ld(BF16, M, N, K, A.to(DEV), K - 8, W.to(DEV), ldw, None, -1, 1.0, 2, out, ws)    # stride below K


@pytest.mark.parametrize("M,N,K", [(4, 2048, 256), (37, 1024, 256), (100, 768, 1024), (3, 52, 24)])
def test_gemm_f32(M, N, K):
    A = rnd((M, K), 5, 1.0, torch.float32)
    W = rnd((N, K), 6, 0.05, torch.float32)
    b = rnd((N,), 7, 0.5, torch.float32)
    out = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    exe.exe_op_gemm(F32, M, N, K, A.to(DEV), W.to(DEV), b.to(DEV), 1, 1.0, 0, out, None)
    torch.cuda.synchronize()
    ref = prim().act(prim().linear(A.numpy(), W.numpy(), b.numpy()), 1)
    assert relerr(out.cpu().numpy(), ref) < 2e-6


def test_gemm_no_bias_and_determinism():
    M, N, K = 48, 5120, 20480            # 64x128 tiles with split-K
    A, W = rnd((M, K), 8), rnd((N, K), 9, 0.02)
    Ad, Wd = A.to(DEV), W.to(DEV)
    ws = torch.zeros(exe.exe_op_gemm_workspace(BF16, M, N, K) // 4 + 1, dtype=torch.float32, device=DEV)
    outs = []
    for _ in range(2):
        out = torch.zeros((M, N), dtype=torch.float32, device=DEV)
        exe.exe_op_gemm(BF16, M, N, K, Ad, Wd, None, -1, 1.0, 2, out, ws)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])       # fixed summation order: bitwise reproducible
    rows = [0, 15, 16, 47]
    ref = prim().linear(A.float().numpy()[rows], W.float().numpy(), None)
    assert relerr(outs[0][rows], ref) < 1e-5


# ------------------------------------------------------------------ norms
@pytest.mark.parametrize("dtype", [BF16, F32])
@pytest.mark.parametrize("rms", [0, 1])
@pytest.mark.parametrize("d", [256, 5120, 12288])
def test_norm(dtype, rms, d):
    td = torch.float32 if dtype == F32 else torch.bfloat16
    rows = 7
    x = rnd((11, d), 10, 3.0, torch.float32) + 0.7
    g = (1 + rnd((d,), 11, 0.1, torch.float32)).to(td)
    b = rnd((d,), 12, 0.1, torch.float32).to(td)
    idx = torch.tensor([10, 0, 3, 3, 7, 1, 9], dtype=torch.int32)
    out = torch.zeros((rows, d), dtype=td, device=DEV)
    eps = 1e-6 if rms else 1e-5
    exe.exe_op_norm(dtype, rms, x.to(DEV), idx.to(DEV), rows, d, g.to(DEV), b.to(DEV), eps, 0.5, out)
    torch.cuda.synchronize()
    xs = x.numpy()[idx.numpy()]
    e = float(np.float32(eps))
    ref = (prim().rmsnorm(xs, g.float().numpy(), e) if rms else
           prim().layernorm(xs, g.float().numpy(), b.float().numpy(), e)) * 0.5
    assert relerr(out.float().cpu().numpy(), ref) < (2e-6 if dtype == F32 else 2.0 ** -8)


# ------------------------------------------------------------------ argmax
def test_argmax_lowest_index_on_ties():
    n = 50272
    x = rnd((5, n), 13, 1.0, torch.float32)
    x[1, 40000] = 9.0; x[1, 123] = 9.0; x[1, 50271] = 9.0
    x[2, :] = 0.25
    x[3, n - 1] = 7.0
    x[4, 0] = 7.0
    out = torch.zeros(5, dtype=torch.int32, device=DEV)
    exe.exe_op_argmax(x.to(DEV), 5, n, out)
    torch.cuda.synchronize()
    want = [prim().argmax(x[i].numpy()) for i in range(5)]
    assert out.cpu().tolist() == want
    assert want[1:] == [123, 0, n - 1, 0]


def test_probe_peaks_are_plausible():
    pk = exe.exe_probe_peaks()
    assert 2e12 < pk["hbm_read_bytes_per_s"] < 8.5e12            # below the nominal 8 TB/s, well above a PCIe-class rate
    assert 0.5e15 < pk["mfma_bf16_flops_per_s"] < 2.6e15         # below the nominal 2.5 PFLOP/s


# ------------------------------------------------------------------ attention
def oracle_attention(q, K, V, scale, bias=None):
    return prim().attention_row(q, K, V, scale, bias)[0]


def bias_table(H, R, seed):
    """Arbitrary per-head table over clamped distances (the kernel only indexes it)."""
    return rnd((H, 2 * R + 1), seed, 0.5, torch.float32)


@pytest.mark.parametrize("dtype,dh,H", [(BF16, 128, 5), (BF16, 64, 3), (F32, 64, 4), (F32, 128, 2)])
@pytest.mark.parametrize("use_bias", [0, 1])
def test_decode_attention(dtype, dh, H, use_bias):
    td = torch.float32 if dtype == F32 else torch.bfloat16
    lens = [1, 2, 63, 64, 65, 300, 1023, 17, 2560, 1281]      # up to the longest K/V of configs[3] (2048 + 512)
    B = len(lens)
    caps = [((L + 9) // 8) * 8 for L in lens]
    offs, tot = [], 0
    for c in caps:
        offs.append(tot)
        tot += 2 * H * c * dh + 64        # gaps between extents
    pool = rnd((tot,), 14, 1.0, td)
    q = rnd((B, H * dh), 15, 1.0, td)
    R = 128
    tab = bias_table(H, R, 16) if use_bias else None
    qpos = [L - 1 for L in lens]
    qpos[5] = 40                            # cross-attention style: query position unrelated to the length
    out = torch.zeros((B, H * dh), dtype=td, device=DEV)
    i64 = lambda a: torch.tensor(a, dtype=torch.int64, device=DEV)
    i32 = lambda a: torch.tensor(a, dtype=torch.int32, device=DEV)
    scale = 1.0 / np.sqrt(dh)
    exe.exe_op_decode_attention(dtype, B, q.to(DEV), H * dh, pool.to(DEV), i64(offs), i32(caps), i32(lens), i32(qpos),
                                H, dh, scale, None if tab is None else tab.to(DEV), R, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    pf = pool.float().numpy()
    worst = 0.0
    for b in range(B):
        for h in range(H):
            kb = offs[b] + h * caps[b] * dh
            K = pf[kb: kb + lens[b] * dh].reshape(lens[b], dh)
            vb = offs[b] + H * caps[b] * dh + h * caps[b] * dh
            V = pf[vb: vb + lens[b] * dh].reshape(lens[b], dh)
            bias = None
            if use_bias:
                rel = np.clip(np.arange(lens[b]) - qpos[b], -R, R) + R
                bias = tab.numpy()[h][rel]
            ref = oracle_attention(q.float().numpy()[b, h * dh:(h + 1) * dh], K, V, float(np.float32(scale)), bias)
            worst = max(worst, relerr(got[b, h * dh:(h + 1) * dh], ref))
    assert worst < (1e-5 if dtype == F32 else 2.0 ** -7), worst


def test_paged_index_replay_on_the_host():
    """The paged kernel's row indexing, replayed on the host through the kernel's own index functions: for every
    instantiation (type, head size), block size and launch shape, every row read lies in the block its look-up names
    and every cached row is read exactly once.  (bf16 with head size 64 reads 16 rows per step, two blocks of 8.)"""
    for dtype, dh in ((BF16, 64), (BF16, 128), (F32, 64), (F32, 128)):
        for block in (8, 16, 32, 64, 256, 4096):
            for waves in (4, 16):
                for L in list(range(1, 300)) + [1023, 1024, 1025, 2560, 4097]:
                    assert exe.exe_op_paged_index_check(dtype, dh, block, waves, L) == 0, (dtype, dh, block, waves, L)


@pytest.mark.parametrize("dtype,dh,H", [(BF16, 128, 5), (F32, 64, 3), (BF16, 64, 3), (F32, 128, 2)])
@pytest.mark.parametrize("block_size", [8, 16, 64, 256])
@pytest.mark.parametrize("fused_append", [0, 1])
def test_decode_attention_paged(dtype, dh, H, block_size, fused_append):
    """Block-table variant: the same rows scattered over shuffled blocks give the extent kernel's result bit for
    bit (same arithmetic in the same order) and the oracle's within tolerance; with the fused append the newest row
    comes from the projection output and lands in the right block."""
    # (Section 2 of the paper mentions paging of the key/value cache; the oracle is the plain attention definition)
    td = torch.float32 if dtype == F32 else torch.bfloat16
    lens = [1, 8, 9, 15, 16, 17, 63, 64, 65, 300, 1023, 17, 24, 1300]
    B = len(lens)
    inner = H * dh
    nblk = [(L + block_size - 1) // block_size for L in lens]
    max_blocks = max(nblk) + 1
    total = sum(nblk) + 3                                   # a few blocks nobody owns
    perm = np.random.default_rng(41).permutation(total)
    table = np.full((B, max_blocks), -1, dtype=np.int32)    # unused entries must never be read
    nxt = 0
    for b in range(B):
        for i in range(nblk[b]):
            table[b, i] = perm[nxt]
            nxt += 1
    table[table < 0] = 0
    blk_elems = 2 * H * block_size * dh
    # per-sequence contiguous K/V [H][L][dh], the ground truth for both layouts
    Ks = [rnd((H, L, dh), 50 + b, 1.0, td) for b, L in enumerate(lens)]
    Vs = [rnd((H, L, dh), 70 + b, 1.0, td) for b, L in enumerate(lens)]
    qkv = rnd((B, 3 * inner), 15, 1.0, td)                  # q, then the newest key and value rows when fused
    pool = torch.zeros(total * blk_elems, dtype=td)
    pv = pool.view(total, 2, H, block_size, dh)
    for b, L in enumerate(lens):
        if fused_append:                                   # the newest row is what the projection produced
            Ks[b][:, L - 1, :] = qkv[b, inner:2 * inner].view(H, dh)
            Vs[b][:, L - 1, :] = qkv[b, 2 * inner:].view(H, dh)
        in_cache = L - 1 if fused_append else L
        for p in range(in_cache):
            blk = table[b, p // block_size]
            pv[blk, 0, :, p % block_size, :] = Ks[b][:, p, :]
            pv[blk, 1, :, p % block_size, :] = Vs[b][:, p, :]
    qpos = [L - 1 for L in lens]
    scale = 1.0 / np.sqrt(dh)
    i32 = lambda a: torch.tensor(np.asarray(a), dtype=torch.int32, device=DEV)
    pool_d = pool.to(DEV)
    out = torch.zeros((B, inner), dtype=td, device=DEV)
    exe.exe_op_decode_attention_paged(dtype, B, qkv.to(DEV), 3 * inner, pool_d, i32(table), max_blocks, block_size, i32(lens),
                                      i32(qpos), H, dh, scale, None, 0, inner if fused_append else 0, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    # the extent kernel on the same rows
    caps = [((L + 7) // 8) * 8 for L in lens]
    offs, tot = [], 0
    for c in caps:
        offs.append(tot)
        tot += 2 * H * c * dh
    ext = torch.zeros(tot, dtype=td)
    for b, L in enumerate(lens):
        e = ext[offs[b]: offs[b] + 2 * H * caps[b] * dh].view(2, H, caps[b], dh)
        e[0, :, :L, :] = Ks[b]
        e[1, :, :L, :] = Vs[b]
    out2 = torch.zeros((B, inner), dtype=td, device=DEV)
    i64 = lambda a: torch.tensor(a, dtype=torch.int64, device=DEV)
    exe.exe_op_decode_attention(dtype, B, qkv.to(DEV), 3 * inner, ext.to(DEV), i64(offs), i32(caps), i32(lens), i32(qpos), H, dh,
                                scale, None, 0, out2)
    torch.cuda.synchronize()
    if not fused_append:                                   # (the fused append folds the newest row in last: another order)
        assert torch.equal(out, out2)
    else:
        assert relerr(got, out2.float().cpu().numpy()) < (1e-5 if dtype == F32 else 2.0 ** -7)
    if fused_append:                                       # the newest rows were stored where the table says
        back = pool_d.cpu().view(total, 2, H, block_size, dh)
        for b, L in enumerate(lens):
            blk, row = table[b, (L - 1) // block_size], (L - 1) % block_size
            assert torch.equal(back[blk, 0, :, row, :], Ks[b][:, L - 1, :]) and torch.equal(back[blk, 1, :, row, :], Vs[b][:, L - 1, :])
    worst = 0.0
    qf = qkv.float().numpy()
    for b, L in enumerate(lens):
        for h in range(H):
            ref = oracle_attention(qf[b, h * dh:(h + 1) * dh], Ks[b][h].float().numpy(), Vs[b][h].float().numpy(),
                                   float(np.float32(scale)), None)
            worst = max(worst, relerr(got[b, h * dh:(h + 1) * dh], ref))
    assert worst < (1e-5 if dtype == F32 else 2.0 ** -7), worst


@pytest.mark.parametrize("dtype,dh,H,generic", [(BF16, 128, 3, 0), (BF16, 128, 3, 1), (BF16, 64, 2, 0), (F32, 64, 4, 0)])
@pytest.mark.parametrize("causal,use_bias", [(1, 0), (0, 1), (1, 1), (0, 0)])
def test_prefill_attention(dtype, dh, H, generic, causal, use_bias):
    td = torch.float32 if dtype == F32 else torch.bfloat16
    lens = [1, 127, 128, 129, 300, 64, 5]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    inner = H * dh
    qkv = rnd((T, 3 * inner), 17, 1.0, td)
    R = 128
    tab = bias_table(H, R, 18) if use_bias else None
    out = torch.zeros((T, inner), dtype=td, device=DEV)
    scale = 1.0 / np.sqrt(dh) if causal else 0.11
    exe.exe_op_prefill_attention(dtype, cu, qkv.to(DEV), H, dh, scale, causal, None if tab is None else tab.to(DEV), R,
                                 out, force_generic=generic)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    x = qkv.float().numpy()
    rng = np.random.default_rng(19)
    worst = 0.0
    for s, L in enumerate(lens):
        # the MFMA kernel spreads a tile's rows over waves, 16-row blocks and lane groups: every row is checked
        every_row = dtype == BF16 and dh == 128 and not generic
        for i in (range(L) if every_row else sorted(set([0, L - 1] + list(rng.integers(0, L, 4))))):
            for h in range(H):
                t = cu[s] + i
                nk = i + 1 if causal else L
                K = x[cu[s]: cu[s] + nk, inner + h * dh: inner + (h + 1) * dh]
                V = x[cu[s]: cu[s] + nk, 2 * inner + h * dh: 2 * inner + (h + 1) * dh]
                bias = None
                if use_bias:
                    bias = tab.numpy()[h][np.clip(np.arange(nk) - i, -R, R) + R]
                ref = oracle_attention(x[t, h * dh:(h + 1) * dh], K, V, float(np.float32(scale)), bias)
                worst = max(worst, relerr(got[t, h * dh:(h + 1) * dh], ref))
    # bf16: probabilities are rounded to bf16 before the second product in the MFMA kernel
    assert worst < (1e-5 if dtype == F32 else 2.0 ** -6), worst


@pytest.mark.parametrize("causal,use_bias", [(1, 0), (0, 1), (1, 1), (0, 0)])
def test_prefill_attention_long(causal, use_bias):
    """The MFMA kernel at the lengths the benchmarks run: 1024 (OPT-13B and T5-11B inputs, 16 key tiles) and 2048
    (configs[3], 32 key tiles), next to a ragged 700; every row of every sequence against the oracle."""
    H, dh = 2, 128
    lens = [1024, 2048, 700]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    inner = H * dh
    qkv = rnd((T, 3 * inner), 27, 1.0)
    R = 128
    tab = bias_table(H, R, 28) if use_bias else None
    out = torch.zeros((T, inner), dtype=torch.bfloat16, device=DEV)
    scale = 1.0 / np.sqrt(dh) if causal else 0.11
    exe.exe_op_prefill_attention(BF16, cu, qkv.to(DEV), H, dh, scale, causal, None if tab is None else tab.to(DEV), R, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    x = qkv.float().numpy()
    worst = 0.0
    for s, L in enumerate(lens):
        for h in range(H):
            Ks = x[cu[s]: cu[s] + L, inner + h * dh: inner + (h + 1) * dh]
            Vs = x[cu[s]: cu[s] + L, 2 * inner + h * dh: 2 * inner + (h + 1) * dh]
            for i in range(L):
                nk = i + 1 if causal else L
                bias = tab.numpy()[h][np.clip(np.arange(nk) - i, -R, R) + R] if use_bias else None
                ref = oracle_attention(x[cu[s] + i, h * dh:(h + 1) * dh], Ks[:nk], Vs[:nk], float(np.float32(scale)), bias)
                worst = max(worst, relerr(got[cu[s] + i, h * dh:(h + 1) * dh], ref))
    assert worst < 2.0 ** -6, worst


@pytest.mark.parametrize("H,causal,use_bias", [(40, 1, 0), (128, 0, 1)])
def test_prefill_attention_bench_batch_is_order_independent(H, causal, use_bias):
    """At the benchmarks' own sizes (OPT-13B: 32 sequences, 40 heads, causal; T5-11B: 16 sequences, 128 heads, bias) the
    oracle samples a few rows; what holds at any size is that a sequence's rows do not depend on where it stands in the
    batch: the launch order (sequences longest first, heads dealt to XCDs) changes with the permutation, the rows of
    every sequence must stay bit-identical."""
    dh, R = 128, 128
    job = wl.workload_opt13b(256) if causal else wl.workload_t5(64)
    lens = [int(x) for x in job.in_len[:32 if causal else 16]]
    inner = H * dh
    scale = 1.0 / np.sqrt(dh) if causal else 0.11
    tab = bias_table(H, R, 77).to(DEV) if use_bias else None
    g = torch.Generator(device=DEV).manual_seed(5)
    rows = {i: torch.randn((L, 3 * inner), device=DEV, generator=g).to(torch.bfloat16) for i, L in enumerate(lens)}

    def run(order):
        cu = np.concatenate([[0], np.cumsum([lens[i] for i in order])]).astype(np.int32)
        qkv = torch.cat([rows[i] for i in order])
        out = torch.zeros((int(cu[-1]), inner), dtype=torch.bfloat16, device=DEV)
        exe.exe_op_prefill_attention(BF16, cu, qkv, H, dh, scale, causal, tab, R, out)
        torch.cuda.synchronize()
        return {i: out[cu[k]:cu[k + 1]].clone() for k, i in enumerate(order)}, qkv, cu

    base, _, _ = run(list(range(len(lens))))
    perm = list(np.random.default_rng(9).permutation(len(lens)))
    other, _, _ = run([int(i) for i in perm])
    for i in range(len(lens)):
        assert torch.equal(base[i], other[i]), i
    # sampled rows against the oracle: first, last and a middle row of the longest and the shortest sequence, three heads
    worst = 0.0
    for s in (int(np.argmax(lens)), int(np.argmin(lens))):
        L = lens[s]
        x = rows[s].float().cpu().numpy()
        got = base[s].float().cpu().numpy()
        for h in (0, H // 2 + 1, H - 1):
            Ks = x[:, inner + h * dh: inner + (h + 1) * dh]
            Vs = x[:, 2 * inner + h * dh: 2 * inner + (h + 1) * dh]
            for i in (0, L // 2, L - 1):
                nk = i + 1 if causal else L
                bias = tab.cpu().numpy()[h][np.clip(np.arange(nk) - i, -R, R) + R] if use_bias else None
                ref = oracle_attention(x[i, h * dh:(h + 1) * dh], Ks[:nk], Vs[:nk], float(np.float32(scale)), bias)
                worst = max(worst, relerr(got[i, h * dh:(h + 1) * dh], ref))
    assert worst < 2.0 ** -6, worst


def random_prefill_batches():
    rng = np.random.default_rng(91)
    cases = []
    for _ in range(8):
        n = int(rng.integers(1, 9))
        lens = [int(rng.choice([rng.integers(1, 40), rng.integers(40, 300), 64 * rng.integers(1, 8), 64 * rng.integers(1, 8) + 1]))
                for _ in range(n)]
        while sum(lens) > 1500:
            lens.pop()
        cases.append((tuple(lens), int(rng.integers(1, 4)), int(rng.integers(0, 2)), int(rng.integers(0, 2)), int(rng.integers(0, 2**31))))
    # head counts that are multiples of 8 take the launch order that deals heads to XCDs (all three model shapes do)
    cases.append(((300, 129, 64, 5, 1, 200), 8, 1, 0, 4242))
    cases.append(((257, 128, 31, 130), 16, 0, 1, 4343))
    cases.append(((129, 385), 24, 1, 1, 4444))
    return cases


@pytest.mark.parametrize("lens,H,causal,use_bias,seed", random_prefill_batches())
def test_prefill_attention_random_batches(lens, H, causal, use_bias, seed):
    """Seeded random ragged batches (sequence counts, lengths on and off the tile edges, heads, mask and bias) through
    the MFMA kernel; every row of every sequence against the oracle."""
    dh, R = 128, 128
    lens = list(lens)
    print(f"prefill random lens={lens} H={H} causal={causal} bias={use_bias}", flush=True)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, inner = int(cu[-1]), H * dh
    qkv = rnd((T, 3 * inner), seed % 1000 + 100, 1.0)
    tab = bias_table(H, R, seed % 1000 + 101) if use_bias else None
    out = torch.zeros((T, inner), dtype=torch.bfloat16, device=DEV)
    scale = 1.0 / np.sqrt(dh)
    exe.exe_op_prefill_attention(BF16, cu, qkv.to(DEV), H, dh, scale, causal, None if tab is None else tab.to(DEV), R, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    x = qkv.float().numpy()
    worst = 0.0
    for s, L in enumerate(lens):
        for h in range(H):
            Ks = x[cu[s]: cu[s] + L, inner + h * dh: inner + (h + 1) * dh]
            Vs = x[cu[s]: cu[s] + L, 2 * inner + h * dh: 2 * inner + (h + 1) * dh]
            for i in range(L):
                nk = i + 1 if causal else L
                bias = tab.numpy()[h][np.clip(np.arange(nk) - i, -R, R) + R] if use_bias else None
                ref = oracle_attention(x[cu[s] + i, h * dh:(h + 1) * dh], Ks[:nk], Vs[:nk], float(np.float32(scale)), bias)
                worst = max(worst, relerr(got[cu[s] + i, h * dh:(h + 1) * dh], ref))
    assert worst < 2.0 ** -6, worst


def random_decode_batches():
    rng = np.random.default_rng(93)
    cases = []
    for _ in range(10):
        B = int(rng.integers(1, 40))
        top = int(rng.choice([40, 330, 1500]))           # short batches take the 4-wave launch, long ones 16 waves
        lens = tuple(int(x) for x in rng.integers(1, top + 1, size=B))
        dtype, dh = [(BF16, 128), (BF16, 64), (F32, 64), (F32, 128)][int(rng.integers(0, 4))]
        cases.append((lens, dtype, dh, int(rng.integers(1, 6)), int(rng.integers(0, 2)), int(rng.integers(0, 1000))))
    return cases


@pytest.mark.parametrize("lens,dtype,dh,H,use_bias,seed", random_decode_batches())
def test_decode_attention_random_batches(lens, dtype, dh, H, use_bias, seed):
    """Seeded random batches of cached lengths (both launch shapes), element types, head sizes and bias: one query row
    per sequence against the oracle."""
    td = torch.float32 if dtype == F32 else torch.bfloat16
    lens = list(lens)
    B = len(lens)
    print(f"decode random B={B} max len {max(lens)} dtype={dtype} dh={dh} H={H} bias={use_bias}", flush=True)
    caps = [((L + 8) // 8) * 8 for L in lens]
    offs, tot = [], 0
    for c in caps:
        offs.append(tot)
        tot += 2 * H * c * dh + 8 * int((seed + c) % 5)      # uneven gaps between extents
    pool = rnd((tot + 64,), seed + 1, 1.0, td)
    q = rnd((B, H * dh), seed + 2, 1.0, td)
    R = 128
    tab = bias_table(H, R, seed + 3) if use_bias else None
    qpos = [L - 1 for L in lens]
    out = torch.zeros((B, H * dh), dtype=td, device=DEV)
    i64 = lambda a: torch.tensor(a, dtype=torch.int64, device=DEV)
    i32 = lambda a: torch.tensor(a, dtype=torch.int32, device=DEV)
    scale = 1.0 / np.sqrt(dh)
    exe.exe_op_decode_attention(dtype, B, q.to(DEV), H * dh, pool.to(DEV), i64(offs), i32(caps), i32(lens), i32(qpos),
                                H, dh, scale, None if tab is None else tab.to(DEV), R, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    pf, qf = pool.float().numpy(), q.float().numpy()
    worst = 0.0
    for b in range(B):
        for h in range(H):
            kb = offs[b] + h * caps[b] * dh
            K = pf[kb: kb + lens[b] * dh].reshape(lens[b], dh)
            vb = offs[b] + H * caps[b] * dh + h * caps[b] * dh
            V = pf[vb: vb + lens[b] * dh].reshape(lens[b], dh)
            bias = tab.numpy()[h][np.clip(np.arange(lens[b]) - qpos[b], -R, R) + R] if use_bias else None
            ref = oracle_attention(qf[b, h * dh:(h + 1) * dh], K, V, float(np.float32(scale)), bias)
            worst = max(worst, relerr(got[b, h * dh:(h + 1) * dh], ref))
    assert worst < (1e-5 if dtype == F32 else 2.0 ** -7), worst
