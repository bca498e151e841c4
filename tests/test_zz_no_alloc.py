"""exe_op_gemm_noalloc (the entry point for callers that cannot allocate: its split-K partial sums live in a static
device array inside the library) against exe_op_gemm with a caller workspace: the same kernels in the same launch
plan, so the outputs must be bit-identical, on two calls in a row, the second with a smaller input, and in every
epilogue mode; shapes whose partial sums exceed the static array are rejected."""
import numpy as np
import pytest
import torch

import paper_2404_07947_amd as exe
import workload as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF16 = wl.DTYPE_BF16


def rnd(shape, seed, scale=1.0, dtype=torch.bfloat16):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(dtype)


def both(M, N, K, mode, seed):
    A, W, b = rnd((M, K), seed).to(DEV), rnd((N, K), seed + 1, 0.05).to(DEV), rnd((N,), seed + 2, 0.5).to(DEV)
    need = exe.exe_op_gemm_workspace(BF16, M, N, K)
    ws = torch.zeros(max(need // 4, 1), dtype=torch.float32, device=DEV)
    if mode == "t":
        o1 = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        o2 = torch.zeros_like(o1)
        args = (1, 1.0, 0)
    elif mode == "resid":
        o1 = rnd((M, N), seed + 3, 1.0, torch.float32).to(DEV)
        o2 = o1.clone()
        args = (-1, 1.0, 1)
    else:
        o1 = torch.zeros((M, N), dtype=torch.float32, device=DEV)
        o2 = torch.zeros_like(o1)
        args = (-1, 0.37, 2)
    exe.exe_op_gemm(BF16, M, N, K, A, W, b, *args, o1, ws)
    exe.exe_op_gemm_noalloc(BF16, M, N, K, A, W, b, *args, o2)
    torch.cuda.synchronize()
    return o1, o2, need


@pytest.mark.parametrize("mode", ["t", "resid", "f32"])
def test_noalloc_gemm_matches_workspace_gemm_twice_in_a_row(mode):
    # split-K shapes (the only ones that touch the scratch): a larger call first, then a smaller one that finds the
    # first call's partial sums still in the array
    first, second = (130, 12288, 5120), (16, 2048, 512)
    for i, (M, N, K) in enumerate((first, second)):
        assert exe.exe_op_gemm_plan(BF16, M, N, K)["splits"] > 1
        o1, o2, need = both(M, N, K, mode, 100 + 10 * i)
        assert 0 < need <= exe.exe_op_gemm_noalloc_max_workspace()
        assert torch.equal(o1, o2), (mode, M, N, K)
        assert bool(torch.isfinite(o2.float()).all()) and float(o2.float().abs().max()) > 0


def test_noalloc_gemm_without_split_and_float_type():
    o1, o2, need = both(1100, 1024, 512, "t", 7)            # one tile per item, no partial sums
    assert need == 0 and torch.equal(o1, o2)
    M, N, K = 37, 1024, 256                                  # float operands: the plain-FMA kernel
    A, W = rnd((M, K), 1, 1.0, torch.float32).to(DEV), rnd((N, K), 2, 0.05, torch.float32).to(DEV)
    o1 = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    o2 = torch.zeros_like(o1)
    exe.exe_op_gemm(wl.DTYPE_F32, M, N, K, A, W, None, 1, 1.0, 0, o1, None)
    exe.exe_op_gemm_noalloc(wl.DTYPE_F32, M, N, K, A, W, None, 1, 1.0, 0, o2)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)


def test_noalloc_gemm_rejects_what_does_not_fit():
    cap = exe.exe_op_gemm_noalloc_max_workspace()
    assert cap == 64 << 20
    # find a split-K shape whose partial sums exceed the static array (host-side planning only)
    big = None
    for M in (256, 512, 768, 1024):
        for N in (20480, 36864, 49152):
            if exe.exe_op_gemm_workspace(BF16, M, N, 12288) > cap:
                big = (M, N, 12288)
                break
        if big:
            break
    assert big is not None
    M, N, K = big
    A, W = torch.zeros((M, K), dtype=torch.bfloat16, device=DEV), torch.zeros((N, K), dtype=torch.bfloat16, device=DEV)
    out = torch.full((M, N), 3.0, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(exe.ExeError) as e:
        exe.exe_op_gemm_noalloc(BF16, M, N, K, A, W, None, -1, 1.0, 0, out)
    assert e.value.code == -2
    torch.cuda.synchronize()
    assert float(out.float().min()) == 3.0                  # nothing was launched
