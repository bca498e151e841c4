"""Helpers for the GPU parity tests: build the HIP model and the oracle from the same seeded weights."""
import numpy as np
import torch

import oracle
import paper_2404_07947_amd as exe
import workload as wl

DEV = "cuda:0"


def tdtype(shape):
    return torch.float32 if shape.dtype == wl.DTYPE_F32 else torch.bfloat16


def kv_bytes_per_token(shape):
    layers = shape.n_layers if shape.arch == wl.ARCH_DECODER_ONLY else shape.n_dec_layers
    return layers * 2 * shape.inner * (4 if shape.dtype == wl.DTYPE_F32 else 2)


def make_pair(shape, seed, real="double", pool_tokens=8192, max_seqs=64, max_batch_tokens=4096, max_batch_seqs=64,
              gen_device="cpu", kv_block_size=0):
    """Returns (hip model, oracle, device weights).  Weights are drawn once and shared by value."""
    w = wl.make_weights(shape, seed, device=gen_device)
    wd = [t.to(DEV) for t in w]
    cfg = exe.config_from_shape(shape, kv_pool_bytes=pool_tokens * kv_bytes_per_token(shape), max_seqs=max_seqs,
                                max_batch_tokens=max_batch_tokens, max_batch_seqs=max_batch_seqs, kv_block_size=kv_block_size)
    m = exe.Model(cfg, wd)
    o = oracle.Oracle(shape, w, real, max_seqs=max_seqs)
    return m, o, wd


def row_relerr(got, ref):
    """max-norm relative error per row: max|g - o| / max|o|, worst row."""
    got = np.asarray(got, dtype=np.float64).reshape(-1, got.shape[-1])
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, ref.shape[-1])
    return float(np.max(np.max(np.abs(got - ref), axis=1) / np.maximum(np.max(np.abs(ref), axis=1), 1e-30)))


def relerr(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))
