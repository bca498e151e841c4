"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module holds no Transformer arithmetic: only model *shapes*, the fixed order
and shapes of the weight tensors, random weight/tokens/length draws, and the
bookkeeping of which sequence is alive at which decode step.  Both the oracle
binding and the HIP binding convert a `ModelShape` into their own config struct.

Workload protocol follows the paper's evaluation section: input/output lengths are
drawn independently from a (clipped) normal distribution and the output length
is *forced* (decoding continues for the drawn number of tokens, no end-of-sequence
token); finished sequences leave the decode batch (early termination).
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

BASE_SEED = 20240427

ARCH_DECODER_ONLY = 0
ARCH_ENC_DEC = 1
ACT_RELU = 0
ACT_GELU = 1
NORM_LAYERNORM = 0
NORM_RMSNORM = 1
POS_LEARNED = 0
POS_RELBIAS = 1
POS_NONE = 2
DTYPE_F32 = 0
DTYPE_BF16 = 1
SCALE_RSQRT_DH = 0
SCALE_NONE = 1


@dataclass(frozen=True)
class ModelShape:
    """Architecture description (no arithmetic).  Field meanings:

    arch           0 decoder-only, 1 encoder-decoder (T5 style)
    n_layers       decoder-only: layers; enc-dec: encoder layers
    n_dec_layers   enc-dec: decoder layers (0 for decoder-only)
    act            0 ReLU, 1 GELU (erf form)
    norm           0 LayerNorm (gain+shift), 1 RMSNorm (gain only)
    pos            0 learned absolute positions, 1 T5 relative-position bias, 2 none
    cross_rel_bias enc-dec: 1 = cross-attention also adds a relative-position bias
    has_embed      0 = the caller passes hidden states instead of token ids
    has_lm_head    0 = the model returns hidden states (one pipeline stage's share)
    scale_mode     0 scores scaled by 1/sqrt(head_dim), 1 unscaled (T5)
    """
    name: str
    arch: int
    n_layers: int
    n_dec_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    max_pos: int
    act: int
    norm: int
    pos: int
    rel_buckets: int
    rel_max_dist: int
    cross_rel_bias: int
    dtype: int
    has_embed: int
    has_lm_head: int
    scale_mode: int
    norm_eps: float

    @property
    def inner(self) -> int:
        return self.n_heads * self.head_dim

    def replace(self, **kw) -> "ModelShape":
        return dataclasses.replace(self, **kw)


def tiny_shape() -> ModelShape:
    """configs[0]: tiny fp32 decoder-only LM."""
    return ModelShape("tiny", ARCH_DECODER_ONLY, 2, 0, 256, 4, 64, 1024, 2048, 64, ACT_GELU,
                      NORM_LAYERNORM, POS_LEARNED, 0, 0, 0, DTYPE_F32, 1, 1, SCALE_RSQRT_DH, 1e-5)


def opt13b_shape(n_layers: int = 40) -> ModelShape:
    """configs[1]: OPT-13B-shaped bf16 decoder (Table 1 of the paper: 40 layers, hidden 5120, 40 heads)."""
    return ModelShape("opt13b", ARCH_DECODER_ONLY, n_layers, 0, 5120, 40, 128, 20480, 50272, 2048,
                      ACT_RELU, NORM_LAYERNORM, POS_LEARNED, 0, 0, 0, DTYPE_BF16, 1, 1,
                      SCALE_RSQRT_DH, 1e-5)


def t5_11b_shape(n_layers: int = 24, n_dec_layers: int = 24) -> ModelShape:
    """configs[2]: T5-11B-shaped bf16 encoder-decoder (Table 1: 48 layers, hidden 1024, 128 heads)."""
    return ModelShape("t5_11b", ARCH_ENC_DEC, n_layers, n_dec_layers, 1024, 128, 128, 65536, 32128, 0,
                      ACT_RELU, NORM_RMSNORM, POS_RELBIAS, 32, 128, 1, DTYPE_BF16, 1, 1,
                      SCALE_NONE, 1e-6)


def gpt3_175b_share_shape(n_layers: int = 12) -> ModelShape:
    """configs[3]: 12 consecutive layers of a GPT-3-175B-shaped decoder (Table 1: hidden 12288, 96 heads);
    hidden states in, hidden states out."""
    return ModelShape("gpt3_175b_share", ARCH_DECODER_ONLY, n_layers, 0, 12288, 96, 128, 49152, 0, 0,
                      ACT_GELU, NORM_LAYERNORM, POS_NONE, 0, 0, 0, DTYPE_BF16, 0, 0,
                      SCALE_RSQRT_DH, 1e-5)


def small_t5_shape(dtype: int = DTYPE_F32) -> ModelShape:
    """A small T5-style model (same structure as configs[2], narrow) that the oracle finishes in seconds."""
    return ModelShape("t5_small", ARCH_ENC_DEC, 2, 2, 256, 4, 64, 512, 1024, 0, ACT_RELU, NORM_RMSNORM,
                      POS_RELBIAS, 32, 128, 1, dtype, 1, 1, SCALE_NONE, 1e-6)


# --------------------------------------------------------------------------
# weight table: fixed order, names and shapes.  Linear weights are [out, in]
# row-major (each output feature's input weights contiguous).
# --------------------------------------------------------------------------

def weight_specs(s: ModelShape) -> List[Tuple[str, Tuple[int, ...], str]]:
    """Returns [(name, shape, kind)], kind in {"matrix","bias","gain","shift","relbias"}."""
    d, inner, f = s.d_model, s.inner, s.d_ff
    out: List[Tuple[str, Tuple[int, ...], str]] = []
    if s.arch == ARCH_DECODER_ONLY:
        if s.has_embed or s.has_lm_head:
            out.append(("tok_emb", (s.vocab, d), "matrix"))
        if s.has_embed and s.pos == POS_LEARNED:
            out.append(("pos_emb", (s.max_pos, d), "matrix"))
        for l in range(s.n_layers):
            p = f"l{l}."
            out += [(p + "ln1_g", (d,), "gain"), (p + "ln1_b", (d,), "shift"),
                    (p + "w_qkv", (3 * inner, d), "matrix"), (p + "b_qkv", (3 * inner,), "bias"),
                    (p + "w_o", (d, inner), "matrix"), (p + "b_o", (d,), "bias"),
                    (p + "ln2_g", (d,), "gain"), (p + "ln2_b", (d,), "shift"),
                    (p + "w_1", (f, d), "matrix"), (p + "b_1", (f,), "bias"),
                    (p + "w_2", (d, f), "matrix"), (p + "b_2", (d,), "bias")]
        if s.has_lm_head:
            out += [("lnf_g", (d,), "gain"), ("lnf_b", (d,), "shift")]
    else:
        out.append(("tok_emb", (s.vocab, d), "matrix"))
        out.append(("enc_rel_bias", (s.rel_buckets, s.n_heads), "relbias"))
        out.append(("dec_rel_bias", (s.rel_buckets, s.n_heads), "relbias"))
        if s.cross_rel_bias:
            out.append(("cross_rel_bias", (s.rel_buckets, s.n_heads), "relbias"))
        for l in range(s.n_layers):
            p = f"e{l}."
            out += [(p + "rms1_g", (d,), "gain"), (p + "w_qkv", (3 * inner, d), "matrix"),
                    (p + "w_o", (d, inner), "matrix"), (p + "rms2_g", (d,), "gain"),
                    (p + "w_1", (f, d), "matrix"), (p + "w_2", (d, f), "matrix")]
        out.append(("enc_final_g", (d,), "gain"))
        for l in range(s.n_dec_layers):
            p = f"d{l}."
            out += [(p + "rms1_g", (d,), "gain"), (p + "w_qkv", (3 * inner, d), "matrix"),
                    (p + "w_o", (d, inner), "matrix"), (p + "rmsx_g", (d,), "gain"),
                    (p + "w_xq", (inner, d), "matrix"), (p + "w_xkv", (2 * inner, d), "matrix"),
                    (p + "w_xo", (d, inner), "matrix"), (p + "rms3_g", (d,), "gain"),
                    (p + "w_1", (f, d), "matrix"), (p + "w_2", (d, f), "matrix")]
        out.append(("dec_final_g", (d,), "gain"))
    return out


def n_params(s: ModelShape) -> int:
    return int(sum(int(np.prod(shape)) for _, shape, _ in weight_specs(s)))


def make_weights(s: ModelShape, seed: int, device: str = "cpu"):
    """Random-init weights as a list of torch tensors in the storage dtype, in `weight_specs` order.

    Matrices, biases and norm shifts ~ N(0, 0.02); norm gains = 1 + N(0, 0.02); relative-position
    bias tables ~ N(0, 0.5) so that the bias visibly changes the attention weights.  Values are drawn
    in fp32 and rounded once to the storage dtype; every consumer (oracle and HIP path) reads these
    rounded values.  Each tensor has its own seed (seed, index), so a reduced-layer model shares its
    tensors with the corresponding prefix of the full model only by name, not by position.
    """
    import torch
    import zlib
    tdtype = torch.float32 if s.dtype == DTYPE_F32 else torch.bfloat16
    out = []
    for name, shape, kind in weight_specs(s):
        g = torch.Generator(device=device)
        g.manual_seed((seed * 1000003 + zlib.crc32(name.encode())) & 0x7FFFFFFFFFFFFFFF)
        w = torch.empty(shape, dtype=torch.float32, device=device)
        w.normal_(0.0, 0.5 if kind == "relbias" else 0.02, generator=g)
        if kind == "gain":
            w += 1.0
        out.append(w.to(tdtype).contiguous())
        del w
    return out


# --------------------------------------------------------------------------
# lengths, tokens, hidden states
# --------------------------------------------------------------------------

def clipped_normal_lengths(rng: np.random.Generator, n: int, mean: float, std: float,
                           lo: int, hi: int) -> np.ndarray:
    """Draw normal, round to nearest integer, clamp to [lo, hi] (clamp, not resample)."""
    x = rng.normal(mean, std, size=n)
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


def clipped_normal_pmf(mean: float, std: float, lo: int, hi: int) -> np.ndarray:
    """The distribution `clipped_normal_lengths` draws from, as probabilities of the lengths 1 .. hi (index s - 1):
    a normal rounded to the nearest integer, with everything below lo piled up on lo and everything above hi on hi."""
    from math import erf, sqrt
    cdf = lambda x: 0.5 * (1.0 + erf((x - mean) / (std * sqrt(2.0))))
    p = np.zeros(hi, dtype=np.float64)
    for s in range(lo, hi + 1):
        a = -np.inf if s == lo else s - 0.5
        b = np.inf if s == hi else s + 0.5
        p[s - 1] = (1.0 if b == np.inf else cdf(b)) - (0.0 if a == -np.inf else cdf(a))
    return p


def uniform_lengths(rng: np.random.Generator, n: int, lo: int, hi: int) -> np.ndarray:
    return rng.integers(lo, hi + 1, size=n).astype(np.int32)


def random_tokens(rng: np.random.Generator, total: int, vocab: int) -> np.ndarray:
    return rng.integers(0, vocab, size=total).astype(np.int32)


@dataclass
class Workload:
    """One synthetic job: `in_len[i]` input tokens and `out_len[i]` forced output tokens per sequence."""
    name: str
    in_len: np.ndarray          # int32 [n]
    out_len: np.ndarray         # int32 [n]
    tokens: np.ndarray          # int32 [sum(in_len)] packed, sequence after sequence
    encode_batch: int           # sequences per encode call

    @property
    def n(self) -> int:
        return int(self.in_len.shape[0])

    def offsets(self) -> np.ndarray:
        o = np.zeros(self.n + 1, dtype=np.int64)
        np.cumsum(self.in_len, out=o[1:])
        return o

    def seq_tokens(self, i: int) -> np.ndarray:
        o = self.offsets()
        return self.tokens[o[i]:o[i + 1]]


def workload_tiny(seed: int = BASE_SEED) -> Workload:
    """configs[0]: batch 4, input lengths uniform in [8,32], 16 decode steps after the encode."""
    rng = np.random.default_rng(seed)
    n = 4
    il = uniform_lengths(rng, n, 8, 32)
    ol = np.full(n, 17, dtype=np.int32)     # encode emits token 1, then 16 decode steps
    return Workload("tiny", il, ol, random_tokens(rng, int(il.sum()), 2048), 4)


def workload_opt13b(decode_batch: int = 256, seed: int = BASE_SEED + 1, vocab: int = 50272) -> Workload:
    """configs[1]: encode batches of 32, inputs ~ N(512,128) in [64,1024]; outputs ~ N(128,32) in [16,256]."""
    rng = np.random.default_rng(seed)
    il = clipped_normal_lengths(rng, decode_batch, 512, 128, 64, 1024)
    ol = clipped_normal_lengths(rng, decode_batch, 128, 32, 16, 256)
    return Workload("opt13b", il, ol, random_tokens(rng, int(il.sum()), vocab), 32)


def workload_t5(decode_batch: int = 64, seed: int = BASE_SEED + 2, vocab: int = 32128) -> Workload:
    """configs[2]: encode batches of 16, inputs ~ N(768,192) in [128,1024]; outputs ~ N(64,16) in [8,128]."""
    rng = np.random.default_rng(seed)
    il = clipped_normal_lengths(rng, decode_batch, 768, 192, 128, 1024)
    ol = clipped_normal_lengths(rng, decode_batch, 64, 16, 8, 128)
    return Workload("t5_11b", il, ol, random_tokens(rng, int(il.sum()), vocab), 16)


def workload_gpt3_share(decode_batch: int = 512, seed: int = BASE_SEED + 3) -> Workload:
    """configs[3]: encode batches of 8, inputs ~ N(1024,256) in [128,2048]; outputs ~ N(256,64) in [32,512].
    Inputs are hidden states, so `tokens` is empty."""
    rng = np.random.default_rng(seed)
    il = clipped_normal_lengths(rng, decode_batch, 1024, 256, 128, 2048)
    ol = clipped_normal_lengths(rng, decode_batch, 256, 64, 32, 512)
    return Workload("gpt3_175b_share", il, ol, np.zeros(0, dtype=np.int32), 8)


def random_hidden(seed: int, rows: int, d: int, dtype: int, device: str = "cpu"):
    """N(0,1) hidden states [rows, d] in the storage dtype (for models without an embedding)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.empty((rows, d), dtype=torch.float32, device=device).normal_(0.0, 1.0, generator=g)
    return x.to(torch.float32 if dtype == DTYPE_F32 else torch.bfloat16).contiguous()


def alive_at_step(out_len: Sequence[int], step: int, decoder_only: bool) -> np.ndarray:
    """Indices of sequences that take part in decode step `step` (1-based).

    Decoder-only: the encode call already produced generated token #1, so a sequence with o forced
    output tokens takes part in decode steps 1..o-1.  Encoder-decoder: the encode call produces no
    token, so it takes part in steps 1..o.
    """
    ol = np.asarray(out_len)
    last = ol - 1 if decoder_only else ol
    return np.nonzero(last >= step)[0].astype(np.int32)


def n_decode_steps(out_len: Sequence[int], decoder_only: bool) -> int:
    ol = np.asarray(out_len)
    return int(ol.max() - 1 if decoder_only else ol.max())
