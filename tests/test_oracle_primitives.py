"""Pins for the oracle's primitive operations: library routines in float64, closed forms, special
cases and exact integer arithmetic.  None of these re-types the oracle's own formula."""
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle

REALS = ["double", "float"]
TOL = {"double": 1e-12, "float": 2e-5}


def relerr(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


@pytest.mark.parametrize("real", REALS)
def test_linear_matches_library_and_is_not_transposed(real):
    P = oracle.Primitives(real)
    rng = np.random.default_rng(1)
    x = rng.normal(size=(5, 37)).astype(np.float32)
    W = rng.normal(size=(11, 37)).astype(np.float32)      # [out, in], non-square on purpose
    b = rng.normal(size=11).astype(np.float32)
    ref = F.linear(torch.from_numpy(x).double(), torch.from_numpy(W).double(), torch.from_numpy(b).double())
    assert relerr(P.linear(x, W, b), ref.numpy()) < TOL[real]
    ref0 = torch.from_numpy(x).double() @ torch.from_numpy(W).double().T
    assert relerr(P.linear(x, W, None), ref0.numpy()) < TOL[real]
    # one-hot input row k selects column k of W (closed form; catches a swapped index)
    e = np.zeros((1, 37), np.float32); e[0, 5] = 1
    assert np.allclose(P.linear(e, W, None)[0], W[:, 5], rtol=0, atol=1e-7)


@pytest.mark.parametrize("real", REALS)
def test_layernorm(real):
    P = oracle.Primitives(real)
    rng = np.random.default_rng(2)
    x = (rng.normal(size=(4, 96)) * 3 + 1.5).astype(np.float32)
    g = (1 + 0.1 * rng.normal(size=96)).astype(np.float32)
    b = (0.1 * rng.normal(size=96)).astype(np.float32)
    ref = F.layer_norm(torch.from_numpy(x).double(), (96,), torch.from_numpy(g).double(),
                       torch.from_numpy(b).double(), eps=1e-5)
    assert relerr(P.layernorm(x, g, b, 1e-5), ref.numpy()) < TOL[real]
    # a constant row has zero variance: the output is exactly the shift
    const = np.full((1, 96), 2.75, np.float32)
    assert np.allclose(P.layernorm(const, g, b, 1e-5)[0], b, rtol=0, atol=1e-7)
    # output (before gain/shift) has mean 0 and variance var/(var+eps)
    y = P.layernorm(x, np.ones(96, np.float32), np.zeros(96, np.float32), 1e-5).astype(np.float64)
    assert np.max(np.abs(y.mean(axis=1))) < 1e-5
    v = x.astype(np.float64).var(axis=1)
    assert np.allclose(y.var(axis=1), v / (v + 1e-5), rtol=1e-4)


@pytest.mark.parametrize("real", REALS)
def test_rmsnorm(real):
    P = oracle.Primitives(real)
    rng = np.random.default_rng(3)
    x = rng.normal(size=(3, 64)).astype(np.float32)
    g = (1 + 0.1 * rng.normal(size=64)).astype(np.float32)
    ref = F.rms_norm(torch.from_numpy(x).double(), (64,), torch.from_numpy(g).double(), eps=1e-6)
    assert relerr(P.rmsnorm(x, g, 1e-6), ref.numpy()) < TOL[real]
    # one-hot row c*e_k: mean square = c^2/d, so y_k = c / sqrt(c^2/d + eps) * g_k and 0 elsewhere
    e = np.zeros((1, 64), np.float32); e[0, 9] = -3.0
    y = P.rmsnorm(e, g, 1e-6)[0]
    want = np.zeros(64); want[9] = -3.0 / np.sqrt(9.0 / 64 + 1e-6) * g[9]
    assert np.allclose(y, want, rtol=1e-6, atol=0)
    # no mean subtraction: a constant row c maps to c/sqrt(c^2+eps) * g, not to zero
    const = np.full((1, 64), 0.5, np.float32)
    assert np.allclose(P.rmsnorm(const, g, 1e-6)[0], 0.5 / np.sqrt(0.25 + 1e-6) * g, rtol=1e-6)


@pytest.mark.parametrize("real", REALS)
def test_activations(real):
    P = oracle.Primitives(real)
    x = np.linspace(-6, 6, 241).astype(np.float32)
    tx = torch.from_numpy(x).double()
    assert relerr(P.act(x, 0), F.relu(tx).numpy()) == 0
    assert relerr(P.act(x, 1), F.gelu(tx, approximate="none").numpy()) < TOL[real]
    # erf form, not the tanh approximation: they differ by ~1e-3 near |x| ~ 2
    assert relerr(P.act(x, 1), F.gelu(tx, approximate="tanh").numpy()) > 1e-5
    # gelu(x) - gelu(-x) = x  (erf is odd)
    y = P.act(x, 1).astype(np.float64)
    assert np.allclose(y - y[::-1], x, atol=1e-6)


@pytest.mark.parametrize("real", REALS)
def test_attention_row_matches_library(real):
    P = oracle.Primitives(real)
    rng = np.random.default_rng(4)
    nk, dh = 23, 16
    q = rng.normal(size=dh).astype(np.float32)
    K = rng.normal(size=(nk, dh)).astype(np.float32)
    V = rng.normal(size=(nk, dh)).astype(np.float32)
    bias = rng.normal(size=nk).astype(np.float32)
    tq, tK, tV = (torch.from_numpy(a).double() for a in (q, K, V))
    ref = F.scaled_dot_product_attention(tq[None, None, None, :], tK[None, None], tV[None, None],
                                         attn_mask=torch.from_numpy(bias).double()[None, None, None, :],
                                         scale=0.25)
    out, probs, ps = P.attention_row(q, K, V, 0.25, bias)
    assert relerr(out, ref[0, 0, 0].numpy()) < 10 * TOL[real]
    assert abs(ps - 1) < 1e-6 and abs(probs.sum() - 1) < 1e-6
    # unscaled, no bias
    ref = F.scaled_dot_product_attention(tq[None, None, None, :], tK[None, None], tV[None, None], scale=1.0)
    out, _, _ = P.attention_row(q, K, V, 1.0, None)
    assert relerr(out, ref[0, 0, 0].numpy()) < 10 * TOL[real]


@pytest.mark.parametrize("real", REALS)
def test_attention_row_closed_forms(real):
    P = oracle.Primitives(real)
    rng = np.random.default_rng(5)
    nk, dh = 9, 8
    q = rng.normal(size=dh).astype(np.float32)
    V = rng.normal(size=(nk, dh)).astype(np.float32)
    K = np.tile(rng.normal(size=(1, dh)).astype(np.float32), (nk, 1))
    # identical keys -> uniform weights -> context is the mean of the values
    out, probs, _ = P.attention_row(q, K, V, 0.3, None)
    assert np.allclose(probs, 1.0 / nk, atol=1e-7)
    assert np.allclose(out, V.astype(np.float64).mean(axis=0), atol=1e-6)
    # single key -> weight 1
    out, probs, _ = P.attention_row(q, K[:1], V[:1], 0.3, None)
    assert probs[0] == 1 and np.allclose(out, V[0], atol=0)
    # a constant added to every bias entry changes nothing (softmax shift invariance)
    K2 = rng.normal(size=(nk, dh)).astype(np.float32)
    b = rng.normal(size=nk).astype(np.float32)
    o1, _, _ = P.attention_row(q, K2, V, 0.3, b)
    o2, _, _ = P.attention_row(q, K2, V, 0.3, b + 4.0)
    assert np.allclose(o1, o2, atol=1e-5)
    # a very negative bias removes a key (what masking relies on)
    b2 = np.zeros(nk, np.float32); b2[3] = -1e30
    _, p, _ = P.attention_row(q, K2, V, 0.3, b2)
    assert p[3] == 0
    # huge scores do not overflow (maximum is subtracted)
    out, probs, ps = P.attention_row(q * 1e4, K2, V, 1.0, None)
    assert np.isfinite(out).all() and abs(ps - 1) < 1e-6


@pytest.mark.parametrize("real", REALS)
def test_argmax_ties_lowest_index(real):
    P = oracle.Primitives(real)
    assert P.argmax(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    assert P.argmax(np.array([5.0, 5.0, 5.0])) == 0
    rng = np.random.default_rng(6)
    x = rng.normal(size=1000)
    assert P.argmax(x) == int(np.argmax(x))


def exact_bucket(rel, bidirectional, nb=32, md=128):
    """The bucket scheme in exact rational arithmetic: log spacing without any logarithm."""
    base = 0
    if bidirectional:
        nb //= 2
        if rel > 0:
            base = nb
        n = abs(rel)
    else:
        n = max(0, -rel)
    ex = nb // 2
    if n < ex:
        return base + n
    span = nb - ex
    b = 0
    # largest b with (md/ex)^(b/span) <= n/ex
    while Fraction(md, ex) ** (b + 1) <= Fraction(n, ex) ** span:
        b += 1
    return base + min(ex + b, nb - 1)


def test_bucket_exact_and_properties():
    P = oracle.Primitives("double")
    for bid in (0, 1):
        vals = [P.bucket(r, bid) for r in range(-2100, 2101)]
        assert vals == [exact_bucket(r, bid) for r in range(-2100, 2101)]
        assert min(vals) >= 0 and max(vals) <= 31
    # unidirectional: keys after the query (rel > 0) count as distance 0; exact region is identity
    assert [P.bucket(-n, 0) for n in range(16)] == list(range(16))
    assert all(P.bucket(r, 0) == 0 for r in range(0, 50))
    # powers of two in the log region: 16 * 2^m -> 16 + floor(16 m / 3)
    assert [P.bucket(-16 * 2 ** m, 0) for m in range(4)] == [16, 21, 26, 31]
    assert P.bucket(-100000, 0) == 31
    # monotone in distance
    u = [P.bucket(-n, 0) for n in range(0, 3000)]
    assert all(a <= b for a, b in zip(u, u[1:]))
    # bidirectional: 16 per sign, exact up to 8, 8 * 2^m -> 8 + 2m, upper half for keys after the query
    assert [P.bucket(-n, 1) for n in range(8)] == list(range(8))
    assert [P.bucket(n, 1) for n in range(1, 8)] == [16 + n for n in range(1, 8)]
    assert [P.bucket(-8 * 2 ** m, 1) for m in range(5)] == [8, 10, 12, 14, 15]
    assert [P.bucket(8 * 2 ** m, 1) for m in range(5)] == [24, 26, 28, 30, 31]
    assert P.bucket(0, 1) == 0
