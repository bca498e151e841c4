"""Pins for the oracle's model forward passes (decoder-only and T5-style encoder-decoder).

The pins are: an independent float64 forward pass assembled from PyTorch library routines
(layer_norm / rms_norm / linear / scaled_dot_product_attention / gelu / relu) and the exact-integer
bucket function; cached decoding == cache-free recomputation; causality; softmax row sums; the
identity-layer closed form; independence from batch-mates and release history.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workload as wl
from test_oracle_primitives import exact_bucket, relerr


def small_dec_shape():
    return wl.tiny_shape().replace(name="small", d_model=64, n_heads=4, head_dim=16, d_ff=96, vocab=211,
                                   max_pos=40)


def EPS(shape):
    """The config carries eps as a 32-bit float; use that exact value."""
    return float(np.float32(shape.norm_eps))


def named(shape, weights):
    return {n: w.double() for (n, _, _), w in zip(wl.weight_specs(shape), weights)}


# ---------------------------------------------------------------- library re-derivations (float64)

def torch_decoder_only(shape, W, tokens=None, hidden=None):
    """All-position logits (or hidden states) of a pre-LN decoder-only stack, from library routines."""
    d, H, dh = shape.d_model, shape.n_heads, shape.head_dim
    if shape.has_embed:
        t = torch.as_tensor(np.asarray(tokens), dtype=torch.long)
        h = W["tok_emb"][t]
        if shape.pos == wl.POS_LEARNED:
            h = h + W["pos_emb"][: len(t)]
    else:
        h = torch.as_tensor(hidden, dtype=torch.float64)
    n = h.shape[0]
    for l in range(shape.n_layers):
        p = f"l{l}."
        a = F.layer_norm(h, (d,), W[p + "ln1_g"], W[p + "ln1_b"], eps=EPS(shape))
        qkv = F.linear(a, W[p + "w_qkv"], W[p + "b_qkv"])
        q, k, v = (x.reshape(n, H, dh).transpose(0, 1) for x in qkv.split(H * dh, dim=1))
        ctx = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        ctx = ctx.transpose(0, 1).reshape(n, H * dh)
        h = h + F.linear(ctx, W[p + "w_o"], W[p + "b_o"])
        a = F.layer_norm(h, (d,), W[p + "ln2_g"], W[p + "ln2_b"], eps=EPS(shape))
        u = F.linear(a, W[p + "w_1"], W[p + "b_1"])
        u = F.gelu(u) if shape.act == wl.ACT_GELU else F.relu(u)
        h = h + F.linear(u, W[p + "w_2"], W[p + "b_2"])
    if not shape.has_lm_head:
        return h.numpy()
    a = F.layer_norm(h, (d,), W["lnf_g"], W["lnf_b"], eps=EPS(shape))
    return F.linear(a, W["tok_emb"]).numpy()


def bias_matrix(table, nq, nk, bidirectional, q0=0):
    """[H, nq, nk] additive bias from a [buckets, H] table, buckets by exact integer arithmetic."""
    idx = torch.tensor([[exact_bucket(j - (q0 + i), bidirectional) for j in range(nk)] for i in range(nq)])
    return table[idx].permute(2, 0, 1)


def torch_t5(shape, W, tokens, dec_tokens):
    d, H, dh = shape.d_model, shape.n_heads, shape.head_dim
    inner = H * dh

    def heads(x):
        return x.reshape(x.shape[0], H, dh).transpose(0, 1)

    def rms(x, g):
        return F.rms_norm(x, (d,), g, eps=EPS(shape))

    x = torch.as_tensor(np.asarray(tokens), dtype=torch.long)
    n = len(x)
    h = W["tok_emb"][x]
    eb = bias_matrix(W["enc_rel_bias"], n, n, True)
    for l in range(shape.n_layers):
        p = f"e{l}."
        q, k, v = (heads(t) for t in F.linear(rms(h, W[p + "rms1_g"]), W[p + "w_qkv"]).split(inner, dim=1))
        ctx = F.scaled_dot_product_attention(q[None], k[None], v[None], attn_mask=eb[None], scale=1.0)[0]
        h = h + F.linear(ctx.transpose(0, 1).reshape(n, inner), W[p + "w_o"])
        h = h + F.linear(F.relu(F.linear(rms(h, W[p + "rms2_g"]), W[p + "w_1"])), W[p + "w_2"])
    enc = rms(h, W["enc_final_g"])
    y = torch.as_tensor(np.asarray(dec_tokens), dtype=torch.long)
    m = len(y)
    g = W["tok_emb"][y]
    causal = torch.full((m, m), float("-inf"), dtype=torch.float64).triu(1)
    db = bias_matrix(W["dec_rel_bias"], m, m, False) + causal
    xb = bias_matrix(W["cross_rel_bias"], m, n, True) if shape.cross_rel_bias else None
    for l in range(shape.n_dec_layers):
        p = f"d{l}."
        q, k, v = (heads(t) for t in F.linear(rms(g, W[p + "rms1_g"]), W[p + "w_qkv"]).split(inner, dim=1))
        ctx = F.scaled_dot_product_attention(q[None], k[None], v[None], attn_mask=db[None], scale=1.0)[0]
        g = g + F.linear(ctx.transpose(0, 1).reshape(m, inner), W[p + "w_o"])
        q = heads(F.linear(rms(g, W[p + "rmsx_g"]), W[p + "w_xq"]))
        k, v = (heads(t) for t in F.linear(enc, W[p + "w_xkv"]).split(inner, dim=1))
        ctx = F.scaled_dot_product_attention(q[None], k[None], v[None],
                                             attn_mask=None if xb is None else xb[None], scale=1.0)[0]
        g = g + F.linear(ctx.transpose(0, 1).reshape(m, inner), W[p + "w_xo"])
        g = g + F.linear(F.relu(F.linear(rms(g, W[p + "rms3_g"]), W[p + "w_1"])), W[p + "w_2"])
    a = rms(g, W["dec_final_g"]) * d ** -0.5
    return F.linear(a, W["tok_emb"]).numpy(), enc.numpy()


# ---------------------------------------------------------------- decoder-only

@pytest.mark.parametrize("real,tol", [("double", 1e-11), ("float", 2e-4)])
@pytest.mark.parametrize("act", [wl.ACT_GELU, wl.ACT_RELU])
def test_decoder_only_matches_library_forward(real, tol, act):
    s = small_dec_shape().replace(act=act)
    w = wl.make_weights(s, 11)
    o = oracle.Oracle(s, w, real)
    toks = np.random.default_rng(0).integers(0, s.vocab, 19)
    ref = torch_decoder_only(s, named(s, w), toks)
    got = o.full(tokens=toks)
    assert relerr(got, ref) < tol
    nxt, last = o.encode(0, toks)
    assert relerr(last, ref[-1]) < tol
    assert nxt == int(np.argmax(ref[-1]))


def test_hidden_in_hidden_out_share_matches_library():
    s = small_dec_shape().replace(has_embed=0, has_lm_head=0, pos=wl.POS_NONE, vocab=0, max_pos=0)
    w = wl.make_weights(s, 12)
    assert len(w) == 12 * s.n_layers
    o = oracle.Oracle(s, w, "double")
    x = np.random.default_rng(1).normal(size=(9, s.d_model))
    ref = torch_decoder_only(s, named(s, w), hidden=x)
    assert relerr(o.full(hidden_in=x), ref) < 1e-11
    _, hid = o.encode(0, hidden_in=x)
    assert relerr(hid, ref) < 1e-11
    x2 = np.random.default_rng(2).normal(size=(1, s.d_model))
    _, h2 = o.decode(0, hidden_in=x2[0])
    ref2 = torch_decoder_only(s, named(s, w), hidden=np.concatenate([x, x2]))
    assert relerr(h2, ref2[-1]) < 1e-11


@pytest.mark.parametrize("real,tol", [("double", 1e-12), ("float", 1e-5)])
def test_cached_decode_equals_full_recompute(real, tol):
    s = wl.tiny_shape()
    w = wl.make_weights(s, wl.BASE_SEED)
    o = oracle.Oracle(s, w, real)
    job = wl.workload_tiny()
    for i in range(job.n):
        prefix = list(job.seq_tokens(i))
        tok, lg = o.encode(i, prefix)
        for step in range(16):
            full = o.full(tokens=np.array(prefix))
            assert relerr(lg, full[-1]) < tol, (i, step)
            assert tok == int(np.argmax(full[-1]))
            prefix.append(tok)
            tok, lg = o.decode(i, prefix[-1])
        assert o.seq_len(i) == job.in_len[i] + 16
    dev = o.rowsum_dev()
    assert dev < (1e-6 if real == "float" else 1e-13)     # every softmax row sums to 1


def test_causal_masking_is_exact():
    s = wl.tiny_shape()
    o = oracle.Oracle(s, wl.make_weights(s, 3), "double")
    toks = np.random.default_rng(3).integers(0, s.vocab, 24)
    base = o.full(tokens=toks)
    for j in (1, 7, 23):
        t2 = toks.copy()
        t2[j] = (t2[j] + 1) % s.vocab
        alt = o.full(tokens=t2)
        assert np.array_equal(alt[:j], base[:j])          # positions before j cannot see token j
        assert not np.array_equal(alt[j], base[j])


def test_identity_layers_closed_form():
    """With W_o = W_2 = 0 and b_o = b_2 = 0 every layer leaves the residual stream unchanged, so
    logits = LN_f(E_tok[x] + E_pos) E_tok^T, which the library computes in one line."""
    s = small_dec_shape()
    w = wl.make_weights(s, 13)
    for (name, _, _), t in zip(wl.weight_specs(s), w):
        if name.endswith((".w_o", ".b_o", ".w_2", ".b_2")):
            t.zero_()
    W = named(s, w)
    toks = np.random.default_rng(4).integers(0, s.vocab, 12)
    h = W["tok_emb"][torch.as_tensor(toks)] + W["pos_emb"][:12]
    ref = F.linear(F.layer_norm(h, (s.d_model,), W["lnf_g"], W["lnf_b"], eps=EPS(s)), W["tok_emb"]).numpy()
    o = oracle.Oracle(s, w, "double")
    assert relerr(o.full(tokens=toks), ref) < 1e-12
    # and cached decode of a further token sees the right position embedding
    _, lg0 = o.encode(0, toks[:11])
    _, lg1 = o.decode(0, int(toks[11]))
    assert relerr(lg0, ref[10]) < 1e-12 and relerr(lg1, ref[11]) < 1e-12


def test_single_token_sequence():
    s = small_dec_shape()
    w = wl.make_weights(s, 14)
    o = oracle.Oracle(s, w, "double")
    ref = torch_decoder_only(s, named(s, w), [5])
    _, lg = o.encode(0, [5])
    assert relerr(lg, ref[0]) < 1e-12


def test_batch_mates_order_and_release_do_not_matter():
    s = wl.tiny_shape()
    w = wl.make_weights(s, 5)
    job = wl.workload_tiny()
    a = oracle.Oracle(s, w, "float")
    b = oracle.Oracle(s, w, "float")
    # a: sequence 2 alone.  b: all four interleaved, others released midway, in a different order.
    ta, la = a.encode(0, job.seq_tokens(2))
    outs_a = [la]
    for _ in range(6):
        ta, l = a.decode(0, ta)
        outs_a.append(l)
    toks = {}
    for i in (3, 1, 2, 0):
        toks[i], l = b.encode(10 + i, job.seq_tokens(i))
        if i == 2:
            outs_b = [l]
    for step in range(6):
        if step == 2:
            b.release(10 + 3)
            del toks[3]
        if step == 4:
            b.release(10 + 0)
            del toks[0]
            toks[7], _ = b.encode(10 + 3, job.seq_tokens(1))     # slot reuse
        for i in sorted(toks, reverse=(step % 2 == 0)):
            toks[i], l = b.decode(10 + (3 if i == 7 else i), toks[i])
            if i == 2:
                outs_b.append(l)
    for x, y in zip(outs_a, outs_b):
        assert np.array_equal(x, y)


def test_float_and_double_oracles_agree():
    s = wl.tiny_shape()
    w = wl.make_weights(s, wl.BASE_SEED)
    toks = wl.workload_tiny().seq_tokens(3)
    f = oracle.Oracle(s, w, "float").full(tokens=toks)
    d = oracle.Oracle(s, w, "double").full(tokens=toks)
    assert relerr(f, d) < 1e-4


def test_tiny_config_greedy_tokens_are_well_posed():
    """The top-1/top-2 logit margin at every greedy decision of configs[0] exceeds 1e-3 of the largest
    |logit|, so 'identical greedy tokens' does not hinge on rounding."""
    s = wl.tiny_shape()
    o = oracle.Oracle(s, wl.make_weights(s, wl.BASE_SEED), "double")
    job = wl.workload_tiny()
    worst = 1.0
    for i in range(job.n):
        tok, lg = o.encode(i, job.seq_tokens(i))
        for step in range(17):
            top = np.sort(lg)[-2:]
            worst = min(worst, (top[1] - top[0]) / np.max(np.abs(lg)))
            if step < 16:
                tok, lg = o.decode(i, tok)
    assert worst > 1e-3, worst


def test_argument_errors():
    s = small_dec_shape()
    w = wl.make_weights(s, 1)
    o = oracle.Oracle(s, w, "double", max_seqs=2)
    with pytest.raises(ValueError):
        oracle.Oracle(s, w[:-1], "double")
    with pytest.raises(ValueError):
        o.encode(5, [1, 2])                  # slot out of range
    with pytest.raises(ValueError):
        o.encode(0, [1, s.vocab])            # token out of range
    with pytest.raises(ValueError):
        o.decode(1, 3)                       # not encoded
    o.encode(0, [1, 2])
    with pytest.raises(ValueError):
        o.encode(0, [1, 2])                  # still live
    with pytest.raises(ValueError):
        o.encode(1, list(range(s.max_pos + 1)))   # longer than the position table


# ---------------------------------------------------------------- encoder-decoder (T5 style)

@pytest.mark.parametrize("real,tol", [("double", 1e-11), ("float", 3e-4)])
@pytest.mark.parametrize("xbias", [1, 0])
def test_t5_matches_library_forward(real, tol, xbias):
    s = wl.small_t5_shape().replace(d_model=64, n_heads=4, head_dim=16, d_ff=96, vocab=199, cross_rel_bias=xbias)
    w = wl.make_weights(s, 21)
    W = named(s, w)
    rng = np.random.default_rng(5)
    toks = rng.integers(0, s.vocab, 41)
    dec = np.concatenate([[0], rng.integers(0, s.vocab, 20)])     # reaches the log-spaced buckets
    ref_logits, ref_enc = torch_t5(s, W, toks, dec)
    o = oracle.Oracle(s, w, real)
    logits, enc = o.full(tokens=toks, dec_tokens=dec)
    assert relerr(enc, ref_enc) < tol
    assert relerr(logits, ref_logits) < tol
    # cached path: encode once, then feed the same decoder tokens one by one
    _, enc2 = o.encode(0, toks)
    assert relerr(enc2, ref_enc) < tol
    for t in range(len(dec)):
        nxt, lg = o.decode(0, int(dec[t]))
        assert relerr(lg, ref_logits[t]) < tol, t
        assert nxt == int(np.argmax(ref_logits[t]))
    assert o.seq_len(0) == len(dec)
    assert o.rowsum_dev() < (1e-6 if real == "float" else 1e-13)


def test_t5_bias_and_scale_conventions_matter():
    """The pins above would not notice a convention that has no effect; check each one has an effect."""
    s = wl.small_t5_shape().replace(d_model=64, n_heads=4, head_dim=16, d_ff=96, vocab=199)
    w = wl.make_weights(s, 22)
    toks = np.random.default_rng(6).integers(0, s.vocab, 30)
    dec = np.array([0, 5, 9, 100, 42])
    base, _ = oracle.Oracle(s, w, "double").full(tokens=toks, dec_tokens=dec)
    for name in ("enc_rel_bias", "dec_rel_bias", "cross_rel_bias"):
        w2 = [t.clone() for t in w]
        idx = [n for n, _, _ in wl.weight_specs(s)].index(name)
        w2[idx].zero_()
        alt, _ = oracle.Oracle(s, w2, "double").full(tokens=toks, dec_tokens=dec)
        assert relerr(alt, base) > 1e-4, name
    alt, _ = oracle.Oracle(s.replace(scale_mode=wl.SCALE_RSQRT_DH), w, "double").full(tokens=toks, dec_tokens=dec)
    assert relerr(alt, base) > 1e-4


def test_t5_zero_bias_scaled_reduces_to_textbook_attention():
    s = wl.small_t5_shape().replace(d_model=64, n_heads=4, head_dim=16, d_ff=96, vocab=199,
                                    scale_mode=wl.SCALE_RSQRT_DH, cross_rel_bias=0)
    w = wl.make_weights(s, 23)
    names = [n for n, _, _ in wl.weight_specs(s)]
    for nm in ("enc_rel_bias", "dec_rel_bias"):
        w[names.index(nm)].zero_()
    toks = np.random.default_rng(7).integers(0, s.vocab, 17)
    _, enc = oracle.Oracle(s, w, "double").full(tokens=toks, dec_tokens=[0])
    # encoder with library attention at its default 1/sqrt(dh) scale and no mask
    W = named(s, w)
    d, H, dh = s.d_model, s.n_heads, s.head_dim
    h = W["tok_emb"][torch.as_tensor(toks)]
    for l in range(s.n_layers):
        p = f"e{l}."
        q, k, v = (t.reshape(17, H, dh).transpose(0, 1) for t in
                   F.linear(F.rms_norm(h, (d,), W[p + "rms1_g"], eps=EPS(s)), W[p + "w_qkv"]).split(H * dh, 1))
        ctx = F.scaled_dot_product_attention(q[None], k[None], v[None])[0].transpose(0, 1).reshape(17, H * dh)
        h = h + F.linear(ctx, W[p + "w_o"])
        h = h + F.linear(F.relu(F.linear(F.rms_norm(h, (d,), W[p + "rms2_g"], eps=EPS(s)), W[p + "w_1"])),
                         W[p + "w_2"])
    ref = F.rms_norm(h, (d,), W["enc_final_g"], eps=EPS(s)).numpy()
    assert relerr(enc, ref) < 1e-11


def test_t5_sequences_are_independent():
    s = wl.small_t5_shape()
    w = wl.make_weights(s, 24)
    rng = np.random.default_rng(8)
    a_t, b_t = rng.integers(0, s.vocab, 33), rng.integers(0, s.vocab, 12)
    o1 = oracle.Oracle(s, w, "float")
    o2 = oracle.Oracle(s, w, "float")
    o1.encode(0, a_t)
    o2.encode(3, b_t); o2.encode(1, a_t)
    t1 = t2 = tb = 0
    for step in range(5):
        t1, l1 = o1.decode(0, t1)
        tb, _ = o2.decode(3, tb)
        if step == 2:
            o2.release(3); o2.encode(3, b_t); tb = 0
        t2, l2 = o2.decode(1, t2)
        assert np.array_equal(l1, l2)


# ---------------------------------------------------------------- workload generator

def test_workload_generators():
    j1, j2 = wl.workload_opt13b(256), wl.workload_opt13b(256)
    assert np.array_equal(j1.in_len, j2.in_len) and np.array_equal(j1.tokens, j2.tokens)
    assert j1.in_len.min() >= 64 and j1.in_len.max() <= 1024
    assert j1.out_len.min() >= 16 and j1.out_len.max() <= 256
    assert abs(j1.in_len.mean() - 512) < 40 and abs(j1.out_len.mean() - 128) < 10
    assert j1.tokens.min() >= 0 and j1.tokens.max() < 50272 and len(j1.tokens) == j1.in_len.sum()
    t = wl.workload_tiny()
    assert t.n == 4 and t.in_len.min() >= 8 and t.in_len.max() <= 32 and (t.out_len == 17).all()
    t5 = wl.workload_t5(64)
    assert t5.in_len.min() >= 128 and t5.in_len.max() <= 1024 and t5.out_len.max() <= 128
    g = wl.workload_gpt3_share(64)
    assert g.in_len.min() >= 128 and g.in_len.max() <= 2048 and g.out_len.min() >= 32
    # forced output lengths: decoder-only sequences with o outputs take o-1 decode steps
    ol = np.array([1, 2, 5])
    assert list(wl.alive_at_step(ol, 1, True)) == [1, 2]
    assert list(wl.alive_at_step(ol, 4, True)) == [2]
    assert list(wl.alive_at_step(ol, 5, True)) == []
    assert list(wl.alive_at_step(ol, 5, False)) == [2]
    assert wl.n_decode_steps(ol, True) == 4 and wl.n_decode_steps(ol, False) == 5
    # parameter counts of the paper's Table 1 shapes
    assert abs(wl.n_params(wl.opt13b_shape()) / 1e9 - 12.85) < 0.1
    assert abs(wl.n_params(wl.t5_11b_shape()) / 1e9 - 11.3) < 0.3
    assert abs(wl.n_params(wl.gpt3_175b_share_shape(96)) / 1e9 - 174) < 1.5
