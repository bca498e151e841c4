"""End-to-end parity of exe_encode / exe_decode_step (through the C ABI) against the CPU oracle on the same
seeded weights and inputs.  Tolerances: float configs compare at 1e-4 (float accumulation order only);
bf16 configs at the stated bar, max-norm relative error <= 2e-2 per logits row."""
import numpy as np
import pytest
import torch

import paper_2404_07947_amd as exe
import workload as wl
from gpu_util import DEV, make_pair, relerr, row_relerr, tdtype

pytestmark = pytest.mark.gpu
BF16_TOL = 2e-2
F32_TOL = 1e-4


def run_decoder_only(shape, seed, in_lens, n_steps, tol, real="double", check_tokens=False, release_at=None,
                     gen_device="cpu", kv_block_size=0):
    """Encode a batch, then n_steps decode steps feeding the ORACLE's greedy tokens to both sides, so that a
    near-tie cannot make the two sides diverge; compares logits at every step."""
    n = len(in_lens)
    m, o, _ = make_pair(shape, seed, real, gen_device=gen_device, max_batch_tokens=max(4096, int(sum(in_lens))),
                        kv_block_size=kv_block_size)
    rng = np.random.default_rng(seed)
    toks = wl.random_tokens(rng, int(sum(in_lens)), shape.vocab)
    ids = np.arange(n) + 3
    logits = torch.zeros((n, shape.vocab), dtype=torch.float32, device=DEV)
    res = [int(L) + n_steps for L in in_lens]
    print(f"encode {shape.name} lens={list(in_lens)}", flush=True)
    nxt = m.encode(ids, in_lens, toks, reserve_lengths=res, out_device=logits)
    off = np.concatenate([[0], np.cumsum(in_lens)])
    ref_tok, worst = [], 0.0
    for i in range(n):
        t, lg = o.encode(int(ids[i]), toks[off[i]:off[i + 1]])
        ref_tok.append(t)
        worst = max(worst, row_relerr(logits[i].cpu().numpy()[None], lg[None]))
    assert worst < tol, ("encode", worst)
    if check_tokens:
        assert list(nxt) == ref_tok
    alive = list(range(n))
    cur = np.array(ref_tok)
    for step in range(1, n_steps + 1):
        if release_at and step in release_at:
            gone = release_at[step]
            m.seq_release(ids[gone])
            for g in gone:
                o.release(int(ids[g]))
            alive = [a for a in alive if a not in gone]
        kv = [int(in_lens[a]) + step for a in alive]
        lg_d = torch.zeros((len(alive), shape.vocab), dtype=torch.float32, device=DEV)
        nxt = m.decode_step(ids[alive], cur[alive], kv, out_device=lg_d)
        got = lg_d.cpu().numpy()
        for j, a in enumerate(alive):
            t, lg = o.decode(int(ids[a]), int(cur[a]))
            worst = max(worst, row_relerr(got[j][None], lg[None]))
            if check_tokens:
                assert int(nxt[j]) == t, (step, a)
            cur[a] = t
        assert worst < tol, (step, worst)
    m.close()
    return worst


def test_tiny_config_identical_greedy_tokens():
    """configs[0]: fp32, batch 4, lengths U[8,32], encode + 16 greedy decode steps; the HIP path's own
    greedy tokens (fed back to itself) must equal the oracle's."""
    shape = wl.tiny_shape()
    job = wl.workload_tiny()
    m, o, _ = make_pair(shape, wl.BASE_SEED, "float")
    ids = np.arange(job.n)
    got = [m.encode(ids, job.in_len, job.tokens, reserve_lengths=job.in_len + 17)]
    for step in range(1, 17):
        got.append(m.decode_step(ids, got[-1], job.in_len + step))
    got = np.stack(got, axis=1)
    want = []
    for i in range(job.n):
        t, _ = o.encode(i, job.seq_tokens(i))
        seq = [t]
        for _ in range(16):
            t, _ = o.decode(i, t)
            seq.append(t)
        want.append(seq)
    assert got.tolist() == want
    assert [m.seq_length(i) for i in ids] == [int(L) + 16 for L in job.in_len]
    m.close()


def test_tiny_config_logits():
    job = wl.workload_tiny()
    w = run_decoder_only(wl.tiny_shape(), wl.BASE_SEED, job.in_len, 16, F32_TOL, check_tokens=True)
    print("tiny f32 worst row rel err", w)


def test_small_bf16_decoder_ragged_with_release():
    shape = wl.tiny_shape().replace(name="small_bf16", dtype=wl.DTYPE_BF16, max_pos=512, n_layers=3)
    w = run_decoder_only(shape, 5, [1, 37, 128, 129, 300, 64], 6, BF16_TOL, release_at={3: [1, 4], 5: [0]})
    print("small bf16 worst", w)


def test_small_bf16_relu_head128():
    shape = wl.tiny_shape().replace(name="small_bf16_h128", dtype=wl.DTYPE_BF16, max_pos=512, head_dim=128,
                                    n_heads=2, act=wl.ACT_RELU)
    w = run_decoder_only(shape, 6, [5, 200, 131], 4, BF16_TOL)
    print("small bf16 h128 worst", w)


def test_opt13b_width_two_layers():
    """Layer-sliced big-shape parity: full OPT-13B width (d 5120, 40 heads, FFN 20480, vocab 50272), 2 layers,
    a few short sequences the oracle can finish."""
    shape = wl.opt13b_shape(2)
    w = run_decoder_only(shape, 7, [40, 7, 65], 2, BF16_TOL, real="float")
    print("opt13b-width worst", w)


def test_gpt3_share_hidden_in_hidden_out():
    shape = wl.gpt3_175b_share_shape(1).replace(d_model=1024, n_heads=8, d_ff=2048, name="g175_narrow")
    m, o, _ = make_pair(shape, 8, "double")
    lens = [9, 140]
    T = sum(lens)
    x = wl.random_hidden(81, T, shape.d_model, shape.dtype)
    out = torch.zeros((T, shape.d_model), dtype=tdtype(shape), device=DEV)
    m.encode([0, 1], lens, None, reserve_lengths=[32, 160], hidden_in=x.to(DEV), want_tokens=False, out_device=out)
    got = out.float().cpu().numpy()
    xs = x.float().numpy()
    _, r0 = o.encode(0, hidden_in=xs[:9])
    _, r1 = o.encode(1, hidden_in=xs[9:])
    assert row_relerr(got[:9], r0) < BF16_TOL and row_relerr(got[9:], r1) < BF16_TOL
    x2 = wl.random_hidden(82, 2, shape.d_model, shape.dtype)
    out2 = torch.zeros((2, shape.d_model), dtype=tdtype(shape), device=DEV)
    m.decode_step([1, 0], None, [141, 10], hidden_in=x2.to(DEV), want_tokens=False, out_device=out2)
    _, d1 = o.decode(1, hidden_in=x2.float().numpy()[0])
    _, d0 = o.decode(0, hidden_in=x2.float().numpy()[1])
    g2 = out2.float().cpu().numpy()
    assert row_relerr(g2[0][None], d1[None]) < BF16_TOL and row_relerr(g2[1][None], d0[None]) < BF16_TOL
    m.close()


def test_gpt3_share_full_width_one_layer():
    """configs[3] at its own width (paper Table 1: GPT-3 175B, hidden 12288, 96 heads; FFN 49152, GELU), one of the
    share's 12 layers, hidden states in and out: 20 input tokens in two sequences, then two decode steps, against
    the float oracle.  Every projection runs at K = 12288 / 49152 and N = 36864 / 12288 / 49152."""
    if torch.cuda.get_device_properties(0).total_memory < 64e9:
        pytest.skip("needs 64 GB of device memory")
    shape = wl.gpt3_175b_share_shape(1)
    assert (shape.d_model, shape.n_heads, shape.head_dim, shape.d_ff) == (12288, 96, 128, 49152)
    m, o, _ = make_pair(shape, 8, "float", pool_tokens=256, max_seqs=4, max_batch_tokens=64, max_batch_seqs=4, gen_device=DEV)
    lens = [7, 13]
    T = sum(lens)
    x = wl.random_hidden(83, T, shape.d_model, shape.dtype)
    out = torch.zeros((T, shape.d_model), dtype=tdtype(shape), device=DEV)
    print("encode gpt3 share, full width", flush=True)
    m.encode([0, 1], lens, None, reserve_lengths=[16, 24], hidden_in=x.to(DEV), want_tokens=False, out_device=out)
    got = out.float().cpu().numpy()
    xs = x.float().numpy()
    _, r0 = o.encode(0, hidden_in=xs[:7])
    _, r1 = o.encode(1, hidden_in=xs[7:])
    worst = max(row_relerr(got[:7], r0), row_relerr(got[7:], r1))
    assert worst < BF16_TOL, worst
    for step in (1, 2):
        x2 = wl.random_hidden(83 + step, 2, shape.d_model, shape.dtype)
        out2 = torch.zeros((2, shape.d_model), dtype=tdtype(shape), device=DEV)
        m.decode_step([1, 0], None, [13 + step, 7 + step], hidden_in=x2.to(DEV), want_tokens=False, out_device=out2)
        _, d1 = o.decode(1, hidden_in=x2.float().numpy()[0])
        _, d0 = o.decode(0, hidden_in=x2.float().numpy()[1])
        g2 = out2.float().cpu().numpy()
        worst = max(worst, row_relerr(g2[0][None], d1[None]), row_relerr(g2[1][None], d0[None]))
        assert worst < BF16_TOL, (step, worst)
    print("gpt3 share full width worst", worst, flush=True)
    m.close()


def run_t5(shape, seed, in_lens, n_steps, tol, real="double"):
    n = len(in_lens)
    m, o, _ = make_pair(shape, seed, real, max_batch_tokens=max(4096, int(sum(in_lens))))
    rng = np.random.default_rng(seed)
    toks = wl.random_tokens(rng, int(sum(in_lens)), shape.vocab)
    off = np.concatenate([[0], np.cumsum(in_lens)])
    ids = np.arange(n) + 1
    enc = torch.zeros((int(sum(in_lens)), shape.d_model), dtype=tdtype(shape), device=DEV)
    m.encode(ids, in_lens, toks, reserve_lengths=[n_steps] * n, want_tokens=False, out_device=enc)
    g = enc.float().cpu().numpy()
    worst = 0.0
    for i in range(n):
        _, ref = o.encode(int(ids[i]), toks[off[i]:off[i + 1]])
        worst = max(worst, row_relerr(g[off[i]:off[i + 1]], ref))
    assert worst < tol, ("encoder output", worst)
    cur = np.zeros(n, dtype=np.int32)                      # start token
    for step in range(1, n_steps + 1):
        lg = torch.zeros((n, shape.vocab), dtype=torch.float32, device=DEV)
        m.decode_step(ids, cur, [step] * n, out_device=lg)
        got = lg.cpu().numpy()
        for i in range(n):
            t, ref = o.decode(int(ids[i]), int(cur[i]))
            worst = max(worst, row_relerr(got[i][None], ref[None]))
            cur[i] = t
        assert worst < tol, (step, worst)
    m.close()
    return worst


@pytest.mark.parametrize("xbias", [1, 0])
def test_t5_small_f32(xbias):
    w = run_t5(wl.small_t5_shape(wl.DTYPE_F32).replace(cross_rel_bias=xbias), 9, [33, 150, 8], 20, F32_TOL)
    print("t5 f32 worst", w)


def test_t5_small_bf16_head128():
    shape = wl.small_t5_shape(wl.DTYPE_BF16).replace(head_dim=128, n_heads=4, name="t5_small_h128")
    w = run_t5(shape, 10, [129, 40, 260], 5, BF16_TOL)
    print("t5 bf16 worst", w)


def test_t5_11b_width_one_layer_each():
    """Full T5-11B width (d 1024, 128 heads of 128, FFN 65536, vocab 32128), 1 encoder + 1 decoder layer."""
    w = run_t5(wl.t5_11b_shape(1, 1), 11, [20, 45], 2, BF16_TOL, real="float")
    print("t5-11b width worst", w)


def test_batch_composition_and_order_do_not_change_results():
    """A sequence's logits are bit-identical on the HIP path whatever its batch-mates, their order, or when
    they were encoded or released (float config: fixed reduction orders everywhere)."""
    shape = wl.tiny_shape()
    job = wl.workload_tiny()
    m, _, _ = make_pair(shape, 3, "float")
    V = shape.vocab
    la = torch.zeros((1, V), dtype=torch.float32, device=DEV)
    t = m.encode([0], [job.in_len[2]], job.seq_tokens(2), out_device=la)
    alone = [la.cpu().numpy()[0].copy()]
    for s in range(1, 5):
        t = m.decode_step([0], t, [job.in_len[2] + s], out_device=la)
        alone.append(la.cpu().numpy()[0].copy())
    m.seq_release([0])
    lb = torch.zeros((4, V), dtype=torch.float32, device=DEV)
    order = [3, 2, 0, 1]
    toks = np.concatenate([job.seq_tokens(i) for i in order])
    t4 = m.encode([10, 11, 12, 13], job.in_len[order], toks, out_device=lb)
    mixed = [lb.cpu().numpy()[1].copy()]
    live = [10, 11, 12, 13]
    cur = dict(zip(live, t4))
    for s in range(1, 5):
        if s == 2:
            m.seq_release([10]); live.remove(10)
        if s == 3:
            cur[20] = m.encode([20], [job.in_len[0]], job.seq_tokens(0))[0]
            live.insert(0, 20)
        kv = [m.seq_length(i) + 1 for i in live]
        out = torch.zeros((len(live), V), dtype=torch.float32, device=DEV)
        nt = m.decode_step(live, [cur[i] for i in live], kv, out_device=out)
        for i, tk in zip(live, nt):
            cur[i] = tk
        mixed.append(out.cpu().numpy()[live.index(11)].copy())
    for a, b in zip(alone, mixed):
        assert np.array_equal(a, b)
    m.close()


def test_abi_errors_leave_state_unchanged():
    shape = wl.tiny_shape()
    m, _, _ = make_pair(shape, 4, "float", pool_tokens=100, max_seqs=8, max_batch_tokens=128, max_batch_seqs=4)
    E = exe.ExeError

    def code(fn):
        with pytest.raises(E) as e:
            fn()
        return e.value.code

    toks = np.arange(40) % shape.vocab
    assert code(lambda: m.encode([0, 0], [5, 5], toks[:10])) == -4                 # duplicate id
    assert code(lambda: m.encode([9], [5], toks[:5])) == -4                        # id out of range
    assert code(lambda: m.encode([0], [0], toks[:0])) == -5                        # empty input
    assert code(lambda: m.encode([0], [65], np.zeros(65, np.int32))) == -5         # beyond the position table
    assert code(lambda: m.encode([0], [5], np.array([1, 2, 3, 4, shape.vocab]))) == -1
    assert code(lambda: m.encode([0, 1, 2, 3, 4], [1] * 5, toks[:5])) == -1        # more than max_batch_seqs
    assert code(lambda: m.encode([0, 1], [64, 64], np.zeros(128, np.int32), reserve_lengths=[64, 64])) == -3
    assert m.kv_stats()["used_bytes"] == 0 and m.kv_stats()["live_seqs"] == 0      # nothing was admitted
    t = m.encode([0, 1], [10, 20], toks[:30], reserve_lengths=[12, 40])
    used = m.kv_stats()["used_bytes"]
    assert code(lambda: m.encode([1], [5], toks[:5])) == -4                        # still live
    assert code(lambda: m.decode_step([0, 1], t, [11, 22])) == -5                  # wrong kv length
    assert code(lambda: m.decode_step([0, 5], t, [11, 1])) == -4                   # not live
    assert code(lambda: m.decode_step([0, 0], t, [11, 11])) == -4
    assert m.seq_length(0) == 10 and m.seq_length(1) == 20
    t = m.decode_step([0, 1], t, [11, 21])
    for s in range(12, 17):
        t = m.decode_step([0, 1], t, [s, s + 10])
    assert code(lambda: m.decode_step([0, 1], t, [17, 27])) == -3                  # seq 0 reserved 12, rounded to 16
    assert m.seq_length(0) == 16 and m.seq_length(1) == 26
    m.seq_release([0])
    assert code(lambda: m.seq_release([0])) == -4                                  # double release
    assert code(lambda: m.seq_length(0)) == -4
    assert m.kv_stats()["used_bytes"] < used and m.kv_stats()["live_seqs"] == 1
    m.seq_release([1])
    st = m.kv_stats()
    assert st["used_bytes"] == 0 and st["largest_free_bytes"] == st["pool_bytes"]  # extents coalesce
    m.close()
