"""A seeded random serving trace through the C ABI against the oracle (Section 4: sequences enter in encoding batches,
leave the decoding batch one by one, and the batch is refilled): sequences are admitted in batches, advanced in
arbitrary subsets so that their positions drift apart, moved to a new id through host memory, re-reserved, compacted
and released, on an extent pool and on paged pools small enough that space has to be reclaimed.  Sequences are
independent, so whatever the interleaving every logits row must equal the oracle's row for that sequence and position,
a refused call must leave the state as it was, and the library's own counts must agree with the trace's."""
import numpy as np
import pytest
import torch

import paper_2404_07947_amd as exe
import workload as wl
from gpu_util import DEV, kv_bytes_per_token, make_pair, row_relerr, tdtype

pytestmark = pytest.mark.gpu
F32_TOL = 1e-4             # float model: float accumulation order only
BF16_TOL = 2e-2            # bf16 model: the stated bar, max-norm relative error per logits row
OOM = -3


class Trace:
    def __init__(self, seed, kv_block_size, pool_tokens, n_ops, bf16=False, encdec=False):
        self.shape = wl.tiny_shape()
        self.max_in, self.max_more, self.tol = 24, 24, F32_TOL
        self.encdec = encdec
        if encdec:             # encoder-decoder: the input's cross-attention entries and the output's own, both in extents
            self.shape = wl.small_t5_shape(wl.DTYPE_F32)
            self.max_in, self.max_more = 60, 16
        if bf16:               # 3 layers, heads of 64, MFMA GEMMs, inputs long enough for several key tiles
            self.shape = self.shape.replace(name="small_bf16", dtype=wl.DTYPE_BF16, max_pos=512, n_layers=3)
            self.max_in, self.max_more, self.tol = 150, 40, BF16_TOL
        self.paged = kv_block_size > 0
        self.m, self.o, _ = make_pair(self.shape, wl.BASE_SEED + 7, "double", pool_tokens=pool_tokens, max_seqs=64,
                                      max_batch_tokens=512, max_batch_seqs=16, kv_block_size=kv_block_size)
        self.rng = np.random.default_rng(seed)
        self.live = {}                     # library id -> dict(oid, len, cur, reserve, n_in); len = K/V rows of the decoder
        self.next_oid = 0
        self.free_oids = []
        self.worst = 0.0
        self.counts = {"admit": 0, "step": 0, "release": 0, "reserve": 0, "compact": 0, "move": 0, "refused": 0}
        self.n_ops = n_ops

    # ---- helpers
    def free_id(self):
        ids = [i for i in range(64) if i not in self.live]
        return int(self.rng.choice(ids))

    def take_oid(self):
        if self.free_oids:
            return self.free_oids.pop()
        self.next_oid += 1
        assert self.next_oid <= 64
        return self.next_oid - 1

    def drop(self, i):
        s = self.live.pop(i)
        self.o.release(s["oid"])
        self.free_oids.append(s["oid"])

    def evict_one(self):
        i = int(self.rng.choice(sorted(self.live)))
        self.m.seq_release([i])
        self.drop(i)
        self.counts["release"] += 1

    def check_rows(self, got, refs, what):
        for g, r in zip(got, refs):
            self.worst = max(self.worst, row_relerr(g[None], r[None]))
        assert self.worst < self.tol, (what, self.worst)

    # ---- operations
    def admit(self):
        k = int(self.rng.integers(1, 4))
        ids = []
        while len(ids) < k:
            i = self.free_id()
            if i not in ids:
                ids.append(i)
        lens = self.rng.integers(1, self.max_in + 1, size=k)
        more = self.rng.integers(1, self.max_more + 1, size=k)
        reserve = more if self.encdec else np.minimum(self.shape.max_pos, lens + more)
        toks = wl.random_tokens(self.rng, int(lens.sum()), self.shape.vocab)
        if self.encdec:                    # the call returns the encoder's output rows
            logits = torch.zeros((int(lens.sum()), self.shape.d_model), dtype=tdtype(self.shape), device=DEV)
        else:
            logits = torch.zeros((k, self.shape.vocab), dtype=torch.float32, device=DEV)
        for attempt in range(4):
            before = self.m.kv_stats()
            try:
                self.m.encode(ids, lens, toks, reserve_lengths=None if self.paged else reserve,
                              want_tokens=not self.encdec, out_device=logits)
                break
            except exe.ExeError as e:
                assert e.code == OOM, e
                assert self.m.kv_stats() == before                      # nothing was admitted
                self.counts["refused"] += 1
                if attempt == 0 and not self.paged:
                    self.m.kv_compact()
                elif self.live:
                    self.evict_one()
                else:
                    raise
        else:
            return
        got = logits.float().cpu().numpy()
        off = np.concatenate([[0], np.cumsum(lens)])
        refs = []
        for j, i in enumerate(ids):
            oid = self.take_oid()
            t, lg = self.o.encode(oid, toks[off[j]:off[j + 1]])
            refs.append(lg)
            self.live[i] = {"oid": oid, "len": 0 if self.encdec else int(lens[j]), "cur": 0 if self.encdec else int(t),
                            "reserve": int(reserve[j]), "n_in": int(lens[j])}
        if self.encdec:
            got, refs = [got[off[j]:off[j + 1]] for j in range(k)], refs
            for g, r in zip(got, refs):
                self.worst = max(self.worst, row_relerr(g, r))
            assert self.worst < self.tol, ("encoder output", self.worst)
        else:
            self.check_rows(got, refs, "admit")
        self.counts["admit"] += 1

    def step(self):
        limit = lambda s: self.shape.max_pos if self.paged else s["reserve"]       # encoder-decoder: output rows only
        able = [i for i, s in sorted(self.live.items()) if s["len"] + 1 <= limit(s)]
        if not able:
            return
        k = int(self.rng.integers(1, min(len(able), 16) + 1))
        ids = [int(x) for x in self.rng.choice(able, size=k, replace=False)]
        logits = torch.zeros((k, self.shape.vocab), dtype=torch.float32, device=DEV)
        while True:
            try:
                self.m.decode_step(ids, [self.live[i]["cur"] for i in ids], [self.live[i]["len"] + 1 for i in ids],
                                   out_device=logits)
                break
            except exe.ExeError as e:                                    # paged pool: no block left for a sequence
                assert e.code == OOM and self.paged, e
                self.counts["refused"] += 1
                for i in ids:
                    assert self.m.seq_length(i) == self.live[i]["len"]   # the refused step advanced nobody
                gone = ids.pop()
                self.m.seq_release([gone])
                self.drop(gone)
                if not ids:
                    return
                logits = logits[:len(ids)]
        got = logits.cpu().numpy()
        refs = []
        for i in ids:
            s = self.live[i]
            t, lg = self.o.decode(s["oid"], s["cur"])
            refs.append(lg)
            s["len"] += 1
            s["cur"] = int(t)
        self.check_rows(got, refs, "step")
        self.counts["step"] += 1

    def release(self):
        if self.live:
            self.evict_one()

    def reserve(self):
        if self.paged or not self.live:
            return
        i = int(self.rng.choice(sorted(self.live)))
        s = self.live[i]
        top = s["len"] + 2 * self.max_more
        want = int(self.rng.integers(max(s["len"], 1), (top if self.encdec else min(self.shape.max_pos, top)) + 1))
        try:
            self.m.seq_reserve(i, want)
            s["reserve"] = want
            self.counts["reserve"] += 1
        except exe.ExeError as e:
            assert e.code == OOM, e
            self.counts["refused"] += 1

    def compact(self):
        if self.paged:
            return
        used = self.m.kv_stats()["used_bytes"]
        self.m.kv_compact()
        st = self.m.kv_stats()
        assert st["used_bytes"] == used and st["largest_free_bytes"] == st["pool_bytes"] - used
        self.counts["compact"] += 1

    def move(self):
        """Export, release, import under another id: the sequence goes on where it stopped."""
        if not self.live:
            return
        i = int(self.rng.choice(sorted(self.live)))
        s = self.live[i]
        buf, st = self.m.seq_export(i)
        assert st == {"kv_len": s["len"], "cross_len": s["n_in"] if self.encdec else 0}
        assert buf.nbytes == kv_bytes_per_token(self.shape) * (s["len"] + (s["n_in"] if self.encdec else 0))
        self.m.seq_release([i])
        del self.live[i]
        j = self.free_id()
        self.m.seq_import(j, buf, st, reserve_length=0 if self.paged else s["reserve"])      # the space was just freed
        self.live[j] = s
        self.counts["move"] += 1

    def audit(self):
        st = self.m.kv_stats()
        assert st["live_seqs"] == len(self.live)
        for i, s in self.live.items():
            assert self.m.seq_length(i) == s["len"]
        if not self.paged:
            per_token = kv_bytes_per_token(self.shape)
            assert st["used_bytes"] >= per_token * sum(s["len"] + (s["n_in"] if self.encdec else 0) for s in self.live.values())

    def run(self):
        ops = [self.admit, self.step, self.release, self.reserve, self.compact, self.move]
        p = np.array([0.22, 0.50, 0.08, 0.07, 0.05, 0.08])
        for n in range(self.n_ops):
            op = ops[int(self.rng.choice(len(ops), p=p))]
            print(f"op {n}: {op.__name__}, {len(self.live)} live", flush=True)
            op()
            if n % 8 == 7:
                self.audit()
        self.audit()
        if self.live:
            self.m.seq_release(sorted(self.live))
        st = self.m.kv_stats()
        assert st["live_seqs"] == 0 and st["used_bytes"] == 0
        self.m.close()
        return self.counts


@pytest.mark.parametrize("seed,kv_block_size,pool_tokens,bf16", [
    (101, 0, 200, False), (102, 0, 320, False), (103, 8, 160, False), (104, 16, 256, False),
    (105, 0, 1000, True), (106, 8, 800, True), (107, 64, 1536, True)])
def test_random_serving_trace(seed, kv_block_size, pool_tokens, bf16):
    counts = Trace(seed, kv_block_size, pool_tokens, n_ops=90, bf16=bf16).run()
    print("trace", seed, counts, flush=True)
    assert counts["admit"] >= 5 and counts["step"] >= 20 and counts["move"] >= 1
    assert counts["refused"] >= 1                    # the pool was small enough to run out


@pytest.mark.parametrize("seed,pool_tokens", [(201, 260), (202, 400)])
def test_random_serving_trace_encoder_decoder(seed, pool_tokens):
    counts = Trace(seed, 0, pool_tokens, n_ops=90, encdec=True).run()
    print("trace", seed, counts, flush=True)
    assert counts["admit"] >= 5 and counts["step"] >= 20 and counts["move"] >= 1 and counts["refused"] >= 1
