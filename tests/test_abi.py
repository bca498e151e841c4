"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every symbol the header
declares, and its host-only functions agree with the oracle / the workload module."""
import ctypes as C
import os
import re

import pytest

import oracle
import paper_2404_07947_amd as exe
import workload as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not h.endswith(".h"):
            continue
        src = open(os.path.join(ROOT, "include", h)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(exe_[a-z0-9_]+)\s*\(", src))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = exe.lib()
    names = header_functions()
    assert len(names) >= 18
    for n in names:
        assert hasattr(L, n), n
    assert sorted(exe.DECLARED_SYMBOLS) == names          # the binding covers the whole header
    assert "gfx950" in exe.exe_version()


def test_rel_bucket_matches_oracle_everywhere():
    P = oracle.Primitives("double")
    for bid in (0, 1):
        for rel in range(-1500, 1501):
            assert exe.exe_rel_bucket(rel, bid, 32, 128) == P.bucket(rel, bid, 32, 128)
    # other parameters as well
    for rel in range(-300, 301):
        assert exe.exe_rel_bucket(rel, 1, 16, 64) == P.bucket(rel, 1, 16, 64)
        assert exe.exe_rel_bucket(rel, 0, 8, 20) == P.bucket(rel, 0, 8, 20)


@pytest.mark.parametrize("shape", [wl.tiny_shape(), wl.opt13b_shape(), wl.t5_11b_shape(), wl.gpt3_175b_share_shape(),
                                   wl.small_t5_shape(), wl.t5_11b_shape().replace(cross_rel_bias=0)])
def test_expected_weight_count_matches_workload_and_oracle(shape):
    cfg = exe.config_from_shape(shape, 1 << 20, 4, 64, 4)
    n = exe.Model.expected_weights(cfg)
    assert n == len(wl.weight_specs(shape))
    ocfg = oracle._Config(shape.arch, shape.n_layers, shape.n_dec_layers, shape.d_model, shape.n_heads,
                          shape.head_dim, shape.d_ff, shape.vocab, shape.max_pos, shape.act, shape.norm, shape.pos,
                          shape.rel_buckets, shape.rel_max_dist, shape.cross_rel_bias, shape.has_embed,
                          shape.has_lm_head, shape.scale_mode, shape.norm_eps)
    assert oracle._load("double").orc_expected_weights(C.byref(ocfg)) == n


def test_config_errors_are_reported_not_raised_as_crashes():
    good = wl.tiny_shape()
    for bad, code in [(good.replace(head_dim=48), -2), (good.replace(arch=7), -1), (good.replace(d_model=260), -2),
                      (good.replace(act=5), -1), (good.replace(norm=wl.NORM_RMSNORM), -2),
                      (wl.small_t5_shape().replace(rel_buckets=30), -2), (wl.small_t5_shape().replace(n_dec_layers=0), -1)]:
        cfg = exe.config_from_shape(bad, 1 << 20, 4, 64, 4)
        with pytest.raises(exe.ExeError) as e:
            exe.Model.expected_weights(cfg)
        assert e.value.code == code, (bad, str(e.value))
    L = exe.lib()
    assert L.exe_expected_weights(None) == -1
    assert L.exe_model_free(None) == -1
    assert L.exe_seq_release(None, 0, None) == -1
    assert b"null" in L.exe_last_error()


def test_prefill_tile_list_covers_every_query_tile_once_in_launch_order():
    """Host logic of the MFMA prefill launch: every 128-row query tile of every sequence appears exactly once; sequences
    go longest first (ties in the given order), a sequence's tiles together, last rows first."""
    import numpy as np
    rng = np.random.default_rng(5)
    batches = [[1], [128], [129], [1024, 1024, 1024], [64, 1024, 300, 300, 1, 127, 128, 129, 2048]]
    batches += [list(rng.integers(1, 1100, size=int(rng.integers(1, 40)))) for _ in range(20)]
    for lens in batches:
        t = exe.exe_op_prefill_tiles(lens)
        want = {(i, q0) for i, n in enumerate(lens) for q0 in range(0, int(n), 128)}
        got = [tuple(int(v) for v in p) for p in t]
        assert len(got) == len(want) and set(got) == want, lens
        seqs = [i for i, _ in got]
        order = [s for k, s in enumerate(seqs) if k == 0 or seqs[k - 1] != s]
        assert len(order) == len(lens), ("a sequence's tiles are not together", lens)
        assert order == sorted(range(len(lens)), key=lambda i: -int(lens[i])), lens      # stable: ties keep their order
        for i in range(len(lens)):
            q = [q0 for s, q0 in got if s == i]
            assert q == sorted(q, reverse=True)
    with pytest.raises(exe.ExeError) as e:
        exe.exe_op_prefill_tiles([5, 0, 7])
    assert e.value.code == -5
    import ctypes
    n = ctypes.c_int32()
    lens = (ctypes.c_int32 * 2)(300, 5)
    assert exe.lib().exe_op_prefill_tiles(2, lens, None, 0, ctypes.byref(n)) == -1 and n.value == 4
