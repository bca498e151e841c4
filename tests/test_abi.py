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
