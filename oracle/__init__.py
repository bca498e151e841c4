"""ctypes binding of the CPU oracle (oracle/exe_oracle.c).

TEST INFRASTRUCTURE: imported only by tests, by the smoke check and by the benchmark's cpu_baseline
leg.  It imports nothing from the GPU package.  `build()` compiles the C file twice (REAL=float and
REAL=double) with gcc; `Oracle(shape, weights, real="double")` wraps one model.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_BUILD = os.path.join(_HERE, "_build")
_SRC = os.path.join(_HERE, "exe_oracle.c")
_HDR = os.path.join(_HERE, "exe_oracle.h")
_libs = {}


def lib_path(real: str) -> str:
    return os.path.join(_BUILD, f"liboracle_{real}.so")


def build(force: bool = False) -> None:
    """Compile the oracle for both arithmetic types.  Rebuilds when a source is newer than the library."""
    os.makedirs(_BUILD, exist_ok=True)
    for real in ("float", "double"):
        out = lib_path(real)
        if (not force and os.path.exists(out)
                and os.path.getmtime(out) >= max(os.path.getmtime(_SRC), os.path.getmtime(_HDR))):
            continue
        cmd = ["gcc", "-O3", "-mavx2", "-mfma", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall",
               f"-DREAL={real}", "-o", out + ".tmp", _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(out + ".tmp", out)


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("arch", "n_layers", "n_dec_layers", "d_model", "n_heads", "head_dim", "d_ff", "vocab",
                 "max_pos", "act", "norm", "pos", "rel_buckets", "rel_max_dist", "cross_rel_bias",
                 "has_embed", "has_lm_head", "scale_mode")] + [("norm_eps", C.c_float)]


def _load(real: str):
    if real in _libs:
        return _libs[real]
    build()
    lib = C.CDLL(lib_path(real))
    rp = C.c_void_p
    lib.orc_linear.argtypes = [rp, C.c_int, C.c_int, rp, rp, C.c_int, rp]
    lib.orc_linear.restype = None
    rt = C.c_float if real == "float" else C.c_double
    lib.orc_layernorm.argtypes = [rp, C.c_int, C.c_int, rp, rp, rt, rp]
    lib.orc_layernorm.restype = None
    lib.orc_rmsnorm.argtypes = [rp, C.c_int, C.c_int, rp, rt, rp]
    lib.orc_rmsnorm.restype = None
    lib.orc_act.argtypes = [rp, C.c_int64, C.c_int]
    lib.orc_act.restype = None
    lib.orc_attention_row.argtypes = [rp, rp, C.c_int64, rp, C.c_int64, C.c_int, C.c_int, rt, rp, rp, rp]
    lib.orc_attention_row.restype = rt
    lib.orc_argmax.argtypes = [rp, C.c_int]
    lib.orc_argmax.restype = C.c_int
    lib.orc_bucket.argtypes = [C.c_int] * 4
    lib.orc_bucket.restype = C.c_int
    lib.orc_create.argtypes = [C.POINTER(_Config), C.POINTER(C.c_void_p), C.c_int, C.c_int]
    lib.orc_create.restype = C.c_void_p
    lib.orc_free.argtypes = [C.c_void_p]
    lib.orc_free.restype = None
    lib.orc_expected_weights.argtypes = [C.POINTER(_Config)]
    lib.orc_expected_weights.restype = C.c_int
    lib.orc_threads.restype = C.c_int
    lib.orc_real_bytes.restype = C.c_int
    lib.orc_encode.argtypes = [C.c_void_p, C.c_int, C.c_int, rp, rp, rp, rp]
    lib.orc_encode.restype = C.c_int
    lib.orc_decode.argtypes = [C.c_void_p, C.c_int, C.c_int32, rp, rp, rp]
    lib.orc_decode.restype = C.c_int
    lib.orc_release.argtypes = [C.c_void_p, C.c_int]
    lib.orc_release.restype = None
    lib.orc_seq_len.argtypes = [C.c_void_p, C.c_int]
    lib.orc_seq_len.restype = C.c_int
    lib.orc_full.argtypes = [C.c_void_p, C.c_int, rp, rp, C.c_int, rp, rp, rp]
    lib.orc_full.restype = C.c_int
    lib.orc_rowsum_dev.argtypes = [C.c_void_p, C.c_int]
    lib.orc_rowsum_dev.restype = rt
    assert lib.orc_real_bytes() == (4 if real == "float" else 8)
    _libs[real] = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Primitives:
    """The oracle's primitive operations on numpy arrays (for pinning tests)."""

    def __init__(self, real: str = "double"):
        self.real = real
        self.dt = np.float32 if real == "float" else np.float64
        self.lib = _load(real)

    def _r(self, a):
        return np.ascontiguousarray(a, dtype=self.dt)

    @staticmethod
    def _f(a):
        return None if a is None else np.ascontiguousarray(a, dtype=np.float32)

    def linear(self, x, W, b=None):
        x = self._r(x); W = self._f(W); b = self._f(b)
        rows, k = x.shape
        y = np.empty((rows, W.shape[0]), dtype=self.dt)
        self.lib.orc_linear(_ptr(x), rows, k, _ptr(W), _ptr(b), W.shape[0], _ptr(y))
        return y

    def layernorm(self, x, g, b, eps):
        x = self._r(x); g = self._f(g); b = self._f(b)
        y = np.empty_like(x)
        self.lib.orc_layernorm(_ptr(x), x.shape[0], x.shape[1], _ptr(g), _ptr(b), eps, _ptr(y))
        return y

    def rmsnorm(self, x, g, eps):
        x = self._r(x); g = self._f(g)
        y = np.empty_like(x)
        self.lib.orc_rmsnorm(_ptr(x), x.shape[0], x.shape[1], _ptr(g), eps, _ptr(y))
        return y

    def act(self, x, kind):
        y = self._r(x).copy()
        self.lib.orc_act(_ptr(y), y.size, kind)
        return y

    def attention_row(self, q, K, V, scale, bias=None):
        """q [dh], K [nk, dh], V [nk, dh] -> (out [dh], probs [nk], sum of probs)"""
        q = self._r(q); K = self._r(K); V = self._r(V)
        bias = None if bias is None else self._r(bias)
        nk, dh = K.shape
        out = np.empty(dh, dtype=self.dt)
        probs = np.empty(nk, dtype=self.dt)
        ps = self.lib.orc_attention_row(_ptr(q), _ptr(K), dh, _ptr(V), dh, nk, dh, scale, _ptr(bias),
                                        _ptr(out), _ptr(probs))
        return out, probs, ps

    def argmax(self, x):
        x = self._r(x)
        return int(self.lib.orc_argmax(_ptr(x), x.size))

    def bucket(self, rel, bidirectional, n_buckets=32, max_dist=128):
        return int(self.lib.orc_bucket(int(rel), int(bidirectional), n_buckets, max_dist))


def _weights_to_f32(weights) -> List[np.ndarray]:
    out = []
    for w in weights:
        if hasattr(w, "detach"):
            w = w.detach().to("cpu").float().numpy()
        out.append(np.ascontiguousarray(w, dtype=np.float32))
    return out


class Oracle:
    """One oracle model.  `shape` is any object with the ModelShape fields; `weights` is the list of
    tensors/arrays in the documented order (their stored values are upcast to float, nothing else)."""

    def __init__(self, shape, weights: Sequence, real: str = "double", max_seqs: int = 4096):
        self.real = real
        self.dt = np.float32 if real == "float" else np.float64
        self.lib = _load(real)
        self.shape = shape
        self.cfg = _Config(shape.arch, shape.n_layers, shape.n_dec_layers, shape.d_model, shape.n_heads,
                           shape.head_dim, shape.d_ff, shape.vocab, shape.max_pos, shape.act, shape.norm,
                           shape.pos, shape.rel_buckets, shape.rel_max_dist, shape.cross_rel_bias,
                           shape.has_embed, shape.has_lm_head, shape.scale_mode, shape.norm_eps)
        self._w = _weights_to_f32(weights)
        arr = (C.c_void_p * len(self._w))(*[w.ctypes.data for w in self._w])
        self._m = self.lib.orc_create(C.byref(self.cfg), arr, len(self._w), max_seqs)
        if not self._m:
            raise ValueError(f"orc_create failed: got {len(self._w)} weights, expected "
                             f"{self.lib.orc_expected_weights(C.byref(self.cfg))}")

    def close(self):
        if self._m:
            self.lib.orc_free(self._m)
            self._m = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def threads(self) -> int:
        return int(self.lib.orc_threads())

    def encode(self, seq: int, tokens=None, hidden_in=None):
        """Returns (next_token, logits_last or hidden_out).  enc-dec: (0, encoder output [n, d])."""
        s = self.shape
        if tokens is not None:
            tokens = np.ascontiguousarray(tokens, dtype=np.int32)
            n = tokens.shape[0]
        else:
            hidden_in = np.ascontiguousarray(hidden_in, dtype=self.dt)
            n = hidden_in.shape[0]
        logits = hidden = None
        if s.arch == 0 and s.has_lm_head:
            logits = np.empty(s.vocab, dtype=self.dt)
        else:
            hidden = np.empty((n, s.d_model), dtype=self.dt)
        r = self.lib.orc_encode(self._m, seq, n, _ptr(tokens), _ptr(hidden_in), _ptr(logits), _ptr(hidden))
        if r < 0:
            raise ValueError("orc_encode: bad argument")
        return r, (logits if logits is not None else hidden)

    def decode(self, seq: int, token: int = 0, hidden_in=None):
        s = self.shape
        if hidden_in is not None:
            hidden_in = np.ascontiguousarray(hidden_in, dtype=self.dt)
        logits = hidden = None
        if s.has_lm_head:
            logits = np.empty(s.vocab, dtype=self.dt)
        else:
            hidden = np.empty(s.d_model, dtype=self.dt)
        r = self.lib.orc_decode(self._m, seq, int(token), _ptr(hidden_in), _ptr(logits), _ptr(hidden))
        if r < 0:
            raise ValueError("orc_decode: bad argument")
        return r, (logits if logits is not None else hidden)

    def release(self, seq: int):
        self.lib.orc_release(self._m, seq)

    def seq_len(self, seq: int) -> int:
        return int(self.lib.orc_seq_len(self._m, seq))

    def full(self, tokens=None, hidden_in=None, dec_tokens=None):
        """Cache-free recomputation.  decoder-only: logits (or hidden) for all positions.
        enc-dec: (logits [n_dec, V], encoder output [n, d])."""
        s = self.shape
        if tokens is not None:
            tokens = np.ascontiguousarray(tokens, dtype=np.int32)
            n = tokens.shape[0]
        else:
            hidden_in = np.ascontiguousarray(hidden_in, dtype=self.dt)
            n = hidden_in.shape[0]
        if s.arch == 0:
            logits = np.empty((n, s.vocab), dtype=self.dt) if s.has_lm_head else None
            hidden = np.empty((n, s.d_model), dtype=self.dt)
            r = self.lib.orc_full(self._m, n, _ptr(tokens), _ptr(hidden_in), 0, None, _ptr(logits), _ptr(hidden))
            if r < 0:
                raise ValueError("orc_full: bad argument")
            return logits if logits is not None else hidden
        dec_tokens = np.ascontiguousarray(dec_tokens, dtype=np.int32)
        logits = np.empty((dec_tokens.shape[0], s.vocab), dtype=self.dt)
        hidden = np.empty((n, s.d_model), dtype=self.dt)
        r = self.lib.orc_full(self._m, n, _ptr(tokens), None, dec_tokens.shape[0], _ptr(dec_tokens),
                              _ptr(logits), _ptr(hidden))
        if r < 0:
            raise ValueError("orc_full: bad argument")
        return logits, hidden

    def rowsum_dev(self, reset: bool = True) -> float:
        return float(self.lib.orc_rowsum_dev(self._m, int(reset)))
