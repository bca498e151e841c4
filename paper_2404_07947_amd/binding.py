"""ctypes marshalling for include/exe.h.  No arithmetic of the method lives here."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None

DECLARED_SYMBOLS = [
    "exe_expected_weights", "exe_model_load", "exe_model_free", "exe_encode", "exe_decode_step",
    "exe_seq_release", "exe_seq_length", "exe_kv_stats", "exe_seq_export_bytes", "exe_seq_export", "exe_seq_import", "exe_seq_reserve", "exe_kv_compact", "exe_profile", "exe_run_rra", "exe_kernel_timing",
    "exe_kernel_times", "exe_op_gemm", "exe_op_gemm_workspace", "exe_op_gemm_plan", "exe_op_gemm_ld", "exe_op_gemm_noalloc", "exe_op_gemm_noalloc_max_workspace", "exe_op_paged_index_check", "exe_op_norm", "exe_op_prefill_attention", "exe_op_prefill_tiles",
    "exe_op_decode_attention", "exe_op_decode_attention_paged", "exe_probe_peaks", "exe_probe_ingest", "exe_op_argmax", "exe_rel_bucket", "exe_last_error", "exe_version",
    # exe_sched.h (host only)
    "exe_sim_completion", "exe_sim_step_ms", "exe_sim_rra", "exe_sim_waa", "exe_sched_search", "exe_sched_rra",
]
KERNEL_KINDS = ["gemm_tile", "gemm_skinny", "prefill_attn", "decode_attn", "cross_attn", "norm", "other"]


class ExeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"exe error {code}: {msg}")
        self.code = code


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("arch", "n_layers", "n_dec_layers", "d_model", "n_heads", "head_dim", "d_ff", "vocab",
                 "max_pos", "act", "norm", "pos", "rel_buckets", "rel_max_dist", "cross_rel_bias", "dtype",
                 "has_embed", "has_lm_head", "scale_mode")] + \
               [("norm_eps", C.c_float), ("kv_pool_bytes", C.c_uint64), ("max_seqs", C.c_int32),
                ("max_batch_tokens", C.c_int32), ("max_batch_seqs", C.c_int32), ("kv_block_size", C.c_int32)]


class Tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p)]


class ProfileRow(C.Structure):
    _fields_ = [("phase", C.c_int32), ("batch", C.c_int32), ("length", C.c_int32), ("ragged", C.c_int32),
                ("total_tokens", C.c_int32), ("attn_ms_per_layer", C.c_float), ("rest_ms_per_layer", C.c_float),
                ("head_ms", C.c_float), ("full_step_ms", C.c_float), ("std_ms", C.c_float), ("n_timed", C.c_int32)]


class SimTable(C.Structure):
    _fields_ = [("rows", C.POINTER(ProfileRow)), ("n_rows", C.c_int32), ("n_layers_encode", C.c_int32),
                ("n_layers_decode", C.c_int32)]


class SimRraResult(C.Structure):
    _fields_ = [(n, C.c_double) for n in
                ("b_e", "b_d", "completed_fraction", "context_length", "encode_ms", "decode_ms", "cycle_ms",
                 "tokens_per_cycle", "throughput_tok_s", "throughput_seq_s", "latency_ms", "occupancy_exact")]


class SimWaaResult(C.Structure):
    _fields_ = [("b_e", C.c_double), ("b_d", C.c_double), ("encode_ms", C.c_double), ("decode_ms", C.c_double),
                ("gpus_encode", C.c_int32), ("gpus_decode", C.c_int32), ("throughput_seq_s", C.c_double)]


class SchedResult(C.Structure):
    _fields_ = [("found", C.c_int32), ("x1", C.c_int32), ("x2", C.c_int32), ("throughput", C.c_double),
                ("latency", C.c_double), ("evaluations", C.c_int32), ("blocks", C.c_int32)]


class SchedRraResult(C.Structure):
    _fields_ = [("search", SchedResult), ("decode_batch", C.c_int32), ("n_decode", C.c_int32), ("sim", SimRraResult)]


PERF_FN = C.CFUNCTYPE(C.c_int, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double))


class SeqState(C.Structure):
    _fields_ = [("kv_len", C.c_int32), ("cross_len", C.c_int32)]


class LengthDist(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mean", C.c_float), ("std", C.c_float), ("lo", C.c_int32),
                ("hi", C.c_int32), ("seed", C.c_uint64)]


class RraConfig(C.Structure):
    _fields_ = [("decode_batch", C.c_int32), ("n_decode", C.c_int32), ("max_encode_batch", C.c_int32),
                ("adjust", C.c_int32), ("workload_tolerance", C.c_float)]


class RraStats(C.Structure):
    _fields_ = [("wall_s", C.c_double), ("encode_s", C.c_double), ("decode_s", C.c_double),
                ("encoded_tokens", C.c_int64), ("generated_tokens", C.c_int64), ("encode_phases", C.c_int32),
                ("encode_calls", C.c_int32), ("decode_iterations", C.c_int32), ("mean_decode_batch", C.c_double),
                ("latency_mean_s", C.c_double), ("latency_p50_s", C.c_double), ("latency_p99_s", C.c_double),
                ("latency_max_s", C.c_double), ("queue_p99_s", C.c_double)]


class KernelTime(C.Structure):
    _fields_ = [("kind", C.c_int32), ("launches", C.c_int64), ("ms", C.c_double), ("bytes", C.c_double),
                ("flops", C.c_double)]


def lib_path() -> str:
    return os.path.join(_HERE, "libexe.so")


def lib():
    """Loads libexe.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    p = lib_path()
    if not os.path.exists(p):
        raise ImportError(f"{p} is not built; run `python -m paper_2404_07947_amd.build` (needs hipcc)")
    L = C.CDLL(p)
    vp, i32, ip = C.c_void_p, C.c_int32, C.POINTER(C.c_int32)
    L.exe_expected_weights.argtypes = [C.POINTER(Config)]
    L.exe_model_load.argtypes = [C.POINTER(Config), C.POINTER(Tensor), i32, vp, C.POINTER(vp)]
    L.exe_model_free.argtypes = [vp]
    L.exe_encode.argtypes = [vp, i32, ip, ip, ip, ip, vp, ip, vp]
    L.exe_decode_step.argtypes = [vp, i32, ip, ip, ip, vp, ip, vp]
    L.exe_seq_release.argtypes = [vp, i32, ip]
    L.exe_seq_length.argtypes = [vp, i32]
    L.exe_kv_stats.argtypes = [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), ip]
    L.exe_seq_export_bytes.argtypes = [vp, i32]
    L.exe_seq_export_bytes.restype = C.c_int64
    L.exe_seq_export.argtypes = [vp, i32, vp, C.c_uint64, C.POINTER(SeqState)]
    L.exe_seq_import.argtypes = [vp, i32, vp, C.c_uint64, C.POINTER(SeqState), i32]
    L.exe_seq_reserve.argtypes = [vp, i32, i32]
    L.exe_kv_compact.argtypes = [vp, C.POINTER(C.c_uint64)]
    L.exe_profile.argtypes = [vp, i32, ip, i32, ip, i32, C.POINTER(LengthDist), i32, C.POINTER(ProfileRow), i32, ip]
    L.exe_run_rra.argtypes = [vp, C.POINTER(RraConfig), i32, ip, ip, ip, ip, C.POINTER(RraStats)]
    L.exe_kernel_timing.argtypes = [vp, i32]
    L.exe_kernel_times.argtypes = [vp, C.POINTER(KernelTime)]
    L.exe_op_gemm.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, i32, C.c_float, i32, vp, vp, C.c_uint64]
    L.exe_op_gemm_workspace.argtypes = [i32, i32, i32, i32]
    L.exe_op_gemm_workspace.restype = C.c_uint64
    L.exe_op_gemm_plan.argtypes = [i32, i32, i32, i32, ip, ip, ip, ip]
    L.exe_op_gemm_ld.argtypes = [vp, i32, i32, i32, i32, vp, i32, vp, i32, vp, i32, C.c_float, i32, vp, vp, C.c_uint64]
    L.exe_op_paged_index_check.argtypes = [i32, i32, i32, i32, i32]
    L.exe_op_gemm_noalloc.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, i32, C.c_float, i32, vp]
    L.exe_op_gemm_noalloc_max_workspace.restype = C.c_uint64
    L.exe_op_norm.argtypes = [vp, i32, i32, vp, vp, i32, i32, vp, vp, C.c_float, C.c_float, vp]
    L.exe_op_prefill_attention.argtypes = [vp, i32, i32, ip, vp, i32, i32, C.c_float, i32, vp, i32, vp, i32]
    L.exe_op_prefill_tiles.argtypes = [i32, ip, ip, i32, ip]
    L.exe_op_decode_attention.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp, vp, vp, i32, i32, C.c_float, vp, i32, vp]
    L.exe_op_decode_attention_paged.argtypes = [vp, i32, i32, vp, i32, vp, vp, i32, i32, vp, vp, i32, i32, C.c_float, vp, i32,
                                                i32, vp]
    L.exe_op_argmax.argtypes = [vp, vp, i32, i32, vp]
    L.exe_rel_bucket.argtypes = [i32, i32, i32, i32]
    L.exe_last_error.restype = C.c_char_p
    L.exe_version.restype = C.c_char_p
    dp, f64 = C.POINTER(C.c_double), C.c_double
    L.exe_sim_completion.argtypes = [dp, i32, i32, dp, dp]
    L.exe_sim_step_ms.argtypes = [C.POINTER(SimTable), i32, f64, f64, dp]
    L.exe_sim_rra.argtypes = [C.POINTER(SimTable), dp, i32, dp, i32, f64, i32, i32, C.POINTER(SimRraResult)]
    L.exe_sim_waa.argtypes = [C.POINTER(SimTable), dp, i32, dp, i32, f64, i32, C.POINTER(SimWaaResult)]
    L.exe_sched_search.argtypes = [PERF_FN, vp, i32, i32, i32, i32, f64, f64, f64, C.POINTER(SchedResult)]
    L.exe_sched_rra.argtypes = [C.POINTER(SimTable), dp, i32, dp, i32, i32, i32, i32, i32, i32, f64, f64, f64,
                                C.POINTER(SchedRraResult)]
    _lib = L
    return L


def _check(rc: int) -> int:
    if rc < 0:
        raise ExeError(rc, lib().exe_last_error().decode())
    return rc


def _i32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _ip(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_int32))


def _dev(t) -> Optional[int]:
    """Device pointer of a torch tensor (or an int address), None for None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda and t.is_contiguous(), "expected a contiguous device tensor"
    return t.data_ptr()


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def config_from_shape(shape, kv_pool_bytes: int, max_seqs: int, max_batch_tokens: int, max_batch_seqs: int,
                      kv_block_size: int = 0) -> Config:
    """`shape` is any object with the ModelShape fields of the workload module."""
    return Config(shape.arch, shape.n_layers, shape.n_dec_layers, shape.d_model, shape.n_heads, shape.head_dim,
                  shape.d_ff, shape.vocab, shape.max_pos, shape.act, shape.norm, shape.pos, shape.rel_buckets,
                  shape.rel_max_dist, shape.cross_rel_bias, shape.dtype, shape.has_embed, shape.has_lm_head,
                  shape.scale_mode, shape.norm_eps, kv_pool_bytes, max_seqs, max_batch_tokens, max_batch_seqs, kv_block_size)


def exe_version() -> str:
    return lib().exe_version().decode()


def exe_rel_bucket(rel: int, bidirectional: int, n_buckets: int = 32, max_dist: int = 128) -> int:
    return int(lib().exe_rel_bucket(rel, bidirectional, n_buckets, max_dist))


class Model:
    """Owns one exe_model_t.  Methods mirror the C entry points one to one."""

    def __init__(self, cfg: Config, weights: Sequence, stream=None):
        L = lib()
        self.cfg = cfg
        self._weights = list(weights)           # keep the borrowed tensors alive
        arr = (Tensor * len(self._weights))(*[Tensor(_dev(w)) for w in self._weights])
        h = C.c_void_p()
        self._stream = stream
        _check(L.exe_model_load(C.byref(cfg), arr, len(self._weights), _stream_ptr(stream), C.byref(h)))
        self._h = h

    @staticmethod
    def expected_weights(cfg: Config) -> int:
        return _check(lib().exe_expected_weights(C.byref(cfg)))

    def close(self):
        if getattr(self, "_h", None):
            lib().exe_model_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def encode(self, seq_ids, input_lengths, tokens_packed=None, reserve_lengths=None, hidden_in=None,
               want_tokens: bool = True, out_device=None) -> Optional[np.ndarray]:
        ids, lens = _i32(seq_ids), _i32(input_lengths)
        toks, res = _i32(tokens_packed), _i32(reserve_lengths)
        nxt = np.zeros(len(ids), dtype=np.int32) if want_tokens else None
        _check(lib().exe_encode(self._h, len(ids), _ip(ids), _ip(lens), _ip(toks), _ip(res), _dev(hidden_in),
                                _ip(nxt), _dev(out_device)))
        return nxt

    def decode_step(self, seq_ids, tokens_in, kv_lengths, hidden_in=None, want_tokens: bool = True,
                    out_device=None) -> Optional[np.ndarray]:
        ids, toks, kvl = _i32(seq_ids), _i32(tokens_in), _i32(kv_lengths)
        nxt = np.zeros(len(ids), dtype=np.int32) if want_tokens else None
        _check(lib().exe_decode_step(self._h, len(ids), _ip(ids), _ip(toks), _ip(kvl), _dev(hidden_in), _ip(nxt),
                                     _dev(out_device)))
        return nxt

    def seq_release(self, seq_ids) -> None:
        ids = _i32(seq_ids)
        _check(lib().exe_seq_release(self._h, len(ids), _ip(ids)))

    def seq_length(self, seq_id: int) -> int:
        return _check(lib().exe_seq_length(self._h, int(seq_id)))

    def kv_stats(self) -> dict:
        a, b, c, d = C.c_uint64(), C.c_uint64(), C.c_uint64(), C.c_int32()
        _check(lib().exe_kv_stats(self._h, C.byref(a), C.byref(b), C.byref(c), C.byref(d)))
        return {"pool_bytes": a.value, "used_bytes": b.value, "largest_free_bytes": c.value, "live_seqs": d.value}

    def profile(self, phase: int, batch_sizes, lengths, dist: Optional[LengthDist] = None, n_steps: int = 20) -> List[dict]:
        bs, ls = _i32(batch_sizes), _i32(lengths)
        cap = len(bs) * len(ls)
        rows = (ProfileRow * cap)()
        n = C.c_int32()
        _check(lib().exe_profile(self._h, phase, _ip(bs), len(bs), _ip(ls), len(ls),
                                 C.byref(dist) if dist is not None else None, n_steps, rows, cap, C.byref(n)))
        return [{f: getattr(rows[i], f) for f, _ in ProfileRow._fields_} for i in range(n.value)]

    def seq_export(self, seq_id: int):
        """Returns (host buffer as a numpy uint8 array, state dict) of a live sequence's K/V entries."""
        n = int(lib().exe_seq_export_bytes(self._h, seq_id))
        if n < 0:
            _check(n)
        buf = np.empty(max(n, 1), dtype=np.uint8)
        st = SeqState()
        _check(lib().exe_seq_export(self._h, seq_id, buf.ctypes.data_as(C.c_void_p), n, C.byref(st)))
        return buf[:n], {"kv_len": st.kv_len, "cross_len": st.cross_len}

    def seq_import(self, seq_id: int, buf, state: dict, reserve_length: int = 0) -> None:
        buf = np.ascontiguousarray(buf, dtype=np.uint8)
        st = SeqState(state["kv_len"], state["cross_len"])
        _check(lib().exe_seq_import(self._h, seq_id, buf.ctypes.data_as(C.c_void_p), buf.nbytes, C.byref(st), reserve_length))

    def seq_reserve(self, seq_id: int, reserve_length: int) -> None:
        _check(lib().exe_seq_reserve(self._h, seq_id, reserve_length))

    def kv_compact(self) -> int:
        """Returns the bytes moved."""
        moved = C.c_uint64()
        _check(lib().exe_kv_compact(self._h, C.byref(moved)))
        return moved.value

    def run_rra(self, decode_batch: int, n_decode: int, input_lengths, output_lengths, tokens_packed,
                max_encode_batch: int = 32, adjust: bool = False, workload_tolerance: float = 0.25):
        """Returns (generated tokens packed request after request, stats dict)."""
        il, ol, tk = _i32(input_lengths), _i32(output_lengths), _i32(tokens_packed)
        out = np.zeros(int(ol.sum()), dtype=np.int32)
        cfg = RraConfig(decode_batch, n_decode, max_encode_batch, int(adjust), workload_tolerance)
        st = RraStats()
        _check(lib().exe_run_rra(self._h, C.byref(cfg), len(il), _ip(il), _ip(ol), _ip(tk), _ip(out), C.byref(st)))
        return out, {f: getattr(st, f) for f, _ in RraStats._fields_}

    def kernel_timing(self, enable: bool) -> None:
        _check(lib().exe_kernel_timing(self._h, int(enable)))

    def kernel_times(self) -> List[dict]:
        rows = (KernelTime * len(KERNEL_KINDS))()
        _check(lib().exe_kernel_times(self._h, rows))
        return [{"kind": KERNEL_KINDS[r.kind], "launches": r.launches, "ms": r.ms, "bytes": r.bytes, "flops": r.flops}
                for r in rows]


# ---- single-operation entry points (device tensors in, enqueued on the current torch stream) ----

def exe_op_gemm_workspace(dtype: int, M: int, N: int, K: int) -> int:
    return int(lib().exe_op_gemm_workspace(dtype, M, N, K))


def exe_op_gemm(dtype, M, N, K, A, W, bias, act, alpha, out_mode, out, workspace=None, stream=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().exe_op_gemm(_stream_ptr(stream), dtype, M, N, K, _dev(A), _dev(W), _dev(bias), act, alpha, out_mode,
                             _dev(out), _dev(workspace), ws_bytes))


GEMM_CFG_NAMES = ["64x256", "128x256", "256x256", "64x128", "128x128", "256x128"]


def exe_op_gemm_plan(dtype: int, M: int, N: int, K: int) -> dict:
    r, c, s, f = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
    _check(lib().exe_op_gemm_plan(dtype, M, N, K, C.byref(r), C.byref(c), C.byref(s), C.byref(f)))
    return {"route": r.value, "cfg": c.value, "splits": s.value, "rows_first": f.value}


def exe_op_gemm_ld(dtype, M, N, K, A, lda, W, ldw, bias, act, alpha, out_mode, out, workspace=None, stream=None):
    """A and W are device tensors (or addresses) whose rows are lda / ldw elements apart."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ptr = lambda t: t if isinstance(t, int) or t is None else t.data_ptr()
    _check(lib().exe_op_gemm_ld(_stream_ptr(stream), dtype, M, N, K, ptr(A), lda, ptr(W), ldw, _dev(bias), act, alpha,
                                out_mode, _dev(out), _dev(workspace), ws_bytes))


def exe_op_gemm_noalloc(dtype, M, N, K, A, W, bias, act, alpha, out_mode, out, stream=None):
    _check(lib().exe_op_gemm_noalloc(_stream_ptr(stream), dtype, M, N, K, _dev(A), _dev(W), _dev(bias), act, alpha, out_mode,
                                     _dev(out)))


def exe_op_gemm_noalloc_max_workspace() -> int:
    return int(lib().exe_op_gemm_noalloc_max_workspace())


def exe_op_paged_index_check(dtype: int, dh: int, block_size: int, n_waves: int, length: int) -> int:
    return _check(lib().exe_op_paged_index_check(dtype, dh, block_size, n_waves, length))


def exe_op_norm(dtype, rms, x, row_index, rows, d, gain, shift, eps, out_scale, out, stream=None):
    _check(lib().exe_op_norm(_stream_ptr(stream), dtype, rms, _dev(x), _dev(row_index), rows, d, _dev(gain),
                             _dev(shift), eps, out_scale, _dev(out)))


def exe_op_prefill_tiles(lengths):
    """The (sequence, first query row) pairs of the prefill kernel's query tiles, in launch order (host only)."""
    lens = np.ascontiguousarray(lengths, dtype=np.int32)
    cap = int((lens.astype(np.int64) + 127).sum() // 128 + len(lens))
    out = np.zeros((max(cap, 1), 2), dtype=np.int32)
    n = C.c_int32()
    _check(lib().exe_op_prefill_tiles(len(lens), _ip(lens), _ip(out), cap, C.byref(n)))
    return out[:n.value].copy()


def exe_op_prefill_attention(dtype, cu_seqlens, qkv, H, dh, scale, causal, bias_by_dist, bias_radius, out,
                             force_generic=0, stream=None):
    cu = _i32(cu_seqlens)
    _check(lib().exe_op_prefill_attention(_stream_ptr(stream), dtype, len(cu) - 1, _ip(cu), _dev(qkv), H, dh, scale,
                                          causal, _dev(bias_by_dist), bias_radius, _dev(out), force_generic))


def exe_op_decode_attention(dtype, B, q, q_stride, kv, k_offset, cap, length, qpos, H, dh, scale, bias_by_dist,
                            bias_radius, out, stream=None):
    _check(lib().exe_op_decode_attention(_stream_ptr(stream), dtype, B, _dev(q), q_stride, _dev(kv), _dev(k_offset),
                                         _dev(cap), _dev(length), _dev(qpos), H, dh, scale, _dev(bias_by_dist),
                                         bias_radius, _dev(out)))


def exe_op_decode_attention_paged(dtype, B, q, q_stride, kv_blocks, block_table, max_blocks, block_size, length, qpos, H,
                                  dh, scale, bias_by_dist, bias_radius, new_kv_offset, out, stream=None):
    _check(lib().exe_op_decode_attention_paged(_stream_ptr(stream), dtype, B, _dev(q), q_stride, _dev(kv_blocks),
                                               _dev(block_table), max_blocks, block_size, _dev(length), _dev(qpos), H, dh,
                                               scale, _dev(bias_by_dist), bias_radius, new_kv_offset, _dev(out)))


def exe_probe_peaks(read_bytes: int = 0, stream=None) -> dict:
    """Measured streaming-read and bf16 MFMA rates of the current device."""
    L = lib()
    L.exe_probe_peaks.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    r, f = C.c_double(), C.c_double()
    _check(L.exe_probe_peaks(_stream_ptr(stream), read_bytes, C.byref(r), C.byref(f)))
    return {"hbm_read_bytes_per_s": r.value, "mfma_bf16_flops_per_s": f.value}


def exe_probe_ingest(mode: int, region_bytes: int, passes: int, waves: int, loads_per_batch: int, row_bytes: int = 0,
                     stream=None) -> float:
    """Bytes per second that one workgroup per compute unit takes in (see include/exe.h)."""
    L = lib()
    L.exe_probe_ingest.argtypes = [C.c_void_p, C.c_int32, C.c_uint64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                   C.POINTER(C.c_double)]
    r = C.c_double()
    _check(L.exe_probe_ingest(_stream_ptr(stream), mode, region_bytes, passes, waves, loads_per_batch, row_bytes, C.byref(r)))
    return r.value


def exe_op_argmax(logits, rows, n, out, stream=None):
    _check(lib().exe_op_argmax(_stream_ptr(stream), _dev(logits), rows, n, _dev(out)))


# ---- schedule simulator and scheduling search (exe_sched.h; host only, no GPU needed) ----

def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _as_dict(st):
    out = {}
    for f, _ in st._fields_:
        v = getattr(st, f)
        out[f] = _as_dict(v) if isinstance(v, C.Structure) else v
    return out


def make_sim_table(rows: Sequence[dict], n_layers_encode: int, n_layers_decode: int):
    """rows: dicts as Model.profile returns them (phase, batch, length, attn_ms_per_layer, rest_ms_per_layer, head_ms
    are read).  Returns an object to pass as `table`; it owns the row storage."""
    arr = (ProfileRow * len(rows))()
    for i, r in enumerate(rows):
        for f, _ in ProfileRow._fields_:
            if f in r:
                setattr(arr[i], f, r[f])
    t = SimTable(arr, len(rows), n_layers_encode, n_layers_decode)
    t._keep = arr
    return t


def exe_sim_completion(p_out, n_decode: int):
    p = _f64(p_out)
    pu = np.zeros(n_decode, dtype=np.float64)
    frac = C.c_double()
    _check(lib().exe_sim_completion(_dp(p), len(p), n_decode, _dp(pu), C.byref(frac)))
    return pu, frac.value


def exe_sim_step_ms(table, phase: int, batch: float, length: float) -> float:
    ms = C.c_double()
    _check(lib().exe_sim_step_ms(C.byref(table), phase, batch, length, C.byref(ms)))
    return ms.value


def exe_sim_rra(table, p_in, p_out, decode_batch: float, n_decode: int, latency_len: int) -> dict:
    pi, po = _f64(p_in), _f64(p_out)
    r = SimRraResult()
    _check(lib().exe_sim_rra(C.byref(table), _dp(pi), len(pi), _dp(po), len(po), decode_batch, n_decode, latency_len,
                             C.byref(r)))
    return _as_dict(r)


def exe_sim_waa(table, p_in, p_out, encode_batch: float, n_gpus: int) -> dict:
    pi, po = _f64(p_in), _f64(p_out)
    r = SimWaaResult()
    _check(lib().exe_sim_waa(C.byref(table), _dp(pi), len(pi), _dp(po), len(po), encode_batch, n_gpus, C.byref(r)))
    return _as_dict(r)


def exe_sched_search(perf, r1, r2, eps_throughput: float, eps_latency: float, latency_bound: float) -> dict:
    """perf(x1, x2) -> (latency, throughput)."""
    def cb(x1, x2, user, lat, thr):
        try:
            lat[0], thr[0] = perf(x1, x2)
            return 0
        except Exception:                                  # reported by the library as a failed evaluation
            return 1
    r = SchedResult()
    _check(lib().exe_sched_search(PERF_FN(cb), None, r1[0], r1[1], r2[0], r2[1], eps_throughput, eps_latency,
                                  latency_bound, C.byref(r)))
    return _as_dict(r)


def exe_sched_rra(table, p_in, p_out, bd_range, nd_range, latency_len: int, latency_bound_ms: float,
                  eps_throughput: float = 0.0, eps_latency_ms: float = 0.0) -> dict:
    pi, po = _f64(p_in), _f64(p_out)
    r = SchedRraResult()
    _check(lib().exe_sched_rra(C.byref(table), _dp(pi), len(pi), _dp(po), len(po), bd_range[0], bd_range[1],
                               nd_range[0], nd_range[1], latency_len, latency_bound_ms, eps_throughput,
                               eps_latency_ms, C.byref(r)))
    return _as_dict(r)
