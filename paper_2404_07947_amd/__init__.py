"""exe: batched Transformer execution (encode once, decode iteratively over ragged K/V caches) on MI355X.

Thin ctypes binding of libexe.so (include/exe.h).  Every step of the path runs in the library's HIP
kernels; this package only marshals arguments.  PyTorch is used by callers for device memory and
streams.  Importing the package does not load the library; the first call does, and raises if the
library has not been built (python -m paper_2404_07947_amd.build).
"""
from .binding import (ExeError, Model, config_from_shape, exe_op_argmax, exe_op_decode_attention, exe_op_decode_attention_paged, exe_probe_peaks, exe_probe_ingest,  # noqa: F401
                      exe_op_gemm, exe_op_gemm_workspace, exe_op_gemm_plan, exe_op_gemm_ld, exe_op_gemm_noalloc, exe_op_gemm_noalloc_max_workspace, exe_op_paged_index_check,
                      GEMM_CFG_NAMES, exe_op_norm, exe_op_prefill_attention, exe_op_prefill_tiles,
                      exe_rel_bucket, exe_version, lib, lib_path, DECLARED_SYMBOLS, KERNEL_KINDS,
                      make_sim_table, exe_sim_completion, exe_sim_step_ms, exe_sim_rra, exe_sim_waa,
                      exe_sched_search, exe_sched_rra)
