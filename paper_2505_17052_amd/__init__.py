"""MI355X-native batched speculative verification (sev).

Thin Python binding over the C-ABI library `libsev.so` (hand-written HIP kernels for
gfx950).  The binding only marshals arguments; PyTorch is used for device memory and
streams.  There is no CPU or PyTorch fallback: if the library is missing or no GPU is
present, calls fail.
"""
from .binding import (SevError, lib, lib_path, Model, KVCache, verify, verify_ex, verify_sample, verify_sample_static, prefill, kv_commit, kv_rollback,
                      Scheduler, calibrate_depth, edge_align, SEV_F32, SEV_BF16, W_KINDS)

__all__ = ["SevError", "lib", "lib_path", "Model", "KVCache", "verify", "verify_ex", "verify_sample", "verify_sample_static", "prefill", "kv_commit", "kv_rollback", "Scheduler", "calibrate_depth", "edge_align",
           "SEV_F32", "SEV_BF16", "W_KINDS"]
