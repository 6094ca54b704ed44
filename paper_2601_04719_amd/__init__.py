"""kvq: per-channel symmetric INT8 KV-cache quantization for MI355X (gfx950).

The compute path lives in the C-ABI shared library built from csrc/ (hand
written HIP); `paper_2601_04719_amd.kvq` is its thin ctypes binding.  Importing
the package loads nothing: the library is opened on first use and a missing
library raises (there is no CPU fallback).
"""
__all__ = ["kvq", "workloads"]
