"""SurfaceLogicKV prefill KV-compression pass for AMD MI355X (gfx950).

The compute lives in the C-ABI library built from csrc/ (libslkv.so); binding.py
is a thin ctypes layer with the same entry-point names.  The library is loaded
on first use and a missing build raises: there is no CPU fallback.
"""

__all__ = ["binding", "workloads"]
