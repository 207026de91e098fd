"""ctypes binding of libslkv.so: argument marshalling only.

Function names match the C ABI (include/slkv.h).  Device buffers are torch
tensors (torch owns memory and streams); host descriptors are numpy arrays.
Every step of the compression pass runs inside the library's HIP kernels; if
the library has not been built, loading raises instead of falling back.
"""

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libslkv.so")

SLKV_F32, SLKV_BF16, SLKV_F16, SLKV_BF16_KV_FP8 = 0, 1, 2, 3
SLKV_POOL_NONE, SLKV_POOL_MAX, SLKV_POOL_AVG = 0, 1, 2
SLKV_BUDGET_EXACT, SLKV_BUDGET_PAPER_LITERAL, SLKV_BUDGET_EXACT_PER_QUERY_HEAD = 0, 1, 2
SLKV_AGG_MICRO, SLKV_AGG_MACRO = 0, 1

STATUS_NAMES = {0: "SLKV_OK", 1: "SLKV_ERR_NULL", 2: "SLKV_ERR_BAD_ARG", 3: "SLKV_ERR_BAD_VALUE",
                4: "SLKV_ERR_UNSUPPORTED", 5: "SLKV_ERR_WORKSPACE", 6: "SLKV_ERR_CAPACITY", 7: "SLKV_ERR_HIP"}

EXPORTS = ["slkv_status_str", "slkv_last_error", "slkv_version", "slkv_init", "slkv_score_heads", "slkv_score_heads_ex", "slkv_score_heads_qk",
           "slkv_score_heads_qk_workspace_bytes",
           "slkv_score_heads_workspace_bytes", "slkv_allocate_budgets", "slkv_fixed_from_beta",
           "slkv_compacted_sizes", "slkv_workspace_bytes", "slkv_compress_layer", "slkv_compress_layer_static",
           "slkv_recompress_sizes", "slkv_recompress_workspace_bytes", "slkv_recompress_layer",
           "slkv_profile_begin", "slkv_profile_end"]

KERNEL_NAMES = ["score_stats", "combine", "score_accum", "select", "gather", "row_cells", "head_reduce", "qk_cells",
                "qk_fallback"]


class SlkvError(RuntimeError):
    def __init__(self, status, detail):
        self.status = status
        super().__init__("%s: %s" % (STATUS_NAMES.get(status, status), detail))


class KernelTime(C.Structure):
    _fields_ = [("kernel", C.c_int32), ("ms", C.c_float)]


class ScoreParams(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("aggregation", C.c_int32), ("use_wo", C.c_int32), ("use_wd", C.c_int32),
                ("use_ws", C.c_int32), ("reserved", C.c_int32)]


class LayerDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("dtype", C.c_int32),
                ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32), ("w", C.c_int32),
                ("pool_kernel", C.c_int32), ("pool", C.c_int32), ("reserved", C.c_int32),
                ("h_cu_seqlens", C.POINTER(C.c_int64)),
                ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
                ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
                ("h_budgets", C.POINTER(C.c_int32))]


class RaggedDesc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("dtype", C.c_int32),
                ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32), ("w", C.c_int32),
                ("pool_kernel", C.c_int32), ("pool", C.c_int32), ("reserved", C.c_int32),
                ("h_in_offsets", C.POINTER(C.c_int64)),
                ("h_budgets", C.POINTER(C.c_int32))]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2508_15806_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libslkv.so is missing: build it with `python -m paper_2508_15806_amd.build` "
                               "(there is no CPU fallback)")
        # torch owns device memory and streams, so its HIP runtime has to be the one this process
        # uses: load it before the library (loaded the other way round, the library would pull in
        # the system runtime first and the two would not see each other's devices and streams)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.slkv_status_str.restype = C.c_char_p
        L.slkv_status_str.argtypes = [C.c_int]
        L.slkv_last_error.restype = C.c_char_p
        L.slkv_version.restype = C.c_int32
        L.slkv_fixed_from_beta.restype = C.c_int32
        L.slkv_fixed_from_beta.argtypes = [C.c_int32, C.c_double]
        L.slkv_allocate_budgets.restype = C.c_int
        L.slkv_allocate_budgets.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_int32, C.c_void_p]
        L.slkv_compacted_sizes.restype = C.c_int
        L.slkv_compacted_sizes.argtypes = [C.POINTER(LayerDesc), C.c_void_p, C.c_void_p]
        L.slkv_workspace_bytes.restype = C.c_int
        L.slkv_workspace_bytes.argtypes = [C.POINTER(LayerDesc), C.POINTER(C.c_size_t)]
        L.slkv_compress_layer.restype = C.c_int
        L.slkv_compress_layer.argtypes = [C.POINTER(LayerDesc)] + [C.c_void_p] * 9 + [C.c_int64, C.c_void_p,
                                                                                      C.c_size_t, C.c_void_p]
        L.slkv_compress_layer_static.restype = C.c_int
        L.slkv_compress_layer_static.argtypes = [C.POINTER(LayerDesc)] + [C.c_void_p] * 9 + [C.c_int64, C.c_void_p]
        L.slkv_recompress_sizes.restype = C.c_int
        L.slkv_recompress_sizes.argtypes = [C.POINTER(RaggedDesc), C.c_void_p, C.c_void_p]
        L.slkv_recompress_workspace_bytes.restype = C.c_int
        L.slkv_recompress_workspace_bytes.argtypes = [C.POINTER(RaggedDesc), C.POINTER(C.c_size_t)]
        L.slkv_recompress_layer.restype = C.c_int
        L.slkv_recompress_layer.argtypes = [C.POINTER(RaggedDesc)] + [C.c_void_p] * 11 + [C.c_int64, C.c_void_p,
                                                                                          C.c_size_t, C.c_void_p]
        L.slkv_score_heads_workspace_bytes.restype = C.c_size_t
        L.slkv_score_heads_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int64]
        L.slkv_score_heads.restype = C.c_int
        L.slkv_score_heads.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int32,
                                       C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.slkv_score_heads_ex.restype = C.c_int
        L.slkv_score_heads_ex.argtypes = [C.POINTER(ScoreParams)] + L.slkv_score_heads.argtypes
        L.slkv_score_heads_qk_workspace_bytes.restype = C.c_size_t
        L.slkv_score_heads_qk_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int64]
        L.slkv_score_heads_qk.restype = C.c_int
        L.slkv_score_heads_qk.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64,
                                          C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_size_t, C.c_void_p]
        L.slkv_profile_begin.restype = C.c_int
        L.slkv_profile_begin.argtypes = [C.c_int32]
        L.slkv_profile_end.restype = C.c_int
        L.slkv_profile_end.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
        _lib = L
    return _lib


def _check(status):
    if status != 0:
        raise SlkvError(status, lib().slkv_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def slkv_version():
    return int(lib().slkv_version())


def slkv_init():
    """One-time set-up on the current device (optional; see the header)."""
    _check(lib().slkv_init())


def slkv_fixed_from_beta(avg_budget, beta):
    return int(lib().slkv_fixed_from_beta(int(avg_budget), float(beta)))


def slkv_allocate_budgets(inf, Hkv, avg_budget, fixed_budget, mode=SLKV_BUDGET_EXACT):
    """inf: [L, Hq] float64 INF_sc map (host).  Returns int32 [L, Hkv] capacities."""
    inf = np.ascontiguousarray(inf, dtype=np.float64)
    L, Hq = inf.shape
    out = np.zeros((L, Hkv), dtype=np.int32)
    _check(lib().slkv_allocate_budgets(inf.ctypes.data, L, Hq, Hkv, int(avg_budget), int(fixed_budget), int(mode),
                                       out.ctypes.data))
    return out


class Layer:
    """Host-side descriptor of one layer call; keeps the numpy arrays it points to alive."""

    def __init__(self, dtype, B, Hq, Hkv, d, w, cu_seqlens, budgets, k_strides, v_strides,
                 pool_kernel=7, pool=SLKV_POOL_MAX):
        self.cu = np.ascontiguousarray(cu_seqlens, dtype=np.int64)
        self.budgets = np.ascontiguousarray(budgets, dtype=np.int32)
        self.desc = LayerDesc(C.sizeof(LayerDesc), int(dtype), B, Hq, Hkv, d, w, pool_kernel, pool, 0,
                              self.cu.ctypes.data_as(C.POINTER(C.c_int64)),
                              k_strides[0], k_strides[1], v_strides[0], v_strides[1],
                              self.budgets.ctypes.data_as(C.POINTER(C.c_int32)))
        self.B, self.Hkv = B, Hkv


def slkv_compacted_sizes(layer):
    """Returns (out_offsets int64 [B*Hkv+1], total_kept)."""
    offs = np.zeros(layer.B * layer.Hkv + 1, dtype=np.int64)
    total = C.c_int64(0)
    _check(lib().slkv_compacted_sizes(C.byref(layer.desc), offs.ctypes.data, C.addressof(total)))
    return offs, int(total.value)


def slkv_workspace_bytes(layer):
    n = C.c_size_t(0)
    _check(lib().slkv_workspace_bytes(C.byref(layer.desc), C.byref(n)))
    return int(n.value)


def slkv_compress_layer(layer, qwin, k, v, k_out, v_out, kept_idx, workspace, out_offsets=None,
                        importance=None, pooled=None, stream=None):
    """Enqueues one layer's compression on `stream` (torch stream; default: current)."""
    _check(lib().slkv_compress_layer(C.byref(layer.desc), _ptr(qwin), _ptr(k), _ptr(v), _ptr(k_out), _ptr(v_out),
                                     _ptr(kept_idx), _ptr(out_offsets), _ptr(importance), _ptr(pooled),
                                     int(k_out.shape[0]), _ptr(workspace), int(workspace.numel() * workspace.element_size()),
                                     _stream(stream)))


def slkv_compress_layer_static(layer, qwin, k, v, k_out, v_out, kept_idx, out_offsets=None,
                               importance=None, pooled=None, stream=None):
    """As slkv_compress_layer, with the library's own static scratch buffer instead of a workspace."""
    _check(lib().slkv_compress_layer_static(C.byref(layer.desc), _ptr(qwin), _ptr(k), _ptr(v), _ptr(k_out), _ptr(v_out),
                                            _ptr(kept_idx), _ptr(out_offsets), _ptr(importance), _ptr(pooled),
                                            int(k_out.shape[0]), _stream(stream)))


class Ragged:
    """Host-side descriptor of one re-compression call; keeps the numpy arrays it points to alive."""

    def __init__(self, dtype, B, Hq, Hkv, d, w, in_offsets, budgets, pool_kernel=7, pool=SLKV_POOL_MAX):
        self.offs = np.ascontiguousarray(in_offsets, dtype=np.int64)
        self.budgets = np.ascontiguousarray(budgets, dtype=np.int32)
        self.desc = RaggedDesc(C.sizeof(RaggedDesc), int(dtype), B, Hq, Hkv, d, w, pool_kernel, pool, 0,
                               self.offs.ctypes.data_as(C.POINTER(C.c_int64)),
                               self.budgets.ctypes.data_as(C.POINTER(C.c_int32)))
        self.B, self.Hkv = B, Hkv


def slkv_recompress_sizes(rag):
    """Returns (out_offsets int64 [B*Hkv+1], total_kept)."""
    offs = np.zeros(rag.B * rag.Hkv + 1, dtype=np.int64)
    total = C.c_int64(0)
    _check(lib().slkv_recompress_sizes(C.byref(rag.desc), offs.ctypes.data, C.addressof(total)))
    return offs, int(total.value)


def slkv_recompress_workspace_bytes(rag):
    n = C.c_size_t(0)
    _check(lib().slkv_recompress_workspace_bytes(C.byref(rag.desc), C.byref(n)))
    return int(n.value)


def slkv_recompress_layer(rag, qwin, k_in, v_in, k_out, v_out, kept_idx, workspace, pos_in=None, pos_out=None,
                          out_offsets=None, importance=None, pooled=None, stream=None):
    """Enqueues one re-compression of a ragged cache on `stream` (torch stream; default: current)."""
    _check(lib().slkv_recompress_layer(C.byref(rag.desc), _ptr(qwin), _ptr(k_in), _ptr(v_in), _ptr(pos_in),
                                       _ptr(k_out), _ptr(v_out), _ptr(kept_idx), _ptr(pos_out), _ptr(out_offsets),
                                       _ptr(importance), _ptr(pooled), int(k_out.shape[0]), _ptr(workspace),
                                       int(workspace.numel() * workspace.element_size()), _stream(stream)))


def slkv_score_heads_workspace_bytes(L, H, T, n):
    return int(lib().slkv_score_heads_workspace_bytes(L, H, T, n))


def slkv_score_heads(rows, needle_start, needle_len, topk, acc, scores, workspace, stream=None):
    """rows: [L, H, T, n] fp32 device tensor; acc [L, H, 5] float64 (in/out); scores [L, H, 3] float64 or None."""
    L, H, T, n = rows.shape
    _check(lib().slkv_score_heads(_ptr(rows), L, H, T, n, int(needle_start), int(needle_len), int(topk), _ptr(acc),
                                  _ptr(scores), _ptr(workspace), int(workspace.numel() * workspace.element_size()),
                                  _stream(stream)))


def slkv_score_heads_ex(rows, needle_start, needle_len, topk, acc, scores, workspace, aggregation=SLKV_AGG_MICRO,
                        components=(True, True, True), stream=None):
    """As slkv_score_heads with acc [L, H, 8]; aggregation and the (WO, WD, WS) switches of the ablation."""
    L, H, T, n = rows.shape
    prm = ScoreParams(C.sizeof(ScoreParams), int(aggregation), int(bool(components[0])), int(bool(components[1])),
                      int(bool(components[2])), 0)
    _check(lib().slkv_score_heads_ex(C.byref(prm), _ptr(rows), L, H, T, n, int(needle_start), int(needle_len), int(topk),
                                     _ptr(acc), _ptr(scores), _ptr(workspace),
                                     int(workspace.numel() * workspace.element_size()), _stream(stream)))


def slkv_score_heads_qk_workspace_bytes(L, Hq, T, n):
    return int(lib().slkv_score_heads_qk_workspace_bytes(L, Hq, T, n))


def slkv_score_heads_qk(q, k, needle_start, needle_len, topk, acc, scores, workspace, stream=None):
    """q: [L, Hq, T, d], k: [L, Hkv, n, d] bf16 device tensors; acc [L, Hq, 5] float64 (in/out); scores [L, Hq, 3] or None."""
    L, Hq, T, d = q.shape
    Hkv, n = k.shape[1], k.shape[2]
    _check(lib().slkv_score_heads_qk(_ptr(q), _ptr(k), L, Hq, Hkv, T, n, d, int(needle_start), int(needle_len), int(topk),
                                     _ptr(acc), _ptr(scores), _ptr(workspace),
                                     int(workspace.numel() * workspace.element_size()), _stream(stream)))


def slkv_profile_begin(max_records):
    _check(lib().slkv_profile_begin(int(max_records)))


def slkv_profile_end(capacity):
    """Returns a list of (kernel name, milliseconds) in launch order."""
    recs = (KernelTime * capacity)()
    cnt = C.c_int32(0)
    _check(lib().slkv_profile_end(C.cast(recs, C.c_void_p), capacity, C.byref(cnt)))
    return [(KERNEL_NAMES[recs[i].kernel], float(recs[i].ms)) for i in range(min(cnt.value, capacity))]
