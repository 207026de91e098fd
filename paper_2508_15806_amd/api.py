"""Convenience layer over binding.py: uploads host arrays, allocates outputs and
workspace with torch, calls the library.  No arithmetic of the method lives here."""

import numpy as np
import torch

from . import binding as B


# name -> (slkv_dtype, torch dtype of the queries, torch dtype of keys and values)
DTYPES = {"f32": (B.SLKV_F32, torch.float32, torch.float32), "bf16": (B.SLKV_BF16, torch.bfloat16, torch.bfloat16),
          "f16": (B.SLKV_F16, torch.float16, torch.float16),
          "bf16_kv8": (B.SLKV_BF16_KV_FP8, torch.bfloat16, torch.uint8)}   # E4M3 bytes travel as uint8


def to_device(arr, dtype, device="cuda"):
    """numpy fp32 / fp16 array, uint16 array of bfloat16 bit patterns or uint8 array of E4M3 bytes -> device tensor."""
    if dtype == "bf16_kv8":
        arr = np.ascontiguousarray(arr)
        if arr.dtype == np.uint8:
            return torch.from_numpy(arr).to(device)
        dtype = "bf16"
    if dtype == "bf16":
        t = torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).to(device)
        return t.view(torch.bfloat16)
    if dtype == "f16":
        return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float16)).to(device)
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(device)


def to_host(t):
    """device tensor -> numpy (bfloat16 comes back as uint16 bit patterns)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class LayerCall:
    """Device buffers + descriptor for repeated calls on one layer's shapes."""

    def __init__(self, dtype, B_, Hq, Hkv, d, w, cu_seqlens, budgets, pool_kernel=7, pool=B.SLKV_POOL_MAX,
                 device="cuda", debug_scores=False, k_strides=None, v_strides=None):
        """k_strides / v_strides: (token stride, head stride) in elements; default = head-major
        contiguous [Hkv][T][d]."""
        T = int(cu_seqlens[-1])
        self.dtype = dtype
        self.layer = B.Layer(DTYPES[dtype][0], B_, Hq, Hkv, d, w, cu_seqlens,
                             budgets, k_strides or (d, T * d), v_strides or (d, T * d), pool_kernel, pool)
        self.offsets, self.total_kept = B.slkv_compacted_sizes(self.layer)
        tdt = DTYPES[dtype][2]
        rows = max(self.total_kept, 1)
        self.k_out = torch.empty((rows, d), dtype=tdt, device=device)
        self.v_out = torch.empty((rows, d), dtype=tdt, device=device)
        self.kept_idx = torch.empty((rows,), dtype=torch.int32, device=device)
        self.out_offsets = torch.empty((B_ * Hkv + 1,), dtype=torch.int64, device=device)
        self.workspace = torch.zeros((B.slkv_workspace_bytes(self.layer),), dtype=torch.uint8, device=device)   # zero-filled once
        self.importance = self.pooled = None
        if debug_scores:
            self.importance = torch.zeros((max(Hkv * T, 1),), dtype=torch.float32, device=device)
            self.pooled = torch.zeros((max(Hkv * T, 1),), dtype=torch.float32, device=device)

    def run(self, qwin, k, v, stream=None):
        B.slkv_compress_layer(self.layer, qwin, k, v, self.k_out, self.v_out, self.kept_idx, self.workspace,
                              self.out_offsets, self.importance, self.pooled, stream)


class RaggedCall:
    """Device buffers + descriptor for repeated re-compression calls on one ragged cache shape."""

    def __init__(self, dtype, B_, Hq, Hkv, d, w, in_offsets, budgets, pool_kernel=7, pool=B.SLKV_POOL_MAX,
                 device="cuda", debug_scores=False, positions=True):
        rows_in = int(in_offsets[-1])
        self.rag = B.Ragged(DTYPES[dtype][0], B_, Hq, Hkv, d, w, in_offsets, budgets,
                            pool_kernel, pool)
        self.offsets, self.total_kept = B.slkv_recompress_sizes(self.rag)
        tdt = DTYPES[dtype][2]
        rows = max(self.total_kept, 1)
        self.k_out = torch.empty((rows, d), dtype=tdt, device=device)
        self.v_out = torch.empty((rows, d), dtype=tdt, device=device)
        self.kept_idx = torch.empty((rows,), dtype=torch.int32, device=device)
        self.pos_out = torch.empty((rows,), dtype=torch.int32, device=device) if positions else None
        self.out_offsets = torch.empty((B_ * Hkv + 1,), dtype=torch.int64, device=device)
        self.workspace = torch.zeros((B.slkv_recompress_workspace_bytes(self.rag),), dtype=torch.uint8, device=device)
        self.importance = self.pooled = None
        if debug_scores:
            self.importance = torch.zeros((max(rows_in, 1),), dtype=torch.float32, device=device)
            self.pooled = torch.zeros((max(rows_in, 1),), dtype=torch.float32, device=device)

    def run(self, qwin, k_in, v_in, pos_in=None, stream=None):
        B.slkv_recompress_layer(self.rag, qwin, k_in, v_in, self.k_out, self.v_out, self.kept_idx, self.workspace,
                                pos_in, self.pos_out if pos_in is not None else None, self.out_offsets,
                                self.importance, self.pooled, stream)


def score_heads(rows, needle_start, needle_len, topk, acc=None, stream=None):
    """rows: [L,H,T,n] fp32 device tensor.  Returns (acc [L,H,5], scores [L,H,3]) float64 device tensors."""
    L, H, T, n = rows.shape
    if acc is None:
        acc = torch.zeros((L, H, 5), dtype=torch.float64, device=rows.device)
    scores = torch.empty((L, H, 3), dtype=torch.float64, device=rows.device)
    ws = torch.empty((max(B.slkv_score_heads_workspace_bytes(L, H, T, n), 16),), dtype=torch.uint8, device=rows.device)
    B.slkv_score_heads(rows, needle_start, needle_len, topk, acc, scores, ws, stream)
    return acc, scores


def score_heads_ex(rows, needle_start, needle_len, topk, aggregation=B.SLKV_AGG_MICRO, components=(True, True, True),
                   acc=None, stream=None):
    """As score_heads through slkv_score_heads_ex: acc is [L,H,8]."""
    L, H, T, n = rows.shape
    if acc is None:
        acc = torch.zeros((L, H, 8), dtype=torch.float64, device=rows.device)
    scores = torch.empty((L, H, 3), dtype=torch.float64, device=rows.device)
    ws = torch.empty((max(B.slkv_score_heads_workspace_bytes(L, H, T, n), 16),), dtype=torch.uint8, device=rows.device)
    B.slkv_score_heads_ex(rows, needle_start, needle_len, topk, acc, scores, ws, aggregation, components, stream)
    return acc, scores


def score_heads_qk(q, k, needle_start, needle_len, topk, acc=None, stream=None):
    """q [L,Hq,T,d], k [L,Hkv,n,d] bf16 device tensors.  Returns (acc [L,Hq,5], scores [L,Hq,3]) float64 device tensors."""
    L, Hq, T, d = q.shape
    n = k.shape[2]
    if acc is None:
        acc = torch.zeros((L, Hq, 5), dtype=torch.float64, device=q.device)
    scores = torch.empty((L, Hq, 3), dtype=torch.float64, device=q.device)
    ws = torch.empty((B.slkv_score_heads_qk_workspace_bytes(L, Hq, T, n),), dtype=torch.uint8, device=q.device)
    B.slkv_score_heads_qk(q, k, needle_start, needle_len, topk, acc, scores, ws, stream)
    return acc, scores
