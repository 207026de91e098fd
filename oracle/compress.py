"""Oracle for Stage 2b of SurfaceLogicKV: KV entry selection (test infrastructure).

Follows Section 3.1 (Eq. 2-4), Section 3.4 (Eq. 7-8) and Algorithm 3 of the
paper, in float64, one (sequence, KV head) segment at a time, with no tiling,
fusion or reordering.  The paper leaves several points open; the readings used
here are:

  * softmax runs over the history keys only (Algorithm 3 forms the history H
    first and takes Softmax(Q_window H^T / sqrt(d_k)) of it);
  * the w x m probability matrix is reduced to one score per history key by
    summing over the w window rows, and under grouped-query attention over the
    G query heads that share the KV head ("window-summed importance");
  * scores are smoothed by a 1-D stride-1 same-length pool (max by default,
    window clipped at the edges) before ranking;
  * TopK ranks larger scores first, equal scores by lower position, and the
    kept history positions are emitted in ascending order, followed by the
    window (Concat(H', W));
  * history budget C_H = C - w is clamped to [0, m]: the window is always kept.

Inputs are fp32 arrays or uint16 arrays holding bfloat16 bit patterns; both are
widened exactly to float64.  Outputs K/V rows are bit copies in the input dtype.
"""

import math

import numpy as np

POOL_NONE = 0
POOL_MAX = 1
POOL_AVG = 2


def fp8_e4m3_to_f64(b):
    """OCP 8-bit floating point E4M3 (bytes, uint8) -> float64: 1 sign, 4 exponent (bias 7), 3 mantissa
    bits; exponent 0 = subnormal (m * 2^-9); no infinities; exponent 15 with mantissa 7 = NaN."""
    b = np.asarray(b, dtype=np.uint8).astype(np.int64)
    sign = np.where(b >> 7, -1.0, 1.0)
    e = (b >> 3) & 15
    m = (b & 7).astype(np.float64)
    mag = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    mag = np.where((e == 15) & ((b & 7) == 7), np.nan, mag)
    return sign * mag


def bf16_bits_to_f64(a):
    """Exact widening to float64 of bfloat16 bit patterns (uint16), E4M3 bytes (uint8), fp16 or fp32 values."""
    a = np.asarray(a)
    if a.dtype == np.uint8:
        return fp8_e4m3_to_f64(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if a.dtype == np.float16 or a.dtype == np.float32 or a.dtype == np.float64:
        return a.astype(np.float64)
    raise TypeError("expected float32, float16, uint16 (bf16 bits) or uint8 (E4M3 bytes), got %s" % a.dtype)


def window_importance(q_group, k_hist):
    """Window-summed softmax importance of every history key (Eq. 2-4, Eq. 7).

    q_group: [G, w, d] window queries of the G query heads sharing this KV head.
    k_hist : [m, d]    history keys.
    Returns I[m] = sum over the G*w query rows of softmax_j(q . k_j / sqrt(d)).
    """
    q = bf16_bits_to_f64(q_group)
    k = bf16_bits_to_f64(k_hist)
    d = q.shape[-1]
    rows = q.reshape(-1, d)
    s = (rows @ k.T) / math.sqrt(d)               # Eq. (3)
    s = s - s.max(axis=1, keepdims=True)          # shift does not change Eq. (4)
    e = np.exp(s)
    p = e / e.sum(axis=1, keepdims=True)          # Eq. (4) over the m history keys
    return p.sum(axis=0)


def pool_1d(x, kernel, mode=POOL_MAX):
    """Stride-1 same-length 1-D pooling of a score vector (odd kernel).

    MAX: out[j] = max(x[j-r .. j+r]) with the window clipped to [0, m).
    AVG: out[j] = sum(x[j-r .. j+r], zeros outside) / kernel.
    """
    x = np.asarray(x, dtype=np.float64)
    if mode == POOL_NONE or kernel == 1:
        return x.copy()
    if kernel < 1 or kernel % 2 == 0:
        raise ValueError("pool kernel must be odd and >= 1")
    r = kernel // 2
    if mode == POOL_MAX:
        padded = np.pad(x, r, constant_values=-np.inf)   # clipped window == -inf padding
        return np.lib.stride_tricks.sliding_window_view(padded, kernel).max(axis=-1)
    if mode == POOL_AVG:
        padded = np.pad(x, r, constant_values=0.0)
        return np.lib.stride_tricks.sliding_window_view(padded, kernel).sum(axis=-1) / kernel
    raise ValueError("unknown pool mode")


def select_topk(scores, k):
    """Positions of the k largest scores; ties to the lower position; ascending.

    Returns (idx, tau) with tau the k-th largest score (None when k == 0).
    """
    scores = np.asarray(scores, dtype=np.float64)
    m = scores.shape[0]
    if not 0 <= k <= m:
        raise ValueError("k out of range")
    if k == 0:
        return np.empty(0, dtype=np.int64), None
    order = np.argsort(-scores, kind="stable")     # equal scores keep ascending position
    top = order[:k]
    tau = float(scores[top[-1]])
    return np.sort(top).astype(np.int64), tau


def kept_count(n, w, cap):
    """Rows kept for a segment of n tokens, window w, capacity cap (Algorithm 3)."""
    if n <= w or n <= cap:
        return n
    return max(cap, w)


def compress_segment(q_group, k_seg, v_seg, w, cap, pool_kernel=7, pool_mode=POOL_MAX, scores=None):
    """Algorithm 3 for one sequence and one KV head.

    q_group: [G, w, d]; k_seg, v_seg: [n, d]; cap: the head's capacity C.
    scores: optional (importance, pooled) pair returned by an earlier call on the same
    inputs and pooling (they do not depend on the capacity); reused instead of recomputed.
    Returns a dict: kept_idx (int64, ascending history then window), k_out,
    v_out (bit copies), importance, pooled (None on the early-out path), tau, k.
    """
    n = k_seg.shape[0]
    if n <= w or n <= cap:                         # length within capacity: keep all
        idx = np.arange(n, dtype=np.int64)
        return dict(kept_idx=idx, k_out=k_seg[idx].copy(), v_out=v_seg[idx].copy(),
                    importance=None, pooled=None, tau=None, k=None)
    m = n - w                                      # history / window split
    k_keep = min(max(cap - w, 0), m)               # C_H = C - window, clamped
    if scores is None:
        imp = window_importance(q_group, k_seg[:m])
        pooled = pool_1d(imp, pool_kernel, pool_mode)
    else:
        imp, pooled = scores
    hist_idx, tau = select_topk(pooled, k_keep)
    idx = np.concatenate([hist_idx, np.arange(m, n, dtype=np.int64)])
    return dict(kept_idx=idx, k_out=k_seg[idx].copy(), v_out=v_seg[idx].copy(),
                importance=imp, pooled=pooled, tau=tau, k=k_keep)


def compress_layer(qwin, k, v, cu_seqlens, budgets, w, pool_kernel=7, pool_mode=POOL_MAX, score_cache=None):
    """One layer over a ragged batch.

    qwin: [B, Hq, w, d]; k, v: [Hkv, T, d] with sequences packed along T at
    cu_seqlens[B+1]; budgets: [Hkv] capacities of this layer.
    score_cache: optional dict that keeps (importance, pooled) per (b, h) between calls on the
    same inputs and pooling with other budgets (memoisation only: the scores do not depend on
    the capacities).
    Returns dict: segments (list over b*Hkv+h of compress_segment results),
    out_offsets (int64 [B*Hkv+1]), k_out, v_out ([total_kept, d] packed).
    """
    qwin = np.asarray(qwin)
    B, Hq = qwin.shape[0], qwin.shape[1]
    Hkv = k.shape[0]
    G = Hq // Hkv
    segs = []
    offs = [0]
    for b in range(B):
        t0, t1 = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        for h in range(Hkv):
            cached = score_cache.get((b, h)) if score_cache is not None else None
            r = compress_segment(qwin[b, h * G:(h + 1) * G], k[h, t0:t1], v[h, t0:t1],
                                 w, int(budgets[h]), pool_kernel, pool_mode, scores=cached)
            if score_cache is not None and r["importance"] is not None:
                score_cache[(b, h)] = (r["importance"], r["pooled"])
            segs.append(r)
            offs.append(offs[-1] + r["kept_idx"].shape[0])
    k_out = np.concatenate([s["k_out"] for s in segs], axis=0)
    v_out = np.concatenate([s["v_out"] for s in segs], axis=0)
    return dict(segments=segs, out_offsets=np.asarray(offs, dtype=np.int64),
                k_out=k_out, v_out=v_out)


def recompress_layer(qwin, k_rows, v_rows, in_offsets, budgets, w, pool_kernel=7, pool_mode=POOL_MAX,
                     pos_in=None):
    """Algorithm 3 applied to a cache that is already ragged (Section 3.4: the selection runs
    whenever a head's cache length exceeds its capacity, so also on a compacted cache that has
    grown during generation).

    qwin: [B, Hq, w, d] queries of the latest w tokens; k_rows, v_rows: [rows, d] packed cache,
    segment s = b*Hkv + h at rows in_offsets[s]..in_offsets[s+1] (its last w rows are the
    window); budgets: [Hkv]; pos_in: optional [rows] original token position of every cached row.
    Returns the dict of compress_layer plus pos_out (pos_in at the kept rows) when pos_in is given.
    """
    qwin = np.asarray(qwin)
    B, Hq = qwin.shape[0], qwin.shape[1]
    Hkv = len(budgets)
    G = Hq // Hkv
    segs = []
    offs = [0]
    pos_out = []
    for b in range(B):
        for h in range(Hkv):
            s = b * Hkv + h
            r0, r1 = int(in_offsets[s]), int(in_offsets[s + 1])
            r = compress_segment(qwin[b, h * G:(h + 1) * G], k_rows[r0:r1], v_rows[r0:r1],
                                 w, int(budgets[h]), pool_kernel, pool_mode)
            segs.append(r)
            offs.append(offs[-1] + r["kept_idx"].shape[0])
            if pos_in is not None:
                pos_out.append(np.asarray(pos_in)[r0 + r["kept_idx"]])
    out = dict(segments=segs, out_offsets=np.asarray(offs, dtype=np.int64),
               k_out=np.concatenate([s["k_out"] for s in segs], axis=0),
               v_out=np.concatenate([s["v_out"] for s in segs], axis=0))
    if pos_in is not None:
        out["pos_out"] = np.concatenate(pos_out)
    return out
