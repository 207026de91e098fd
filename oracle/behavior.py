"""Oracle for Stage 1 of SurfaceLogicKV: attention behaviour analysis (test infrastructure).

Follows Section 3.2 and Algorithm 1 of the paper.  For one attention-weight row
W over n context positions, a needle span N and the set T_k of the K largest
weights, the row's mass splits into four cells:

  WO (correct)      = sum of W over N and T_k
  WD (distracted)   = sum of W over T_k without N
  WS (subconscious) = max(0, TNW - WO) with TNW the sum of W over N
  Wide              = everything else

and SF = WO/(WO+WD), LG = WO/(WO+WS), INF = 2 SF LG / (SF + LG).

Readings where the paper is silent: K is a parameter (the needle length by
default); equal weights rank by lower position; a head's scores come from the
four cells summed over all of its rows (micro average), then divided once;
0/0 is 0.  Rows are fp32 and are widened to float64 before any sum.
"""

import numpy as np


def row_weights(row, needle_start, needle_len, topk):
    """The four cells of Algorithm 1 (steps 1-4) for one row.  Returns
    (WO, WD, WS, Wide) as Python floats (float64)."""
    wts = np.asarray(row, dtype=np.float64)
    n = wts.shape[0]
    if not (0 <= needle_start and needle_start + needle_len <= n):
        raise ValueError("needle outside the row")
    if not 1 <= topk <= n:
        raise ValueError("topk out of range")
    order = np.argsort(-wts, kind="stable")        # larger first, ties by lower position
    top = order[:topk]
    in_needle = (top >= needle_start) & (top < needle_start + needle_len)
    WO = float(wts[top[in_needle]].sum())
    WD = float(wts[top[~in_needle]].sum())
    TNW = float(wts[needle_start:needle_start + needle_len].sum())
    WS = max(0.0, TNW - WO)
    wide = float(wts.sum()) - WO - WD - WS
    return WO, WD, WS, wide


def finalize_scores(WO, WD, WS):
    """Steps 5-7 of Algorithm 1 with 0/0 = 0.  Returns (SF, LG, INF)."""
    SF = WO / (WO + WD) if (WO + WD) > 0.0 else 0.0
    LG = WO / (WO + WS) if (WO + WS) > 0.0 else 0.0
    INF = 2.0 * SF * LG / (SF + LG) if (SF + LG) > 0.0 else 0.0
    return SF, LG, INF


def score_heads(rows, needle_start, needle_len, topk, acc=None):
    """rows: [L, H, T, n] fp32 attention rows.  Adds this call's cells into
    acc[L, H, 5] = (sum WO, sum WD, sum WS, sum Wide, row count) (created when
    None) and returns (acc, scores[L, H, 3] = SF, LG, INF)."""
    rows = np.asarray(rows)
    L, H, T, _ = rows.shape
    if acc is None:
        acc = np.zeros((L, H, 5), dtype=np.float64)
    for l in range(L):
        for h in range(H):
            for t in range(T):
                WO, WD, WS, wide = row_weights(rows[l, h, t], needle_start, needle_len, topk)
                acc[l, h, 0] += WO
                acc[l, h, 1] += WD
                acc[l, h, 2] += WS
                acc[l, h, 3] += wide
                acc[l, h, 4] += 1.0
    scores = np.zeros((L, H, 3), dtype=np.float64)
    for l in range(L):
        for h in range(H):
            scores[l, h] = finalize_scores(acc[l, h, 0], acc[l, h, 1], acc[l, h, 2])
    return acc, scores
