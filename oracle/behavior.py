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

Variants (score_heads_modes): the ablation of Section 4.2 / Table 4 keeps or
removes each of WO, WD, WS; the paper prints no formula for the ablated score,
so a removed component is read as the value 0 in steps 5-6.  A "macro"
aggregation takes SF and LG of every row first, averages them over the head's
rows and applies step 7 to the two means (the default "micro" aggregation sums
the cells first).
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


def finalize_scores(WO, WD, WS, components=(True, True, True)):
    """Steps 5-7 of Algorithm 1 with 0/0 = 0.  Returns (SF, LG, INF).
    components = (use WO, use WD, use WS): a component that is switched off (the
    "-" entries of Table 4) enters steps 5-6 as 0."""
    WO = WO if components[0] else 0.0
    WD = WD if components[1] else 0.0
    WS = WS if components[2] else 0.0
    SF = WO / (WO + WD) if (WO + WD) > 0.0 else 0.0
    LG = WO / (WO + WS) if (WO + WS) > 0.0 else 0.0
    INF = harmonic(SF, LG)
    return SF, LG, INF


def harmonic(SF, LG):
    """Step 7 of Algorithm 1 (0/0 = 0)."""
    return 2.0 * SF * LG / (SF + LG) if (SF + LG) > 0.0 else 0.0


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


def score_heads_modes(rows, needle_start, needle_len, topk, aggregation="micro", components=(True, True, True), acc=None):
    """As score_heads, with the aggregation over a head's rows and the ablation of Table 4 as
    parameters.  acc[L, H, 8] = (sum WO, sum WD, sum WS, sum Wide, row count, sum of per-row SF,
    sum of per-row LG, 0); the per-row SF / LG use the same `components`.
    aggregation "micro": scores from the summed cells; "macro": SF, LG = means of the per-row
    values, INF = step 7 on the two means."""
    if aggregation not in ("micro", "macro"):
        raise ValueError("aggregation must be 'micro' or 'macro'")
    rows = np.asarray(rows)
    L, H, T, _ = rows.shape
    if acc is None:
        acc = np.zeros((L, H, 8), dtype=np.float64)
    for l in range(L):
        for h in range(H):
            for t in range(T):
                WO, WD, WS, wide = row_weights(rows[l, h, t], needle_start, needle_len, topk)
                sf, lg, _ = finalize_scores(WO, WD, WS, components)
                acc[l, h, 0] += WO
                acc[l, h, 1] += WD
                acc[l, h, 2] += WS
                acc[l, h, 3] += wide
                acc[l, h, 4] += 1.0
                acc[l, h, 5] += sf
                acc[l, h, 6] += lg
    scores = np.zeros((L, H, 3), dtype=np.float64)
    for l in range(L):
        for h in range(H):
            if aggregation == "micro":
                scores[l, h] = finalize_scores(acc[l, h, 0], acc[l, h, 1], acc[l, h, 2], components)
            else:
                cnt = acc[l, h, 4]
                sf = acc[l, h, 5] / cnt if cnt > 0 else 0.0
                lg = acc[l, h, 6] / cnt if cnt > 0 else 0.0
                scores[l, h] = (sf, lg, harmonic(sf, lg))
    return acc, scores


def attention_rows(q, k):
    """Attention-weight rows of Section 3.1 (Eq. 2-4) for decode queries against a fixed context.

    q: [L, Hq, T, d] queries of T decode steps (fp32, or uint16 bfloat16 bit patterns);
    k: [L, Hkv, n, d] keys of the context; the Hq / Hkv query heads of a group share a KV head.
    Returns float64 rows [L, Hq, T, n]: softmax over the n keys of q . k / sqrt(d)."""
    from .compress import bf16_bits_to_f64
    q64, k64 = bf16_bits_to_f64(q), bf16_bits_to_f64(k)
    L, Hq, T, d = q64.shape
    Hkv, n = k64.shape[1], k64.shape[2]
    G = Hq // Hkv
    rows = np.empty((L, Hq, T, n), dtype=np.float64)
    for l in range(L):
        for h in range(Hq):
            s = (q64[l, h] @ k64[l, h // G].T) / np.sqrt(float(d))     # Eq. (3)
            s = s - s.max(axis=1, keepdims=True)
            e = np.exp(s)
            rows[l, h] = e / e.sum(axis=1, keepdims=True)                # Eq. (4)
    return rows


def score_heads_from_qk(q, k, needle_start, needle_len, topk, acc=None):
    """Stage 1 when the attention rows are not given but implied by queries and keys: the rows
    of attention_rows() go through Algorithm 1 exactly as in score_heads (float64 throughout)."""
    return score_heads(attention_rows(q, k), needle_start, needle_len, topk, acc)
