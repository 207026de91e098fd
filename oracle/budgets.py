"""Oracle for Stage 2a of SurfaceLogicKV: per-head KV capacities (test infrastructure).

Follows Section 3.3 (Eq. 6) and Algorithm 2 of the paper.

The printed formula does not spend the dynamic pool exactly (the 0.01 minimum
layer share breaks normalisation, and Algorithm 2 rounds each head on its own),
while the compression pass needs integer capacities that sum to the total.  Two
modes therefore exist:

allocate_budgets (EXACT)
    Reading of Eq. (6): a layer's share of the dynamic pool is proportional to
    0.01 + L_i (L_i = the layer's part of the summed INF_sc), and inside the
    layer a head's share is proportional to its INF_sc ("relative importance of
    the j-th head within the i-th layer").  Both levels are apportioned with
    the largest-remainder rule in exact integer arithmetic, so capacities are
    integers, each >= the fixed part, and sum to avg * L * Hkv exactly.
    Under grouped-query attention the INF_sc of the G query heads of a KV head
    are averaged first, and quantised to a 2^-30 grid so every later step is
    integer.

allocate_budgets_literal (PAPER_LITERAL)
    Algorithm 2 as printed: head shares normalised by the global sum, the
    0.01 offset left un-normalised, independent round-half-up per head.  Kept
    only as a cross-check; it does not sum to the total.
"""

from fractions import Fraction
import math

FIXED_POINT_BITS = 30


def fixed_from_beta(avg_budget, beta):
    """Fixed part b_c (1 - 1/beta) of Algorithm 2, rounded half up to an integer."""
    return int(math.floor(avg_budget * (1.0 - 1.0 / beta) + 0.5))


def _group_means(inf_map, Hq, Hkv):
    """Average INF_sc over the G query heads of each KV head (left-to-right sum / G)."""
    G = Hq // Hkv
    out = []
    for row in inf_map:
        means = []
        for g in range(Hkv):
            acc = 0.0
            for t in range(G):
                acc = acc + float(row[g * G + t])
            means.append(acc / G)
        out.append(means)
    return out


def _largest_remainder(total, weights):
    """Split the integer `total` over integer weights: floor of the exact quota,
    leftover units to the largest fractional remainders, ties to the lower index.
    All-zero weights count as equal weights."""
    n = len(weights)
    if sum(weights) == 0:
        weights = [1] * n
    wsum = sum(weights)
    quotas = [Fraction(total * wgt, wsum) for wgt in weights]
    seats = [q.numerator // q.denominator for q in quotas]
    rem = [q - s for q, s in zip(quotas, seats)]
    left = total - sum(seats)
    order = sorted(range(n), key=lambda i: (-rem[i], i))
    for i in order[:left]:
        seats[i] += 1
    return seats


def allocate_budgets(inf_map, Hq, Hkv, avg_budget, fixed_budget):
    """EXACT mode.  inf_map: L rows of Hq INF_sc values in [0, 1].
    Returns L rows of Hkv integer capacities."""
    L = len(inf_map)
    if Hq % Hkv != 0:
        raise ValueError("Hq must be a multiple of Hkv")
    if not 0 <= fixed_budget <= avg_budget:
        raise ValueError("need 0 <= fixed <= avg")
    for row in inf_map:
        if len(row) != Hq:
            raise ValueError("row length != Hq")
        for val in row:
            if not (0.0 <= float(val) <= 1.0):
                raise ValueError("INF_sc outside [0, 1]")
    means = _group_means(inf_map, Hq, Hkv)
    scale = float(1 << FIXED_POINT_BITS)
    x = [[int(math.floor(m * scale + 0.5)) for m in row] for row in means]
    A = [sum(row) for row in x]
    T = sum(A)
    pool = (avg_budget - fixed_budget) * L * Hkv
    # layer share proportional to 0.01 + A_l / T, i.e. to T + 100 * A_l
    layer_w = [T + 100 * a for a in A] if T > 0 else [1] * L
    layer_pool = _largest_remainder(pool, layer_w)
    out = []
    for l in range(L):
        dyn = _largest_remainder(layer_pool[l], x[l])
        out.append([fixed_budget + dv for dv in dyn])
    return out


def allocate_budgets_literal(inf_map, Hq, Hkv, avg_budget, fixed_budget):
    """PAPER_LITERAL mode: Algorithm 2 step by step in float64 with
    beta = avg / (avg - fixed) and H = Hkv after the group mean."""
    L = len(inf_map)
    means = _group_means(inf_map, Hq, Hkv)
    b_c = float(avg_budget)
    if avg_budget == fixed_budget:
        return [[int(fixed_budget)] * Hkv for _ in range(L)]
    beta = b_c / (avg_budget - fixed_budget)
    b_fixed = b_c * (1.0 - 1.0 / beta)
    B_total = b_c / beta * L * Hkv
    layer_sum = [sum(row) for row in means]
    L_s = sum(layer_sum)
    out = []
    for i in range(L):
        row = []
        for j in range(Hkv):
            if L_s > 0.0:
                S = means[i][j] / L_s
                Li = layer_sum[i] / L_s
            else:
                S, Li = 0.0, 0.0
            b = b_fixed + B_total * (0.01 + Li) * S
            row.append(int(math.floor(max(0.0, b) + 0.5)))
        out.append(row)
    return out


def allocate_budgets_per_query_head(inf_map, Hq, Hkv, avg_budget, fixed_budget):
    """Algorithm 2 speaks of the heads of a layer without grouped-query attention in mind; read
    with its heads = the Hq QUERY heads, every query head gets a capacity (average avg_budget,
    fixed part fixed_budget, EXACT rule over the L x Hq map), and a KV head, whose cache serves
    its G query heads, keeps the sum of their capacities.  Returns L rows of Hkv capacities that
    sum to avg * L * Hq."""
    per_q = allocate_budgets(inf_map, Hq, Hq, avg_budget, fixed_budget)
    G = Hq // Hkv
    return [[sum(row[g * G:(g + 1) * G]) for g in range(Hkv)] for row in per_q]
