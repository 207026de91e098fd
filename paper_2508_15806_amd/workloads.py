"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random tensors; it holds none of the compression
method's arithmetic, so both the GPU library's tests and the CPU oracle can be
fed from it without sharing any of the computation under test.

Shapes follow the Llama-3-8B-Instruct setting of the paper (32 layers x 32
query heads, 8 KV heads, head_dim 128; Section 4 and Figure 2), prefix lengths
span its benchmarks (1k-18k for LongBench, up to 129k for LongBench v2), KV
sizes 64..1024 follow Appendix H, and the INF_sc maps copy the skew of Figures
4 and 8 (a few high heads, most near zero, layer 1 very low).  The real
datasets, prompts and model weights are not used anywhere.

All generators use numpy's Philox bit generator; seeds are BASE_SEED + config
(+ layer).  bfloat16 tensors are produced on the host by round-to-nearest-even
from fp32 and returned as uint16 bit patterns.
"""

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20250815


def _rng(*key):
    ss = np.random.SeedSequence([int(k) for k in key])
    return np.random.Generator(np.random.Philox(ss))


def to_bf16_bits(x):
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def _e4m3_magnitudes():
    """The 127 finite non-negative E4M3 values (code = index), ascending."""
    code = np.arange(127)
    e, m = code >> 3, code & 7
    return np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))


def to_fp8_e4m3_bits(x):
    """fp32 -> OCP E4M3 bytes (uint8): round to nearest, ties to the even code, saturating at 448."""
    x = np.asarray(x, dtype=np.float32)
    mags = _e4m3_magnitudes()
    a = np.minimum(np.abs(x).astype(np.float64), mags[-1])
    hi = np.clip(np.searchsorted(mags, a, side="left"), 0, 126)
    lo = np.maximum(hi - 1, 0)
    dlo, dhi = a - mags[lo], mags[hi] - a
    code = np.where(dlo < dhi, lo, np.where(dhi < dlo, hi, np.where(lo % 2 == 0, lo, hi)))
    return (code | (np.signbit(x).astype(np.int64) << 7)).astype(np.uint8)


def bf16_bits_to_f32(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class LayerInputs:
    """One layer's inputs for the compression pass.

    qwin [B, Hq, w, d]; k, v [Hkv, T, d] (sequences packed along T);
    cu_seqlens [B+1] int64.  dtype "f32" (float32 arrays), "f16" (float16 arrays), "bf16_kv8" (queries as
    bf16 bit patterns, keys and values as E4M3 bytes) or "bf16" (uint16 bit
    patterns)."""
    dtype: str
    B: int
    Hq: int
    Hkv: int
    d: int
    w: int
    cu_seqlens: np.ndarray
    qwin: np.ndarray
    k: np.ndarray
    v: np.ndarray
    meta: dict = field(default_factory=dict)


def make_layer(seed_key, seqlens, Hq, Hkv, d, w, dtype="bf16", bias_frac=0.0, bias_sigma=4.0):
    """Q/K/V ~ N(0,1).  With bias_frac > 0 that fraction of each sequence's
    history positions (per KV head, drawn without replacement) has its key
    shifted by bias_sigma times the unit vector of one random window query of a
    random query head in the group, which raises that query's logit by about
    bias_sigma and makes the position stand out."""
    rng = _rng(*seed_key)
    seqlens = [int(s) for s in seqlens]
    B = len(seqlens)
    cu = np.zeros(B + 1, dtype=np.int64)
    cu[1:] = np.cumsum(seqlens)
    T = int(cu[-1])
    G = Hq // Hkv
    q = rng.standard_normal((B, Hq, w, d), dtype=np.float32)
    k = rng.standard_normal((Hkv, T, d), dtype=np.float32)
    v = rng.standard_normal((Hkv, T, d), dtype=np.float32)
    if bias_frac > 0.0:
        for b in range(B):
            m = seqlens[b] - w
            if m <= 0:
                continue
            cnt = int(round(bias_frac * m))
            for h in range(Hkv):
                pos = rng.choice(m, size=cnt, replace=False)
                qh = rng.integers(0, G, size=cnt) + h * G
                qi = rng.integers(0, w, size=cnt)
                qv = q[b, qh, qi, :]
                qv = qv / np.linalg.norm(qv, axis=1, keepdims=True)
                k[h, cu[b] + pos, :] += np.float32(bias_sigma) * qv
    if dtype == "bf16":
        q, k, v = to_bf16_bits(q), to_bf16_bits(k), to_bf16_bits(v)
    elif dtype == "f16":
        q, k, v = q.astype(np.float16), k.astype(np.float16), v.astype(np.float16)
    elif dtype == "bf16_kv8":
        q, k, v = to_bf16_bits(q), to_fp8_e4m3_bits(k), to_fp8_e4m3_bits(v)
    elif dtype != "f32":
        raise ValueError("dtype must be 'f32', 'bf16', 'f16' or 'bf16_kv8'")
    return LayerInputs(dtype, B, Hq, Hkv, d, w, cu, q, k, v)


class RaggedCache(object):
    """A compacted cache that has grown: segment s = b*Hkv + h holds seg_lens[s] rows of K and V
    (packed [rows, d]); pos_in is the original token position of every row (ascending inside a
    segment, the last w rows of a segment being the newest tokens of its sequence)."""

    def __init__(self, dtype, B, Hq, Hkv, d, w, in_offsets, qwin, k_rows, v_rows, pos_in):
        self.dtype, self.B, self.Hq, self.Hkv, self.d, self.w = dtype, B, Hq, Hkv, d, w
        self.in_offsets, self.qwin, self.k_rows, self.v_rows, self.pos_in = in_offsets, qwin, k_rows, v_rows, pos_in


def make_ragged_cache(seed_key, seg_lens, B, Hq, Hkv, d, w, dtype="bf16", bias_frac=0.0, bias_sigma=4.0,
                      seq_len=1 << 20):
    """Rows ~ N(0,1) as in make_layer (same biased positions recipe, per segment).  seg_lens has
    B*Hkv entries.  Positions: a sorted sample of [0, seq_len - w) for the history rows of the
    segment, then the last w positions of the sequence."""
    rng = _rng(*seed_key)
    seg_lens = [int(x) for x in seg_lens]
    assert len(seg_lens) == B * Hkv
    offs = np.zeros(B * Hkv + 1, dtype=np.int64)
    offs[1:] = np.cumsum(seg_lens)
    rows = int(offs[-1])
    G = Hq // Hkv
    q = rng.standard_normal((B, Hq, w, d), dtype=np.float32)
    k = rng.standard_normal((rows, d), dtype=np.float32)
    v = rng.standard_normal((rows, d), dtype=np.float32)
    pos = np.zeros(rows, dtype=np.int32)
    for s, n in enumerate(seg_lens):
        b, h = divmod(s, Hkv)
        r0 = int(offs[s])
        m = max(n - w, 0)
        if n > w:
            pos[r0:r0 + m] = np.sort(rng.choice(seq_len - w, size=m, replace=False))
            pos[r0 + m:r0 + n] = np.arange(seq_len - w, seq_len)
        else:
            pos[r0:r0 + n] = np.arange(seq_len - n, seq_len)
        cnt = int(round(bias_frac * m))
        if cnt > 0:
            at = rng.choice(m, size=cnt, replace=False)
            qh = rng.integers(0, G, size=cnt) + h * G
            qi = rng.integers(0, w, size=cnt)
            qv = q[b, qh, qi, :]
            qv = qv / np.linalg.norm(qv, axis=1, keepdims=True)
            k[r0 + at, :] += np.float32(bias_sigma) * qv
    if dtype == "bf16":
        q, k, v = to_bf16_bits(q), to_bf16_bits(k), to_bf16_bits(v)
    elif dtype == "f16":
        q, k, v = q.astype(np.float16), k.astype(np.float16), v.astype(np.float16)
    elif dtype == "bf16_kv8":
        q, k, v = to_bf16_bits(q), to_fp8_e4m3_bits(k), to_fp8_e4m3_bits(v)
    elif dtype != "f32":
        raise ValueError("dtype must be 'f32', 'bf16', 'f16' or 'bf16_kv8'")
    return RaggedCache(dtype, B, Hq, Hkv, d, w, offs, q, k, v, pos)


def config6(head_lens, batch=32):
    """Decode-time re-compression: `batch` sequences of Llama-3-8B shape (32q / 8kv heads, d 128,
    window 64), bf16; head h of every sequence holds head_lens[h] cached rows (what its capacity
    kept after prefill plus the tokens generated since; the caller computes the lengths)."""
    head_lens = [int(x) for x in head_lens]
    assert len(head_lens) == 8
    rc = make_ragged_cache((BASE_SEED + 6, batch), head_lens * batch, batch, 32, 8, 128, 64, dtype="bf16",
                           bias_frac=0.02, seq_len=32768 + 4096)
    rc.meta = dict(name="c6", avg=256, fixed=16, pool=7)
    return rc


# ---------------------------------------------------------------- INF_sc maps

def inf_uniform(seed_key, L, Hq):
    return _rng(*seed_key).uniform(0.0, 1.0, size=(L, Hq))


def inf_beta(seed_key, L, Hq, a=0.5, b=5.0):
    return _rng(*seed_key).beta(a, b, size=(L, Hq))


def inf_spiky(seed_key, L=32, Hq=32, spike_frac=0.02, low_layer=1, low_scale=0.05):
    """98% of the cells near zero, U(0, 0.02); 2% spikes, U(0.6, 0.9), at seeded
    cells; one layer (layer 1 by default) scaled down to be very low."""
    rng = _rng(*seed_key)
    m = rng.uniform(0.0, 0.02, size=(L, Hq))
    n_spike = int(round(spike_frac * L * Hq))
    cells = rng.choice(L * Hq, size=n_spike, replace=False)
    m.reshape(-1)[cells] = rng.uniform(0.6, 0.9, size=n_spike)
    if 0 <= low_layer < L:
        m[low_layer] *= low_scale
    return m


# ---------------------------------------------------------------- the five configurations

def config1():
    """Tiny fp32 layer: 4 query / 4 KV heads, d 64, n 1024, w 32, pool 7,
    average budget 128 (fixed 32), INF_sc ~ U(0,1)."""
    seed = BASE_SEED + 1
    lay = make_layer((seed, 0), [1024], 4, 4, 64, 32, dtype="f32")
    lay.meta = dict(name="c1", avg=128, fixed=32, pool=7, inf=inf_uniform((seed, 1), 1, 4))
    return lay


def config2():
    """One Llama-3-8B-shaped bf16 layer: 32q/8kv, d 128, n 8192, w 32, 2% biased
    keys, average budget 128 (fixed 32), INF_sc ~ Beta(0.5, 5)."""
    seed = BASE_SEED + 2
    lay = make_layer((seed, 0), [8192], 32, 8, 128, 32, dtype="bf16", bias_frac=0.02)
    lay.meta = dict(name="c2", avg=128, fixed=32, pool=7, inf=inf_beta((seed, 1), 1, 32))
    return lay


C3_BUDGETS = (64, 256, 1024)


def config3_inf():
    return inf_spiky((BASE_SEED + 3, 1000), 32, 32)


def config3_layer(layer, n=32768):
    """Layer `layer` of the 32-layer prefill: 32q/8kv, d 128, n 32768, w 64,
    2% biased keys.  Budgets: average 64 / 256 / 1024, fixed 16, from
    config3_inf()."""
    seed = BASE_SEED + 3
    lay = make_layer((seed, layer), [n], 32, 8, 128, 64, dtype="bf16", bias_frac=0.02)
    lay.meta = dict(name="c3", layer=layer, fixed=16, pool=7)
    return lay


def config5(seqlens=(131072, 65536, 100000, 20000)):
    """Ragged long-context batch, bf16, 32q/8kv, d 128, w 64, average budget 512
    (fixed 64); budgets come from config 3's map (the caller picks the row of
    the lowest layer >= 2 that holds a spike)."""
    seed = BASE_SEED + 5
    lay = make_layer((seed, 0), list(seqlens), 32, 8, 128, 64, dtype="bf16", bias_frac=0.02)
    lay.meta = dict(name="c5", avg=512, fixed=64, pool=7)
    return lay


def config5_layer_row(inf_map, threshold=0.5):
    """Index of the lowest layer >= 2 whose row holds a spike (> threshold)."""
    for l in range(2, inf_map.shape[0]):
        if (inf_map[l] > threshold).any():
            return l
    return 2


# ---------------------------------------------------------------- Stage 1 rows (configuration 4)

@dataclass
class NeedleRows:
    """rows [L, H, T, n] fp32 attention rows; the needle occupies
    [needle_start, needle_start + needle_len); token_ids is bookkeeping only."""
    rows: np.ndarray
    needle_start: int
    needle_len: int
    topk: int
    token_ids: np.ndarray


def config4(L=32, H=32, T=16, n=16384, needle_len=32, vocab=128000, seed_extra=0):
    """Synthetic needle-in-a-haystack decode rows.  Each row is softmax(z),
    z ~ N(0,1).  With probability 0.005 the row is a "surface" row (z at the
    needle token being emitted, start + t, raised by 12); with probability
    0.015 it is a "logic" row (z raised by 6 on 8 positions drawn from the
    needle's other tokens and the 16 tokens on either side); otherwise it stays
    diffuse."""
    seed = BASE_SEED + 4
    rng = _rng(seed, seed_extra)
    token_ids = rng.integers(0, vocab, size=n, dtype=np.int64)
    start = int(rng.integers(0, n - needle_len + 1))
    rows = np.empty((L, H, T, n), dtype=np.float32)
    for l in range(L):
        z = rng.standard_normal((H, T, n), dtype=np.float32)
        kind = rng.random((H, T))
        for h in range(H):
            for t in range(T):
                if kind[h, t] < 0.005:
                    z[h, t, start + (t % needle_len)] += np.float32(12.0)
                elif kind[h, t] < 0.020:
                    lo = max(0, start - 16)
                    hi = min(n, start + needle_len + 16)
                    cand = np.array([p for p in range(lo, hi) if p != start + (t % needle_len)])
                    pos = rng.choice(cand, size=min(8, cand.shape[0]), replace=False)
                    z[h, t, pos] += np.float32(6.0)
        z64 = z.astype(np.float64)
        z64 -= z64.max(axis=-1, keepdims=True)
        e = np.exp(z64)
        rows[l] = (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)
    return NeedleRows(rows, start, needle_len, needle_len, token_ids)


@dataclass
class NeedleQK:
    """Decode queries q [L, Hq, T, d] and context keys k [L, Hkv, n, d] (uint16 bfloat16 bit
    patterns) of a needle-in-a-haystack run; the needle occupies [needle_start, +needle_len)."""
    q: np.ndarray
    k: np.ndarray
    needle_start: int
    needle_len: int
    topk: int


def config4_qk(L=32, Hq=32, Hkv=8, T=16, n=16384, d=128, needle_len=32, seed_extra=0, tie_rows=0):
    """The queries and keys behind rows like those of config4(): K ~ N(0,1); a query is N(0,1),
    and with probability 0.005 ("surface") it is pulled towards the key of the needle token being
    emitted (start + t), with probability 0.015 ("logic") towards the mean of 8 keys drawn from
    the needle's other tokens and the 16 tokens on either side; the pull is 12 (6) times the unit
    key direction times sqrt(d), which raises those logits by about 12 (6 x the overlap).
    tie_rows > 0: the first `tie_rows` KV heads of layer 0 get identical keys everywhere (every
    logit of their rows ties)."""
    rng = _rng(BASE_SEED + 4, 77, seed_extra)
    G = Hq // Hkv
    start = int(rng.integers(0, n - needle_len + 1))
    k = rng.standard_normal((L, Hkv, n, d), dtype=np.float32)
    for h in range(min(tie_rows, Hkv)):
        k[0, h, :, :] = k[0, h, :1, :]
    q = rng.standard_normal((L, Hq, T, d), dtype=np.float32)
    kind = rng.random((L, Hq, T))
    scale = np.float32(np.sqrt(d))
    for l, h, t in zip(*np.nonzero(kind < 0.020)):
        kv = h // G
        if kind[l, h, t] < 0.005:
            tgt = k[l, kv, start + (t % needle_len)]
            q[l, h, t] += np.float32(12.0) * scale * tgt / np.linalg.norm(tgt) ** 2
        else:
            lo, hi = max(0, start - 16), min(n, start + needle_len + 16)
            cand = np.array([p for p in range(lo, hi) if p != start + (t % needle_len)])
            pos = rng.choice(cand, size=min(8, cand.shape[0]), replace=False)
            tgt = k[l, kv, pos].mean(axis=0)
            q[l, h, t] += np.float32(6.0) * scale * tgt / np.linalg.norm(tgt) ** 2
    return NeedleQK(to_bf16_bits(q), to_bf16_bits(k), start, needle_len, needle_len)
