"""CPU oracle for the VL-Cache hot path (numpy, fp64).  TEST INFRASTRUCTURE ONLY.

A plain, slow, by-the-definitions implementation of what the GPU path computes:
post-vision attention, accumulated post-vision scores, ThresholdFilter sparsity,
sparsity-aware layer budgets, per-head TopK, gather, and decode attention over the
compressed cache.  It exists so that tests, the smoke check and the benchmark's
`cpu_baseline` leg have something independent to compare against.  It shares no
code with the HIP path and must never be imported by the product package.

Shapes are per (request, layer): q_win [Hq, tau, d] are the queries of the last tau
prompt tokens (the post-vision window), k, v [Hkv, m, d] the prompt's keys/values.
Query head h reads KV head h // g, g = Hq / Hkv.  All arithmetic, the ThresholdFilter
decision of Eq. 1 included, is fp64 on the values handed in.

Pins (see tests/test_oracle_pins.py): softmax rows sum to 1; sum_j psi_j = tau;
equal logits give harmonic-number scores; one dominant key per row gives nnz = tau;
two-level logits give a counted nnz; equal sparsity gives equal budgets; the
worked two-layer budget example; TopK equals a full sort; decode equals a library
scaled-dot-product attention; full-budget decode equals uncompressed attention;
every routine equals the pure-loop brute force on tiny inputs; the decode-query attention equals
a library softmax; CacheHitRate is 1 for the optimal policy, 0 for a disjoint set, k/m-bounded
and equal to a brute-force set intersection; the E4M3 table equals torch's float8_e4m3fn, the
row quantiser equals torch's conversion of the scaled row, is idempotent and within half a step;
the window attention equals a library scaled-dot-product attention under the same mask, returns
V's row for a one-key prompt and 1 for constant V; the column sweep from given statistics equals
the scores, and scales as 1/Z and exp(-M) in the statistics it is given.

Parity unpinned by the paper (self-consistency only): the reduction of the g query
heads of a GQA group into one KV-head score (sum; also used for the decode-query attention of
CacheHitRate), the forced recent window and its rounding, and the integer apportionment of budgets
into token counts.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------------------
# Post-vision attention  (Alg. 1, ComputeSparsity: Q' = Q[m-tau:m], A' = softmax(Q'K^T/sqrt d))
# --------------------------------------------------------------------------------------

def causal_valid(m: int, tau: int) -> np.ndarray:
    """[tau, m] mask of the region i + m - tau >= j of Alg. 1: window row i is prompt
    position m - tau + i and sees keys up to and including itself."""
    i = np.arange(tau)[:, None]
    j = np.arange(m)[None, :]
    return j <= (m - tau + i)


def region_size(m: int, tau: int) -> int:
    """|{(i, j): i + m - tau >= j}| = tau (m - tau) + tau (tau + 1) / 2."""
    return tau * (m - tau) + tau * (tau + 1) // 2


def logits(q_win: np.ndarray, k: np.ndarray, scale: float) -> np.ndarray:
    """s[h, i, j] = scale * <q_win[h, i], k[h // g, j]>  (Alg. 1: Q'K^T / sqrt d; the
    scale defaults to 1/sqrt(d) at the call sites and carries the synthetic per-layer
    temperature otherwise)."""
    q = np.asarray(q_win, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    Hq, Hkv = q.shape[0], kk.shape[0]
    g = Hq // Hkv
    s = np.empty((Hq, q.shape[1], kk.shape[1]), dtype=np.float64)
    for h in range(Hq):
        s[h] = q[h] @ kk[h // g].T
    return s * float(scale)


def post_vision_attention(q_win, k, scale) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """A' (masked entries are 0), logits s, row max M and row sum Z (the two statistics
    App. A.3 stores: pre-exponentiation max and post-exponentiation sum)."""
    s = logits(q_win, k, scale)
    tau, m = s.shape[1], s.shape[2]
    valid = causal_valid(m, tau)[None]
    sm = np.where(valid, s, -np.inf)
    M = sm.max(axis=2)
    e = np.where(valid, np.exp(sm - M[:, :, None]), 0.0)
    Z = e.sum(axis=2)
    return e / Z[:, :, None], s, M, Z


def score(q_win, k, scale):
    """Accumulated post-vision attention (Sec. 3.2): psi_h[j] = sum_i A'_{ij} per query
    head, and psi_kv = sum over the g query heads of a KV group (reading: one TopK per
    KV head needs one score row per KV head).  Returns (psi_kv [Hkv,m], psi_h [Hq,m], M, Z)."""
    A, _, M, Z = post_vision_attention(q_win, k, scale)
    psi_h = A.sum(axis=1)
    Hq = psi_h.shape[0]
    Hkv = np.asarray(k).shape[0]
    psi_kv = psi_h.reshape(Hkv, Hq // Hkv, -1).sum(axis=1)
    return psi_kv, psi_h, M, Z


def window_attention(q_win, k, v, scale) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Causal prefill attention of the post-vision window rows: O[h, i] = sum_j A'_{ij} v[h // g, j]
    (Sec. 2.1, prefill phase, restricted to the last tau prompt positions), together with the two
    row statistics M and Z of the same softmax.  This is what a prefill attention kernel that also
    emits its running max and sum for those rows would hand to the scoring sweep (App. A.3: the
    first kernel computes exactly the reductions a fused-softmax attention kernel carries)."""
    A, _, M, Z = post_vision_attention(q_win, k, scale)
    vv = np.asarray(v, dtype=np.float64)
    Hq, Hkv = A.shape[0], vv.shape[0]
    g = Hq // Hkv
    out = np.empty((Hq, A.shape[1], vv.shape[2]), dtype=np.float64)
    for h in range(Hq):
        out[h] = A[h] @ vv[h // g]
    return out, M, Z


def score_from_stats(q_win, k, scale, M: np.ndarray, Z: np.ndarray):
    """The column sweep alone (App. A.3, second kernel): psi from logits and GIVEN row statistics,
    psi_h[j] = sum_i exp(s_ij - M_i) / Z_i over the causal region.  Returns (psi_kv, psi_h)."""
    s = logits(q_win, k, scale)
    tau, m = s.shape[1], s.shape[2]
    valid = causal_valid(m, tau)[None]
    e = np.where(valid, np.exp(np.where(valid, s, -np.inf) - np.asarray(M, dtype=np.float64)[:, :, None]), 0.0)
    psi_h = (e / np.asarray(Z, dtype=np.float64)[:, :, None]).sum(axis=1)
    Hq, Hkv = psi_h.shape[0], np.asarray(k).shape[0]
    return psi_h.reshape(Hkv, Hq // Hkv, -1).sum(axis=1), psi_h


# --------------------------------------------------------------------------------------
# ThresholdFilter sparsity  (Eq. 1, Eq. 2 restricted to the post-vision rows as in Alg. 1)
# --------------------------------------------------------------------------------------

def sparsity(q_win, k, scale, p: float = 0.01, want_margin: bool = False):
    """nnz[h] = number of entries of the causal region that ThresholdFilter keeps, i.e.
    A'_{ij} >= p max_j A'_{ij}; gamma[h] = 1 - nnz[h] / region_size.

    Since A'_{ij} / max_j A'_{ij} = exp(s_ij - M_i), the test is s_ij - M_i >= ln p (Eq. 1 is a
    statement in real arithmetic: it is decided on the fp64 logits).  With want_margin the
    distance |s_ij - M_i - ln p| of every valid entry is returned too (masked entries get +inf)
    so a harness can list the decisions that a lower-precision evaluation may take the other way."""
    s = logits(q_win, k, scale)
    tau, m = s.shape[1], s.shape[2]
    valid = causal_valid(m, tau)[None]
    M = np.where(valid, s, -np.inf).max(axis=2)
    gap = s - M[:, :, None] - math.log(p)
    keep = valid & (gap >= 0.0)
    nnz = keep.sum(axis=(1, 2)).astype(np.int64)
    gamma = 1.0 - nnz / float(region_size(m, tau))
    if not want_margin:
        return nnz, gamma
    margin = np.where(valid, np.abs(gap), np.inf)
    return nnz, gamma, margin, keep


# --------------------------------------------------------------------------------------
# Sparsity-aware budget allocation  (Alg. 1, SkewedCacheBudgetAllocation)
# --------------------------------------------------------------------------------------

def allocate_float(gamma_lh: np.ndarray, alpha: float) -> np.ndarray:
    """Alg. 1 as printed: gamma' = mean over heads, Z = sum_l (1 - gamma'_l),
    beta_l = clip((1 - gamma'_l) / Z * alpha * L, 0.01, 1).  No renormalisation after the clip."""
    g = np.asarray(gamma_lh, dtype=np.float64).mean(axis=1)
    L = g.shape[0]
    Z = (1.0 - g).sum()
    return np.clip((1.0 - g) / Z * alpha * L, 0.01, 1.0)


def k_min(m: int) -> int:
    """Token count of the lower clip 0.01 (at least one token)."""
    return max(1, -(-m // 100))


def allocate(nnz_lh: np.ndarray, m: int, alpha_num: int, alpha_den: int) -> Tuple[np.ndarray, np.ndarray]:
    """Integer form of Alg. 1 for one request.  1 - gamma'_l is proportional to
    n_l = sum_h nnz[l, h], so beta_l m = n_l / N * alpha L m with N = sum_l n_l.  The
    whole budget B_tot = floor(alpha L m) is apportioned by largest remainder:
    floor quotas q_l = floor(n_l B_tot / N), then +1 to the B_tot - sum q_l layers with
    the largest remainders (ties to the lower layer), then the clip to [k_min, m].
    Returns (k [L] int64, beta [L] = k / m)."""
    nn = [int(sum(int(x) for x in row)) for row in np.asarray(nnz_lh)]
    L = len(nn)
    N = sum(nn)
    B_tot = (alpha_num * L * m) // alpha_den
    if N == 0:
        quota = [B_tot // L] * L
        rem = [0] * L
    else:
        quota = [(n * B_tot) // N for n in nn]
        rem = [(n * B_tot) % N for n in nn]
    extra = B_tot - sum(quota)
    order = sorted(range(L), key=lambda l: (-rem[l], l))
    for l in order[:extra]:
        quota[l] += 1
    lo = k_min(m)
    kk = np.array([min(max(q, lo), m) for q in quota], dtype=np.int64)
    return kk, kk / float(m)


# --------------------------------------------------------------------------------------
# Token eviction: TopK + gather  (Sec. 2.2 scoring policy / top-k set; Sec. 4.2; App. A.4 copy)
# --------------------------------------------------------------------------------------

def topk(psi: np.ndarray, k: int, n_recent: int = 0) -> np.ndarray:
    """Indices of the k largest scores, ties to the lower index, returned ascending.
    With n_recent = r the last r positions are kept unconditionally and the remaining
    k - r slots are filled from the other positions."""
    psi = np.asarray(psi, dtype=np.float64)
    m = psi.shape[0]
    if not (1 <= k <= m):
        raise ValueError("k out of range")
    r = min(n_recent, k)
    head = psi[: m - r]
    order = np.argsort(-head, kind="stable")      # descending score, equal scores by index
    chosen = np.concatenate([order[: k - r], np.arange(m - r, m)])
    return np.sort(chosen).astype(np.int64)


def recent_count(k: int, num: int, den: int) -> int:
    """Size of the forced recent window when it is a fixed fraction of the layer's budget
    (Sec. 5 'Implementation Details': 10 % of the budget), rounded down: floor(k * num / den).
    The paper does not say how the product is rounded; floor is this build's reading."""
    if not (0 <= num <= den and den >= 1):
        raise ValueError("fraction out of range")
    return (int(k) * int(num)) // int(den)


def compact(k: np.ndarray, v: np.ndarray, idx: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Survivors copied to contiguous memory in ascending position: Kc = K[idx], Vc = V[idx]."""
    return np.asarray(k)[idx].copy(), np.asarray(v)[idx].copy()


# --------------------------------------------------------------------------------------
# CacheHitRate  (Def. 3.1)
# --------------------------------------------------------------------------------------

def decode_query_attention(q_next: np.ndarray, k: np.ndarray, scale: float) -> np.ndarray:
    """A_{m+1} of Def. 3.1, per KV head: softmax over all m prompt keys of the first decode
    query's logits, summed over the g query heads of the group.  q_next [Hq, d], k [Hkv, m, d]
    -> [Hkv, m]."""
    q = np.asarray(q_next, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    Hq, Hkv = q.shape[0], kk.shape[0]
    g = Hq // Hkv
    out = np.zeros((Hkv, kk.shape[1]))
    for h in range(Hq):
        s = (kk[h // g] @ q[h]) * float(scale)
        e = np.exp(s - s.max())
        out[h // g] += e / e.sum()
    return out


def cache_hit_rate(psi_star: np.ndarray, kept: np.ndarray, k: int) -> Tuple[int, float]:
    """Def. 3.1: S* = the k positions with the largest psi_star (ties to the lower position),
    hits = |kept ∩ S*|, CacheHitRate = hits / |S*|.  `kept` are the positions a policy preserved."""
    s_star = set(topk(psi_star, int(k)).tolist())
    hits = len(s_star.intersection(int(j) for j in np.asarray(kept).tolist()))
    return hits, hits / float(len(s_star))


# --------------------------------------------------------------------------------------
# FP8 storage of the compressed cache  (App. A.2 names FP8 KV-cache quantisation as an
# orthogonal technique that can be combined with sparsification; the format is this build's)
# --------------------------------------------------------------------------------------

def e4m3_values() -> np.ndarray:
    """The 256 values of the OCP FP8 E4M3 format (1 sign, 4 exponent bits with bias 7, 3 mantissa
    bits, no infinities, 0x7f / 0xff are NaN), from the format's definition."""
    out = np.empty(256)
    for c in range(256):
        e, mnt = (c >> 3) & 0xF, c & 7
        if e == 0xF and mnt == 7:
            v = np.nan
        elif e == 0:
            v = mnt * 2.0 ** -9
        else:
            v = (1 + mnt / 8.0) * 2.0 ** (e - 7)
        out[c] = -v if c & 0x80 else v
    return out


def quantize_e4m3_rows(x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Per-row scaled E4M3: for every row (last axis) scale = absmax / 448 in fp32 (1 for an
    all-zero row), code = the E4M3 value nearest to fp32(x / scale), ties to the even code,
    magnitudes clamped to 448.  Returns (codes uint8, scales float32)."""
    x = np.asarray(x, dtype=np.float32)
    absmax = np.max(np.abs(x), axis=-1, keepdims=True).astype(np.float32)
    scale = np.where(absmax > 0, absmax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    y = (x / scale).astype(np.float32)
    a = np.minimum(np.abs(y), np.float32(448.0)).astype(np.float64)
    pos = e4m3_values()[:0x7F]                       # the 127 finite non-negative values, ascending
    hi = np.searchsorted(pos, a, side="left")        # pos[hi - 1] < a <= pos[hi]
    hi = np.minimum(hi, len(pos) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - pos[lo], pos[hi] - a
    code = np.where(d_lo < d_hi, lo, np.where(d_lo > d_hi, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(a == pos[hi], hi, code).astype(np.uint8)
    code = np.where(np.signbit(y), code | 0x80, code).astype(np.uint8)
    return code, scale[..., 0]


def dequantize_e4m3_rows(code: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """x_hat = value(code) * scale, in fp64."""
    return e4m3_values()[np.asarray(code, dtype=np.uint8)] * np.asarray(scale, dtype=np.float64)[..., None]


# --------------------------------------------------------------------------------------
# Decode attention over the compressed cache  (Sec. 2.1 decoding phase)
# --------------------------------------------------------------------------------------

def decode_attn(q: np.ndarray, kc: Sequence[np.ndarray], vc: Sequence[np.ndarray], scale: float) -> np.ndarray:
    """o[h] = softmax(scale * q[h] Kc[h//g]^T) Vc[h//g] over every cached slot.
    q [Hq, d]; kc, vc: per KV head arrays [n, d] (all heads of a layer hold n slots)."""
    q = np.asarray(q, dtype=np.float64)
    Hq = q.shape[0]
    Hkv = len(kc)
    g = Hq // Hkv
    out = np.empty_like(q)
    for h in range(Hq):
        K = np.asarray(kc[h // g], dtype=np.float64)
        V = np.asarray(vc[h // g], dtype=np.float64)
        s = (K @ q[h]) * float(scale)
        e = np.exp(s - s.max())
        out[h] = (e / e.sum()) @ V
    return out


class CompressedCache:
    """The ragged per-layer cache of one request batch, as plain lists:
    kc[b][l][hkv] is an [n, d] array.  Decode steps append the new key/value first and
    then attend over all slots; nothing is evicted during decode (allocation happens
    once, right after prefill)."""

    def __init__(self, B: int, L: int, Hkv: int, fp8: bool = False):
        self.B, self.L, self.Hkv = B, L, Hkv
        self.fp8 = fp8            # rows are stored as per-row scaled E4M3 and attended as dequantised
        self.kc: List[List[List[Optional[np.ndarray]]]] = [[[None] * Hkv for _ in range(L)] for _ in range(B)]
        self.vc: List[List[List[Optional[np.ndarray]]]] = [[[None] * Hkv for _ in range(L)] for _ in range(B)]
        self.idx: List[List[List[Optional[np.ndarray]]]] = [[[None] * Hkv for _ in range(L)] for _ in range(B)]

    def fill_layer(self, b: int, l: int, psi_kv: np.ndarray, k_l: int, k: np.ndarray, v: np.ndarray,
                   n_recent: int = 0) -> None:
        for h in range(self.Hkv):
            idx = topk(psi_kv[h], int(k_l), n_recent)
            self.idx[b][l][h] = idx
            self.kc[b][l][h], self.vc[b][l][h] = compact(k[h], v[h], idx)
            if self.fp8:
                self.kc[b][l][h] = dequantize_e4m3_rows(*quantize_e4m3_rows(self.kc[b][l][h]))
                self.vc[b][l][h] = dequantize_e4m3_rows(*quantize_e4m3_rows(self.vc[b][l][h]))

    def decode_layer(self, l: int, q: np.ndarray, k_new: Optional[np.ndarray], v_new: Optional[np.ndarray],
                     scale: float) -> np.ndarray:
        """q [B, Hq, d], k_new, v_new [B, Hkv, d] (None: attend without appending) -> o [B, Hq, d]."""
        out = np.empty(np.asarray(q).shape, dtype=np.float64)
        for b in range(self.B):
            if k_new is not None:
                for h in range(self.Hkv):
                    kn, vn = np.asarray(k_new)[b, h][None], np.asarray(v_new)[b, h][None]
                    if self.fp8:              # quantised on append, attended as stored
                        kn = dequantize_e4m3_rows(*quantize_e4m3_rows(kn))
                        vn = dequantize_e4m3_rows(*quantize_e4m3_rows(vn))
                    self.kc[b][l][h] = np.concatenate([self.kc[b][l][h], kn], axis=0)
                    self.vc[b][l][h] = np.concatenate([self.vc[b][l][h], vn], axis=0)
            out[b] = decode_attn(q[b], self.kc[b][l], self.vc[b][l], scale)
        return out


# --------------------------------------------------------------------------------------
# Whole compression pass of one request (the order the path runs in)
# --------------------------------------------------------------------------------------

def compress_request(layers, scales, m: int, alpha_num: int, alpha_den: int, p: float = 0.01):
    """layers: sequence over l of dicts with q_win, k (v not needed here).
    Returns (psi_kv per layer, nnz [L, Hq], k [L]).  Scores and counts come first for every
    layer, because the budgets need every layer's sparsity."""
    psis, nnzs = [], []
    for l, t in enumerate(layers):
        psi_kv, _, _, _ = score(t["q_win"], t["k"], scales[l])
        nnz, _ = sparsity(t["q_win"], t["k"], scales[l], p)
        psis.append(psi_kv)
        nnzs.append(nnz)
    nnz = np.stack(nnzs)
    kk, _ = allocate(nnz, m, alpha_num, alpha_den)
    return psis, nnz, kk
