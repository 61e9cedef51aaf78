"""Pure-loop brute force of the VL-Cache definitions, for inputs of a few dozen tokens.
TEST INFRASTRUCTURE ONLY: it is what the numpy oracle is checked against.

Everything is written entry by entry with Python floats (fp64) and the formulas are
the paper's literal ones: the ThresholdFilter compares attention scores
(A_ij >= p max_j A_ij, Eq. 1), sparsity counts zeroed entries of the causal region
(Eq. 2 / Alg. 1), budgets are the printed float formula, TopK is a full sort.
"""
from __future__ import annotations

import math
from typing import List


def attention_rows(q_win, k, scale) -> List[List[List[float]]]:
    """A'[h][i][j] for j <= m - tau + i, 0 elsewhere (Alg. 1: softmax(Q'K^T / sqrt d), causal)."""
    Hq, tau, d = len(q_win), len(q_win[0]), len(q_win[0][0])
    Hkv, m = len(k), len(k[0])
    g = Hq // Hkv
    A = []
    for h in range(Hq):
        rows = []
        for i in range(tau):
            last = m - tau + i
            s = []
            for j in range(last + 1):
                acc = 0.0
                for e in range(d):
                    acc += float(q_win[h][i][e]) * float(k[h // g][j][e])
                s.append(acc * scale)
            mx = max(s)
            ex = [math.exp(x - mx) for x in s]
            z = sum(ex)
            rows.append([x / z for x in ex] + [0.0] * (m - last - 1))
        A.append(rows)
    return A


def scores_kv(q_win, k, scale) -> List[List[float]]:
    """psi_kv[hkv][j] = sum over the group's query heads and window rows of A'."""
    A = attention_rows(q_win, k, scale)
    Hq, Hkv, m = len(q_win), len(k), len(k[0])
    g = Hq // Hkv
    out = [[0.0] * m for _ in range(Hkv)]
    for h in range(Hq):
        for row in A[h]:
            for j, a in enumerate(row):
                out[h // g][j] += a
    return out


def sparsity_literal(q_win, k, scale, p):
    """Eq. 1 + Eq. 2 on the post-vision rows: count entries of the causal region with
    A_ij < p max_j A_ij (zeroed by the filter), divide by the region's size."""
    A = attention_rows(q_win, k, scale)
    tau, m = len(q_win[0]), len(k[0])
    gammas, nnzs = [], []
    for h in range(len(A)):
        zeroed = 0
        size = 0
        for i in range(tau):
            last = m - tau + i
            mx = max(A[h][i][: last + 1])
            for j in range(last + 1):
                size += 1
                if not (A[h][i][j] >= p * mx):
                    zeroed += 1
        gammas.append(zeroed / size)
        nnzs.append(size - zeroed)
    return nnzs, gammas


def budgets_literal(gamma_lh, alpha):
    """Alg. 1 as printed (floats)."""
    L = len(gamma_lh)
    gm = [sum(row) / len(row) for row in gamma_lh]
    Z = sum(1.0 - x for x in gm)
    return [min(max((1.0 - x) / Z * alpha * L, 0.01), 1.0) for x in gm]


def topk_sorted(psi, k):
    """Full sort by (score descending, index ascending), first k, returned ascending."""
    order = sorted(range(len(psi)), key=lambda j: (-psi[j], j))
    return sorted(order[:k])


def attend(q, K, V, scale):
    """Textbook attention of one query vector over n slots."""
    n, d = len(K), len(q)
    s = [scale * sum(float(q[e]) * float(K[r][e]) for e in range(d)) for r in range(n)]
    mx = max(s)
    ex = [math.exp(x - mx) for x in s]
    z = sum(ex)
    return [sum(ex[r] / z * float(V[r][e]) for r in range(n)) for e in range(len(V[0]))]
