"""Block-wise memory allocation of the oracle (test infrastructure): sensitivities (Sec. 3.2, Eq. 5) and the
integer program that assigns one bit-width to every transformer block under a memory budget (Sec. 3.2, Eq. 6).
"""
from __future__ import annotations

import itertools

import numpy as np

from .quantizer import quantize, dequantize


def sensitivity(K: np.ndarray, V: np.ndarray, b: int, group: int, GK: np.ndarray | None = None,
                GV: np.ndarray | None = None):
    """s_{i,b} of Eq. 5 for one block, as its two terms: (|| G_K * (K - Q_b(K)) ||_1, || G_V * (V - Q_b(V)) ||_1),
    Q_b the b-bit quantizer of Eq. 1-2 followed by de-quantization, * the element-wise product.  G_K, G_V are the
    gradients of the loss with respect to K and V; None stands for all-ones (no model: plain L1 reconstruction error).
    K, V fp16 [batch, n_kv_heads, T, D]; gradients fp32 of the same shape.  Sums in fp64.  b = 16 gives (0, 0)."""
    out = []
    for X, G in ((K, GK), (V, GV)):
        if b == 16:
            out.append(0.0)
            continue
        c, S, Z = quantize(X, b, group)
        d = np.abs(dequantize(c, S, Z, group) - X.astype(np.float64))
        if G is not None:
            d = d * np.abs(G.astype(np.float64))
        out.append(float(d.sum()))
    return tuple(out)


def allocate_bits_bruteforce(s: np.ndarray, mem: np.ndarray, budget: int):
    """Eq. 6 by enumeration: choose one column per row of s [N, C] (x_{i,b} one-hot) minimising the sum of the chosen
    s under sum of the chosen mem [N, C] <= budget.  Returns (choice [N] or None if nothing fits, total s, total mem).
    Ties are broken towards the smaller memory, then the lexicographically smaller choice."""
    N, C = s.shape
    best = None
    for ch in itertools.product(range(C), repeat=N):
        m = int(sum(int(mem[i, c]) for i, c in enumerate(ch)))
        if m > budget:
            continue
        cost = float(sum(float(s[i, c]) for i, c in enumerate(ch)))
        key = (cost, m, ch)
        if best is None or key < best:
            best = key
    if best is None:
        return None, float("inf"), 0
    return np.array(best[2], np.int32), best[0], best[1]


def allocate_bits_dp(s: np.ndarray, mem: np.ndarray, budget: int):
    """Eq. 6 by dynamic programming over the budget in units of the greatest common divisor of all memory sizes
    (the textbook multiple-choice knapsack recurrence); exact.  Same return as the enumeration (cost ties may pick
    another, equally good, choice)."""
    N, C = s.shape
    g = int(np.gcd.reduce(mem.astype(np.int64).ravel()))
    g = max(g, 1)
    W = int(budget // g)
    w = (mem.astype(np.int64) // g)
    INF = float("inf")
    best = np.full((N + 1, W + 1), INF)
    best[0, :] = 0.0
    pick = np.full((N + 1, W + 1), -1, np.int32)
    for i in range(N):
        for cap in range(W + 1):
            for c in range(C):
                if w[i, c] <= cap and best[i, cap - w[i, c]] + s[i, c] < best[i + 1, cap]:
                    best[i + 1, cap] = best[i, cap - w[i, c]] + s[i, c]
                    pick[i + 1, cap] = c
    if not np.isfinite(best[N, W]):
        return None, INF, 0
    ch = np.empty(N, np.int32)
    cap = W
    for i in range(N, 0, -1):
        ch[i - 1] = pick[i, cap]
        cap -= w[i - 1, ch[i - 1]]
    total_mem = int(sum(int(mem[i, ch[i]]) for i in range(N)))
    return ch, float(best[N, W]), total_mem
