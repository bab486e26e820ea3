"""Single-token grouped-query attention in fp64 (oracle, test infrastructure)."""
from __future__ import annotations

import numpy as np


def decode_attention_fp64(q: np.ndarray, K_hat: np.ndarray, V_hat: np.ndarray, scale: float | None = None):
    """softmax(q K_hat^T * scale) V_hat for one query token per sequence.

    q: [B, Hq, D]; K_hat, V_hat: [B, Hkv, T, D] (already de-quantized); query head h reads
    KV head h // (Hq // Hkv).  No mask: every cached token is attended.  scale defaults to
    1/sqrt(D).  Two-pass softmax with the maximum subtracted, all in fp64.
    Returns [B, Hq, D] float64.
    """
    q = q.astype(np.float64)
    K_hat = K_hat.astype(np.float64)
    V_hat = V_hat.astype(np.float64)
    B, Hq, D = q.shape
    Hkv = K_hat.shape[1]
    g = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.empty((B, Hq, D), np.float64)
    for b in range(B):
        for h in range(Hq):
            s = (K_hat[b, h // g] @ q[b, h]) * scale          # [T]
            p = np.exp(s - s.max())
            p /= p.sum()
            out[b, h] = p @ V_hat[b, h // g]
    return out
