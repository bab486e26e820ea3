"""Seeded synthetic inputs for the PM-KVQ hot path (keys, values, queries, workload shapes).

This module serves both the CPU oracle's tests and the HIP path's tests/bench.  It holds
input generation only: Gaussian draws, the persistent outlier-channel gain the paper
describes for key tensors (Sec. 3.3, first paragraph), and the rotary embedding that the
keys and queries carry when they reach the cache (Sec. 3.3, Eq. 9).  None of the method's
own arithmetic (quantizer, packing, bit-width shrinking, attention) lives here.
"""
from __future__ import annotations

import dataclasses
import numpy as np

HEAD_DIM = 128


def rope_rotate(x: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing (Sec. 3.3, Eq. 9).

    Channel i is paired with channel i + d/2 and the pair is rotated by the angle
    m * theta_i with theta_i = base ** (-2 i / d), m the token position.
    x: [..., T, d] float64/float32, positions: [T].  Returns the same shape/dtype.
    """
    d = x.shape[-1]
    half = d // 2
    i = np.arange(half, dtype=np.float64)
    theta = base ** (-2.0 * i / d)
    ang = positions.astype(np.float64)[:, None] * theta[None, :]
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = a * c - b * s
    out[..., half:] = a * s + b * c
    return out


def _unit_rng(seed: int, layer: int, b: int, h: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(layer), int(b), int(h), int(stream)])


def rope_tables(positions: np.ndarray, base: float, d: int = HEAD_DIM):
    """cos(m theta_i), sin(m theta_i) as fp32 [len(positions), d/2], theta_i = base ** (-2 i / d) (Sec. 3.3, Eq. 9);
    positions may be fractional (interpolated, Eq. 10).  Angles and functions are evaluated in fp64."""
    i = np.arange(d // 2, dtype=np.float64)
    ang = np.asarray(positions, np.float64)[:, None] * (base ** (-2.0 * i / d))[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def outlier_channels(seed: int, h: int, d: int = HEAD_DIM, n_out: int = 4) -> np.ndarray:
    """The seeded outlier channel set of KV head h (same set for every token and layer)."""
    return np.sort(np.random.default_rng([int(seed), 9001, int(h)]).choice(d, n_out, replace=False))


def make_kv_unit(seed: int, layer: int, b: int, h: int, t0: int, t1: int, d: int = HEAD_DIM,
                 rope_base: float | None = 1.0e6, outlier_gain: float = 20.0, n_out: int = 4,
                 pos_scale: float = 1.0):
    """K and V (fp16, [t1-t0, d]) of one (layer, sequence b, KV head h) for tokens t0..t1-1.

    Every 1024-token block of a unit has its own counter-based stream, so any token range
    can be produced without generating the tokens before it.  pos_scale: token m is rotated
    at position pos_scale * m (positional interpolation of calibration data, Sec. 3.3, Eq. 10).
    """
    BLK = 1024
    ks, vs = [], []
    gain = np.ones(d)
    gain[outlier_channels(seed, h, d, n_out)] = outlier_gain
    for blk in range(t0 // BLK, (t1 + BLK - 1) // BLK):
        rk = _unit_rng(seed, layer, b, h, 2 * blk)
        rv = _unit_rng(seed, layer, b, h, 2 * blk + 1)
        k = rk.standard_normal((BLK, d), dtype=np.float32).astype(np.float64) * gain
        v = rv.standard_normal((BLK, d), dtype=np.float32)
        if rope_base is not None:
            k = rope_rotate(k, pos_scale * np.arange(blk * BLK, (blk + 1) * BLK), rope_base)
        lo, hi = max(t0, blk * BLK) - blk * BLK, min(t1, (blk + 1) * BLK) - blk * BLK
        ks.append(k[lo:hi].astype(np.float16))
        vs.append(v[lo:hi].astype(np.float16))
    if not ks:
        return np.zeros((0, d), np.float16), np.zeros((0, d), np.float16)
    return np.concatenate(ks, 0), np.concatenate(vs, 0)


def make_kv(seed: int, layer: int, batch: int, n_kv: int, t0: int, t1: int, d: int = HEAD_DIM,
            rope_base: float | None = 1.0e6, outlier_gain: float = 20.0, pos_scale: float = 1.0):
    """K, V fp16 [batch, n_kv, t1-t0, d] for one layer."""
    K = np.empty((batch, n_kv, t1 - t0, d), np.float16)
    V = np.empty_like(K)
    for b in range(batch):
        for h in range(n_kv):
            K[b, h], V[b, h] = make_kv_unit(seed, layer, b, h, t0, t1, d, rope_base, outlier_gain, pos_scale=pos_scale)
    return K, V


def make_q(seed: int, layer: int, batch: int, n_q: int, pos: int, d: int = HEAD_DIM,
           rope_base: float | None = 1.0e6) -> np.ndarray:
    """One decode step's queries, fp16 [batch, n_q, d], rotated at position pos."""
    r = np.random.default_rng([int(seed), int(layer), 7777, int(pos)])
    q = r.standard_normal((batch, n_q, 1, d), dtype=np.float32).astype(np.float64)
    if rope_base is not None:
        q = rope_rotate(q, np.array([pos]), rope_base)
    return q[:, :, 0, :].astype(np.float16)


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one synthetic cache state: tiers are (n_tokens, bits) oldest to newest."""
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    tiers: tuple          # ((n_tokens, bits), ...) oldest -> newest; per-layer override below
    page_tokens: int
    seed: int
    rope_base: float | None = 1.0e6
    group: int = 32
    head_dim: int = HEAD_DIM
    layer_bits: tuple | None = None   # 14B-shaped: bulk bit-width drawn per layer

    @property
    def n_tokens(self) -> int:
        return sum(n for n, _ in self.tiers)

    def tiers_of_layer(self, layer: int):
        if self.layer_bits is None:
            return self.tiers
        return tuple((n, self.layer_bits[layer] if b == 0 else b) for n, b in self.tiers)


def _layer_bits_14b(n_layers: int, seed: int):
    return tuple(int(x) for x in np.random.default_rng([seed, 4242]).choice([2, 4, 8], n_layers))


WORKLOADS = {
    # 1 layer, 8 q / 2 kv heads, 4 x 1,024 tokens at 2/4/8/16 bits, outlier gain applied directly, no RoPE
    "tiny": Workload("tiny", 1, 1, 8, 2, ((1024, 2), (1024, 4), (1024, 8), (1024, 16)), 256, 0, rope_base=None),
    "7b": Workload("7b", 28, 16, 28, 4, ((32256, 4), (512, 16)), 256, 7),
    "14b": Workload("14b", 48, 8, 40, 8, ((32256, 0), (512, 16)), 256, 14, layer_bits=_layer_bits_14b(48, 14)),
    "32b": Workload("32b", 64, 4, 40, 8, ((16384, 2), (8192, 4), (8064, 8), (128, 16)), 128, 32),
    "70b": Workload("70b", 80, 1, 64, 8, ((81920, 2), (40960, 4), (7168, 8), (1024, 16)), 1024, 70),
}
