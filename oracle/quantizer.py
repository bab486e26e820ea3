"""Quantizer, packing and bit-width shrinking of the oracle (test infrastructure).

Notation follows the paper: X the 16-bit tensor, Z the zero point, S the scaling factor,
b the bit-width, X_b the b-bit integer tensor.
"""
from __future__ import annotations

import numpy as np

LEVELS = {16: 65535, 8: 255, 4: 15, 2: 3}


def quantize(x: np.ndarray, b: int, group: int):
    """Asymmetric uniform group-wise quantization (Sec. 2.2, Eq. 1 and Eq. 2).

    x: fp16 [..., D]; a group is `group` consecutive channels of one token of one head.
    Z = min(X) per group, S = (max(X) - Z) / (2^b - 1); both are stored as fp16.  The
    subtraction and the division for S are single IEEE fp32 operations and S is rounded
    to nearest-even into fp16; the codes are round-to-nearest-even of (X - Z) / S in fp32
    with the *stored* S, clamped to [0, 2^b - 1].  A group with S == 0 has all codes 0.
    Returns (codes uint8 [..., D], S fp16 [..., D/group], Z fp16 [..., D/group]).

    b = 16 is the integer 16-bit tier (the "INT16 format" of Sec. 4.1.2, the X_2b of the appendix theorem at
    b = 8): same formulas with 2^16 - 1 levels, codes uint16.  With S held in fp16 the clamp is essential there:
    S rounded down by up to 2^-11 puts (max - Z) / S as far as ~32 above 65535, and below a group range of ~4 the
    scale is an fp16 subnormal with fewer significant bits still.
    """
    assert x.dtype == np.float16 and b in LEVELS and x.shape[-1] % group == 0
    assert np.all(np.isfinite(x))
    g = x.reshape(x.shape[:-1] + (x.shape[-1] // group, group))
    Z = g.min(axis=-1)
    mx = g.max(axis=-1)
    S32 = (mx.astype(np.float32) - Z.astype(np.float32)) / np.float32(LEVELS[b])
    S = S32.astype(np.float16)
    assert np.all(np.isfinite(S))
    Sf = S.astype(np.float32)[..., None]
    num = g.astype(np.float32) - Z.astype(np.float32)[..., None]
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.rint(num / Sf)
    r = np.where(Sf == 0, np.float32(0), r)
    codes = np.clip(r, 0, LEVELS[b]).astype(np.uint16 if b == 16 else np.uint8)
    return codes.reshape(x.shape), S, Z


def dequantize(codes: np.ndarray, S: np.ndarray, Z: np.ndarray, group: int) -> np.ndarray:
    """X_hat = X_b * S + Z in fp64 (the product is exact: a code of at most 16 bits times an 11-bit significand)."""
    ng = codes.shape[-1] // group
    c = codes.reshape(codes.shape[:-1] + (ng, group)).astype(np.float64)
    out = c * S.astype(np.float64)[..., None] + Z.astype(np.float64)[..., None]
    return out.reshape(codes.shape)


def shrink_codes(x2b: np.ndarray, b: int) -> np.ndarray:
    """Equivalent Right Shift (Sec. 3.1, Eq. 3): X_b = ((2^{2b} - 2^b + 1)(X_{2b} + 2^{b-1})) >> 3b.

    x2b holds 2b-bit codes; b is the target width.  Evaluated in unsigned 64-bit integers.  The result keeps the
    dtype of x2b, except that 16-bit codes (uint16) come back as the uint8 every narrower width is held in.
    """
    assert b in (8, 4, 2)
    x = x2b.astype(np.uint64)
    mult = np.uint64((1 << (2 * b)) - (1 << b) + 1)
    y = (mult * (x + np.uint64(1 << (b - 1)))) >> np.uint64(3 * b)
    return y.astype(np.uint8 if x2b.dtype == np.uint16 else x2b.dtype)


def shrink_scale(S2b: np.ndarray, b: int) -> np.ndarray:
    """S_b = (2^b + 1) S_{2b} (Sec. 3.1, below Eq. 3); the fp32 product is rounded to fp16.  Z is kept."""
    out = (S2b.astype(np.float32) * np.float32((1 << b) + 1)).astype(np.float16)
    assert np.all(np.isfinite(out))
    return out


LAMBDA_FLOOR = np.float32(1.0e-5)   # |K| maxima below this count as this (a channel that is zero everywhere)


def calibrate_lambda(K_calib: np.ndarray, alpha: float) -> np.ndarray:
    """Channel-wise reparameterization factors (Sec. 3.3, Eq. 8): lambda_i = (max_m |K_{m,i}|)^alpha.

    K_calib: fp16 [batch, n_kv_heads, T, D] (rotated keys of the calibration sequences); the maximum runs over
    the sequences and token positions m of one KV head.  The maximum of the magnitude is taken (an outlier
    channel may be negative), floored at LAMBDA_FLOOR.  Returns fp32 [n_kv_heads, D]; pow is evaluated in fp64
    and rounded to fp32.
    """
    assert K_calib.dtype == np.float16 and K_calib.ndim == 4
    mx = np.abs(K_calib.astype(np.float32)).max(axis=(0, 2))
    mx = np.maximum(mx, LAMBDA_FLOOR)
    return np.power(mx.astype(np.float64), float(alpha)).astype(np.float32)


def reparam_keys(K: np.ndarray, lam: np.ndarray) -> np.ndarray:
    """K Lambda^{-1} of Eq. 7: every channel i of KV head h is multiplied by the fp32 reciprocal 1/lambda_{h,i}
    (one correctly rounded fp32 division per channel, one fp32 product per element), rounded to fp16."""
    assert K.dtype == np.float16 and lam.dtype == np.float32 and lam.shape == (K.shape[1], K.shape[3])
    r = (np.float32(1.0) / lam)[None, :, None, :]
    out = (K.astype(np.float32) * r).astype(np.float16)
    assert np.all(np.isfinite(out))
    return out


def reparam_queries(q: np.ndarray, lam: np.ndarray, n_kv_heads: int) -> np.ndarray:
    """Q Lambda of Eq. 7: query head h uses the factors of KV head h // (n_q_heads / n_kv_heads); fp32 product
    rounded to fp16.  q: fp16 [batch, n_q_heads, D]."""
    assert q.dtype == np.float16 and lam.dtype == np.float32
    g = q.shape[1] // n_kv_heads
    out = (q.astype(np.float32) * np.repeat(lam, g, axis=0)[None]).astype(np.float16)
    assert np.all(np.isfinite(out))
    return out


def rope_rotate_keys(K: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotary embedding of un-rotated keys (Sec. 3.3, Eq. 9), channel i paired with i + D/2:
        K~_i       = K_i cos_i - K_{i+D/2} sin_i
        K~_{i+D/2} = K_i sin_i + K_{i+D/2} cos_i
    K: fp16 [batch, n_kv_heads, T, D]; cos, sin: fp32 [T, D/2], the values of cos(m theta_i), sin(m theta_i) for the
    T token positions (inputs: whoever produces them decides positions, base and interpolation).  Every product
    and the sum are separate IEEE fp32 operations (no fused multiply-add); the result is rounded to fp16."""
    assert K.dtype == np.float16 and cos.dtype == np.float32 and sin.dtype == np.float32
    half = K.shape[-1] // 2
    assert cos.shape == sin.shape == (K.shape[2], half)
    a, b = K[..., :half].astype(np.float32), K[..., half:].astype(np.float32)
    c, s = cos[None, None], sin[None, None]
    lo = (a * c).astype(np.float32) - (b * s).astype(np.float32)
    hi = (a * s).astype(np.float32) + (b * c).astype(np.float32)
    return np.concatenate([lo, hi], -1).astype(np.float16)


SHIFT_EQUIVALENT, SHIFT_DIRECT, SHIFT_MODIFIED = 0, 1, 2


def shrink_step(x2b: np.ndarray, S2b: np.ndarray, Z2b: np.ndarray, b: int, strategy: int):
    """One 2b -> b bit-width shrinking step under one of the three strategies of the ablation in Sec. 4.3.1.

    Equivalent Right Shift (the method's own, Eq. 3): X_b = ((2^{2b} - 2^b + 1)(X_{2b} + 2^{b-1})) >> 3b,
        S_b = (2^b + 1) S_{2b}, Z_b = Z_{2b}.
    Direct Right Shift: X_b = X_{2b} >> b (the upper b bits), S_b = (2^b + 1) S_{2b}, Z_b = Z_{2b}: the dynamic
        range [Z, Z + (2^{2b} - 1) S_{2b}] is preserved.
    Modified Right Shift: X_b = X_{2b} >> b, S_b = 2^b S_{2b}, Z_b = Z_{2b} + (S_b - S_{2b}) / 2: a b-bit level is the
        mean of the 2b-bit levels that share its upper b bits.
    S and Z are fp16: products and the sum are formed in fp32 (the products are exact there) and rounded to
    nearest-even into fp16.  Returns (X_b, S_b, Z_b).
    """
    assert b in (8, 4, 2) and strategy in (SHIFT_EQUIVALENT, SHIFT_DIRECT, SHIFT_MODIFIED)
    Sf, Zf = S2b.astype(np.float32), Z2b.astype(np.float32)
    if strategy == SHIFT_EQUIVALENT:
        return shrink_codes(x2b, b), shrink_scale(S2b, b), Z2b.copy()
    xb = (x2b.astype(np.uint64) >> np.uint64(b)).astype(np.uint8 if x2b.dtype == np.uint16 else x2b.dtype)
    if strategy == SHIFT_DIRECT:
        return xb, shrink_scale(S2b, b), Z2b.copy()
    Sb32 = Sf * np.float32(1 << b)
    half = np.float32(0.5) * (Sb32 - Sf)          # = S_2b (2^b - 1) / 2, exact in fp32
    Sb, Zb = Sb32.astype(np.float16), (Zf + half).astype(np.float16)
    assert np.all(np.isfinite(Sb)) and np.all(np.isfinite(Zb))
    return xb, Sb, Zb


def pack_codes(codes: np.ndarray, b: int) -> np.ndarray:
    """Canonical packing: element i of a row sits at bit offset (i*b) mod 8 of byte (i*b)//8, low bits first
    (16-bit codes: two bytes, low byte first)."""
    if b == 16:
        c = codes.astype(np.uint16)
        return np.stack([(c & 0xff).astype(np.uint8), (c >> 8).astype(np.uint8)], -1).reshape(c.shape[:-1] + (2 * c.shape[-1],))
    per = 8 // b
    c = codes.reshape(codes.shape[:-1] + (codes.shape[-1] // per, per)).astype(np.uint16)
    out = np.zeros(c.shape[:-1], np.uint16)
    for j in range(per):
        out |= c[..., j] << (j * b)
    return out.astype(np.uint8)


def unpack_codes(packed: np.ndarray, b: int) -> np.ndarray:
    if b == 16:
        p = packed.reshape(packed.shape[:-1] + (packed.shape[-1] // 2, 2)).astype(np.uint16)
        return p[..., 0] | (p[..., 1] << 8)
    per = 8 // b
    out = np.empty(packed.shape + (per,), np.uint8)
    for j in range(per):
        out[..., j] = (packed >> (j * b)) & ((1 << b) - 1)
    return out.reshape(packed.shape[:-1] + (packed.shape[-1] * per,))


def bytes_per_token_head(bits: int, head_dim: int, group: int, count_metadata: bool, int16_tier: bool = False) -> int:
    """Bytes one cached token of one KV head occupies, K and V together.

    Codes: 2 * head_dim * bits / 8.  Quantized widths also carry one fp16 (S, Z) pair per
    group for K and for V when metadata is counted; 16-bit tokens do when the 16-bit tier holds integer codes.
    """
    n = 2 * head_dim * bits // 8
    if count_metadata and (bits < 16 or int16_tier):
        n += 2 * (head_dim // group) * 4
    return n
