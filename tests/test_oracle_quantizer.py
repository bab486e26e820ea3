"""Pins of the oracle's quantizer, packing and Equivalent Right Shift (CPU only)."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import quantize, dequantize, pack_codes, unpack_codes, shrink_codes, shrink_scale, LEVELS
from oracle.quantizer import bytes_per_token_head

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def _half_up(fr: Fraction) -> int:
    """The rounding the appendix proof uses: X - 1/2 <= X~ < X + 1/2."""
    return (2 * fr.numerator + fr.denominator) // (2 * fr.denominator)


@pytest.mark.parametrize("b", [2, 4, 8])
def test_eq3_equals_rounded_division_exhaustive(b):
    """Appendix theorem: Eq. 3 == round(X_2b / (2^b + 1)) for every 2b-bit code; range is exactly [0, 2^b - 1]."""
    x = np.arange(1 << (2 * b), dtype=np.uint32)
    got = shrink_codes(x, b)
    want = np.array([_half_up(Fraction(int(v), (1 << b) + 1)) for v in x], dtype=np.uint32)
    assert np.array_equal(got, want)
    assert got.min() == 0 and got.max() == (1 << b) - 1
    assert np.all(np.diff(got.astype(np.int64)) >= 0)


def test_eq3_constants_match_paper():
    g = GOLD["equivalent_right_shift"]
    for b, m, o, s, f in zip(g["b"], g["multiplier"], g["offset"], g["shift"], g["scale_factor"]):
        assert m == (1 << (2 * b)) - (1 << b) + 1 and o == 1 << (b - 1) and s == 3 * b and f == (1 << b) + 1
        # (2^{2b} - 2^b + 1)(2^b + 1) = 2^{3b} + 1, the identity behind the proof
        assert m * f == (1 << (3 * b)) + 1
        # a few literal values through the oracle
        for x in (0, o, f - 1, f, (1 << (2 * b)) - 1):
            assert int(shrink_codes(np.array([x], np.uint32), b)[0]) == (m * (x + o)) >> s
    # b = 8 needs more than a signed 32-bit product
    assert 65281 * (65535 + 128) > 2 ** 31


@pytest.mark.parametrize("b", [2, 4, 8])
def test_theorem_in_exact_rationals(b):
    """quantize_b(X) == Eq.3(quantize_2b(X)) with the shared Z and max of the theorem, exact arithmetic."""
    rng = np.random.default_rng(100 + b)
    for _ in range(40):
        vals = [Fraction(float(v)) for v in rng.standard_normal(32).astype(np.float16)]
        Z, mx = min(vals), max(vals)
        if mx == Z:
            continue
        S2b = (mx - Z) / ((1 << (2 * b)) - 1)
        Sb = (mx - Z) / ((1 << b) - 1)
        assert Sb == ((1 << b) + 1) * S2b
        x2b = np.array([_half_up((v - Z) / S2b) for v in vals], np.uint32)
        xb = np.array([_half_up((v - Z) / Sb) for v in vals], np.uint32)
        assert np.array_equal(shrink_codes(x2b, b), xb)


@pytest.mark.parametrize("b", [2, 4, 8])
@pytest.mark.parametrize("group", [32, 64, 128])
def test_quantizer_roundtrip_bound_and_endpoints(b, group):
    """|x - x_hat| <= S/2 plus the fp16 rounding of S at the top code; min -> code 0 -> Z exactly; max -> top code."""
    rng = np.random.default_rng(b * 1000 + group)
    x = (rng.standard_normal((3, 5, 128)) * rng.choice([0.01, 1.0, 30.0], (3, 5, 1))).astype(np.float16)
    codes, S, Z = quantize(x, b, group)
    xh = dequantize(codes, S, Z, group)
    ng = 128 // group
    Sg = np.repeat(S.astype(np.float64), group, -1)
    err = np.abs(x.astype(np.float64) - xh)
    bound = Sg / 2 + LEVELS[b] * Sg * 2.0 ** -11 + 1e-12
    assert np.all(err <= bound)
    xg = x.reshape(3, 5, ng, group)
    cg = codes.reshape(3, 5, ng, group)
    imin, imax = xg.argmin(-1), xg.argmax(-1)
    assert np.all(np.take_along_axis(cg, imin[..., None], -1) == 0)
    assert np.all(np.take_along_axis(cg, imax[..., None], -1) == LEVELS[b])
    assert np.array_equal(Z, xg.min(-1))
    assert np.array_equal(np.take_along_axis(xh.reshape(3, 5, ng, group), imin[..., None], -1)[..., 0],
                          Z.astype(np.float64))
    # S is the fp16 rounding of the exact (max - Z)/(2^b - 1) up to one fp32 rounding before it
    exact = (xg.max(-1).astype(np.float64) - Z.astype(np.float64)) / LEVELS[b]
    assert np.all(np.abs(S.astype(np.float64) - exact) <= np.abs(exact) * (2.0 ** -11 + 2.0 ** -22) + 2.0 ** -25)
    # codes are monotone in x within a group
    order = np.argsort(xg, -1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(cg, order, -1).astype(np.int32), axis=-1) >= 0)


def test_quantizer_nearest_level():
    """Each code is a nearest lattice point of the stored (S, Z) lattice: no other code is strictly closer."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal((64, 128)).astype(np.float16)
    for b in (2, 4, 8):
        codes, S, Z = quantize(x, b, 32)
        Sg = np.repeat(S.astype(np.float64), 32, -1)
        Zg = np.repeat(Z.astype(np.float64), 32, -1)
        xd = x.astype(np.float64)
        e0 = np.abs(xd - (codes * Sg + Zg))
        for d in (-1, 1):
            c2 = np.clip(codes.astype(np.int32) + d, 0, LEVELS[b])
            e1 = np.abs(xd - (c2 * Sg + Zg))
            # fp32 evaluation of (x - Z)/S may flip a near-tie: allow a relative 2^-20 slack
            assert np.all(e0 <= e1 + Sg * 2.0 ** -20)


def test_constant_group_and_tie_rule():
    x = np.full((1, 128), 0.75, np.float16)
    codes, S, Z = quantize(x, 4, 32)
    assert np.all(codes == 0) and np.all(S == 0) and np.all(Z == np.float16(0.75))
    assert np.array_equal(dequantize(codes, S, Z, 32), np.full((1, 128), 0.75))
    assert np.all(shrink_scale(S, 2) == 0)
    # ties go to even: group spanning 0..3 at b = 2 has S = 1; 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    g = np.zeros(32, np.float16)
    g[:5] = [0.0, 3.0, 0.5, 1.5, 2.5]
    codes, S, Z = quantize(g[None], 2, 32)
    assert S[0, 0] == 1 and Z[0, 0] == 0
    assert codes[0, :5].tolist() == [0, 3, 0, 2, 2]


def test_shrink_chain_keeps_dynamic_range_and_bound():
    """After 8 -> 4 -> 2 the top code still de-quantizes to ~max and the error bound is S_b/2 (+ fp16 terms)."""
    rng = np.random.default_rng(11)
    x = rng.standard_normal((200, 128)).astype(np.float16)
    codes, S, Z = quantize(x, 8, 32)
    for b in (4, 2):
        codes, S = shrink_codes(codes, b), shrink_scale(S, b)
        assert codes.max() <= LEVELS[b]
        xh = dequantize(codes, S, Z, 32)
        Sg = np.repeat(S.astype(np.float64), 32, -1)
        assert np.all(np.abs(x.astype(np.float64) - xh) <= Sg / 2 + 4 * LEVELS[b] * Sg * 2.0 ** -11 + 1e-12)
    # shrinking the codes of a direct 2b-bit quantization gives the direct b-bit codes except where the
    # fp16 rounding of S moves a value across a rounding boundary: rare, and never by more than one level
    c4, _, _ = quantize(x, 4, 32)
    c2, _, _ = quantize(x, 2, 32)
    diff = np.abs(shrink_codes(c4, 2).astype(np.int32) - c2.astype(np.int32))
    assert diff.max() <= 1 and (diff != 0).mean() < 0.02


def test_scale_update_is_exact_product():
    S = np.array([0.1234, 1.0, 3.0e-4, 17.5], np.float16)
    for b, f in ((8, 257), (4, 17), (2, 5)):
        want = np.array([np.float16(np.float32(float(s) * f)) for s in S], np.float16)
        assert np.array_equal(shrink_scale(S, b), want)
        # products of an 11-bit and a <= 9-bit significand are exact in fp32, so only one rounding happens
        for s in S:
            assert float(np.float32(s) * np.float32(f)) == float(s) * f


@pytest.mark.parametrize("b", [2, 4, 8])
def test_packing_layout(b):
    rng = np.random.default_rng(b)
    codes = rng.integers(0, 1 << b, (4, 3, 128), dtype=np.uint8)
    p = pack_codes(codes, b)
    assert p.shape == (4, 3, 128 * b // 8) and p.dtype == np.uint8
    assert np.array_equal(unpack_codes(p, b), codes)
    # element i lives at bit (i*b) % 8 of byte (i*b)//8, low bits first
    for i in (0, 1, 5, 127):
        byte, sh = (i * b) // 8, (i * b) % 8
        assert np.array_equal((p[..., byte] >> sh) & ((1 << b) - 1), codes[..., i])


def test_packing_literals():
    assert pack_codes(np.array([[1, 2, 3, 0]], np.uint8), 2).tolist() == [[0x39]]
    assert pack_codes(np.array([[0xA, 0x5]], np.uint8), 4).tolist() == [[0x5A]]
    assert pack_codes(np.array([[200, 7]], np.uint8), 8).tolist() == [[200, 7]]


def test_table1_byte_counts():
    """Table 1: 16-bit KV cache of batch 16 x 32K context is 64 / 128 / 160 GB."""
    t = GOLD["table1_kv_cache_gb"]
    for row in t["rows"]:
        per = bytes_per_token_head(16, row["head_dim"], 128, True)
        assert per == 512
        total = row["layers"] * row["kv_heads"] * per * t["context"] * t["batch"]
        assert total == row["kv_gb"] * 2 ** 30
    assert [bytes_per_token_head(b, 128, 32, True) for b in (16, 8, 4, 2)] == [512, 288, 160, 96]
    assert [bytes_per_token_head(b, 128, 128, True) for b in (16, 8, 4, 2)] == [512, 264, 136, 72]
    assert [bytes_per_token_head(b, 128, 32, False) for b in (16, 8, 4, 2)] == [512, 256, 128, 64]


# ---------------------------------------------------------------- the ablation's two other shift strategies (Sec. 4.3.1)
def test_direct_and_modified_shift_properties_stated_by_the_paper():
    """Direct Right Shift keeps the upper b bits and the dynamic range (Z_b = Z_2b, S_b = (2^b + 1) S_2b);
    Modified Right Shift maps levels that share their upper b bits to their mean (S_b = 2^b S_2b,
    Z_b = Z_2b + (S_b - S_2b) / 2).  Checked in exact rationals for every 2b-bit code."""
    from fractions import Fraction
    from oracle import shrink_step, SHIFT_DIRECT, SHIFT_MODIFIED
    S2, Z2 = Fraction(3, 64), Fraction(-7, 8)          # exactly representable in fp16
    for b in (4, 2):
        codes = np.arange(1 << (2 * b), dtype=np.uint8 if b < 8 else np.uint16)
        S16, Z16 = np.array([float(S2)], np.float16), np.array([float(Z2)], np.float16)
        xd, Sd, Zd = shrink_step(codes, S16, Z16, b, SHIFT_DIRECT)
        xm, Sm, Zm = shrink_step(codes, S16, Z16, b, SHIFT_MODIFIED)
        assert np.array_equal(xd, codes >> b) and np.array_equal(xm, codes >> b)
        Sd_, Zd_, Sm_, Zm_ = (Fraction(float(v[0])) for v in (Sd, Zd, Sm, Zm))
        assert Sd_ == ((1 << b) + 1) * S2 and Zd_ == Z2
        # dynamic range kept: the top and bottom levels de-quantize to the same values as before
        assert Zd_ + int(xd[-1]) * Sd_ == Z2 + int(codes[-1]) * S2 and Zd_ + int(xd[0]) * Sd_ == Z2
        assert Sm_ == (1 << b) * S2 and Zm_ == Z2 + (Sm_ - S2) / 2
        for k in range(1 << b):                         # bucket k: codes k 2^b .. k 2^b + 2^b - 1
            bucket = [Z2 + c * S2 for c in range(k << b, (k + 1) << b)]
            assert Zm_ + k * Sm_ == sum(bucket) / len(bucket)


def test_shift_strategies_reconstruction_error_ordering_on_uniform_codes():
    """Closed forms for codes uniform over [0, 2^{2b}): mean squared distance between a 2b-bit level and its
    b-bit image, in units of S_2b^2.  Modified = (4^b - 1)/12 (within-bucket variance); Equivalent =
    round-to-nearest on a grid of step 2^b + 1; Direct is the largest of the three.  These fix the arithmetic of
    all three strategies independently of the implementation."""
    from oracle import shrink_step, SHIFT_EQUIVALENT, SHIFT_DIRECT, SHIFT_MODIFIED
    one, zero = np.array([1.0], np.float16), np.array([0.0], np.float16)
    for b in (4, 2):
        n = 1 << (2 * b)
        codes = np.arange(n, dtype=np.uint8)
        mse = {}
        for st in (SHIFT_EQUIVALENT, SHIFT_DIRECT, SHIFT_MODIFIED):
            xb, S, Z = shrink_step(codes, one, zero, b, st)
            rec = xb.astype(np.float64) * float(S[0]) + float(Z[0])
            mse[st] = float(np.mean((rec - codes) ** 2))
        assert mse[SHIFT_MODIFIED] == pytest.approx(((1 << b) ** 2 - 1) / 12.0)
        brute_eq = np.mean([(((2 ** b) + 1) * round_half_up(c / ((2 ** b) + 1)) - c) ** 2 for c in range(n)])
        assert mse[SHIFT_EQUIVALENT] == pytest.approx(brute_eq)
        brute_dir = np.mean([(((2 ** b) + 1) * (c >> b) - c) ** 2 for c in range(n)])
        assert mse[SHIFT_DIRECT] == pytest.approx(brute_dir)
        assert mse[SHIFT_DIRECT] > mse[SHIFT_EQUIVALENT] and mse[SHIFT_DIRECT] > mse[SHIFT_MODIFIED]


def round_half_up(x):
    import math
    return math.floor(x + 0.5)


# ------------------------------------------------------------------------------- rotary embedding of the keys (Eq. 9)
def test_rope_rotation_of_keys():
    """The fp32 rotation agrees with the fp64 rotation of the input generator to fp16 rounding, keeps the norm of
    every (i, i + D/2) pair, is the identity at position 0, and a quarter turn swaps the pair with a sign."""
    import kvq_synth
    from oracle import rope_rotate_keys
    rng = np.random.default_rng(9)
    K = rng.standard_normal((1, 2, 40, 128)).astype(np.float16)
    pos = np.arange(1000, 1040)
    cos, sin = kvq_synth.rope_tables(pos, 1.0e4)
    got = rope_rotate_keys(K, cos, sin).astype(np.float64)
    want = kvq_synth.rope_rotate(K.astype(np.float64), pos, 1.0e4)
    assert np.abs(got - want).max() <= 2.0 ** -10 * np.abs(want).max()
    n0 = K.astype(np.float64)[..., :64] ** 2 + K.astype(np.float64)[..., 64:] ** 2
    n1 = got[..., :64] ** 2 + got[..., 64:] ** 2
    assert np.allclose(n0, n1, rtol=4e-3, atol=1e-5)
    c0, s0 = kvq_synth.rope_tables(np.zeros(40), 1.0e4)
    assert np.array_equal(rope_rotate_keys(K, c0, s0), K)
    cq, sq = np.zeros((40, 64), np.float32), np.ones((40, 64), np.float32)      # quarter turn: (a, b) -> (-b, a)
    r = rope_rotate_keys(K, cq, sq)
    assert np.array_equal(r[..., :64], -K[..., 64:]) and np.array_equal(r[..., 64:], K[..., :64])
