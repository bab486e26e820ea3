"""Pins of the oracle's integer 16-bit tier (the INT16 format of Sec. 4.1.2; X_2b of the appendix theorem at b = 8)."""
from fractions import Fraction

import numpy as np
import pytest

import kvq_synth
from oracle import (OracleCache, CacheConfig, BudgetError, POLICY_PAPER, POLICY_OLDEST_FIRST, TIER16_INT16, TIER16_FP16,
                    quantize, dequantize, shrink_codes, shrink_scale, shrink_step, pack_codes, unpack_codes,
                    bytes_per_token_head, decode_attention_fp64, SHIFT_EQUIVALENT, SHIFT_DIRECT, SHIFT_MODIFIED)


def _data(seed, n=400):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, 128)) * rng.choice([0.05, 1.0, 30.0], (n, 1))).astype(np.float16)


@pytest.mark.parametrize("group", [32, 128])
def test_int16_codes_are_the_nearest_levels_of_the_stored_lattice(group):
    """Every code is what exact arithmetic gives for round((x - Z) / S) with the *stored* fp16 S and Z, clamped to
    [0, 65535] (ties aside: the fp32 quotient may land on the other side of a half); the minimum maps to code 0."""
    x = _data(1)
    codes, S, Z = quantize(x, 16, group)
    assert codes.dtype == np.uint16 and S.dtype == np.float16 and Z.dtype == np.float16
    xg = x.reshape(-1, 128 // group, group)
    assert np.array_equal(Z, xg.min(-1))
    cg = codes.reshape(xg.shape)
    rng = np.random.default_rng(2)
    for _ in range(3000):
        r, g, e = rng.integers(xg.shape[0]), rng.integers(xg.shape[1]), rng.integers(group)
        s, z, v = Fraction(float(S[r, g])), Fraction(float(Z[r, g])), Fraction(float(xg[r, g, e]))
        if s == 0:
            assert cg[r, g, e] == 0
            continue
        t = (v - z) / s
        want = min(65535, max(0, (2 * t.numerator + t.denominator) // (2 * t.denominator)))
        frac = t - (t.numerator // t.denominator)
        if abs(frac - Fraction(1, 2)) < Fraction(1, 64):   # fp32 quotient near a half: either neighbour
            assert abs(int(cg[r, g, e]) - want) <= 1
        else:
            assert int(cg[r, g, e]) == want
    assert np.all(np.take_along_axis(cg, xg.argmin(-1)[..., None], -1) == 0)


def test_int16_round_trip_error_and_the_clamp():
    """|x - x_hat| <= S/2 where no clamp acts; where the fp16 rounding of S pushes (max - Z) / S above 65535 the
    clamp costs at most the overshoot, which stays below 65535 * (relative rounding error of S): 2^-11 for a normal
    S, half an fp16 subnormal step (2^-25) in absolute terms below that."""
    x = _data(3, 2000)
    codes, S, Z = quantize(x, 16, 32)
    xh = dequantize(codes, S, Z, 32)
    Sd, Zd = S.astype(np.float64), Z.astype(np.float64)
    xg = x.reshape(-1, 4, 32).astype(np.float64)
    err = np.abs(xh.reshape(xg.shape) - xg)
    over = np.maximum(0.0, (xg.max(-1) - Zd) - 65535.0 * Sd)       # how far the top of the lattice falls short
    # (the quotient is formed in fp32, whose step near 65535 is 2^-8: a value that close to a half may go either way)
    assert np.all(err <= Sd[..., None] * (0.5 + 2.0 ** -8) + over[..., None] + 1e-12)
    exact = (xg.max(-1) - Zd) / 65535.0
    s_err = np.maximum(np.abs(exact) * (2.0 ** -11 + 2.0 ** -22), 2.0 ** -25)
    assert np.all(np.abs(Sd - exact) <= s_err * (1 + 1e-6))
    assert np.all(over <= 65535.0 * s_err * (1 + 1e-6))
    assert (over > 0.5 * Sd).mean() > 0.2     # the clamp is not a corner case: S rounds down about half the time
    # unclamped groups reconstruct to within S/2, i.e. far below what 8 bits give
    c8, S8, Z8 = quantize(x, 8, 32)
    e8 = np.abs(dequantize(c8, S8, Z8, 32) - x.astype(np.float64))
    assert (err ** 2).mean() < (e8 ** 2).mean() / 1000


def test_theorem_at_b8_through_the_fp16_scales():
    """Appendix theorem, b = 8: Eq. 3 on the INT16 codes gives the codes of the direct 8-bit quantization.  In exact
    arithmetic they are identical (pinned elsewhere in exact rationals); with S stored in fp16 the two lattices
    differ by the rounding of S (2^-11 relative, more for subnormal S), which moves few codes, by few levels, and
    leaves the reconstruction error unchanged to within a few percent."""
    x = _data(5, 2000)
    c16, S16, Z16 = quantize(x, 16, 32)
    c8d, S8d, Z8d = quantize(x, 8, 32)
    c8s, S8s, Z8s = shrink_step(c16, S16, Z16, 8, SHIFT_EQUIVALENT)
    assert c8s.dtype == np.uint8 and np.array_equal(Z8s, Z8d)
    assert np.array_equal(c8s, shrink_codes(c16, 8)) and np.array_equal(S8s, shrink_scale(S16, 8))
    d = np.abs(c8d.astype(np.int32) - c8s.astype(np.int32)).reshape(-1, 4, 32)
    assert (d == 0).mean() > 0.75 and d.max() <= 5
    ed = ((dequantize(c8d, S8d, Z8d, 32) - x) ** 2).mean()
    es = ((dequantize(c8s, S8s, Z8s, 32) - x) ** 2).mean()
    assert abs(es / ed - 1) < 0.05
    # the product of Eq. 3 at b = 8 does not fit a signed 32-bit integer but fits an unsigned one
    assert 2 ** 31 < 65281 * (65535 + 128) < 2 ** 32
    top = shrink_codes(np.array([65535, 65535 - 129, 0, 128, 129], np.uint16), 8)
    assert top.tolist() == [255, 254, 0, 0, 1]


def test_theorem_at_b8_is_exact_when_the_scales_are():
    """Groups built so that both scales are exact fp16 numbers: Z = -63 and max = 1 - 2^-10 give
    S_16 = 63.9990234375 / 65535 = 2^-10 and S_8 = 257 * 2^-10; values are multiples of 2^-9, so the 16-bit codes are
    the integers (x + 63) * 1024 and no 8-bit quotient is a tie (257 is odd).  Then Eq. 3 on the INT16 codes must
    reproduce the direct 8-bit codes in every element, and the 16-bit round trip is lossless."""
    rng = np.random.default_rng(9)
    x = (np.round(rng.uniform(-63, 1, (500, 128)).astype(np.float16).astype(np.float64) * 512) / 512).astype(np.float16)
    x = np.clip(x, np.float16(-63), np.float16(1 - 2.0 ** -10))
    x[:, 0::32] = np.float16(-63)
    x[:, 1::32] = np.float16(1 - 2.0 ** -10)
    c16, S16, Z16 = quantize(x, 16, 32)
    assert np.all(S16 == np.float16(2.0 ** -10)) and np.all(Z16 == np.float16(-63))
    assert np.array_equal(c16, ((x.astype(np.float64) + 63) * 1024).astype(np.uint16))
    assert np.array_equal(dequantize(c16, S16, Z16, 32), x.astype(np.float64))
    c8d, S8d, Z8d = quantize(x, 8, 32)
    c8s, S8s, Z8s = shrink_step(c16, S16, Z16, 8, SHIFT_EQUIVALENT)
    assert np.all(S8d == np.float16(257 * 2.0 ** -10)) and np.array_equal(S8s, S8d) and np.array_equal(Z8s, Z8d)
    assert np.array_equal(c8s, c8d)
    assert c8d.min() == 0 and c8d.max() == 255 and len(np.unique(c8d)) == 256


def test_direct_and_modified_shift_from_16_bits():
    c16 = np.array([[0, 255, 256, 0x1234, 0xffff] + [0] * 27], np.uint16)
    S = np.array([[0.001]], np.float16); Z = np.array([[-1.5]], np.float16)
    xb, Sb, Zb = shrink_step(c16, S, Z, 8, SHIFT_DIRECT)
    assert xb[0, :5].tolist() == [0, 0, 1, 0x12, 0xff] and Sb[0, 0] == np.float16(np.float32(S[0, 0]) * 257) and Zb[0, 0] == Z[0, 0]
    xb, Sb, Zb = shrink_step(c16, S, Z, 8, SHIFT_MODIFIED)
    assert xb[0, :5].tolist() == [0, 0, 1, 0x12, 0xff] and Sb[0, 0] == np.float16(np.float32(S[0, 0]) * 256)
    assert Zb[0, 0] == np.float16(np.float32(Z[0, 0]) + np.float32(0.5) * (np.float32(S[0, 0]) * 256 - np.float32(S[0, 0])))


def test_packing_of_16_bit_codes():
    assert pack_codes(np.array([[0x1234, 0x00ff]], np.uint16), 16).tolist() == [[0x34, 0x12, 0xff, 0x00]]
    c = np.random.default_rng(0).integers(0, 65536, (3, 2, 128)).astype(np.uint16)
    p = pack_codes(c, 16)
    assert p.shape == (3, 2, 256) and p.dtype == np.uint8 and np.array_equal(unpack_codes(p, 16), c)
    assert [bytes_per_token_head(16, 128, g, True, True) for g in (32, 64, 128)] == [544, 528, 520]
    assert bytes_per_token_head(16, 128, 32, False, True) == 512 and bytes_per_token_head(8, 128, 32, True, True) == 288


def test_int16_tier_cache_chain_window_and_attention():
    """A block with an INT16 sink and window under the paper's policy: evicted pages go 16 -> 8 -> (4) by successive
    Eq. 3 steps, bytes are counted with the tier's metadata, and attention over the cache stays close to exact."""
    P, W, T = 32, 64, 640
    cfg = CacheConfig(1, 2, 4, 2, page_tokens=P, max_tokens=2048, window=W, n_sink=P, policy=POLICY_PAPER,
                      tier16=TIER16_INT16)
    per = {b: bytes_per_token_head(b, 128, 32, True, True) for b in (16, 8, 4, 2)}
    assert per[16] == 544
    budget = 2 * 2 * (600 * per[4] + (W + 2 * P) * per[16])
    c = OracleCache(cfg, [budget], [4])
    K, V = kvq_synth.make_kv(11, 0, 2, 2, 0, T)
    q = kvq_synth.make_q(12, 0, 2, 4, T)
    t = 0
    while t < T:
        try:
            c.append(0, K[:, :, t:t + 16], V[:, :, t:t + 16])
            t += 16
        except BudgetError:
            c.requant(0)
        assert c.bytes_used(0) <= budget
        assert c.bytes_used(0) == sum((t1 - t0) * 4 * per[b] for t0, t1, b in c.segments(0))
    segs = c.segments(0)
    assert segs[0] == (0, P, 16) and segs[-1][2] == 16 and segs[-1][1] == T and T - segs[-1][0] >= W
    assert c.current_bits(0) == 4 and {b for _, _, b in segs} == {16, 4}
    # a page evicted from the window equals the manual chain on its tokens
    t0 = segs[1][0]
    kc, ks, kz = quantize(K[:, :, t0:t0 + P], 16, 32)
    for b in (8, 4):
        kc, ks, kz = shrink_step(kc, ks, kz, b, SHIFT_EQUIVALENT)
    codes, S, Z = c.export_segment(0, 1, "K")
    assert np.array_equal(codes[:, :, :P], pack_codes(kc, 4)) and np.array_equal(S[:, :, :P], ks) and np.array_equal(Z[:, :, :P], kz)
    # the 16-bit runs export as little-endian 16-bit codes with their metadata
    codes, S, Z = c.export_segment(0, 0, "V")
    vc, vs, vz = quantize(V[:, :, :P], 16, 32)
    assert np.array_equal(unpack_codes(codes, 16), vc) and np.array_equal(S, vs) and np.array_equal(Z, vz)
    # attention: all-INT16 cache against the exact fp64 attention over the fp16 tensors
    cfg2 = CacheConfig(1, 2, 4, 2, page_tokens=P, max_tokens=2048, policy=POLICY_OLDEST_FIRST, tier16=TIER16_INT16)
    c2 = OracleCache(cfg2, [1 << 40], [16])
    c2.append(0, K, V)
    assert c2.segments(0) == [(0, T, 16)] and c2.bytes_used(0) == T * 4 * 544
    exact = decode_attention_fp64(q, K.astype(np.float64), V.astype(np.float64))
    assert np.abs(c2.attention(0, q) - exact).max() < 2e-3
    c8 = OracleCache(CacheConfig(1, 2, 4, 2, page_tokens=P, max_tokens=2048, policy=POLICY_OLDEST_FIRST), [1 << 40], [8])
    c8.append(0, K, V, entry_bits=8)
    assert np.abs(c2.attention(0, q) - exact).max() < 0.5 * np.abs(c8.attention(0, q) - exact).max()
    # requant of the whole INT16 run by segment: one Eq. 3 step to 8 bits
    assert c2.requant(0, segment=0) == T // P and c2.segments(0) == [(0, T, 8)]
    vc, vs, vz = shrink_step(*quantize(V, 16, 32), 8, SHIFT_EQUIVALENT)
    codes, S, Z = c2.export_segment(0, 0, "V")
    assert np.array_equal(codes, vc) and np.array_equal(S, vs) and np.array_equal(Z, vz)


def test_fp16_tier_is_unchanged_by_the_option():
    cfg = CacheConfig(1, 1, 2, 1, page_tokens=32, max_tokens=256, policy=POLICY_OLDEST_FIRST, tier16=TIER16_FP16)
    c = OracleCache(cfg, [1 << 30], [16])
    K, V = kvq_synth.make_kv(3, 0, 1, 1, 0, 64)
    c.append(0, K, V)
    vals, S, Z = c.export_segment(0, 0, "K")
    assert S is None and Z is None and np.array_equal(vals, K) and c.bytes_used(0) == 64 * 512
