"""Pins of the oracle's bookkeeping: shrink schedule, budgets, window, policies (CPU only)."""
import json
import os

import numpy as np
import pytest

import kvq_synth
from oracle import (OracleCache, CacheConfig, BudgetError, StateError, POLICY_PAPER, POLICY_OLDEST_FIRST,
                    bytes_per_token_head)

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def _feed(c, K, V, chunk, on_budget):
    T = K.shape[2]
    t = 0
    while t < T:
        n = min(chunk, T - t)
        try:
            c.append(0, K[:, :, t:t + n], V[:, :, t:t + n])
            t += n
        except BudgetError:
            on_budget(t)


def test_paper_schedule_fbit2_32k():
    """Fbit = 2, maximum context 32K: the cache is full at 4K x 16 bit, 8K x 8 bit, 16K x 4 bit and ends at 32K x 2 bit."""
    g = GOLD["progressive_schedule"]
    Tmax = g["max_context"]
    cfg = CacheConfig(1, 1, 1, 1, page_tokens=128, max_tokens=Tmax, window=0, n_sink=0,
                      policy=POLICY_PAPER, count_metadata_in_budget=0)
    budget = Tmax * bytes_per_token_head(g["fbit"], 128, 32, False)
    c = OracleCache(cfg, [budget], [g["fbit"]])
    rng = np.random.default_rng(0)
    K = rng.standard_normal((1, 1, Tmax, 128)).astype(np.float16)
    points, widths = [], []

    def on_budget(t):
        points.append(t)
        c.requant(0)
        widths.append(c.current_bits(0))
        assert c.bytes_used(0) <= budget

    _feed(c, K, K, 64, on_budget)
    assert points == g["shrink_points"] and widths == [8, 4, 2]
    assert c.layers[0].T == Tmax and c.bytes_used(0) == budget
    assert c.segments(0) == [(0, Tmax, 2)]
    with pytest.raises(BudgetError):
        c.requant(0)          # already at Fbit
    with pytest.raises(StateError):
        c.append(0, K[:, :, :1], K[:, :, :1])   # beyond max_tokens


def test_paper_policy_window_and_sink():
    P, W = 32, 64
    cfg = CacheConfig(1, 1, 2, 1, page_tokens=P, max_tokens=2048, window=W, n_sink=P, policy=POLICY_PAPER)
    per = {b: bytes_per_token_head(b, 128, 32, True) for b in (16, 8, 4, 2)}
    budget = 600 * per[4]
    c = OracleCache(cfg, [budget], [4])
    K, V = kvq_synth.make_kv(21, 0, 1, 1, 0, 700)
    events = []

    def on_budget(t):
        n = c.requant(0)
        events.append((t, c.current_bits(0), n))

    hit = []
    t = 0
    while t < 700:
        try:
            c.append(0, K[:, :, t:t + 1], V[:, :, t:t + 1])
            t += 1
        except BudgetError:
            try:
                on_budget(t)
            except BudgetError:
                hit.append(t)
                break
        # invariants after every step
        assert c.bytes_used(0) <= budget
        segs = c.segments(0)
        assert segs[0][2] == 16 and segs[0][1] >= min(t, P)            # sink page stays 16-bit
        tail = segs[-1]
        assert tail[2] == 16 and (t < W or W <= t - tail[0] < W + P or c.current_bits(0) == 16)
    assert [e[1] for e in events] == [8, 4]
    assert hit, "the budget must eventually be exhausted at Fbit"
    # widths are monotone non-increasing from newest to oldest outside the sink
    bits = [s[2] for s in c.segments(0)[1:]]
    assert bits == sorted(bits)


def test_oldest_first_policy():
    P = 32
    cfg = CacheConfig(1, 1, 2, 1, page_tokens=P, max_tokens=1024, window=P, policy=POLICY_OLDEST_FIRST)
    per = {b: bytes_per_token_head(b, 128, 32, True) for b in (16, 8, 4, 2)}
    budget = 8 * P * per[16]
    c = OracleCache(cfg, [budget], [4])
    K, V = kvq_synth.make_kv(22, 0, 1, 1, 0, 1024)
    c.append(0, K[:, :, :8 * P], V[:, :, :8 * P])
    with pytest.raises(BudgetError):
        c.append(0, K[:, :, 8 * P:9 * P], V[:, :, 8 * P:9 * P])
    assert c.layers[0].T == 8 * P                                     # unchanged
    n = c.requant(0, reserve_tokens=P)
    # one page 16 -> 8 frees 32*(512-288) = 7168 B < 32*512: needs page 0 down to 4 bits (2 steps) and page 1 16->8->4 ...
    used = c.bytes_used(0)
    assert used + P * per[16] <= budget and n >= 2
    segs = c.segments(0)
    assert segs[0][2] == 4 and segs[-1][2] == 16
    bits = [s[2] for s in segs]
    assert bits == sorted(bits)
    c.append(0, K[:, :, 8 * P:9 * P], V[:, :, 8 * P:9 * P])
    # exhaust: eventually nothing is left above Fbit outside the window
    with pytest.raises(BudgetError):
        for i in range(9, 32):
            try:
                c.append(0, K[:, :, i * P:(i + 1) * P], V[:, :, i * P:(i + 1) * P])
            except BudgetError:
                c.requant(0, reserve_tokens=P)
                c.append(0, K[:, :, i * P:(i + 1) * P], V[:, :, i * P:(i + 1) * P])
    assert c.bytes_used(0) <= budget


def test_width_change_inside_page_is_rejected_and_budget_failure_leaves_state():
    cfg = CacheConfig(1, 1, 2, 1, page_tokens=64, max_tokens=512)
    c = OracleCache(cfg, [10 ** 9], [2])
    K, V = kvq_synth.make_kv(23, 0, 1, 1, 0, 200)
    c.append(0, K[:, :, :40], V[:, :, :40], 8)
    with pytest.raises(StateError):
        c.append(0, K[:, :, 40:50], V[:, :, 40:50], 4)
    c.append(0, K[:, :, 40:64], V[:, :, 40:64], 8)
    c.append(0, K[:, :, 64:100], V[:, :, 64:100], 4)
    assert c.segments(0) == [(0, 64, 8), (64, 100, 4)]
    assert c.bytes_used(0) == 64 * 288 + 36 * 160


def test_shift_strategy_chains_and_reconstruction_error():
    """The cache applies the configured strategy to every 2b -> b step; the reconstruction error of a cache is the
    squared distance of its de-quantized content from the tensors it was built from (zero for the 16-bit tier, and
    within the round-trip bound S/2 per element after direct quantization)."""
    from oracle import (quantize, dequantize, shrink_step, SHIFT_EQUIVALENT, SHIFT_DIRECT, SHIFT_MODIFIED)
    import kvq_synth
    B, H, T, P = 1, 2, 128, 64
    K, V = kvq_synth.make_kv(55, 0, B, H, 0, T)
    for st in (SHIFT_EQUIVALENT, SHIFT_DIRECT, SHIFT_MODIFIED):
        oc = OracleCache(CacheConfig(1, B, 2 * H, H, page_tokens=P, max_tokens=T, shift_strategy=st), [1 << 40], [2])
        oc.append(0, K, V, 16)
        assert oc.reconstruction_sq_error(0, K, V) == (0.0, 0.0)
        oc.requant(0, segment=0)                                   # 16 -> 8: Eq. 1-2 whatever the strategy
        kc, ks, kz = quantize(K, 8, 32)
        ek, ev = oc.reconstruction_sq_error(0, K, V)
        assert ek == pytest.approx(float(np.sum((dequantize(kc, ks, kz, 32) - K.astype(np.float64)) ** 2)))
        bound = np.sum((np.repeat(ks.astype(np.float64), 32, -1) * (0.5 + 255 * 2.0 ** -11)) ** 2)
        assert ek <= bound
        for b in (4, 2):
            oc.requant(0, segment=0)
            kc, ks, kz = shrink_step(kc, ks, kz, b, st)
            codes, S, Z = oc.export_segment(0, 0, "K")
            assert np.array_equal(S, ks) and np.array_equal(Z, kz)
            ek2, _ = oc.reconstruction_sq_error(0, K, V)
            assert ek2 == pytest.approx(float(np.sum((dequantize(kc, ks, kz, 32) - K.astype(np.float64)) ** 2)))
            assert ek2 > ek


# ------------------------------------------------------------ channel-wise reparameterization (Sec. 3.3, Eq. 7-8)
def test_reparam_lambda_formula_on_hand_made_keys():
    from oracle import calibrate_lambda, LAMBDA_FLOOR
    K = np.zeros((2, 1, 5, 128), np.float16)
    K[0, 0, 3, 0] = 4.0          # max |K| = 4
    K[1, 0, 1, 1] = -9.0         # the largest magnitude is negative
    K[0, 0, 0, 2] = 0.25
    K[1, 0, 4, 2] = 0.125
    lam = calibrate_lambda(K, 0.5)
    assert lam.shape == (1, 128) and lam.dtype == np.float32
    assert lam[0, 0] == 2.0 and lam[0, 1] == 3.0 and lam[0, 2] == 0.5
    assert lam[0, 3] == pytest.approx(float(LAMBDA_FLOOR) ** 0.5, rel=1e-6)     # an all-zero channel
    assert np.array_equal(calibrate_lambda(K, 0.0), np.ones((1, 128), np.float32))
    assert calibrate_lambda(K, 1.0)[0, 1] == 9.0


def test_reparam_is_exact_for_power_of_two_factors_and_close_otherwise():
    """Q Lambda (K Lambda^-1)^T = Q K^T: with power-of-two factors both scalings are exact in fp16 (up to elements
    that fall into the fp16 subnormal range), so a 16-bit cache reproduces the outputs to 1e-6; with arbitrary
    factors the fp16 rounding of K / lambda and q * lambda moves the result by about 1e-3."""
    import kvq_synth
    B, H, g, T = 1, 2, 3, 96
    K, V = kvq_synth.make_kv(56, 0, B, H, 0, T)
    q = kvq_synth.make_q(56, 0, B, H * g, T - 1)
    cfg = CacheConfig(1, B, H * g, H, page_tokens=32, max_tokens=T)
    base = OracleCache(cfg, [1 << 40], [2]); base.append(0, K, V, 16)
    want = base.attention(0, q)
    rng = np.random.default_rng(1)
    lam2 = (2.0 ** rng.integers(-2, 3, (H, 128))).astype(np.float32)
    oc = OracleCache(cfg, [1 << 40], [2]); oc.set_reparam(0, lam2); oc.append(0, K, V, 16)
    assert np.abs(oc.attention(0, q) - want).max() < 1e-6
    lam = rng.uniform(0.5, 3.0, (H, 128)).astype(np.float32)
    oc = OracleCache(cfg, [1 << 40], [2]); oc.set_reparam(0, lam); oc.append(0, K, V, 16)
    d = np.abs(oc.attention(0, q) - want).max()
    assert 1e-6 < d < 5e-3
    with pytest.raises(StateError):
        oc.set_reparam(0, lam2)                      # not on a block that already holds tokens


def test_reparam_moves_outliers_out_of_the_keys():
    """The motivation of Sec. 3.3 on the synthetic keys (4 channels per head x20): with lambda from Eq. 8 at
    alpha = 0.5 the stored keys' outlier channels shrink by sqrt(their maximum), and 4-bit attention gets closer to
    the exact attention over the raw tensors."""
    import kvq_synth
    from oracle import calibrate_lambda, reparam_keys, decode_attention_fp64
    B, H, g, T = 1, 2, 2, 512
    K, V = kvq_synth.make_kv(57, 0, B, H, 0, T)
    q = kvq_synth.make_q(57, 0, B, H * g, T - 1)
    lam = calibrate_lambda(K, 0.5)
    out_ch = kvq_synth.outlier_channels(57, 0, 128, 4)
    Kp = reparam_keys(K, lam)
    ratio = np.abs(K[0, 0]).max(0)[out_ch] / np.abs(Kp[0, 0]).max(0)[out_ch]
    assert np.allclose(ratio, lam[0, out_ch], rtol=2e-3)
    exact = decode_attention_fp64(q, K.astype(np.float64), V.astype(np.float64))
    cfg = CacheConfig(1, B, H * g, H, page_tokens=64, max_tokens=T)
    errs = []
    for use in (False, True):
        oc = OracleCache(cfg, [1 << 40], [2])
        if use:
            oc.set_reparam(0, lam)
        oc.append(0, K, V, 4)
        errs.append(float(np.linalg.norm(oc.attention(0, q) - exact) / np.linalg.norm(exact)))
    assert errs[1] < errs[0]
