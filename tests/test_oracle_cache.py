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
