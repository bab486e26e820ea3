"""Pins of the oracle's ragged-batch decode step: every sequence attends over its own cache only."""
import numpy as np
import pytest

import kvq_synth
from oracle import (OracleCache, CacheConfig, BudgetError, POLICY_PAPER, POLICY_OLDEST_FIRST, bytes_per_token_head,
                    decode_step_batch)


def _cache(B, T, seed, budget=1 << 40, window=0, policy=POLICY_OLDEST_FIRST, b0=0, bits=None):
    cfg = CacheConfig(1, B, 4, 2, page_tokens=32, max_tokens=1024, window=window, policy=policy)
    c = OracleCache(cfg, [budget], [2])
    K, V = kvq_synth.make_kv(seed, 0, b0 + B, 2, 0, T + 1)
    K, V = K[b0:], V[b0:]
    if bits:
        t = 0
        for n, b in bits:
            c.append(0, K[:, :, t:t + n], V[:, :, t:t + n], b)
            t += n
        assert t == T
    else:
        c.append(0, K[:, :, :T], V[:, :, :T])
    return c, K[:, :, T:T + 1], V[:, :, T:T + 1]


def test_equal_lengths_reduce_to_the_batched_cache():
    """Three one-sequence caches built from the rows of one three-sequence cache: the ragged step gives what the
    (separately pinned) batched attention gives."""
    T = 150
    big, kb, vb = _cache(3, T, 5, bits=((64, 4), (64, 8), (22, 16)))
    q = kvq_synth.make_q(5, 0, 3, 4, T)
    parts = [_cache(1, T, 5, b0=i, bits=((64, 4), (64, 8), (22, 16))) for i in range(3)]
    outs = decode_step_batch([p[0] for p in parts], 0, [p[1] for p in parts], [p[2] for p in parts],
                             [q[i:i + 1] for i in range(3)])
    big.append(0, kb, vb)
    want = big.attention(0, q)
    for i in range(3):
        assert np.allclose(outs[i][0], want[i], rtol=0, atol=1e-14)


def test_ragged_lengths_are_independent_and_order_free():
    specs = [(1, 40, 11), (2, 333, 12), (1, 97, 13), (1, 1, 14)]
    def run(order):
        caches = [_cache(B, T, s) for B, T, s in specs]
        qs = [kvq_synth.make_q(s, 0, B, 4, T) for B, T, s in specs]
        outs = decode_step_batch([caches[i][0] for i in order], 0, [caches[i][1] for i in order],
                                 [caches[i][2] for i in order], [qs[i] for i in order])
        return {i: o for i, o in zip(order, outs)}, caches
    a, _ = run([0, 1, 2, 3])
    b, _ = run([3, 1, 0, 2])
    for i in range(4):
        assert np.array_equal(a[i], b[i])
    # each alone
    for i, (B, T, s) in enumerate(specs):
        c, k, v = _cache(B, T, s)
        alone = decode_step_batch([c], 0, [k], [v], [kvq_synth.make_q(s, 0, B, 4, T)])[0]
        assert np.array_equal(alone, a[i])
        assert c.layers[0].T == T + 1
    # a one-token cache attends to its single token: the output is that token's V
    c, k, v = _cache(1, 1, 14)
    o = decode_step_batch([c], 0, [k], [v], [kvq_synth.make_q(14, 0, 1, 4, 1)])[0]
    Kh, Vh = c.dequantized(0)
    assert Vh.shape[2] == 2 and np.all((o[0, 0] >= Vh[0, 0].min(0) - 1e-12) & (o[0, 0] <= Vh[0, 0].max(0) + 1e-12))


def test_all_or_nothing_when_one_cache_is_full():
    per16 = bytes_per_token_head(16, 128, 32, True)
    ok, k0, v0 = _cache(1, 50, 21)
    full, k1, v1 = _cache(1, 64, 22, budget=2 * 64 * per16)      # exactly full at 64 tokens
    q = [kvq_synth.make_q(21, 0, 1, 4, 50), kvq_synth.make_q(22, 0, 1, 4, 64)]
    with pytest.raises(BudgetError):
        decode_step_batch([ok, full], 0, [k0, k1], [v0, v1], q)
    assert ok.layers[0].T == 50 and full.layers[0].T == 64
    full.requant(0, reserve_tokens=1)
    outs = decode_step_batch([ok, full], 0, [k0, k1], [v0, v1], q)
    assert ok.layers[0].T == 51 and full.layers[0].T == 65 and len(outs) == 2
