"""Pins of the oracle's block-wise memory allocation (Sec. 3.2, Eq. 5-6)."""
import numpy as np
import pytest

import kvq_synth
from oracle import (sensitivity, allocate_bits_bruteforce, allocate_bits_dp, quantize, dequantize,
                    bytes_per_token_head)


def test_sensitivity_terms():
    K, V = kvq_synth.make_kv(60, 0, 1, 2, 0, 64)
    assert sensitivity(K, V, 16, 32) == (0.0, 0.0)
    sk, sv = sensitivity(K, V, 4, 32)
    c, S, Z = quantize(K, 4, 32)
    assert sk == pytest.approx(float(np.abs(dequantize(c, S, Z, 32) - K.astype(np.float64)).sum()))
    # per element the error is at most S/2 (+ fp16 rounding of S): the L1 norm obeys the summed bound
    assert sk <= float((np.repeat(S.astype(np.float64), 32, -1) * (0.5 + 15 * 2.0 ** -11)).sum())
    s2, s8 = sensitivity(K, V, 2, 32), sensitivity(K, V, 8, 32)
    assert s2[0] > sk > s8[0] and s2[1] > sv > s8[1]
    # gradients weigh the error element-wise; a constant gradient scales the norm, its sign does not matter
    G = np.full(K.shape, -3.0, np.float32)
    gk, gv = sensitivity(K, V, 4, 32, G, G)
    assert gk == pytest.approx(3 * sk) and gv == pytest.approx(3 * sv)
    G0 = np.zeros(K.shape, np.float32); G0[:, :, :, 5] = 1.0
    gk0, _ = sensitivity(K, V, 4, 32, G0, G0)
    assert gk0 == pytest.approx(float(np.abs(dequantize(c, S, Z, 32) - K.astype(np.float64))[..., 5].sum()))


def test_allocation_hand_solved_instance():
    """Three blocks, widths {2, 4}: costs s = [[9, 1], [5, 4], [7, 2]], memory [[1, 2]] * 3, budget 5: the two 4-bit
    upgrades worth most (blocks 0 and 2: gains 8 and 5) fit, a third does not.  Total cost 1 + 5 + 2 = 8."""
    s = np.array([[9.0, 1.0], [5.0, 4.0], [7.0, 2.0]])
    mem = np.array([[1, 2]] * 3)
    for solve in (allocate_bits_bruteforce, allocate_bits_dp):
        ch, cost, m = solve(s, mem, 5)
        assert list(ch) == [1, 0, 1] and cost == 8.0 and m == 5
        assert list(solve(s, mem, 6)[0]) == [1, 1, 1]            # everything fits: the best width everywhere
        assert list(solve(s, mem, 3)[0]) == [0, 0, 0]            # only the smallest widths fit
        assert solve(s, mem, 2)[0] is None                       # nothing fits


def test_allocation_uniform_two_bit_fits_uniform_four_bit_does_not():
    """The situation of Sec. 3.2: memory between uniform 2 and uniform 4 bits is used by giving 4 bits to the most
    sensitive blocks.  32 tokens... sizes are real bytes per block (T tokens x units x bytes per token-head)."""
    N, T, units = 6, 1024, 8
    mem = np.array([[T * units * bytes_per_token_head(b, 128, 32, True) for b in (2, 4)]] * N)
    rng = np.random.default_rng(2)
    s2 = rng.uniform(5, 10, N)
    s = np.stack([s2, s2 * 0.2], 1)
    budget = int(mem[:, 0].sum() + 2.5 * (mem[0, 1] - mem[0, 0]))      # room for two upgrades, not three
    for solve in (allocate_bits_bruteforce, allocate_bits_dp):
        ch, cost, m = solve(s, mem, budget)
        assert ch.sum() == 2 and m <= budget
        assert set(np.nonzero(ch)[0]) == set(np.argsort(-s2)[:2])       # the two most sensitive blocks


def test_allocation_enumeration_and_recurrence_agree_on_random_instances():
    rng = np.random.default_rng(3)
    for trial in range(40):
        N, C = int(rng.integers(1, 7)), int(rng.integers(2, 5))
        mem = np.sort(rng.integers(1, 20, (N, C)), 1) * int(rng.choice([1, 3, 64]))
        s = -np.sort(-rng.uniform(0, 10, (N, C)), 1)                    # more memory, less sensitivity
        if trial % 5 == 0:
            s = rng.uniform(0, 10, (N, C))                              # ... or no structure at all
        budget = int(rng.integers(mem[:, 0].sum() - 2, mem[:, -1].sum() + 3))
        a, b = allocate_bits_bruteforce(s, mem, budget), allocate_bits_dp(s, mem, budget)
        assert (a[0] is None) == (b[0] is None)
        if a[0] is not None:
            assert a[1] == pytest.approx(b[1]) and a[2] <= budget and b[2] <= budget
