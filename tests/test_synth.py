"""Pins of the synthetic input generator (CPU only)."""
import json
import math
import os

import numpy as np

import kvq_synth

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def test_rope_lowest_frequency_period_matches_paper():
    g = GOLD["rope_lowest_frequency_period_tokens"]
    d = g["head_dim"]
    theta_last = g["base"] ** (-2.0 * (d // 2 - 1) / d)
    assert int(2 * math.pi / theta_last) == g["value"]
    # the generator's slowest pair really has that period: rotating by `period` tokens is ~ the identity on it
    x = np.zeros((1, d)); x[0, d // 2 - 1] = 1.0
    y = kvq_synth.rope_rotate(np.repeat(x, 2, 0), np.array([0, 54410]), g["base"])
    assert abs(y[1, d // 2 - 1] - 1.0) < 1e-8 and abs(y[1, d - 1]) < 1e-4


def test_rope_is_complex_rotation_and_keeps_pair_norms():
    rng = np.random.default_rng(0)
    d = 128
    x = rng.standard_normal((5, d))
    pos = np.array([0, 1, 17, 4096, 32767])
    y = kvq_synth.rope_rotate(x, pos, 1e6)
    z = (x[:, :d // 2] + 1j * x[:, d // 2:]) * np.exp(1j * pos[:, None] * (1e6 ** (-2.0 * np.arange(d // 2) / d))[None])
    assert np.allclose(y[:, :d // 2], z.real) and np.allclose(y[:, d // 2:], z.imag)
    assert np.allclose(y[:, :d // 2] ** 2 + y[:, d // 2:] ** 2, x[:, :d // 2] ** 2 + x[:, d // 2:] ** 2)
    assert np.allclose(y[0], x[0])


def test_generator_is_seeded_and_range_addressable():
    a, av = kvq_synth.make_kv_unit(5, 2, 1, 3, 0, 3000)
    b, bv = kvq_synth.make_kv_unit(5, 2, 1, 3, 1000, 2100)
    assert np.array_equal(a[1000:2100], b) and np.array_equal(av[1000:2100], bv)
    c, _ = kvq_synth.make_kv_unit(6, 2, 1, 3, 0, 100)
    assert not np.array_equal(a[:100], c)
    ch = kvq_synth.outlier_channels(5, 3)
    assert len(ch) == 4
    amp = np.abs(kvq_synth.make_kv_unit(5, 0, 0, 3, 0, 2048, rope_base=None)[0].astype(np.float64)).mean(0)
    assert set(np.argsort(amp)[-4:]) == set(ch)


def test_workload_shapes_match_configs():
    w = kvq_synth.WORKLOADS
    assert w["tiny"].n_tokens == 4096 and w["32b"].n_tokens == 32768 and w["70b"].n_tokens == 131072
    assert w["7b"].n_tokens == 32768 and w["14b"].n_tokens == 32768
    for x in w.values():
        assert all(n % x.page_tokens == 0 for n, _ in x.tiers)
    assert set(w["14b"].layer_bits) <= {2, 4, 8} and len(w["14b"].layer_bits) == 48
