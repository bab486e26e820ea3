"""Pins of the oracle's attention and of attention over mixed-width caches (CPU only)."""
import itertools
import math

import numpy as np
import pytest
import torch

import kvq_synth
from oracle import (OracleCache, CacheConfig, decode_attention_fp64, quantize, shrink_codes, shrink_scale)


def _sdpa_fp64(q, K, V):
    """Library routine: torch scaled_dot_product_attention in fp64 on CPU, GQA by head repetition."""
    g = q.shape[1] // K.shape[1]
    qt = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    kt = torch.from_numpy(K.astype(np.float64)).repeat_interleave(g, dim=1)
    vt = torch.from_numpy(V.astype(np.float64)).repeat_interleave(g, dim=1)
    return torch.nn.functional.scaled_dot_product_attention(qt, kt, vt)[:, :, 0, :].numpy()


def test_16bit_passthrough_equals_library_attention():
    K, V = kvq_synth.make_kv(3, 0, 2, 2, 0, 700, rope_base=1e4)
    q = kvq_synth.make_q(3, 0, 2, 8, 699, rope_base=1e4)
    cfg = CacheConfig(1, 2, 8, 2, page_tokens=128, max_tokens=1024)
    c = OracleCache(cfg, [10 ** 12], [2])
    c.append(0, K[:, :, :300], V[:, :, :300], 16)
    c.append(0, K[:, :, 300:], V[:, :, 300:], 16)
    got = c.attention(0, q)
    assert np.allclose(got, _sdpa_fp64(q, K, V), rtol=0, atol=1e-12)
    assert np.allclose(decode_attention_fp64(q, K, V), _sdpa_fp64(q, K, V), rtol=0, atol=1e-12)


def _brute(q, toks, g, D):
    """Independent scalar loops over hand-de-quantized tokens: toks[b][hkv] = list of (k_vec, v_vec) python lists."""
    B, Hq = len(q), len(q[0])
    out = [[[0.0] * D for _ in range(Hq)] for _ in range(B)]
    for b in range(B):
        for h in range(Hq):
            tl = toks[b][h // g]
            s = [sum(q[b][h][d] * k[d] for d in range(D)) / math.sqrt(D) for k, _ in tl]
            m = max(s)
            w = [math.exp(x - m) for x in s]
            tot = sum(w)
            for d in range(D):
                out[b][h][d] = sum(wi * v[d] for wi, (_, v) in zip(w, tl)) / tot
    return np.array(out)


def test_bruteforce_tiny_mixed_tiers_all_orders():
    """T = 8 tokens, D = G = 32, every order of the four widths; scalar loops vs the oracle cache."""
    D = 32
    rng = np.random.default_rng(5)
    K = rng.standard_normal((1, 2, 8, D)).astype(np.float16)
    V = rng.standard_normal((1, 2, 8, D)).astype(np.float16)
    q = rng.standard_normal((1, 4, D)).astype(np.float16)
    for order in itertools.permutations([16, 8, 4, 2]):
        cfg = CacheConfig(1, 1, 4, 2, head_dim=D, group=32, page_tokens=32, max_tokens=256)
        # page_tokens = 32 but only 2 tokens per width: use one layer per width? No: widths change only at page
        # boundaries, so build four caches of one page each and concatenate by hand for the brute force.
        toks = [[[], []]]
        Kh, Vh = [], []
        for i, bits in enumerate(order):
            c = OracleCache(cfg, [10 ** 9], [2])
            c.append(0, K[:, :, 2 * i:2 * i + 2], V[:, :, 2 * i:2 * i + 2], bits)
            kh, vh = c.dequantized(0)
            Kh.append(kh); Vh.append(vh)
            for h in range(2):
                for t in range(2):
                    kv, vv = K[0, h, 2 * i + t], V[0, h, 2 * i + t]
                    if bits == 16:
                        kd, vd = [float(x) for x in kv], [float(x) for x in vv]
                    else:
                        kd, vd = [], []
                    for src, dst in ((kv, kd), (vv, vd)):
                        if bits == 16:
                            continue
                        lo, hi = float(src.min()), float(src.max())
                        S = float(np.float16(np.float32(np.float32(hi) - np.float32(lo)) / np.float32(2 ** bits - 1)))
                        for x in src:
                            code = 0 if S == 0 else min(max(int(np.rint(np.float32(np.float32(x) - np.float32(lo)) / np.float32(S))), 0), 2 ** bits - 1)
                            dst.append(code * S + lo)
                    toks[0][h].append((kd, vd))
        want = _brute(q.astype(np.float64).tolist(), toks, 2, D)
        got = decode_attention_fp64(q, np.concatenate(Kh, 2), np.concatenate(Vh, 2))
        assert np.allclose(got, want, rtol=0, atol=1e-12)


def _mixed_cache(page_tokens, splits, seed=9, B=1, Hkv=2, Hq=8, T=1024):
    K, V = kvq_synth.make_kv(seed, 0, B, Hkv, 0, T, rope_base=None)
    cfg = CacheConfig(1, B, Hq, Hkv, page_tokens=page_tokens, max_tokens=T)
    c = OracleCache(cfg, [10 ** 12], [2])
    t = 0
    for n, bits in splits:
        c.append(0, K[:, :, t:t + n], V[:, :, t:t + n], bits)
        t += n
    return c, K, V


def test_closed_forms():
    c, K, V = _mixed_cache(128, [(256, 2), (256, 4), (256, 8), (256, 16)])
    Kh, Vh = c.dequantized(0)
    # q = 0 -> uniform weights -> mean of V_hat
    o = c.attention(0, np.zeros((1, 8, 128), np.float16))
    assert np.allclose(o, np.repeat(Vh.mean(2), 4, 1), atol=1e-12)
    # identical V rows -> output is that row
    Vc = np.broadcast_to(Vh[:, :, :1], Vh.shape)
    q = kvq_synth.make_q(9, 0, 1, 8, 0, rope_base=None)
    assert np.allclose(decode_attention_fp64(q, Kh, Vc), np.repeat(Vc[:, :, 0], 4, 1), atol=1e-12)
    # one key with a huge logit dominates
    Kd = Kh.copy() * 1e-3
    t_star = 777
    Kd[:, :, t_star] = q.astype(np.float64).reshape(1, 2, 4, 128)[:, :, 0] * 50.0
    o = decode_attention_fp64(q, Kd, Vh)
    assert np.allclose(o[:, ::4], Vh[:, :, t_star], atol=1e-9)


def test_code_space_identity():
    """q . K_hat = sum_g S_g (q_g . c_g) + Z_g sum(q_g): the form the GPU kernel evaluates."""
    rng = np.random.default_rng(2)
    k = rng.standard_normal((1, 1, 16, 128)).astype(np.float16)
    q = rng.standard_normal(128)
    for b in (2, 4, 8):
        codes, S, Z = quantize(k, b, 32)
        c = OracleCache(CacheConfig(1, 1, 1, 1, page_tokens=32, max_tokens=32), [10 ** 9], [2])
        c.append(0, k, k, b)
        Kh, _ = c.dequantized(0)
        lhs = Kh[0, 0] @ q
        cg = codes[0, 0].reshape(16, 4, 32).astype(np.float64)
        qg = q.reshape(4, 32)
        rhs = (S[0, 0].astype(np.float64) * np.einsum("tgc,gc->tg", cg, qg)).sum(-1) \
            + (Z[0, 0].astype(np.float64) * qg.sum(-1)).sum(-1)
        assert np.allclose(lhs, rhs, atol=1e-10)


def test_invariance_to_page_size_and_append_chunking():
    a, K, V = _mixed_cache(128, [(256, 2), (256, 4), (256, 8), (256, 16)])
    b, _, _ = _mixed_cache(256, [(256, 2), (256, 4), (256, 8), (256, 16)])
    q = kvq_synth.make_q(9, 0, 1, 8, 1023, rope_base=None)
    assert np.array_equal(a.attention(0, q), b.attention(0, q))
    # appending the same tokens in different chunk sizes gives the same cache
    cfg = CacheConfig(1, 1, 8, 2, page_tokens=128, max_tokens=1024)
    c1 = OracleCache(cfg, [10 ** 12], [2]); c2 = OracleCache(cfg, [10 ** 12], [2])
    c1.append(0, K[:, :, :384], V[:, :, :384], 4)
    for t in range(0, 384, 7):
        c2.append(0, K[:, :, t:min(t + 7, 384)], V[:, :, t:min(t + 7, 384)], 4)
    for which in "KV":
        x, y = c1.export_segment(0, 0, which), c2.export_segment(0, 0, which)
        assert all(np.array_equal(p, r) for p, r in zip(x, y))


def test_token_permutation_invariance():
    rng = np.random.default_rng(4)
    K = rng.standard_normal((1, 1, 64, 128)); V = rng.standard_normal((1, 1, 64, 128))
    q = rng.standard_normal((1, 2, 128))
    perm = rng.permutation(64)
    assert np.allclose(decode_attention_fp64(q, K, V), decode_attention_fp64(q, K[:, :, perm], V[:, :, perm]), atol=1e-13)


def test_chain_through_cache_matches_function_chain():
    """16 -> 8 -> 4 -> 2 through the cache equals quantize(8) then Eq. 3 twice on the arrays."""
    K, V = kvq_synth.make_kv(1, 0, 1, 2, 0, 256, rope_base=1e6)
    cfg = CacheConfig(1, 1, 8, 2, page_tokens=128, max_tokens=256)
    c = OracleCache(cfg, [10 ** 12], [2])
    c.append(0, K, V, 16)
    for _ in range(3):
        assert c.requant(0, segment=0) == 2
    assert c.segments(0) == [(0, 256, 2)]
    codes, S, Z = quantize(K, 8, 32)
    for b in (4, 2):
        codes, S = shrink_codes(codes, b), shrink_scale(S, b)
    from oracle import pack_codes
    pc, ps, pz = c.export_segment(0, 0, "K")
    assert np.array_equal(pc, pack_codes(codes, 2)) and np.array_equal(ps, S) and np.array_equal(pz, Z)
    with pytest.raises(Exception):
        c.requant(0, segment=0)
