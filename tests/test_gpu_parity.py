"""GPU parity: the HIP library against the CPU oracle, through the C ABI (run with -m gpu on an MI355X)."""
import numpy as np
import pytest
import torch

import kvq_synth
import paper_2505_18610_amd as kq
from oracle import OracleCache, CacheConfig, BudgetError, POLICY_PAPER, POLICY_OLDEST_FIRST, bytes_per_token_head
from gpu_util import (dev, make_pair, append_both, assert_same_cache, check_attention, attention_errors,
                      MAX_ABS, REL_L2)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits", [16, 8, 4, 2])
def test_append_bit_exact_ragged_chunks(bits):
    B, H, T, P = 2, 2, 427, 128
    K, V = kvq_synth.make_kv(101, 0, B, H, 0, T)
    oc, gc = make_pair(1, B, 2 * H, H, 1024, P)
    t = 0
    for n in (1, 31, 32, 100, 7, 129, 64, 63):
        append_both(oc, gc, 0, K[:, :, t:t + n], V[:, :, t:t + n], bits)
        t += n
    assert t == T
    assert_same_cache(oc, gc, 0)


def test_append_one_shot_equals_token_by_token():
    B, H, T, P = 1, 2, 200, 64
    K, V = kvq_synth.make_kv(102, 0, B, H, 0, T)
    for bits in (4, 2):
        oc, gc = make_pair(1, B, 2 * H, H, 256, P)
        append_both(oc, gc, 0, K, V, bits)
        _, gc2 = make_pair(1, B, 2 * H, H, 256, P)
        for t in range(T):
            gc2.kvq_quantize_append(0, dev(K[:, :, t:t + 1]), dev(V[:, :, t:t + 1]), bits)
        assert_same_cache(oc, gc, 0)
        assert_same_cache(oc, gc2, 0)


def test_quantizer_special_groups():
    """Constant groups (S = 0), a group at the fp16 extremes' scale, tiny ranges, exact ties."""
    B, H, T, P = 1, 1, 64, 32
    rng = np.random.default_rng(3)
    K = rng.standard_normal((B, H, T, 128)).astype(np.float16)
    V = rng.standard_normal((B, H, T, 128)).astype(np.float16)
    K[0, 0, 0, :32] = 0.75            # constant group
    K[0, 0, 1, :] = 0.0               # all-zero token
    K[0, 0, 2, 32:64] = np.linspace(0, 3, 32).astype(np.float16)   # ties at b = 2
    K[0, 0, 3, :32] = (rng.standard_normal(32) * 1e-4).astype(np.float16)   # tiny range
    K[0, 0, 4, 64:96] = (rng.standard_normal(32) * 2000).astype(np.float16)  # large range
    V[0, 0, 5, :] = -2.5
    for bits in (8, 4, 2):
        oc, gc = make_pair(1, B, H, H, 64, P)
        append_both(oc, gc, 0, K, V, bits)
        assert_same_cache(oc, gc, 0)


def test_quantizer_ties_and_near_ties():
    """Groups built on an exact lattice: values at (k + 1/2) S and one fp16 ulp beside it, for every width.  These
    are the inputs where a reciprocal-multiply shortcut and the correctly rounded division of Eq. 1 can disagree."""
    B, H, T, P = 1, 2, 256, 64
    rng = np.random.default_rng(11)
    for bits in (8, 4, 2):
        L = 2 ** bits - 1
        K = np.empty((B, H, T, 128), np.float16)
        for t in range(T):
            for h in range(H):
                for g in range(4):
                    S = np.float16(2.0 ** rng.integers(-6, 3) * rng.choice([1.0, 1.5, 1.25, 0.75]))
                    z = np.float16(rng.integers(-8, 8) * float(S))
                    k = rng.integers(0, L, 32)
                    vals = (k + 0.5) * float(S) + float(z)
                    v16 = vals.astype(np.float16)
                    jitter = rng.integers(-1, 2, 32)
                    v16 = np.where(jitter > 0, np.nextafter(v16, np.float16(np.inf)),
                                   np.where(jitter < 0, np.nextafter(v16, np.float16(-np.inf)), v16)).astype(np.float16)
                    v16[0], v16[1] = z, np.float16(float(z) + L * float(S))     # pin min and max: scale = S
                    K[0, h, t, 32 * g:32 * g + 32] = v16
        assert np.all(np.isfinite(K))
        oc, gc = make_pair(1, B, 2 * H, H, T, P)
        append_both(oc, gc, 0, K, K[:, :, ::-1].copy(), bits)
        assert_same_cache(oc, gc, 0)
        if bits == 8:      # the same data through the fp16 tier and the 16 -> 8 kernel
            oc2, gc2 = make_pair(1, B, 2 * H, H, T, P)
            append_both(oc2, gc2, 0, K, K[:, :, ::-1].copy(), 16)
            assert gc2.kvq_progressive_requant(0, segment=0) == oc2.requant(0, segment=0)
            assert_same_cache(oc2, gc2, 0)


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_quantizer_bulk_random_data_bit_exact(bits):
    """Four million elements per tensor with arbitrary scales: the reciprocal-multiply shortcut of the quantizer meets
    quotients within a few fp32 ulps of a half-integer some tens of times here (8 bits), and every code must still be
    the one the correctly rounded division gives.  Through the append kernel and, for 8 bits, the fp16-page kernel."""
    B, H, T, P = 2, 2, 8192, 256
    rng = np.random.default_rng(900 + bits)
    gain = np.exp(rng.uniform(-4, 4, (B, H, T, 4, 1)))
    K = (rng.standard_normal((B, H, T, 4, 32)) * gain).reshape(B, H, T, 128).astype(np.float16)
    V = (rng.uniform(-1, 1, (B, H, T, 4, 32)) * gain[::-1]).reshape(B, H, T, 128).astype(np.float16)
    oc, gc = make_pair(1, B, 2 * H, H, T, P)
    append_both(oc, gc, 0, K, V, bits)
    assert_same_cache(oc, gc, 0)
    if bits == 8:
        oc2, gc2 = make_pair(1, B, 2 * H, H, T, P)
        append_both(oc2, gc2, 0, K, V, 16)
        assert gc2.kvq_progressive_requant(0, segment=0) == oc2.requant(0, segment=0)
        assert_same_cache(oc2, gc2, 0)


def test_requant_chain_bit_exact():
    B, H, T, P = 2, 2, 512, 128
    K, V = kvq_synth.make_kv(103, 0, B, H, 0, T)
    oc, gc = make_pair(1, B, 2 * H, H, T, P)
    append_both(oc, gc, 0, K, V, 16)
    q = kvq_synth.make_q(103, 0, B, 2 * H, T - 1)
    for want_bits in (8, 4, 2):
        assert gc.kvq_progressive_requant(0, segment=0) == oc.requant(0, segment=0) == T // P
        assert gc.kvq_cache_describe(0)[0] == [(0, T, want_bits)]
        assert_same_cache(oc, gc, 0)
        check_attention(oc, gc, 0, q)
    with pytest.raises(kq.KvqError) as e:
        gc.kvq_progressive_requant(0, segment=0)
    assert e.value.status == kq.KVQ_E_STATE


def test_requant_of_more_pages_than_ride_in_the_kernel_arguments():
    """Short job lists travel in the kernel arguments, long ones through the uploaded table: 210 pages in one call."""
    B, H, P = 1, 1, 32
    T = 210 * P
    K, V = kvq_synth.make_kv(105, 0, B, H, 0, T)
    oc, gc = make_pair(1, B, 2 * H, H, T, P)
    append_both(oc, gc, 0, K, V, 16)
    for want_bits in (8, 4, 2):
        assert gc.kvq_progressive_requant(0, segment=0) == oc.requant(0, segment=0) == 210
        assert gc.kvq_cache_describe(0)[0] == [(0, T, want_bits)]
        assert_same_cache(oc, gc, 0)
    check_attention(oc, gc, 0, kvq_synth.make_q(105, 0, B, 2 * H, T - 1))


def test_shrink_of_directly_quantized_tiers():
    """8 -> 4 and 4 -> 2 starting from tokens that entered at 8 / 4 bits, with a partly filled last page."""
    B, H, P = 1, 2, 64
    K, V = kvq_synth.make_kv(104, 0, B, H, 0, 300)
    oc, gc = make_pair(1, B, 2 * H, H, 512, P)
    append_both(oc, gc, 0, K[:, :, :128], V[:, :, :128], 4)
    append_both(oc, gc, 0, K[:, :, 128:300], V[:, :, 128:300], 8)
    assert gc.kvq_progressive_requant(0, segment=1) == oc.requant(0, segment=1)
    assert gc.kvq_cache_describe(0)[0] == [(0, 300, 4)]
    assert_same_cache(oc, gc, 0)
    assert gc.kvq_progressive_requant(0, segment=0) == oc.requant(0, segment=0)
    assert_same_cache(oc, gc, 0)
    # the partly filled page keeps accepting tokens at the new width
    K2, V2 = kvq_synth.make_kv(104, 0, B, H, 300, 340)
    append_both(oc, gc, 0, K2, V2, 2)
    assert_same_cache(oc, gc, 0)
    check_attention(oc, gc, 0, kvq_synth.make_q(104, 0, B, 2 * H, 339))


@pytest.mark.parametrize("strategy", [0, 1, 2])
def test_shift_strategies_and_reconstruction_error(strategy):
    """The three bit-width shrinking strategies compared in Sec. 4.3.1 (0 Equivalent = Eq. 3, 1 Direct, 2 Modified):
    codes, S and Z after every step of the chain are bit-exact against the oracle (the Modified strategy also
    rewrites Z), attention runs over the result, and the reconstruction error the library reports equals the
    oracle's (fp32 inside a tile, fp64 across tiles: relative 1e-5)."""
    B, H, T, P = 2, 2, 448, 64
    K, V = kvq_synth.make_kv(130 + strategy, 0, B, H, 0, T)
    Kd, Vd = dev(K), dev(V)
    oc, gc = make_pair(1, B, 3 * H, H, 512, P, shift_strategy=strategy)
    append_both(oc, gc, 0, K, V, 16)
    assert gc.kvq_cache_sq_error(0, Kd, Vd) == (0.0, 0.0)
    q = kvq_synth.make_q(130 + strategy, 0, B, 3 * H, T - 1)
    errs = []
    for want_bits in (8, 4, 2):
        assert gc.kvq_progressive_requant(0, segment=0) == oc.requant(0, segment=0)
        assert gc.kvq_cache_describe(0)[0] == [(0, T, want_bits)]
        assert_same_cache(oc, gc, 0)
        check_attention(oc, gc, 0, q)
        got, want = gc.kvq_cache_sq_error(0, Kd, Vd), oc.reconstruction_sq_error(0, K, V)
        assert got[0] == pytest.approx(want[0], rel=1e-5) and got[1] == pytest.approx(want[1], rel=1e-5)
        errs.append(got)
    assert errs[0][0] < errs[1][0] < errs[2][0] and errs[0][1] < errs[1][1] < errs[2][1]
    # a mixed cache: 2-bit pages, then tokens that entered at 8 bits, then a ragged 16-bit tail
    K2, V2 = kvq_synth.make_kv(130 + strategy, 0, B, H, T, T + 50)
    append_both(oc, gc, 0, K2[:, :, :30], V2[:, :, :30], 8)
    Kall, Vall = np.concatenate([K, K2[:, :, :30]], 2), np.concatenate([V, V2[:, :, :30]], 2)
    got, want = gc.kvq_cache_sq_error(0, dev(Kall), dev(Vall)), oc.reconstruction_sq_error(0, Kall, Vall)
    assert got[0] == pytest.approx(want[0], rel=1e-5) and got[1] == pytest.approx(want[1], rel=1e-5)


def test_channel_reparameterization_matches_oracle():
    """Sec. 3.3, Eq. 7-8: lambda from the calibration kernel equals the oracle's (pow in fp64: one fp32 ulp); with the
    same lambda on both sides the stored keys K / lambda are bit-exact at every width and through the shrink chain,
    and attention with q * lambda matches.  The factors cannot be changed once a block holds tokens."""
    from oracle import calibrate_lambda
    B, H, g, T, P = 2, 2, 3, 300, 64
    K, V = kvq_synth.make_kv(140, 0, B, H, 0, T)
    Kc, _ = kvq_synth.make_kv(141, 0, B, H, 0, 128, pos_scale=8.0)       # short calibration keys, interpolated positions
    lam = calibrate_lambda(Kc, 0.5)
    lam_dev = torch.empty((H, 128), dtype=torch.float32, device="cuda")
    kq.kvq_calibrate_lambda(dev(Kc), 0.5, lam_dev)
    assert np.allclose(lam_dev.cpu().numpy(), lam, rtol=3e-7, atol=0)
    q = kvq_synth.make_q(140, 0, B, H * g, T - 1)
    for bits in (16, 8, 4, 2):
        oc, gc = make_pair(1, B, H * g, H, 512, P)
        oc.set_reparam(0, lam)
        gc.kvq_cache_set_reparam(0, dev(lam))
        t = 0
        for n in (1, 70, 129, 100):
            append_both(oc, gc, 0, K[:, :, t:t + n], V[:, :, t:t + n], bits)
            t += n
        assert_same_cache(oc, gc, 0)
        check_attention(oc, gc, 0, q)
        if bits == 16:
            for _ in range(3):
                assert gc.kvq_progressive_requant(0, segment=0) == oc.requant(0, segment=0)
                assert_same_cache(oc, gc, 0)
                check_attention(oc, gc, 0, q)
        with pytest.raises(kq.KvqError) as e:
            gc.kvq_cache_set_reparam(0, None)
        assert e.value.status == kq.KVQ_E_STATE
    # switched off again on an empty block: identical to a cache that never had factors
    oc, gc = make_pair(1, B, H * g, H, 512, P)
    gc.kvq_cache_set_reparam(0, dev(lam))
    gc.kvq_cache_set_reparam(0, None)
    append_both(oc, gc, 0, K, V, 4)
    assert_same_cache(oc, gc, 0)
    check_attention(oc, gc, 0, q)


def test_sensitivity_terms_match_oracle():
    """Sec. 3.2, Eq. 5: || G * (X - Q_b(X)) ||_1 for K and V of a block held at width b, with and without gradient
    tensors, against the oracle (fp32 inside a tile, fp64 across: relative 1e-5); a ragged last tile is covered."""
    from oracle import sensitivity
    B, H, T, P = 2, 2, 427, 64
    K, V = kvq_synth.make_kv(150, 0, B, H, 0, T)
    rng = np.random.default_rng(150)
    GK = rng.standard_normal(K.shape).astype(np.float32)
    GV = (rng.standard_normal(V.shape) ** 2).astype(np.float32)
    Kd, Vd, GKd, GVd = dev(K), dev(V), dev(GK), dev(GV)
    for bits in (16, 8, 4, 2):
        oc, gc = make_pair(1, B, 2 * H, H, 512, P)
        append_both(oc, gc, 0, K, V, bits)
        for gk, gv, gkd, gvd in ((None, None, None, None), (GK, GV, GKd, GVd)):
            got, want = gc.kvq_cache_sensitivity(0, Kd, Vd, gkd, gvd), sensitivity(K, V, bits, 32, gk, gv)
            assert got[0] == pytest.approx(want[0], rel=1e-5, abs=1e-12)
            assert got[1] == pytest.approx(want[1], rel=1e-5, abs=1e-12)


def test_rope_fused_into_the_append():
    """Un-rotated keys plus cos/sin rows of the new tokens' positions: the append kernels rotate (Sec. 3.3, Eq. 9)
    before quantizing, bit-identically to the oracle's fp32 rotation followed by a plain append - at every width,
    across ragged chunks, with the channel-wise reparameterization on top, and with interpolated positions."""
    from oracle import rope_rotate_keys, calibrate_lambda
    B, H, g, T, P = 2, 2, 2, 333, 64
    rng = np.random.default_rng(170)
    K0 = (rng.standard_normal((B, H, T, 128)) * np.where(np.arange(128) % 37 == 0, 12.0, 1.0)).astype(np.float16)
    V = rng.standard_normal((B, H, T, 128)).astype(np.float16)
    for scale, use_lambda in ((1.0, False), (7.5, True)):
        cos, sin = kvq_synth.rope_tables(scale * np.arange(T), 1.0e6)
        Krot = rope_rotate_keys(K0, cos, sin)
        cs = dev(np.concatenate([cos, sin], 1))
        lam = calibrate_lambda(Krot[:, :, :128], 0.5) if use_lambda else None
        q = kvq_synth.make_q(170, 0, B, H * g, T - 1)
        for bits in (16, 8, 4, 2):
            oc, gc = make_pair(1, B, H * g, H, 512, P)
            if use_lambda:
                oc.set_reparam(0, lam)
                gc.kvq_cache_set_reparam(0, dev(lam))
            t = 0
            for n in (1, 63, 200, 69):
                oc.append(0, Krot[:, :, t:t + n], V[:, :, t:t + n], bits)
                gc.kvq_quantize_append_rope(0, dev(K0[:, :, t:t + n]), dev(V[:, :, t:t + n]), cs[t:t + n].contiguous(), bits)
                t += n
            assert_same_cache(oc, gc, 0)
            check_attention(oc, gc, 0, q)


@pytest.mark.parametrize("P,W,splits,det,extras", [(64, 64, 0, 0, False), (96, 96, 1, 0, False), (32, 32, 3, 1, False),
                                                   (64, 128, 0, 0, True)])
def test_fused_append_and_attention_step(P, W, splits, det, extras):
    """kvq_append_decode_attention against the two separate calls and the oracle over a decode loop that crosses
    tile and page boundaries and evicts window pages: identical cache contents at every check point, outputs within
    the tolerance (the chunk-to-wavefront assignment differs, so only the summation order moves).  Variants: pages
    of three tiles, one split (no merge), several splits in deterministic mode, and un-rotated keys with RoPE and the
    channel-wise reparameterization applied inside the fused launch."""
    from oracle import rope_rotate_keys, calibrate_lambda
    B, H, g, T0, steps = 2, 2, 3, P + W + 29, 2 * P + 9
    budget = B * H * (T0 + steps + 2 * P) * 512
    K, V = kvq_synth.make_kv(180, 0, B, H, 0, T0 + steps, rope_base=None if extras else 1.0e6)
    cos, sin = kvq_synth.rope_tables(np.arange(T0 + steps), 1.0e6)
    Kin = rope_rotate_keys(K, cos, sin) if extras else K          # what the oracle and the plain calls are given
    cs = dev(np.concatenate([cos, sin], 1))
    lam = calibrate_lambda(Kin[:, :, :64], 0.5) if extras else None
    caches = []
    for _ in range(2):
        oc, gc = make_pair(1, B, H * g, H, T0 + steps + P, P, budgets=[budget], fbits=[2], window=W)
        if extras:
            oc.set_reparam(0, lam)
            gc.kvq_cache_set_reparam(0, dev(lam))
        gc.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, splits)
        gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, det)
        oc.append(0, Kin[:, :, :T0], V[:, :, :T0])
        gc.kvq_quantize_append(0, dev(Kin[:, :, :T0]), dev(V[:, :, :T0]))
        assert gc.kvq_progressive_requant(0) == oc.requant(0)     # the bulk goes to 8 bits; the window stays 16
        caches.append((oc, gc))
    (oc, plain), (_, fused) = caches
    out_p = torch.empty((B, H * g, 128), dtype=torch.float32, device="cuda")
    out_f = torch.empty_like(out_p)
    for i in range(steps):
        t = T0 + i
        q = kvq_synth.make_q(180, 0, B, H * g, t)
        k1, v1 = dev(Kin[:, :, t:t + 1]), dev(V[:, :, t:t + 1])
        oc.append(0, Kin[:, :, t:t + 1], V[:, :, t:t + 1])
        plain.kvq_quantize_append(0, k1, v1)
        plain.kvq_decode_attention(0, dev(q), out_p)
        if extras:
            fused.kvq_append_decode_attention(0, dev(K[:, :, t:t + 1]), v1, dev(q), out_f, cos_sin=cs[t:t + 1].contiguous())
        else:
            fused.kvq_append_decode_attention(0, k1, v1, dev(q), out_f)
        torch.cuda.synchronize()
        a, b = out_p.cpu().numpy(), out_f.cpu().numpy()
        assert np.abs(a - b).max() <= 1e-3, (i, np.abs(a - b).max())
        if i % 23 == 0 or i == steps - 1 or (t + 1) % P in (0, 1):
            mx, rl = attention_errors(b, oc.attention(0, q))
            assert mx <= MAX_ABS and rl <= REL_L2, (i, mx, rl)
            assert_same_cache(oc, fused, 0)
    assert_same_cache(oc, plain, 0)
    assert any(bits == 8 for _, _, bits in fused.kvq_cache_describe(0)[0])


@pytest.mark.parametrize("group", [64, 128])
def test_group_sizes_64_and_128(group):
    """Quantization groups of 64 and 128 channels (128 is the paper's setting, Sec. 4.1.2): ragged appends at every
    width, the fp16 tier taken down the whole 16 -> 8 -> 4 -> 2 chain, byte accounting with D/G metadata pairs per
    token-head, attention over the result.  Codes, scales and zero points are compared bit for bit in the canonical
    [token][D/G] format."""
    B, H, T, P = 2, 2, 331, 64
    K, V = kvq_synth.make_kv(120 + group, 0, B, H, 0, T)
    for bits in (8, 4, 2):
        oc, gc = make_pair(1, B, 3 * H, H, 512, P, group=group)
        t = 0
        for n in (1, 63, 64, 130, 73):
            append_both(oc, gc, 0, K[:, :, t:t + n], V[:, :, t:t + n], bits)
            t += n
        assert t == T
        assert_same_cache(oc, gc, 0)
        assert gc.kvq_cache_describe(0)[1] == T * B * H * bytes_per_token_head(bits, 128, group, True)
        check_attention(oc, gc, 0, kvq_synth.make_q(120 + group, 0, B, 3 * H, T - 1))
    oc, gc = make_pair(1, B, 3 * H, H, 512, P, group=group)
    append_both(oc, gc, 0, K[:, :, :256], V[:, :, :256], 16)
    q = kvq_synth.make_q(120 + group, 0, B, 3 * H, 255)
    for want_bits in (8, 4, 2):
        assert gc.kvq_progressive_requant(0, segment=0) == oc.requant(0, segment=0)
        assert gc.kvq_cache_describe(0)[0] == [(0, 256, want_bits)]
        assert_same_cache(oc, gc, 0)
        check_attention(oc, gc, 0, q)


@pytest.mark.parametrize("policy,W,sink,fbit", [(POLICY_PAPER, 0, 0, 2), (POLICY_PAPER, 64, 32, 2),
                                                (POLICY_OLDEST_FIRST, 32, 0, 2)])
def test_progressive_decode_run_matches_oracle(policy, W, sink, fbit):
    """A decode loop under a byte budget: append, shrink when the budget is hit, attend; state and outputs match."""
    P, B, H, Tmax = 32, 1, 2, 640
    budget = B * H * (420 * bytes_per_token_head(fbit, 128, 32, True) + (W + sink + 2 * P) * 512)
    oc, gc = make_pair(1, B, 2 * H, H, Tmax, P, budgets=[budget], fbits=[fbit], window=W, n_sink=sink, policy=policy)
    K, V = kvq_synth.make_kv(105, 0, B, H, 0, Tmax)
    rng = np.random.default_rng(5)
    t, events = 0, 0
    while t < Tmax:
        n = min(int(rng.integers(1, 24)), Tmax - t)
        try:
            oc.append(0, K[:, :, t:t + n], V[:, :, t:t + n])
        except BudgetError:
            with pytest.raises(kq.KvqError) as e:
                gc.kvq_quantize_append(0, dev(K[:, :, t:t + n]), dev(V[:, :, t:t + n]))
            assert e.value.status == kq.KVQ_E_BUDGET
            try:
                done = oc.requant(0, reserve_tokens=n)
            except BudgetError:
                with pytest.raises(kq.KvqError) as e:       # steps taken before running out stay, on both sides
                    gc.kvq_progressive_requant(0, reserve_tokens=n)
                assert e.value.status == kq.KVQ_E_BUDGET
                break
            assert gc.kvq_progressive_requant(0, reserve_tokens=n) == done
            events += 1
            assert_same_cache(oc, gc, 0)
            check_attention(oc, gc, 0, kvq_synth.make_q(105, 0, B, 2 * H, t))
            continue
        gc.kvq_quantize_append(0, dev(K[:, :, t:t + n]), dev(V[:, :, t:t + n]))
        t += n
    assert events >= 2
    assert_same_cache(oc, gc, 0)
    check_attention(oc, gc, 0, kvq_synth.make_q(105, 0, B, 2 * H, t))


def _build_workload(w, layer=0, B=None, rope=True):
    B = B or w.batch
    oc, gc = make_pair(1, B, w.n_q_heads, w.n_kv_heads, w.n_tokens, w.page_tokens)
    t = 0
    for n, bits in w.tiers_of_layer(layer):
        K, V = kvq_synth.make_kv(w.seed, layer, B, w.n_kv_heads, t, t + n, rope_base=w.rope_base)
        append_both(oc, gc, 0, K, V, bits)
        t += n
    return oc, gc


def test_attention_tiny_config():
    """BASELINE config 'Tiny': 8 q / 2 kv heads, 4 x 1,024 tokens at 2/4/8/16 bits, outlier channels x20, seed 0."""
    w = kvq_synth.WORKLOADS["tiny"]
    oc, gc = _build_workload(w)
    assert_same_cache(oc, gc, 0)
    q = kvq_synth.make_q(w.seed, 0, 1, 8, 4095, rope_base=None)
    for dt in (torch.float32, torch.float16):
        mx, rl = check_attention(oc, gc, 0, q, dt)
        print("tiny", dt, mx, rl)


@pytest.mark.parametrize("bits", [16, 8, 4, 2])
@pytest.mark.parametrize("gqa", [1, 5, 8, 16])
def test_attention_each_tier_and_group_size(bits, gqa):
    B, H, T, P = 2, 2, 1000, 128
    K, V = kvq_synth.make_kv(200 + bits, 0, B, H, 0, T)
    oc, gc = make_pair(1, B, gqa * H, H, 1024, P)
    append_both(oc, gc, 0, K, V, bits)
    q = kvq_synth.make_q(200 + bits, 0, B, gqa * H, T - 1)
    check_attention(oc, gc, 0, q)


def test_attention_16bit_is_exact_attention():
    B, H, T, P = 1, 2, 777, 64
    K, V = kvq_synth.make_kv(300, 0, B, H, 0, T)
    oc, gc = make_pair(1, B, 4 * H, H, 1024, P)
    append_both(oc, gc, 0, K, V, 16)
    q = kvq_synth.make_q(300, 0, B, 4 * H, T - 1)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    gc.kvq_decode_attention(0, dev(q), out)
    from oracle import decode_attention_fp64
    want = decode_attention_fp64(q, K, V)
    mx, rl = attention_errors(out.cpu().numpy(), want)
    assert mx <= 1e-3 and rl <= 5e-4, (mx, rl)


@pytest.mark.parametrize("T", [1, 2, 31, 32, 33, 127, 129])
def test_attention_short_caches(T):
    B, H, P = 1, 1, 32
    K, V = kvq_synth.make_kv(400 + T, 0, B, H, 0, T)
    for bits in (16, 4):
        oc, gc = make_pair(1, B, 4, H, 256, P)
        append_both(oc, gc, 0, K, V, bits)
        check_attention(oc, gc, 0, kvq_synth.make_q(400, 0, B, 4, T - 1))


def test_large_value_scales_take_the_overflow_proof_path():
    """V ranges far beyond anything an attention layer produces (scales >= 256) switch the kernel to its second
    V path; outputs stay within the tolerance scaled to the magnitude of V, before and after the switch."""
    B, H, T, P = 1, 2, 512, 64
    K, V = kvq_synth.make_kv(600, 0, B, H, 0, T)
    Vbig = (V.astype(np.float32) * 600.0).astype(np.float16)
    oc, gc = make_pair(1, B, 4 * H, H, T, P)
    q = kvq_synth.make_q(600, 0, B, 4 * H, T - 1)

    def check(scale_v):
        out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
        gc.kvq_decode_attention(0, dev(q), out)
        want = oc.attention(0, q)
        mx, rl = attention_errors(out.cpu().numpy(), want)
        assert rl <= REL_L2 and mx <= MAX_ABS * scale_v, (mx, rl)

    append_both(oc, gc, 0, K[:, :, :256], V[:, :, :256], 2)        # ordinary values: fast path
    check(1.0)
    append_both(oc, gc, 0, K[:, :, 256:384], Vbig[:, :, 256:384], 2)   # 2-bit scales ~ 1000: marks the cache
    append_both(oc, gc, 0, K[:, :, 384:], Vbig[:, :, 384:], 4)
    assert_same_cache(oc, gc, 0)
    check(600.0)
    assert gc.kvq_progressive_requant(0, segment=1) == oc.requant(0, segment=1)    # 4 -> 2 keeps it marked
    check(600.0)


def test_empty_cache_is_a_state_error():
    _, gc = make_pair(1, 1, 4, 1, 256, 32)
    out = torch.empty((1, 4, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(kq.KvqError) as e:
        gc.kvq_decode_attention(0, out, out)
    assert e.value.status == kq.KVQ_E_STATE


def test_split_count_and_merge_variant_invariance():
    w = kvq_synth.WORKLOADS["tiny"]
    oc, gc = _build_workload(w)
    q = kvq_synth.make_q(w.seed, 0, 1, 8, 4095, rope_base=None)
    ref = None
    for fused in (0, 1):
        gc.kvq_cache_set_option(kq.KVQ_OPT_FUSED_MERGE, fused)
        for n in (1, 2, 3, 7, 32, 128, 0):
            gc.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, n)
            out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
            for _ in range(3):       # repeated launches reuse the arrival counters
                out.zero_()
                gc.kvq_decode_attention(0, dev(q), out)
            torch.cuda.synchronize()
            o = out.cpu().numpy()
            if ref is None:
                ref = o
                check_attention(oc, gc, 0, q)
            assert np.abs(o - ref).max() <= 5e-4, (fused, n, np.abs(o - ref).max())


def test_ranges_longer_than_the_descriptor_window():
    """A workgroup keeps 256 page descriptors in LDS at a time; one split over 300 pages (and two over 150 + 150
    with odd tile counts) walks several windows.  Mixed widths, odd pages of 96 tokens (three tiles: single-tile
    chunks), deterministic and dynamic claiming."""
    B, H, P, n_pages = 1, 1, 96, 300
    T = P * n_pages - 17
    K, V = kvq_synth.make_kv(160, 0, B, H, 0, T)
    oc, gc = make_pair(1, B, 4 * H, H, P * n_pages, P, policy=POLICY_OLDEST_FIRST)  # new tokens enter at 16 bits
    t = 0
    for n, bits in ((P * 90, 2), (P * 60, 4), (P * 100, 8), (T - P * 250, 16)):
        append_both(oc, gc, 0, K[:, :, t:t + n], V[:, :, t:t + n], bits)
        t += n
    q = kvq_synth.make_q(160, 0, B, 4 * H, T - 1)
    for det in (0, 1):
        gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, det)
        for n in (1, 2, 3, 0):
            gc.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, n)
            check_attention(oc, gc, 0, q)
    # decode steps on the same cache: the launch appends its token, whose tile is in the last of the windows
    K2, V2 = kvq_synth.make_kv(161, 0, B, H, T, T + 6)
    out = torch.empty((B, 4 * H, 128), dtype=torch.float32, device="cuda")
    for i, (det, n) in enumerate(((0, 1), (1, 1), (0, 2), (1, 2), (0, 3), (0, 0))):
        gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, det)
        gc.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, n)
        k1, v1 = K2[:, :, i:i + 1], V2[:, :, i:i + 1]
        q = kvq_synth.make_q(161, 0, B, 4 * H, T + i)
        oc.append(0, k1, v1)
        gc.kvq_append_decode_attention(0, dev(k1), dev(v1), dev(q), out)
        torch.cuda.synchronize()
        mx, rl = attention_errors(out.cpu().numpy(), oc.attention(0, q))
        assert mx <= MAX_ABS and rl <= REL_L2, (det, n, mx, rl)
    assert_same_cache(oc, gc, 0)


def test_softmax_scale_and_multi_layer():
    B, H, T, P = 1, 2, 300, 64
    oc, gc = make_pair(3, B, 2 * H, H, 512, P)
    for layer, bits in enumerate((8, 2, 16)):
        K, V = kvq_synth.make_kv(500, layer, B, H, 0, T)
        append_both(oc, gc, layer, K, V, bits)
    for layer in range(3):
        q = kvq_synth.make_q(500, layer, B, 2 * H, T - 1)
        check_attention(oc, gc, layer, q, scale=0.05)
        assert_same_cache(oc, gc, layer)


def test_full_size_32b_layer_sampled_units():
    """One block of the 32B-shaped workload at full size, in the launch configuration the bench uses; the oracle
    checks sampled (sequence, KV head) units one by one."""
    w = kvq_synth.WORKLOADS["32b"]
    B, Hkv, g = w.batch, w.n_kv_heads, w.n_q_heads // w.n_kv_heads
    cfg = kq.KvqConfig(1, B, w.n_q_heads, Hkv, w.n_tokens, page_tokens=w.page_tokens)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, w.n_tokens * B * Hkv * 320), dtype=torch.uint8, device="cuda")
    gc = kq.KvqCache(cfg, [1 << 50], [2], arena=arena)
    t = 0
    for n, bits in w.tiers:
        K, V = kvq_synth.make_kv(w.seed, 0, B, Hkv, t, t + n)
        gc.kvq_quantize_append(0, dev(K), dev(V), bits)
        t += n
    q = kvq_synth.make_q(w.seed, 0, B, w.n_q_heads, w.n_tokens - 1)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    gc.kvq_decode_attention(0, dev(q), out)
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    # deterministic mode: the two merge variants do the same arithmetic in the same order, so outputs are
    # bit-identical launch after launch; default mode: only the summation order moves (far below the tolerance)
    for det in (1, 0):
        gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, det)
        outs = []
        for fused in (0, 1):
            gc.kvq_cache_set_option(kq.KVQ_OPT_FUSED_MERGE, fused)
            res = []
            for _ in range(6):
                o = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
                gc.kvq_decode_attention(0, dev(q), o)
                res.append(o)
            torch.cuda.synchronize()
            outs += [r.cpu().numpy() for r in res]
        for r in outs:
            if det:
                assert np.array_equal(r, outs[0])
            else:
                assert np.abs(r - got).max() <= 1e-3   # fp16 rounding of p relative to a schedule-dependent maximum
    for b, h in ((0, 0), (3, 7), (1, 4)):
        oc = OracleCache(CacheConfig(1, 1, g, 1, page_tokens=w.page_tokens, max_tokens=w.n_tokens), [1 << 50], [2])
        t = 0
        for n, bits in w.tiers:
            k, v = kvq_synth.make_kv_unit(w.seed, 0, b, h, t, t + n)
            oc.append(0, k[None, None], v[None, None], bits)
            t += n
        want = oc.attention(0, q[b:b + 1, h * g:(h + 1) * g])
        mx, rl = attention_errors(got[b:b + 1, h * g:(h + 1) * g], want)
        print("32b unit", b, h, mx, rl)
        assert mx <= MAX_ABS and rl <= REL_L2, (b, h, mx, rl)


def _sampled_full_size(w, B, units_to_check, layer=0):
    """Build one block of workload w (batch B) through the library and check sampled (sequence, KV head) units
    against the oracle, which builds only those units."""
    Hkv, g = w.n_kv_heads, w.n_q_heads // w.n_kv_heads
    tiers = w.tiers_of_layer(layer)
    cfg = kq.KvqConfig(1, B, w.n_q_heads, Hkv, w.n_tokens, page_tokens=w.page_tokens)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, w.n_tokens * B * Hkv * 560), dtype=torch.uint8, device="cuda")
    gc = kq.KvqCache(cfg, [1 << 50], [2], arena=arena)
    t = 0
    for n, bits in tiers:
        for t0 in range(t, t + n, 16384):          # bounded host memory per append
            t1 = min(t0 + 16384, t + n)
            K, V = kvq_synth.make_kv(w.seed, layer, B, Hkv, t0, t1)
            gc.kvq_quantize_append(0, dev(K), dev(V), bits)
        t += n
    q = kvq_synth.make_q(w.seed, layer, B, w.n_q_heads, w.n_tokens - 1)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    gc.kvq_decode_attention(0, dev(q), out)
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    segs = gc.kvq_cache_describe(0)[0]
    assert [(b - a, bits) for a, b, bits in segs] == [(n, bits) for n, bits in tiers]
    for b, h in units_to_check:
        oc = OracleCache(CacheConfig(1, 1, g, 1, page_tokens=w.page_tokens, max_tokens=w.n_tokens), [1 << 50], [2])
        t = 0
        for n, bits in tiers:
            k, v = kvq_synth.make_kv_unit(w.seed, layer, b, h, t, t + n)
            oc.append(0, k[None, None], v[None, None], bits)
            t += n
        want = oc.attention(0, q[b:b + 1, h * g:(h + 1) * g])
        mx, rl = attention_errors(got[b:b + 1, h * g:(h + 1) * g], want)
        print(w.name, "unit", b, h, mx, rl)
        assert mx <= MAX_ABS and rl <= REL_L2, (w.name, b, h, mx, rl)


def test_full_size_70b_layer_sampled_units():
    """One block of the 70B-shaped workload: 128K tokens, 64 q / 8 kv heads, mostly 2- and 4-bit."""
    _sampled_full_size(kvq_synth.WORKLOADS["70b"], 1, ((0, 0), (0, 5)))


def test_cache_reset_and_reuse():
    """A block that held one sequence is emptied and takes another: contents and attention are those of a fresh cache."""
    B, H, T, P = 1, 2, 300, 64
    oc, gc = make_pair(2, B, 2 * H, H, 512, P)
    K, V = kvq_synth.make_kv(950, 0, B, H, 0, T)
    append_both(oc, gc, 1, K, V, 4)
    gc.kvq_progressive_requant(1, segment=0)
    free_before = gc.kvq_cache_arena_free_bytes()
    gc.kvq_cache_reset(1)
    assert gc.kvq_cache_arena_free_bytes() > free_before and gc.kvq_cache_describe(1)[2] == 0
    oc2, _ = make_pair(2, B, 2 * H, H, 512, P)
    K2, V2 = kvq_synth.make_kv(951, 0, B, H, 0, 200)
    for n, bits in ((64, 2), (64, 8), (72, 16)):
        t = oc2.layers[1].T
        oc2.append(1, K2[:, :, t:t + n], V2[:, :, t:t + n], bits)
        gc.kvq_quantize_append(1, dev(K2[:, :, t:t + n]), dev(V2[:, :, t:t + n]), bits)
    assert_same_cache(oc2, gc, 1)
    check_attention(oc2, gc, 1, kvq_synth.make_q(951, 0, B, 2 * H, 199))


def test_attention_launches_replay_from_a_hip_graph():
    """kvq_decode_attention enqueues kernels only (arguments by value, no copies, no clears), so a sweep over blocks can
    be captured into a HIP graph: replays, interleaved with eager launches and synchronisations, reproduce the eager
    outputs bit for bit in deterministic mode, also after q has been overwritten in place."""
    L, B, H, g, T, P = 3, 2, 2, 4, 700, 64
    oc, gc = make_pair(L, B, H * g, H, 1024, P)
    gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, 1)
    for layer in range(L):
        K, V = kvq_synth.make_kv(960 + layer, layer, B, H, 0, T)
        t = 0
        for n, bits in ((256, 2), (192, 4), (128, 8), (124, 16)):
            append_both(oc, gc, layer, K[:, :, t:t + n], V[:, :, t:t + n], bits)
            t += n
    q = dev(kvq_synth.make_q(960, 0, B, H * g, T - 1))
    outs = [torch.empty((B, H * g, 128), dtype=torch.float32, device="cuda") for _ in range(L)]
    eager = []
    for layer in range(L):
        gc.kvq_decode_attention(layer, q, outs[layer])
    torch.cuda.synchronize()
    eager = [o.clone() for o in outs]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            for layer in range(L):
                gc.kvq_decode_attention(layer, q, outs[layer], stream=torch.cuda.current_stream())
    for rep in range(4):
        for o in outs:
            o.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(outs, eager)), rep
        gc.kvq_decode_attention(rep % L, q, outs[rep % L])           # eager work between the replays
        torch.cuda.synchronize()
    q2 = dev(kvq_synth.make_q(961, 0, B, H * g, T - 1))
    q.copy_(q2)                                                       # same buffer, new queries
    graph.replay()
    torch.cuda.synchronize()
    for layer in range(L):
        mx, rl = attention_errors(outs[layer].cpu().numpy(), oc.attention(layer, q2.cpu().numpy()))
        assert mx <= MAX_ABS and rl <= REL_L2, (layer, mx, rl)
