"""GPU parity of the ragged-batch entry points: several caches of different lengths and states, one attention launch."""
import numpy as np
import pytest
import torch

import kvq_synth
import paper_2505_18610_amd as kq
from oracle import BudgetError, POLICY_PAPER, POLICY_OLDEST_FIRST, TIER16_INT16, bytes_per_token_head, decode_step_batch
from gpu_util import dev, make_pair, append_both, assert_same_cache, attention_errors, MAX_ABS, REL_L2

pytestmark = pytest.mark.gpu


def _build(spec, Hq, Hkv, tier16=0):
    """spec: (batch, page_tokens, seed, ((n_tokens, bits), ...), window)"""
    B, P, seed, tiers, window = spec
    T = sum(n for n, _ in tiers)
    oc, gc = make_pair(1, B, Hq, Hkv, T + 300, P, window=window, policy=POLICY_OLDEST_FIRST, tier16=tier16)
    K, V = kvq_synth.make_kv(seed, 0, B, Hkv, 0, T + 200)
    t = 0
    for n, b in tiers:
        append_both(oc, gc, 0, K[:, :, t:t + n], V[:, :, t:t + n], b)
        t += n
    return oc, gc, K, V, T


SPECS = [(1, 32, 401, ((1, 16),), 0),                                   # a sequence that has just started
         (2, 64, 402, ((640, 2), (320, 4), (128, 8), (77, 16)), 0),     # long, all widths, ragged last tile
         (1, 96, 403, ((288, 4), (50, 16)), 0),                          # pages of three tiles
         (1, 32, 404, ((2048, 2), (31, 16)), 0),
         (3, 32, 405, ((64, 8), (33, 16)), 0)]


@pytest.mark.parametrize("det", [0, 1])
def test_ragged_batch_attention_matches_oracle_and_single_calls(det):
    Hq, Hkv = 10, 2
    built = [_build(s, Hq, Hkv) for s in SPECS]
    qs = [kvq_synth.make_q(s[2], 0, s[0], Hq, b[4] - 1) for s, b in zip(SPECS, built)]
    for _, gc, *_ in built:
        gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, det)
    outs = [torch.empty(q.shape, dtype=torch.float32, device="cuda") for q in qs]
    kq.kvq_decode_attention_batch([b[1] for b in built], 0, [dev(q) for q in qs], outs)
    torch.cuda.synchronize()
    for (oc, gc, *_), q, o in zip(built, qs, outs):
        mx, rl = attention_errors(o.cpu().numpy(), oc.attention(0, q))
        assert mx <= MAX_ABS and rl <= REL_L2, (mx, rl)
        single = torch.empty_like(o)
        gc.kvq_decode_attention(0, dev(q), single)
        torch.cuda.synchronize()
        assert (single - o).abs().max().item() <= 1e-3
    # a second launch right away (arrival counters were left at zero), other order, fp16 outputs
    order = [3, 0, 4, 2, 1]
    outs16 = [torch.empty(qs[i].shape, dtype=torch.float16, device="cuda") for i in order]
    kq.kvq_decode_attention_batch([built[i][1] for i in order], 0, [dev(qs[i]) for i in order], outs16)
    torch.cuda.synchronize()
    for i, o in zip(order, outs16):
        assert (o.float() - outs[i]).abs().max().item() <= 1e-3 + 1e-3 * outs[i].abs().max().item()
    if det:   # bit-reproducible per cache, whatever the batch looks like, and with the merge as separate kernels
        again = [torch.empty_like(o) for o in outs]
        kq.kvq_decode_attention_batch([b[1] for b in built], 0, [dev(q) for q in qs], again)
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(again, outs))
        for _, gc, *_ in built:
            gc.kvq_cache_set_option(kq.KVQ_OPT_FUSED_MERGE, 0)
        unfused = [torch.empty_like(o) for o in outs]
        kq.kvq_decode_attention_batch([b[1] for b in built], 0, [dev(q) for q in qs], unfused)
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(unfused, outs))


@pytest.mark.parametrize("tier16", [0, TIER16_INT16])
def test_ragged_batch_decode_steps(tier16):
    """A decode loop over five caches of different lengths with kvq_append_decode_attention_batch: cache contents stay
    bit-identical to the oracle's, outputs within tolerance, through tile and page boundaries."""
    Hq, Hkv = 8, 2
    specs = [(1, 32, 411, ((20, 16),), 0), (2, 64, 412, ((256, 2), (128, 4), (60, 16)), 0),
             (1, 32, 413, ((96, 8), (31, 16)), 0), (1, 64, 414, ((512, 4), (64, 16)), 64), (1, 32, 415, ((33, 16),), 0)]
    built = [_build(s, Hq, Hkv, tier16) for s in specs]
    ocs, gcs = [b[0] for b in built], [b[1] for b in built]
    outs = [torch.empty((s[0], Hq, 128), dtype=torch.float32, device="cuda") for s in specs]
    for step in range(70):
        ks = [b[2][:, :, b[4] + step:b[4] + step + 1] for b in built]
        vs = [b[3][:, :, b[4] + step:b[4] + step + 1] for b in built]
        qs = [kvq_synth.make_q(s[2], 0, s[0], Hq, b[4] + step) for s, b in zip(specs, built)]
        want = decode_step_batch(ocs, 0, ks, vs, qs)
        kq.kvq_append_decode_attention_batch(gcs, 0, [dev(k) for k in ks], [dev(v) for v in vs], [dev(q) for q in qs], outs)
        if step % 9 == 0 or step == 69:
            torch.cuda.synchronize()
            for o, w in zip(outs, want):
                mx, rl = attention_errors(o.cpu().numpy(), w)
                assert mx <= MAX_ABS and rl <= REL_L2, (step, mx, rl)
    for oc, gc in zip(ocs, gcs):
        assert_same_cache(oc, gc, 0)


def test_ragged_batch_append_is_all_or_nothing_and_arguments_are_checked():
    Hq, Hkv, P = 4, 2, 32
    per16 = bytes_per_token_head(16, 128, 32, True)
    oc0, gc0 = make_pair(1, 1, Hq, Hkv, 256, P, policy=POLICY_OLDEST_FIRST)
    oc1, gc1 = make_pair(1, 1, Hq, Hkv, 256, P, budgets=[Hkv * 64 * per16], policy=POLICY_OLDEST_FIRST)
    K, V = kvq_synth.make_kv(420, 0, 1, Hkv, 0, 100)
    append_both(oc0, gc0, 0, K[:, :, :50], V[:, :, :50])
    append_both(oc1, gc1, 0, K[:, :, :64], V[:, :, :64])                 # exactly full
    k, v = dev(K[:, :, 64:65]), dev(V[:, :, 64:65])
    q = dev(kvq_synth.make_q(420, 0, 1, Hq, 64))
    outs = [torch.empty((1, Hq, 128), dtype=torch.float32, device="cuda") for _ in range(2)]
    with pytest.raises(kq.KvqError) as e:
        kq.kvq_append_decode_attention_batch([gc0, gc1], 0, [k, k], [v, v], [q, q], outs)
    assert e.value.status == kq.KVQ_E_BUDGET
    assert gc0.kvq_cache_describe(0)[2] == 50 and gc1.kvq_cache_describe(0)[2] == 64
    assert_same_cache(oc0, gc0, 0)
    with pytest.raises(kq.KvqError) as e:                                  # the same cache twice
        kq.kvq_decode_attention_batch([gc0, gc0], 0, [q, q], outs)
    assert e.value.status == kq.KVQ_E_INVALID
    _, gi = make_pair(1, 1, Hq, Hkv, 256, P, tier16=TIER16_INT16)
    gi.kvq_quantize_append(0, dev(K[:, :, :10]), dev(V[:, :, :10]))
    with pytest.raises(kq.KvqError) as e:                                  # mixed kinds of 16-bit tier
        kq.kvq_decode_attention_batch([gc0, gi], 0, [q, q], outs)
    assert e.value.status == kq.KVQ_E_INVALID
    _, ge = make_pair(1, 1, Hq, Hkv, 256, P)
    with pytest.raises(kq.KvqError) as e:                                  # an empty cache
        kq.kvq_decode_attention_batch([gc0, ge], 0, [q, q], outs)
    assert e.value.status == kq.KVQ_E_STATE
    # after making room the step goes through for both
    assert gc1.kvq_progressive_requant(0, reserve_tokens=1) == oc1.requant(0, reserve_tokens=1)
    want = decode_step_batch([oc0, oc1], 0, [K[:, :, 64:65]] * 2, [V[:, :, 64:65]] * 2,
                             [kvq_synth.make_q(420, 0, 1, Hq, 64)] * 2)
    kq.kvq_append_decode_attention_batch([gc0, gc1], 0, [k, k], [v, v], [q, q], outs)
    torch.cuda.synchronize()
    for o, w in zip(outs, want):
        mx, rl = attention_errors(o.cpu().numpy(), w)
        assert mx <= MAX_ABS and rl <= REL_L2
    assert_same_cache(oc0, gc0, 0)
    assert_same_cache(oc1, gc1, 0)


def test_full_size_ragged_batch_sampled_sequences():
    """The ragged batch the bench times (sixteen 7B-shaped sequences of 2,048 ... 32,768 tokens, 4-bit bulk and a
    512-token raw window, one cache each) at full size, one block: the step in one launch, then sampled sequences
    checked one by one against the oracle (outputs within tolerance, cache contents bit-exact)."""
    from oracle import OracleCache, CacheConfig
    Hq, Hkv, P, W = 28, 4, 256, 512
    lengths = [2048 * (i + 1) for i in range(16)]
    caches, arenas, data = [], [], []
    for i, T in enumerate(lengths):
        cfg = kq.KvqConfig(1, 1, Hq, Hkv, T + 64, page_tokens=P, policy=kq.KVQ_POLICY_OLDEST_FIRST)
        arena = torch.empty(kq.kvq_arena_bytes(cfg, int(Hkv * (T * 160 + (W + 2 * P) * 512) * 1.1) + (8 << 20)),
                            dtype=torch.uint8, device="cuda")
        c = kq.KvqCache(cfg, [1 << 60], [2], arena=arena)
        K, V = kvq_synth.make_kv(500 + i, 0, 1, Hkv, 0, T + 1)
        c.kvq_quantize_append(0, dev(K[:, :, :T - W]), dev(V[:, :, :T - W]), 4)
        c.kvq_quantize_append(0, dev(K[:, :, T - W:T]), dev(V[:, :, T - W:T]), 16)
        caches.append(c); arenas.append(arena); data.append((K, V))
    qs = [kvq_synth.make_q(500 + i, 0, 1, Hq, T) for i, T in enumerate(lengths)]
    outs = [torch.empty((1, Hq, 128), dtype=torch.float32, device="cuda") for _ in lengths]
    kq.kvq_append_decode_attention_batch(caches, 0, [dev(d[0][:, :, T:T + 1]) for d, T in zip(data, lengths)],
                                         [dev(d[1][:, :, T:T + 1]) for d, T in zip(data, lengths)],
                                         [dev(q) for q in qs], outs)
    torch.cuda.synchronize()
    assert all(bool(torch.isfinite(o).all()) for o in outs)
    for i in (0, 6, 15):
        T, (K, V) = lengths[i], data[i]
        oc = OracleCache(CacheConfig(1, 1, Hq, Hkv, page_tokens=P, max_tokens=T + 64, policy=POLICY_OLDEST_FIRST), [1 << 60], [2])
        oc.append(0, K[:, :, :T - W], V[:, :, :T - W], 4)
        oc.append(0, K[:, :, T - W:T], V[:, :, T - W:T], 16)
        want = decode_step_batch([oc], 0, [K[:, :, T:T + 1]], [V[:, :, T:T + 1]], [qs[i]])[0]
        mx, rl = attention_errors(outs[i].cpu().numpy(), want)
        assert mx <= MAX_ABS and rl <= REL_L2, (i, mx, rl)
        if i == 0:
            assert_same_cache(oc, caches[i], 0)
    for c in caches:
        c.close()


def test_maximum_batch_of_64_caches():
    """The largest batch the entry points take: 64 caches (1 or 2 sequences each, 2 KV heads) of 1 ... ~700 tokens in
    every mix of widths, three decode steps in one launch each; every cache stays bit-identical to its oracle and every
    output within the tolerance.  A 65th cache is refused before anything changes."""
    Hq, Hkv, n = 6, 2, 64
    rng = np.random.default_rng(64)
    built = []
    for i in range(n):
        B, P = int(rng.choice([1, 2])), int(rng.choice([32, 64]))
        tiers = []
        for bits in (2, 4, 8):
            if rng.random() < 0.5:
                tiers.append((P * int(rng.integers(1, 5)), bits))
        tiers.append((int(rng.integers(1, 2 * P)), 16))
        built.append(_build((B, P, 600 + i, tuple(tiers), 0), Hq, Hkv) + (B,))
    ocs, gcs = [b[0] for b in built], [b[1] for b in built]
    outs = [torch.empty((b[5], Hq, 128), dtype=torch.float32, device="cuda") for b in built]
    for step in range(3):
        ks = [b[2][:, :, b[4] + step:b[4] + step + 1] for b in built]
        vs = [b[3][:, :, b[4] + step:b[4] + step + 1] for b in built]
        qs = [kvq_synth.make_q(600 + i, 0, b[5], Hq, b[4] + step) for i, b in enumerate(built)]
        want = decode_step_batch(ocs, 0, ks, vs, qs)
        kq.kvq_append_decode_attention_batch(gcs, 0, [dev(k) for k in ks], [dev(v) for v in vs], [dev(q) for q in qs], outs)
        torch.cuda.synchronize()
        for i in range(n):
            mx, rl = attention_errors(outs[i].cpu().numpy(), want[i])
            assert mx <= MAX_ABS and rl <= REL_L2, (step, i, mx, rl)
    for oc, gc in zip(ocs, gcs):
        assert_same_cache(oc, gc, 0)
    extra = _build((1, 32, 699, ((5, 16),), 0), Hq, Hkv)
    q65 = [dev(kvq_synth.make_q(1, 0, o.shape[0], Hq, 0)) for o in outs] + [dev(kvq_synth.make_q(1, 0, 1, Hq, 0))]
    with pytest.raises(kq.KvqError) as e:
        kq.kvq_decode_attention_batch(gcs + [extra[1]], 0, q65, outs + [torch.empty((1, Hq, 128), dtype=torch.float32, device="cuda")])
    assert e.value.status == kq.KVQ_E_INVALID
