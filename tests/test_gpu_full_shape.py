"""Parity at the shapes and launch geometry bench.py runs: whole blocks of the 7B-, 14B- and 70B-shaped workloads at their
full batch, checked on sampled (sequence, KV head) units which the oracle builds one by one; and the progressive
behaviour the workloads name (growth by 4,096-token appends under a real byte budget with both shrink policies; the
whole 16 -> 8 -> 4 -> 2 chain on a 128K-token block) with bit-exact cache contents after the shrinks."""
import numpy as np
import pytest
import torch

import kvq_synth
import paper_2505_18610_amd as kq
from oracle import OracleCache, CacheConfig, BudgetError, POLICY_PAPER, POLICY_OLDEST_FIRST, bytes_per_token_head
from gpu_util import MAX_ABS, REL_L2, attention_errors, dev

pytestmark = pytest.mark.gpu


def _unit_oracle(w, g, b, h, tiers, layer, policy=POLICY_PAPER, budget=1 << 50, page_tokens=None):
    oc = OracleCache(CacheConfig(1, 1, g, 1, page_tokens=page_tokens or w.page_tokens, max_tokens=w.n_tokens,
                                 policy=policy), [budget], [2])
    t = 0
    for n, bits in tiers:
        k, v = kvq_synth.make_kv_unit(w.seed, layer, b, h, t, t + n, rope_base=w.rope_base)
        oc.append(0, k[None, None], v[None, None], bits)
        t += n
    return oc


def _same_unit_contents(oc, gc, b, h, which=("K", "V")):
    _same_contents(gc, [(b, h, oc, which)])


def _same_contents(gc, units):
    """Exported codes, scales and zero points of block 0 against one-unit oracle caches: units = [(b, h, oracle cache,
    which of "K" / "V" to compare)].  Every run is exported once and compared for all the units that ask for it."""
    segs = gc.kvq_cache_describe(0)[0]
    for _, _, oc, _ in units:
        assert segs == oc.segments(0)
    for si in range(len(segs)):
        for name in ("K", "V"):
            takers = [(b, h, oc) for b, h, oc, which in units if name in which]
            if not takers:
                continue
            gcodes, gS, gZ = gc.kvq_cache_export_segment(0, si, kq.KVQ_WHICH_K if name == "K" else kq.KVQ_WHICH_V)
            for b, h, oc in takers:
                ocodes, oS, oZ = oc.export_segment(0, si, name)
                if oS is None:
                    assert np.array_equal(gcodes[b, h].view(np.uint16), ocodes[0, 0].view(np.uint16)), (si, name, b, h)
                else:
                    assert np.array_equal(gcodes[b, h], ocodes[0, 0]), (si, name, b, h, segs[si])
                    assert np.array_equal(gS[b, h].view(np.uint16), oS[0, 0].view(np.uint16)), (si, name, b, h, "scales")
                    assert np.array_equal(gZ[b, h].astype(np.float32), oZ[0, 0].astype(np.float32)), (si, name, b, h, "zeros")


def _full_shape_block(w, units_to_check, layer=0, export_unit=None):
    """One block of workload w at its full batch (the launch bench.py times: batch * KV heads units, the library's own
    split count), sampled units against the oracle; one unit's cache contents bit for bit."""
    B, Hkv, g = w.batch, w.n_kv_heads, w.n_q_heads // w.n_kv_heads
    tiers = w.tiers_of_layer(layer)
    cfg = kq.KvqConfig(1, B, w.n_q_heads, Hkv, w.n_tokens, page_tokens=w.page_tokens)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, w.n_tokens * B * Hkv * 560), dtype=torch.uint8, device="cuda")
    gc = kq.KvqCache(cfg, [1 << 50], [2], arena=arena)
    t = 0
    for n, bits in tiers:
        for t0 in range(t, t + n, 8192):           # bounded host memory per append
            t1 = min(t0 + 8192, t + n)
            K, V = kvq_synth.make_kv(w.seed, layer, B, Hkv, t0, t1, rope_base=w.rope_base)
            gc.kvq_quantize_append(0, dev(K), dev(V), bits)
        t += n
    q = kvq_synth.make_q(w.seed, layer, B, w.n_q_heads, w.n_tokens - 1, rope_base=w.rope_base)
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    gc.kvq_decode_attention(0, dev(q), out)
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    assert [(b_ - a_, bits) for a_, b_, bits in gc.kvq_cache_describe(0)[0]] == [(n, bits) for n, bits in tiers]
    for b, h in units_to_check:
        oc = _unit_oracle(w, g, b, h, tiers, layer)
        want = oc.attention(0, q[b:b + 1, h * g:(h + 1) * g])
        mx, rl = attention_errors(got[b:b + 1, h * g:(h + 1) * g], want)
        print(f"{w.name} layer {layer} ({tiers[0][1]}-bit bulk) unit ({b},{h}): max-abs {mx:.2e} rel-l2 {rl:.2e}", flush=True)
        assert mx <= MAX_ABS and rl <= REL_L2, (w.name, layer, b, h, mx, rl)
        if (b, h) == export_unit:
            _same_unit_contents(oc, gc, b, h)
    gc.close()


def test_7b_block_at_batch_16():
    """7B-shaped: 16 sequences x 4 KV heads = 64 units (4 splits each on 256 compute units), 32,256 4-bit tokens and a
    512-token 16-bit window; four units spread over sequences and heads, one of them with its cache contents."""
    w = kvq_synth.WORKLOADS["7b"]
    assert w.batch == 16
    _full_shape_block(w, ((0, 0), (5, 3), (10, 1), (15, 2)), export_unit=(5, 3))


@pytest.mark.parametrize("bulk_bits", [2, 4, 8])
def test_14b_block_at_batch_8(bulk_bits):
    """14B-shaped: 8 sequences x 8 KV heads = 64 units; one block of each bulk width the workload draws (2, 4 and 8
    bits); four units each, one with its cache contents (2- and 4-bit blocks)."""
    w = kvq_synth.WORKLOADS["14b"]
    assert w.batch == 8 and bulk_bits in w.layer_bits
    layer = w.layer_bits.index(bulk_bits)
    _full_shape_block(w, ((0, 0), (2, 6), (5, 3), (7, 7)), layer=layer, export_unit=(2, 6) if bulk_bits < 8 else None)


def _grow_under_budget(policy, page_tokens, budget_tokens_bits, check_at):
    """A 14B-shaped block (8 x 8 = 64 units) grown by 4,096-token appends to 32,768 tokens under a byte budget; the
    oracle runs the same calls on three sampled units with 1/64 of the budget (all units of a block hold the same
    widths, so the decisions are the same).  After every shrink: segment table and byte accounting; at the
    checkpoints also the sampled units' cache contents bit for bit; attention at the end and at the checkpoints."""
    w = kvq_synth.WORKLOADS["14b"]
    B, Hkv, g, T, step = w.batch, w.n_kv_heads, w.n_q_heads // w.n_kv_heads, w.n_tokens, 4096
    units = B * Hkv
    per_unit_budget = T * bytes_per_token_head(budget_tokens_bits, 128, 32, True)
    cfg = kq.KvqConfig(1, B, w.n_q_heads, Hkv, T, page_tokens=page_tokens, policy=policy)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, int(units * per_unit_budget * 1.6) + units * step * 512 + (64 << 20)),
                        dtype=torch.uint8, device="cuda")
    gc = kq.KvqCache(cfg, [units * per_unit_budget], [2], arena=arena)
    sample = ((0, 0), (3, 5), (7, 2))
    ocs = [OracleCache(CacheConfig(1, 1, g, 1, page_tokens=page_tokens, max_tokens=T, policy=policy), [per_unit_budget], [2])
           for _ in sample]
    events = 0

    def check(t, contents):
        segs, used, T_now, cur = gc.kvq_cache_describe(0)
        for oc in ocs:
            assert segs == oc.segments(0) and used == units * oc.bytes_used(0) and T_now == oc.layers[0].T
            assert cur == oc.current_bits(0)
        if contents:
            q = kvq_synth.make_q(w.seed, 0, B, w.n_q_heads, t - 1)
            out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
            gc.kvq_decode_attention(0, dev(q), out)
            got = out.cpu().numpy()
            _same_contents(gc, [(b, h, oc, ("K", "V") if (b, h) == sample[0] else ("K",)) for (b, h), oc in zip(sample, ocs)])
            for (b, h), oc in zip(sample, ocs):
                mx, rl = attention_errors(got[b:b + 1, h * g:(h + 1) * g], oc.attention(0, q[b:b + 1, h * g:(h + 1) * g]))
                print(f"  t={t} unit ({b},{h}) segments {oc.segments(0)}: max-abs {mx:.2e} rel-l2 {rl:.2e}", flush=True)
                assert mx <= MAX_ABS and rl <= REL_L2, (t, b, h, mx, rl)

    for t0 in range(0, T, step):
        K, V = kvq_synth.make_kv(w.seed, 0, B, Hkv, t0, t0 + step)
        kd, vd = dev(K), dev(V)
        unit_kv = [(K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1]) for b, h in sample]
        try:
            for oc, (k, v) in zip(ocs, unit_kv):
                oc.append(0, k, v)
        except BudgetError:
            with pytest.raises(kq.KvqError) as e:
                gc.kvq_quantize_append(0, kd, vd)
            assert e.value.status == kq.KVQ_E_BUDGET
            done = [oc.requant(0, reserve_tokens=step) for oc in ocs]
            assert gc.kvq_progressive_requant(0, reserve_tokens=step) == done[0] == done[1] == done[2]
            events += 1
            print(f"shrink {events} before token {t0}: {done[0]} pages, now {gc.kvq_cache_describe(0)[0]}", flush=True)
            check(t0, events in check_at)
            for oc, (k, v) in zip(ocs, unit_kv):
                oc.append(0, k, v)
        gc.kvq_quantize_append(0, kd, vd)
    assert events >= 3
    check(T, True)
    gc.close()


def test_14b_block_grows_to_32k_under_the_papers_policy():
    """Policy of Sec. 3.1: budget = 32,768 tokens at 2 bits; the whole block halves its width when an append would not
    fit (16 -> 8 before 8,192 tokens, 8 -> 4 before 12,288, 4 -> 2 before 20,480 with metadata counted).  Pages of 64
    tokens: the last shrink re-quantizes 256 pages, more than ride in the kernel arguments."""
    _grow_under_budget(POLICY_PAPER, 64, 2, check_at=(1, 3))


def test_14b_block_grows_to_32k_oldest_first():
    """Oldest-first policy: budget = 32,768 tokens at 4 bits, new tokens enter at 16 bits, the oldest complete pages go
    down one step at a time until the next 4,096 tokens fit: mixed 2/4/8/16-bit blocks, up to hundreds of page
    re-quantizations per call."""
    _grow_under_budget(POLICY_OLDEST_FIRST, 256, 4, check_at=(2, 5))


def test_70b_block_full_chain_16_8_4_2():
    """70B-shaped block (1 sequence, 8 KV heads, 131,072 tokens) appended at 16 bits and taken through the whole chain
    16 -> 8 -> 4 -> 2 (Eq. 3 after the first step); two units' contents after the last step and attention after each."""
    w = kvq_synth.WORKLOADS["70b"]
    B, Hkv, g, T = w.batch, w.n_kv_heads, w.n_q_heads // w.n_kv_heads, w.n_tokens
    cfg = kq.KvqConfig(1, B, w.n_q_heads, Hkv, T, page_tokens=w.page_tokens)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, int(T * B * Hkv * 512 * 1.7)), dtype=torch.uint8, device="cuda")
    gc = kq.KvqCache(cfg, [1 << 50], [2], arena=arena)
    sample = ((0, 1), (0, 6))
    ocs = [OracleCache(CacheConfig(1, 1, g, 1, page_tokens=w.page_tokens, max_tokens=T), [1 << 50], [2]) for _ in sample]
    for t0 in range(0, T, 16384):
        K, V = kvq_synth.make_kv(w.seed, 0, B, Hkv, t0, t0 + 16384)
        gc.kvq_quantize_append(0, dev(K), dev(V), 16)
        for (b, h), oc in zip(sample, ocs):
            oc.append(0, K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], 16)
    q = kvq_synth.make_q(w.seed, 0, B, w.n_q_heads, T - 1)
    for bits in (8, 4, 2):
        n = gc.kvq_progressive_requant(0, segment=0)
        assert all(oc.requant(0, segment=0) == n for oc in ocs) and n == T // w.page_tokens
        out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
        gc.kvq_decode_attention(0, dev(q), out)
        got = out.cpu().numpy()
        for (b, h), oc in zip(sample, ocs):
            assert gc.kvq_cache_describe(0)[0] == oc.segments(0) == [(0, T, bits)]
            mx, rl = attention_errors(got[b:b + 1, h * g:(h + 1) * g], oc.attention(0, q[b:b + 1, h * g:(h + 1) * g]))
            print(f"70b chain at {bits} bits unit ({b},{h}): max-abs {mx:.2e} rel-l2 {rl:.2e}", flush=True)
            assert mx <= MAX_ABS and rl <= REL_L2, (bits, b, h, mx, rl)
    _same_contents(gc, [(b, h, oc, ("K", "V")) for (b, h), oc in zip(sample, ocs)])
    gc.close()
