"""GPU checks of host-side paths of the library: lowering of partly filled pages, the device flags across a cache
reset, and the pinned staging ring once it has wrapped around."""
import numpy as np
import pytest
import torch

import kvq_synth
import paper_2505_18610_amd as kq
from gpu_util import MAX_ABS, REL_L2, append_both, assert_same_cache, attention_errors, check_attention, dev, make_pair

pytestmark = pytest.mark.gpu


def test_lowering_a_partly_filled_page_touches_only_tiles_that_hold_tokens():
    """An arena full of 0x7c bytes (fp16 NaN patterns), a 256-token page holding 40 tokens, lowered 16 -> 8 -> 4: the
    shrink kernels work on the two tiles that hold tokens and leave the six unwritten ones alone -- in the source page
    they would read garbage, which (as a huge V scale) would switch the cache to its slower attention path for good."""
    B, H, P, n = 1, 2, 256, 40
    oc, gc = make_pair(1, B, 4 * H, H, 1024, P)
    gc.arena.fill_(0x7c)
    K, V = kvq_synth.make_kv(1201, 0, B, H, 0, n)
    append_both(oc, gc, 0, K, V, 16)
    torch.cuda.synchronize()
    units, tiles_used = B * H, (n + 31) // 32
    before = int((gc.arena != 0x7c).sum().item())
    assert gc.kvq_progressive_requant(0, segment=0) == oc.requant(0, segment=0) == 1
    torch.cuda.synchronize()
    after8 = int((gc.arena != 0x7c).sum().item())
    # 8-bit codes (2 x 4 KiB per tile and unit) + metadata (1 KiB): what two tiles per unit may add at most
    assert after8 - before <= units * tiles_used * (2 * 4096 + 1024) + 4096, (before, after8)
    assert gc.kvq_progressive_requant(0, segment=0) == oc.requant(0, segment=0) == 1
    torch.cuda.synchronize()
    after4 = int((gc.arena != 0x7c).sum().item())
    assert after4 - after8 <= units * tiles_used * (2 * 2048) + 4096, (after8, after4)
    assert_same_cache(oc, gc, 0)
    q = kvq_synth.make_q(1201, 0, B, 4 * H, n - 1)
    check_attention(oc, gc, 0, q)
    # the fast attention path is still the one in use: deterministic outputs are bit-identical to those of a cache
    # that holds the same tokens and never saw garbage
    oc2, gc2 = make_pair(1, B, 4 * H, H, 1024, P)
    append_both(oc2, gc2, 0, K, V, 16)
    gc2.kvq_progressive_requant(0, segment=0)
    gc2.kvq_progressive_requant(0, segment=0)
    outs = []
    for c in (gc, gc2):
        c.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, 1)
        o = torch.empty(q.shape, dtype=torch.float32, device="cuda")
        c.kvq_decode_attention(0, dev(q), o)
        outs.append(o.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


def test_reset_of_the_whole_cache_clears_the_large_scale_mark():
    """Values with V scales >= 256 mark a cache for the overflow-proof attention path.  The mark belongs to the data:
    after kvq_cache_reset(-1) and a refill with ordinary values the outputs are again bit-identical (deterministic
    mode) to those of a cache that never held large values."""
    B, H, P, T = 1, 2, 64, 300
    K, V = kvq_synth.make_kv(1202, 0, B, H, 0, T)
    Vbig = (V.astype(np.float32) * 600.0).astype(np.float16)
    q = kvq_synth.make_q(1202, 0, B, 4 * H, T - 1)

    def fill_and_attend(oc, gc, v):
        append_both(oc, gc, 0, K, v, 2)
        o = torch.empty(q.shape, dtype=torch.float32, device="cuda")
        gc.kvq_decode_attention(0, dev(q), o)
        torch.cuda.synchronize()
        return o.cpu().numpy()

    oc_ref, gc_ref = make_pair(1, B, 4 * H, H, 512, P)
    gc_ref.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, 1)
    ref = fill_and_attend(oc_ref, gc_ref, V)
    oc, gc = make_pair(1, B, 4 * H, H, 512, P)
    gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, 1)
    big = fill_and_attend(oc, gc, Vbig)                      # marks the cache
    mx, rl = attention_errors(big, oc.attention(0, q))
    assert rl <= REL_L2 and mx <= MAX_ABS * 600.0
    gc.kvq_cache_reset(-1)
    oc2, _ = make_pair(1, B, 4 * H, H, 512, P)
    again = fill_and_attend(oc2, gc, V)
    assert np.array_equal(again, ref)


def test_staging_ring_wraps_without_losing_uploads():
    """Ragged-batch launches read their parameter blocks from the pinned staging ring (one 256-byte aligned block of
    about 0.75 KiB per cache and launch).  Eight caches x 3,000 launches push about 18 MiB through the 4 MiB ring; page
    table uploads of interleaved appends share it.  Every launch's output must be the one the single-cache call gives."""
    Hq, Hkv, P = 8, 2, 32
    lengths = [37, 64, 100, 129, 200, 31, 77, 160]
    pairs, qs, outs, refs = [], [], [], []
    for i, T in enumerate(lengths):
        oc, gc = make_pair(1, 1, Hq, Hkv, 4096, P)
        gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, 1)
        K, V = kvq_synth.make_kv(1300 + i, 0, 1, Hkv, 0, T)
        append_both(oc, gc, 0, K, V, (2, 4, 8, 16)[i % 4])
        pairs.append((oc, gc))
        qs.append(dev(kvq_synth.make_q(1300 + i, 0, 1, Hq, T - 1)))
        outs.append(torch.empty((1, Hq, 128), dtype=torch.float32, device="cuda"))
    caches = [gc for _, gc in pairs]
    for (oc, gc), q, T in zip(pairs, qs, lengths):
        o = torch.empty((1, Hq, 128), dtype=torch.float32, device="cuda")
        gc.kvq_decode_attention(0, q, o)
        refs.append(o)
    torch.cuda.synchronize()
    K1, V1 = kvq_synth.make_kv(1399, 0, 1, Hkv, 0, 3000)
    k1, v1 = dev(K1), dev(V1)
    kq.kvq_decode_attention_batch(caches, 0, qs, outs)
    torch.cuda.synchronize()
    for o, r in zip(outs, refs):                       # other split counts than the single-cache calls: equal up to rounding
        assert float((o - r).abs().max()) <= 1e-3
    refs = [o.clone() for o in outs]                   # from here on bit for bit (deterministic mode, same launch shape)
    for it in range(3000):
        kq.kvq_decode_attention_batch(caches, 0, qs, outs)
        if it % 500 == 499:
            torch.cuda.synchronize()
            for o, r in zip(outs, refs):
                assert torch.equal(o, r), it
            for o in outs:
                o.fill_(float("nan"))
    # appends (page-table uploads through the same ring) between batch launches, then attention against the oracle
    oc, gc = pairs[0]
    for it in range(600):
        k, v = K1[:, :, it:it + 1], V1[:, :, it:it + 1]
        oc.append(0, k, v, (2, 4, 8, 16)[0])
        gc.kvq_quantize_append(0, k1[:, :, it:it + 1].contiguous(), v1[:, :, it:it + 1].contiguous(), 2)
        kq.kvq_decode_attention_batch(caches, 0, qs, outs)
    torch.cuda.synchronize()
    assert_same_cache(oc, gc, 0)
    want = oc.attention(0, qs[0].cpu().numpy())
    mx, rl = attention_errors(outs[0].cpu().numpy(), want)
    assert mx <= MAX_ABS and rl <= REL_L2, (mx, rl)
    for o, r in list(zip(outs, refs))[1:]:
        assert torch.equal(o, r)
