"""kvq_decode_attention_static: the variant of kvq_decode_attention whose split partials and arrival counters live in
a static array of the library's device image, for callers that cannot allocate.  Checked through the C ABI against
kvq_decode_attention (bit-identical in deterministic mode, where both run the same kernels in the same order; within
the attention tolerance otherwise) and against the oracle, on two calls in a row, the second on a smaller cache."""
import numpy as np
import pytest
import torch

import kvq_synth
import paper_2505_18610_amd as kq
from gpu_util import MAX_ABS, REL_L2, append_both, attention_errors, dev, make_pair

pytestmark = pytest.mark.gpu


def _build(seed, B, Hq, Hkv, P, tiers):
    T = sum(n for n, _ in tiers)
    K, V = kvq_synth.make_kv(seed, 0, B, Hkv, 0, T)
    oc, gc = make_pair(1, B, Hq, Hkv, T, P)
    t = 0
    for n, bits in tiers:
        append_both(oc, gc, 0, K[:, :, t:t + n], V[:, :, t:t + n], bits)
        t += n
    q = kvq_synth.make_q(seed, 0, B, Hq, T - 1)
    return oc, gc, q


def _both(gc, q, fill):
    a = torch.full(q.shape, fill, dtype=torch.float32, device="cuda")
    b = torch.full(q.shape, fill, dtype=torch.float32, device="cuda")
    gc.kvq_decode_attention(0, dev(q), a)
    gc.kvq_decode_attention_static(0, dev(q), b)
    torch.cuda.synchronize()
    return a.cpu().numpy(), b.cpu().numpy()


def test_static_scratch_matches_arena_scratch_twice_second_smaller():
    # first call: 2 sequences x 2 KV heads, 2,085 tokens at four widths, many splits per unit
    big = _build(901, 2, 8, 2, 64, ((1024, 2), (512, 4), (448, 8), (101, 16)))
    # second call: a smaller cache (1 sequence, 1 KV head, 331 tokens) whose partials overwrite part of the first's
    small = _build(902, 1, 5, 1, 32, ((160, 4), (171, 16)))
    for det in (1, 0):
        for oc, gc, q in (big, small):
            gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, det)
            print(f"static scratch: deterministic={det} tokens={oc.layers[0].T}", flush=True)
            want = oc.attention(0, q)
            a, b = _both(gc, q, 7.0)
            if det:
                assert np.array_equal(a, b)
            else:
                assert np.abs(a - b).max() <= 1e-3
            mx, rl = attention_errors(b, want)
            assert mx <= MAX_ABS and rl <= REL_L2, (mx, rl)


def test_static_scratch_other_split_counts_and_merge_variant():
    oc, gc, q = _build(903, 1, 16, 2, 64, ((512, 2), (256, 8), (70, 16)))
    want = oc.attention(0, q)
    gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, 1)
    for fused in (1, 0):
        gc.kvq_cache_set_option(kq.KVQ_OPT_FUSED_MERGE, fused)
        for splits in (1, 3, 26, 0):
            gc.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, splits)
            a, b = _both(gc, q, -3.0)
            assert np.array_equal(a, b), (fused, splits)
            mx, rl = attention_errors(b, want)
            assert mx <= MAX_ABS and rl <= REL_L2, (fused, splits, mx, rl)


def test_static_scratch_rejects_launches_beyond_its_size():
    oc, gc, q = _build(904, 8, 8, 8, 32, ((512, 4),))      # 64 units
    out = torch.zeros(q.shape, dtype=torch.float32, device="cuda")
    gc.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, 9)           # 64 x 9 = 576 workgroups > 512
    with pytest.raises(kq.KvqError) as e:
        gc.kvq_decode_attention_static(0, dev(q), out)
    assert e.value.status == kq.KVQ_E_LIMIT
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0                    # nothing was enqueued
    gc.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, 8)           # 512: the maximum
    gc.kvq_decode_attention_static(0, dev(q), out)
    torch.cuda.synchronize()
    mx, rl = attention_errors(out.cpu().numpy(), oc.attention(0, q))
    assert mx <= MAX_ABS and rl <= REL_L2, (mx, rl)
