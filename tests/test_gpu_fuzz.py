"""Randomized configurations and operation sequences on the GPU: after every run the library's cache is bit-identical to
the oracle's, attention and fused decode steps stay within the benchmark spec's tolerance, and the two agree on every refusal
(budget full, nothing left to lower).  Covers what the hand-written cases fix: GQA ratios 1..16, 1..4 KV heads, pages of
32..256 tokens (odd and even tile counts), groups of 32/64/128, both policies, window, sink, both 16-bit tiers, the three
shift strategies, metadata in or out of the budget, split overrides, the unfused merge and static claims."""
import numpy as np
import pytest
import torch

import kvq_synth
import paper_2505_18610_amd as kq
from oracle import BudgetError
from gpu_util import make_pair, assert_same_cache, check_attention, dev, MAX_ABS

pytestmark = pytest.mark.gpu


def _run(trial):
    rng = np.random.default_rng(1000 + trial)
    Hkv, g, B = int(rng.choice([1, 2, 3, 4])), int(rng.choice([1, 2, 4, 5, 7, 8, 16])), int(rng.choice([1, 2, 3]))
    P, group = int(rng.choice([32, 64, 96, 128, 160, 256])), int(rng.choice([32, 64, 128]))
    policy, tier16, meta = int(rng.choice([0, 1])), int(rng.choice([0, 1])), int(rng.choice([0, 1]))
    window, sink = int(rng.choice([0, P, 2 * P])), int(rng.choice([0, P]))
    strat, fbit = int(rng.choice([0, 0, 1, 2])), int(rng.choice([2, 4, 8]))
    Tmax = P * int(rng.integers(6, 24))
    per16 = kq.kvq_bytes_per_token_head(16, 128, group, meta, tier16) * B * Hkv
    budget = int(per16 * Tmax * rng.uniform(0.2, 0.6))
    what = dict(trial=trial, Hkv=Hkv, g=g, B=B, P=P, group=group, policy=policy, window=window, sink=sink, tier16=tier16,
                meta=meta, strat=strat, Tmax=Tmax, fbit=fbit, budget=budget)
    oc, gc = make_pair(1, B, Hkv * g, Hkv, Tmax, P, budgets=[budget], fbits=[fbit], window=window, n_sink=sink,
                       policy=policy, meta=meta, group=group, shift_strategy=strat, tier16=tier16)
    if rng.random() < 0.3:
        gc.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, int(rng.integers(1, 9)))
    if rng.random() < 0.2:
        gc.kvq_cache_set_option(kq.KVQ_OPT_FUSED_MERGE, 0)
    if rng.random() < 0.2:
        gc.kvq_cache_set_option(kq.KVQ_OPT_DETERMINISTIC, 1)
    K, V = kvq_synth.make_kv(5000 + trial, 0, B, Hkv, 0, Tmax)
    out = torch.empty((B, Hkv * g, 128), dtype=torch.float32, device="cuda")
    t = 0
    while t < Tmax:
        n = min(int(rng.choice([1, 1, 1, 3, 17, P, 2 * P + 5])), Tmax - t)
        fused = n == 1 and rng.random() < 0.5
        k, v = K[:, :, t:t + n], V[:, :, t:t + n]
        q = kvq_synth.make_q(5000 + trial, 0, B, Hkv * g, t)

        def library_step():
            if fused:
                gc.kvq_append_decode_attention(0, dev(k), dev(v), dev(q), out)
            else:
                gc.kvq_quantize_append(0, dev(k), dev(v))

        stuck = False
        while True:
            try:
                oc.append(0, k, v)
            except BudgetError:
                with pytest.raises(kq.KvqError) as e:      # the library refuses the same append and changes nothing
                    library_step()
                assert e.value.status == kq.KVQ_E_BUDGET, what
                try:
                    oc.requant(0, reserve_tokens=n)
                except BudgetError:                         # nothing left to lower: the library says so too
                    with pytest.raises(kq.KvqError) as e:
                        gc.kvq_progressive_requant(0, reserve_tokens=n)
                    assert e.value.status == kq.KVQ_E_BUDGET, what
                    stuck = True
                    break
                gc.kvq_progressive_requant(0, reserve_tokens=n)
                continue
            library_step()
            if fused:
                torch.cuda.synchronize()
                d = np.abs(out.cpu().numpy().astype(np.float64) - oc.attention(0, q)).max()
                assert d <= MAX_ABS, (what, t, d)
            break
        if stuck:
            break
        t += n
        if rng.random() < 0.15:
            check_attention(oc, gc, 0, kvq_synth.make_q(5000 + trial, 1, B, Hkv * g, t),
                            out_dtype=torch.float16 if rng.random() < 0.3 else torch.float32)
        if rng.random() < 0.05:
            assert_same_cache(oc, gc, 0)
    assert_same_cache(oc, gc, 0)
    if oc.layers[0].T > 0:
        check_attention(oc, gc, 0, kvq_synth.make_q(5000 + trial, 2, B, Hkv * g, 0))
    gc.close()


@pytest.mark.parametrize("block", range(4))
def test_random_configurations_and_sequences(block):
    for trial in range(16 * block, 16 * block + 16):
        _run(trial)
