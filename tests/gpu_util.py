"""Helpers shared by the GPU parity tests: build the same cache state in the HIP library and in the oracle."""
import numpy as np
import torch

import paper_2505_18610_amd as kq
from oracle import OracleCache, CacheConfig

MAX_ABS = 2e-3   # spec tolerance of attention outputs (fp16 in, fp32 accumulate) against the fp64 oracle
REL_L2 = 1e-3


def dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def make_pair(n_layers, B, Hq, Hkv, max_tokens, P, budgets=None, fbits=None, window=0, n_sink=0, policy=0,
              meta=1, payload_bytes=None, group=32, shift_strategy=0, tier16=0):
    budgets = budgets or [1 << 50] * n_layers
    fbits = fbits or [2] * n_layers
    ocfg = CacheConfig(n_layers, B, Hq, Hkv, page_tokens=P, max_tokens=max_tokens, window=window, n_sink=n_sink,
                       policy=policy, count_metadata_in_budget=meta, group=group, shift_strategy=shift_strategy,
                       tier16=tier16)
    oc = OracleCache(ocfg, budgets, fbits)
    cfg = kq.KvqConfig(n_layers, B, Hq, Hkv, max_tokens, page_tokens=P, window=window, n_sink=n_sink, policy=policy,
                       count_metadata_in_budget=meta, group=group)
    if payload_bytes is None:
        pages = (max_tokens + P - 1) // P + 4
        payload_bytes = n_layers * pages * P * B * Hkv * 512 + (64 << 20)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, payload_bytes), dtype=torch.uint8, device="cuda")
    gc = kq.KvqCache(cfg, budgets, fbits, arena=arena)
    if shift_strategy:
        gc.kvq_cache_set_option(kq.KVQ_OPT_SHIFT_STRATEGY, shift_strategy)
    if tier16:
        gc.kvq_cache_set_option(kq.KVQ_OPT_TIER16, tier16)
    return oc, gc


def append_both(oc, gc, layer, K, V, entry_bits=0):
    oc.append(layer, K, V, entry_bits)
    gc.kvq_quantize_append(layer, dev(K), dev(V), entry_bits)


def assert_same_cache(oc, gc, layer):
    """Bit-exact comparison of segment tables, byte accounting, packed codes, scales and zero points."""
    segs, used, T, cur = gc.kvq_cache_describe(layer)
    assert segs == oc.segments(layer)
    assert used == oc.bytes_used(layer) and T == oc.layers[layer].T and cur == oc.current_bits(layer)
    for si in range(len(segs)):
        for which, name in ((kq.KVQ_WHICH_K, "K"), (kq.KVQ_WHICH_V, "V")):
            gcodes, gS, gZ = gc.kvq_cache_export_segment(layer, si, which)
            ocodes, oS, oZ = oc.export_segment(layer, si, name)
            if oS is None:
                assert gS is None and np.array_equal(gcodes.view(np.uint16), ocodes.view(np.uint16)), (si, name)
            else:
                assert np.array_equal(gcodes, ocodes), (si, name, segs[si])
                assert np.array_equal(gS.view(np.uint16), oS.view(np.uint16)), (si, name, "scales")
                assert np.array_equal(gZ.astype(np.float32), oZ.astype(np.float32)), (si, name, "zeros")


def attention_errors(got: np.ndarray, want: np.ndarray):
    d = got.astype(np.float64) - want
    return float(np.abs(d).max()), float(np.linalg.norm(d) / max(np.linalg.norm(want), 1e-30))


def check_attention(oc, gc, layer, q, out_dtype=torch.float32, scale=0.0):
    out = torch.empty(q.shape, dtype=out_dtype, device="cuda")
    gc.kvq_decode_attention(layer, dev(q), out, softmax_scale=scale)
    torch.cuda.synchronize()
    want = oc.attention(layer, q, None if scale == 0.0 else scale)
    mx, rl = attention_errors(out.float().cpu().numpy(), want)
    extra = 1e-3 * float(np.abs(want).max()) if out_dtype == torch.float16 else 0.0  # fp16 output rounding
    assert mx <= MAX_ABS + extra and rl <= REL_L2 + (5e-4 if out_dtype == torch.float16 else 0.0), (mx, rl)
    return mx, rl
