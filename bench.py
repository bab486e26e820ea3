#!/usr/bin/env python3
"""Benchmark of the PM-KVQ hot path on one MI355X.

A step is one decode step of the whole path over all transformer blocks: for every block, quantize-append
one new token (K, V) and run single-token GQA attention over the block's mixed-width cache (the shrink step
runs whenever the block's budget asks for it; in the steady state timed here it does not trigger, so its
throughput is measured separately after the timed region and reported under "requant").

Prints ONE JSON line.  value = KV tokens/s = batch * cached tokens * blocks / step time, inputs resident in HBM.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak


def tier_bytes(tiers, units, bpth):
    return sum(n * units * bpth(b) for n, b in tiers)


def build_state(kq, torch, w, steps_total):
    """All blocks of workload w resident in HBM, short of the final context by the tokens the steps will append."""
    import kvq_synth
    B, Hkv, L = w.batch, w.n_kv_heads, w.n_layers
    units = B * Hkv
    tiers0 = list(w.tiers)
    assert steps_total < tiers0[-1][0], "timed steps must fit into the newest tier"
    payload = 0
    for layer in range(L):
        payload += sum(n * units * kq.kvq_bytes_per_token_head(b) for n, b in w.tiers_of_layer(layer))
    payload = int(payload * 1.02) + L * w.page_tokens * units * 512 + (256 << 20)
    cfg = kq.KvqConfig(L, B, w.n_q_heads, Hkv, w.n_tokens, page_tokens=w.page_tokens,
                       policy=kq.KVQ_POLICY_OLDEST_FIRST)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, payload), dtype=torch.uint8, device="cuda")
    cache = kq.KvqCache(cfg, [1 << 60] * L, [2] * L, arena=arena)
    t0 = time.time()
    K, V = kvq_synth.make_kv(w.seed, 0, B, Hkv, 0, w.n_tokens, rope_base=w.rope_base)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    gen_s = time.time() - t0
    append_stats = {}
    filler = QueueFiller(torch, cache)
    for layer in range(L):
        t = 0
        tiers = list(w.tiers_of_layer(layer))
        tiers[-1] = (tiers[-1][0] - steps_total, tiers[-1][1])
        for n, bits in tiers:
            k = Kd[:, :, t:t + n].contiguous()
            v = Vd[:, :, t:t + n].contiguous()
            if layer == 1:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                filler()
                e0.record()
            cache.kvq_quantize_append(layer, k, v, bits)
            if layer == 1:
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1)
                moved = n * units * (512 + kq.kvq_bytes_per_token_head(bits))
                # one-shot construction appends of this workload's tiers; a tier of a few hundred tokens is a
                # launch-bound call, so the token count is part of the key
                append_stats[f"bulk_{bits}bit_{n}tok_GBps"] = round(moved / ms / 1e6, 1)
            t += n
        del k, v
    torch.cuda.synchronize()
    tail = (Kd[:, :, -steps_total:].contiguous(), Vd[:, :, -steps_total:].contiguous())
    del Kd, Vd, filler
    return cache, arena, tail, gen_s, append_stats, (K, V)


class QueueFiller:
    """Keeps the stream busy for a few hundred microseconds (one plain read of 2 GiB) so that a one-shot library
    call measured with events is already queued when the GPU reaches the first event: the host's enqueue time
    (allocator walk, table upload, launch) then stays out of the measured interval."""

    def __init__(self, torch, cache):
        self.cache = cache
        self.buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
        self.buf.fill_(1)

    def __call__(self):
        self.cache.kvq_stream_read_probe(self.buf, 2048)


def measure_requant(kq, torch):
    """16 -> 8 -> 4 -> 2 on 14B-shaped blocks of 16,384 tokens (64 units); GB/s = (read + written) / time.  Each
    shrink of a block can run only once, so one event pair brackets the same step of six blocks, queued back to
    back behind a filler kernel; the time per call includes the call's small job-table upload."""
    B, Hkv, T, P, L = 8, 8, 16384, 256, 6
    units = B * Hkv
    cfg = kq.KvqConfig(L, B, 40, Hkv, T, page_tokens=P)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, int(L * T * units * 512 * 1.7)), dtype=torch.uint8, device="cuda")
    cache = kq.KvqCache(cfg, [1 << 60] * L, [2] * L, arena=arena)
    g = torch.Generator(device="cuda").manual_seed(14)
    k = torch.randn((B, Hkv, T, 128), device="cuda", generator=g).half()
    v = torch.randn((B, Hkv, T, 128), device="cuda", generator=g).half()
    for layer in range(L):
        cache.kvq_quantize_append(layer, k, v, 16)
    del k, v
    elems = T * units * 256
    per_elem = {8: 3.125, 4: 1.75, 2: 1.0}      # algorithmic bytes per element, read + write, group 32
    filler = QueueFiller(torch, cache)
    out = {}
    for b in (8, 4, 2):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        filler()
        e0.record()
        for layer in range(L):
            cache.kvq_progressive_requant(layer, segment=0)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / L
        gbps = elems * per_elem[b] / ms / 1e6
        out[f"{2 * b}to{b}"] = {"ms": round(ms, 4), "GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}
    cache.close()
    return out


def measure_bulk_append(kq, torch):
    """Bulk quantize-on-append of 14B-shaped blocks of 16,384 tokens (64 units) at every entry width; GB/s = (fp16 read
    + codes and metadata written) / time.  Per width a fresh cache on the same arena: one untimed append, then five
    blocks queued back to back behind a filler kernel and one event pair.  K and V inputs are 268 MB each."""
    B, Hkv, T, P, L = 8, 8, 16384, 256, 6
    units = B * Hkv
    cfg = kq.KvqConfig(L, B, 40, Hkv, T, page_tokens=P)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, int(L * T * units * 512 * 1.2)), dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(15)
    k = torch.randn((B, Hkv, T, 128), device="cuda", generator=g).half()
    v = torch.randn((B, Hkv, T, 128), device="cuda", generator=g).half()
    out = {}
    for bits in (16, 8, 4, 2):
        cache = kq.KvqCache(cfg, [1 << 60] * L, [2] * L, arena=arena)
        filler = QueueFiller(torch, cache)
        cache.kvq_quantize_append(0, k, v, bits)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        filler()
        e0.record()
        for layer in range(1, L):
            cache.kvq_quantize_append(layer, k, v, bits)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / (L - 1)
        moved = T * units * (512 + kq.kvq_bytes_per_token_head(bits))
        gbps = moved / ms / 1e6
        out[f"{bits}bit"] = {"ms": round(ms, 4), "MB_moved": round(moved / 1e6, 1), "GBps": round(gbps, 1),
                             "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}
        cache.close()
    return out


def int16_tier(kq, torch, kvq_synth):
    """The integer 16-bit tier (INT16 format of Sec. 4.1.2) beside the raw fp16 tier.
    requant_16to8: Eq. 3 at b = 8 on 14B-shaped blocks of 16,384 tokens (64 units), six blocks behind one event pair as
    in measure_requant; algorithmic bytes per element: 2 read + 1 written + 0.125 of scales re-written (group 32).
    bulk_append: Eq. 1-2 with 65,535 levels, 2 read + 2 written + 0.125 metadata per element.
    attention: trains of launches over 8 blocks of a 7B-shaped block (32,256 4-bit tokens + a 512-token 16-bit window,
    64 units), window raw fp16 against window INT16, alternating, fastest train of each; the error of the two outputs
    against each other (taken before any token is added); and the whole decode step of a block, new token included."""
    B, Hkv, T, P, L = 8, 8, 16384, 256, 6
    units = B * Hkv
    cfg = kq.KvqConfig(L, B, 40, Hkv, T, page_tokens=P)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, int(L * T * units * 544 * 1.7)), dtype=torch.uint8, device="cuda")
    cache = kq.KvqCache(cfg, [1 << 60] * L, [2] * L, arena=arena)
    cache.kvq_cache_set_option(kq.KVQ_OPT_TIER16, kq.KVQ_TIER16_INT16)
    g = torch.Generator(device="cuda").manual_seed(16)
    k = torch.randn((B, Hkv, T, 128), device="cuda", generator=g).half()
    v = torch.randn((B, Hkv, T, 128), device="cuda", generator=g).half()
    filler = QueueFiller(torch, cache)
    elems = T * units * 256
    out = {}
    cache.kvq_quantize_append(0, k, v)                      # first launch of the kernel stays out of the timing
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    filler()
    e0.record()
    for layer in range(1, L):
        cache.kvq_quantize_append(layer, k, v)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / (L - 1)
    out["bulk_append"] = {"ms": round(ms, 4), "GBps": round(elems * 4.125 / ms / 1e6, 1)}
    del k, v
    cache.kvq_progressive_requant(0, segment=0)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    filler()
    e0.record()
    for layer in range(1, L):
        cache.kvq_progressive_requant(layer, segment=0)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / (L - 1)
    gbps = elems * 3.125 / ms / 1e6
    out["requant_16to8"] = {"ms": round(ms, 4), "GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}
    cache.close()
    del arena, filler

    B, Hkv, Hq, Tb, W, P, L = 16, 4, 28, 32256, 512, 256, 8
    units = B * Hkv
    K, V = kvq_synth.make_kv(7, 0, B, Hkv, 0, Tb + W)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    q = torch.from_numpy(kvq_synth.make_q(7, 0, B, Hq, Tb + W - 1)).cuda()
    cfg = kq.KvqConfig(L, B, Hq, Hkv, Tb + W + 64, page_tokens=P, policy=kq.KVQ_POLICY_OLDEST_FIRST)
    res, built = {}, {}
    for name, tier in (("fp16_window", kq.KVQ_TIER16_FP16), ("int16_window", kq.KVQ_TIER16_INT16)):
        arena = torch.empty(kq.kvq_arena_bytes(cfg, int(L * units * (Tb * 160 + W * 544) * 1.1) + (64 << 20)),
                            dtype=torch.uint8, device="cuda")
        cache = kq.KvqCache(cfg, [1 << 60] * L, [2] * L, arena=arena)
        cache.kvq_cache_set_option(kq.KVQ_OPT_TIER16, tier)
        for layer in range(L):
            cache.kvq_quantize_append(layer, Kd[:, :, :Tb].contiguous(), Vd[:, :, :Tb].contiguous(), 4)
            cache.kvq_quantize_append(layer, Kd[:, :, Tb:].contiguous(), Vd[:, :, Tb:].contiguous(), 16)
        built[name] = (cache, arena, torch.empty((B, Hq, 128), dtype=torch.float32, device="cuda"))
    best = {name: 1e9 for name in built}
    for rnd in range(3):                      # alternate the two variants; the fastest train of each counts
        for name, (cache, _, o) in built.items():
            trains = []
            for rep in range(4):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for layer in range(L):
                    cache.kvq_decode_attention(layer, q, o)
                e1.record()
                trains.append((e0, e1))
            torch.cuda.synchronize()
            best[name] = min(best[name], min(a.elapsed_time(b) for a, b in trains[1:]) / L)
    for name, (cache, _, o) in built.items():
        nbytes = cache.kvq_cache_describe(0)[1]
        res[name] = {"us_per_launch": round(best[name] * 1e3, 2), "GBps": round(nbytes / best[name] / 1e6, 1), "out": o.clone()}
    # the whole decode step of a block (one new token + attention, kvq_append_decode_attention: one launch in both tiers)
    k1, v1 = Kd[:, :, :1].contiguous(), Vd[:, :, :1].contiguous()
    step = {name: 1e9 for name in built}
    for rnd in range(3):
        for name, (cache, _, o) in built.items():
            trains = []
            for rep in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for layer in range(L):
                    cache.kvq_append_decode_attention(layer, k1, v1, q, o)
                e1.record()
                trains.append((e0, e1))
            torch.cuda.synchronize()
            step[name] = min(step[name], min(a.elapsed_time(b) for a, b in trains[1:]) / L)
    for name, (cache, _, o) in built.items():
        res[name]["step_us_per_block"] = round(step[name] * 1e3, 2)
        cache.close()
    del built
    a, b = res["fp16_window"].pop("out"), res["int16_window"].pop("out")
    res["rel_l2_between_outputs"] = float(f"{(torch.linalg.norm(a - b) / torch.linalg.norm(a)).item():.3e}")
    out["attention_7b_block"] = res
    return out


def ragged_batch(kq, torch, kvq_synth):
    """Sixteen 7B-shaped sequences (28 q / 4 KV heads) of different lengths, 2,048 ... 32,768 tokens (4-bit bulk + a
    512-token raw window), every sequence in a cache of its own, 8 blocks each: decode attention of one block of all
    sequences as sixteen single-cache launches against one kvq_decode_attention_batch launch, and the whole decode
    step (one new token per sequence + attention) the same two ways; trains over the 8 blocks, HIP events."""
    Hq, Hkv, P, L, W = 28, 4, 256, 8, 512
    lengths = [2048 * (i + 1) for i in range(16)]
    Tmax = max(lengths)
    K, V = kvq_synth.make_kv(7, 0, 1, Hkv, 0, Tmax + 64)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    caches, arenas = [], []
    for T in lengths:
        cfg = kq.KvqConfig(L, 1, Hq, Hkv, T + 64, page_tokens=P, policy=kq.KVQ_POLICY_OLDEST_FIRST)
        arena = torch.empty(kq.kvq_arena_bytes(cfg, int(L * Hkv * (T * 160 + (W + 2 * P) * 512) * 1.1) + (8 << 20)),
                            dtype=torch.uint8, device="cuda")
        c = kq.KvqCache(cfg, [1 << 60] * L, [2] * L, arena=arena)
        for layer in range(L):
            c.kvq_quantize_append(layer, Kd[:, :, :T - W].contiguous(), Vd[:, :, :T - W].contiguous(), 4)
            c.kvq_quantize_append(layer, Kd[:, :, T - W:T].contiguous(), Vd[:, :, T - W:T].contiguous(), 16)
        caches.append(c)
        arenas.append(arena)
    nbytes = sum(c.kvq_cache_describe(0)[1] for c in caches)
    qs = [torch.from_numpy(kvq_synth.make_q(7, 0, 1, Hq, T)).cuda() for T in lengths]
    outs = [torch.empty((1, Hq, 128), dtype=torch.float16, device="cuda") for _ in lengths]
    ks = [Kd[:, :, T:T + 1].contiguous() for T in lengths]
    vs = [Vd[:, :, T:T + 1].contiguous() for T in lengths]

    def train(fn, reps=4):
        times = []
        for rep in range(reps + 1):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for layer in range(L):
                fn(layer)
            e1.record()
            times.append((e0, e1))
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in times[1:]])) / L

    def single(layer):
        for c, q, o in zip(caches, qs, outs):
            c.kvq_decode_attention(layer, q, o)

    def batched(layer):
        kq.kvq_decode_attention_batch(caches, layer, qs, outs)

    def step_single(layer):
        for c, k, v, q, o in zip(caches, ks, vs, qs, outs):
            c.kvq_append_decode_attention(layer, k, v, q, o)

    def step_batched(layer):
        kq.kvq_append_decode_attention_batch(caches, layer, ks, vs, qs, outs)

    res = {"sequences": len(lengths), "tokens_total": sum(lengths), "MB_per_block": round(nbytes / 1e6, 1)}
    for name, fn in (("attention_16_launches", single), ("attention_1_launch", batched)):
        ms = train(fn)
        res[name] = {"us_per_block": round(ms * 1e3, 1), "GBps": round(nbytes / ms / 1e6, 1)}
    # steps append tokens: 5 trains x 8 blocks add 5 tokens per block and sequence, far inside the 64 spare ones
    for name, fn in (("step_16_launches", step_single), ("step_1_launch", step_batched)):
        ms = train(fn)
        res[name] = {"us_per_block": round(ms * 1e3, 1)}
    for c in caches:
        c.close()
    return res


def compare_shift_strategies(kq, torch, kvq_synth):
    """Sec. 4.3.1 without a model: mean squared reconstruction error of K and V after the 16 -> 8 -> 4 -> 2 chain under
    the three bit-width shrinking strategies, on a 14B-shaped slice of the synthetic recipe (8 KV heads, 2 sequences,
    4,096 tokens, RoPE-rotated K with 4 outlier channels per head); all arithmetic runs in the library's kernels."""
    B, Hkv, T, P = 2, 8, 4096, 256
    K, V = kvq_synth.make_kv(14, 0, B, Hkv, 0, T)
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    n = float(K.size)
    cfg = kq.KvqConfig(1, B, 40, Hkv, T, page_tokens=P)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, int(T * B * Hkv * 512 * 1.7)), dtype=torch.uint8, device="cuda")
    out = {}
    for name, st in (("equivalent", kq.KVQ_SHIFT_EQUIVALENT), ("direct", kq.KVQ_SHIFT_DIRECT),
                     ("modified", kq.KVQ_SHIFT_MODIFIED)):
        cache = kq.KvqCache(cfg, [1 << 60], [2], arena=arena)
        cache.kvq_cache_set_option(kq.KVQ_OPT_SHIFT_STRATEGY, st)
        cache.kvq_quantize_append(0, Kd, Vd, 16)
        row = {}
        for b in (8, 4, 2):
            cache.kvq_progressive_requant(0, segment=0)
            ek, ev = cache.kvq_cache_sq_error(0, Kd, Vd)
            row[f"{b}bit"] = {"mse_K": float(f"{ek / n:.4e}"), "mse_V": float(f"{ev / n:.4e}")}
        out[name] = row
        cache.close()
    return out


def reparam_effect(kq, torch, kvq_synth):
    """Sec. 3.3 on the synthetic recipe (4 key channels per head x20): relative L2 error of decode attention over a
    b-bit cache against the same library's attention over the 16-bit cache, without and with the channel-wise
    reparameterization (lambda from 512 calibration tokens rotated at 64x interpolated positions, alpha = 0.5);
    and what the extra multiply costs a bulk append."""
    B, Hkv, Hq, T, P = 2, 8, 40, 8192, 256
    K, V = kvq_synth.make_kv(14, 0, B, Hkv, 0, T)
    # calibration keys: the same heads (same outlier channels), another block's values
    Kc, _ = kvq_synth.make_kv(14, 1, B, Hkv, 0, 512, pos_scale=64.0)
    q = torch.from_numpy(kvq_synth.make_q(14, 0, B, Hq, T - 1)).cuda()
    Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    lam = torch.empty((Hkv, 128), dtype=torch.float32, device="cuda")
    kq.kvq_calibrate_lambda(torch.from_numpy(Kc).cuda(), 0.5, lam)
    cfg = kq.KvqConfig(1, B, Hq, Hkv, T, page_tokens=P)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, int(T * B * Hkv * 512 * 1.2)), dtype=torch.uint8, device="cuda")

    def run(bits, use_lambda, timed=False):
        cache = kq.KvqCache(cfg, [1 << 60], [2], arena=arena)
        if use_lambda:
            cache.kvq_cache_set_reparam(0, lam)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        cache.kvq_quantize_append(0, Kd, Vd, bits)
        e1.record()
        out = torch.empty((B, Hq, 128), dtype=torch.float32, device="cuda")
        cache.kvq_decode_attention(0, q, out)
        torch.cuda.synchronize()
        cache.close()
        return out, e0.elapsed_time(e1)

    exact, _ = run(16, False)
    res = {}
    for bits in (8, 4, 2):
        row = {}
        for name, use in (("plain", False), ("reparam", True)):
            run(bits, use)                                   # warm-up of this variant
            out, ms = run(bits, use)
            row[name + "_rel_l2"] = float(f"{(torch.linalg.norm(out - exact) / torch.linalg.norm(exact)).item():.4e}")
            row[name + "_append_ms"] = round(ms, 4)
        res[f"{bits}bit"] = row
    return res


def allocation_demo(kq, torch, kvq_synth):
    """Sec. 3.2 end to end on synthetic blocks: the library measures s_{i,b} (Eq. 5 with all-ones gradients) of 16
    blocks whose keys differ in outlier strength, and solves Eq. 6 for a budget half-way between uniform 2 and uniform
    4 bits (the situation of Sec. 3.2: uniform 2 bits wastes memory, uniform 4 bits does not fit)."""
    B, Hkv, T, P, N, widths = 1, 8, 2048, 256, 16, (2, 4, 8)
    cfg = kq.KvqConfig(1, B, 40, Hkv, T, page_tokens=P)
    arena = torch.empty(kq.kvq_arena_bytes(cfg, int(T * B * Hkv * 512 * 1.2)), dtype=torch.uint8, device="cuda")
    s, mem = [], []
    for i in range(N):
        K, V = kvq_synth.make_kv(14, i, B, Hkv, 0, T, outlier_gain=1.0 + 2.0 * i)
        Kd, Vd = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
        row = []
        for b in widths:
            cache = kq.KvqCache(cfg, [1 << 60], [2], arena=arena)
            cache.kvq_quantize_append(0, Kd, Vd, b)
            sk, sv = cache.kvq_cache_sensitivity(0, Kd, Vd)
            row.append(sk + sv)
            cache.close()
        s.append(row)
        mem.append([T * B * Hkv * kq.kvq_bytes_per_token_head(b) for b in widths])
    budget = (sum(m[0] for m in mem) + sum(m[1] for m in mem)) // 2
    t0 = time.perf_counter()
    ch, cost, used = kq.kvq_allocate_bits(s, mem, budget)
    solve_ms = (time.perf_counter() - t0) * 1e3
    return {"blocks": N, "widths": list(widths), "budget_bytes": budget, "used_bytes": used,
            "fbit": [widths[c] for c in ch], "total_sensitivity": float(f"{cost:.6e}"),
            "uniform_2bit_sensitivity": float(f"{sum(r[0] for r in s):.6e}"),
            "uniform_4bit_sensitivity": float(f"{sum(r[1] for r in s):.6e}"), "solve_ms": round(solve_ms, 3)}


def measure_read_ceiling(kq, torch, cache):
    """Plain streaming-read kernel over 4 GiB (far beyond the last-level cache): the practical HBM read ceiling."""
    buf = torch.empty(4 << 30, dtype=torch.uint8, device="cuda")
    buf.fill_(1)
    best = 0.0
    for wgs in (512, 2048, 4096, 8192, 16384):
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            cache.kvq_stream_read_probe(buf, wgs)
            e1.record()
            torch.cuda.synchronize()
            if rep:
                best = max(best, buf.numel() / e0.elapsed_time(e1) / 1e6)
    del buf
    return round(best, 1)


def read_clock_state():
    """Clock levels and power policy of the first GPU as the kernel driver exposes them (sysfs; the level marked
    current is the one at the moment of reading, right behind the timed steps).  Empty where sysfs has no such files."""
    import glob
    state = {}
    for card in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        for key, name in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk"), ("performance_level", "power_dpm_force_performance_level")):
            try:
                text = open(os.path.join(card, name)).read().strip()
            except OSError:
                continue
            if key == "performance_level":
                state[key] = text
            else:
                lines = [l.strip() for l in text.splitlines() if l.strip()]
                state[key + "_levels"] = [l.split(":", 1)[1].replace("*", "").strip() for l in lines if ":" in l]
                state[key + "_current"] = next((l.split(":", 1)[1].replace("*", "").strip() for l in lines if l.endswith("*")), None)
        if state:
            break
    return state


def library_source_sha16():
    """Hash of the library's sources (kernels, host code, public header): ties stored counter results to the code."""
    import glob
    import hashlib
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(ROOT, "paper_2505_18610_amd", "csrc", "*.h")) +
                   glob.glob(os.path.join(ROOT, "paper_2505_18610_amd", "csrc", "*.hip")) +
                   glob.glob(os.path.join(ROOT, "paper_2505_18610_amd", "csrc", "*.cpp")) +
                   [os.path.join(ROOT, "include", "kvq.h")])
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def other_workloads(kq, torch, kvq_synth, skip):
    """The decode step's launch (kvq_append_decode_attention) on the other workloads of the configuration list: a few
    distinct resident blocks each (more than a gigabyte, far beyond the last-level cache), trains of back-to-back
    launches, HIP events around the trains.  Cache values are seeded Gaussian draws made on the device (the launch time
    does not depend on them; parity at these shapes is the job of the GPU tests).  14B-shaped: three blocks of each bulk
    width, timed per width; the mean weights the widths as the workload's 48 blocks draw them."""
    res = {}
    for name in ("7b", "14b", "32b", "70b"):
        if name == skip:
            continue
        w = kvq_synth.WORKLOADS[name]
        B, Hkv, Hq, T, P = w.batch, w.n_kv_heads, w.n_q_heads, w.n_tokens, w.page_tokens
        units = B * Hkv
        if w.layer_bits is None:
            layer_tiers = [list(w.tiers)] * {"7b": 4, "32b": 8, "70b": 8}[name]
        else:
            layer_tiers = [[(n, b if b_ == 0 else b_) for n, b_ in w.tiers] for b in (2, 2, 2, 4, 4, 4, 8, 8, 8)]
        L, spare = len(layer_tiers), 64
        payload = sum(n * units * kq.kvq_bytes_per_token_head(b) for tiers in layer_tiers for n, b in tiers)
        cfg = kq.KvqConfig(L, B, Hq, Hkv, T + spare, page_tokens=P, policy=kq.KVQ_POLICY_OLDEST_FIRST)
        arena = torch.empty(kq.kvq_arena_bytes(cfg, int(payload * 1.03) + L * 2 * P * units * 512 + (64 << 20)),
                            dtype=torch.uint8, device="cuda")
        cache = kq.KvqCache(cfg, [1 << 60] * L, [2] * L, arena=arena)
        g = torch.Generator(device="cuda").manual_seed(w.seed)
        chunk = 8192
        kbuf = torch.randn((B, Hkv, chunk, 128), device="cuda", generator=g).half()
        vbuf = torch.randn((B, Hkv, chunk, 128), device="cuda", generator=g).half()
        for layer, tiers in enumerate(layer_tiers):
            for n, bits in tiers:
                for t0 in range(0, n, chunk):
                    m = min(chunk, n - t0)
                    cache.kvq_quantize_append(layer, kbuf[:, :, :m].contiguous(), vbuf[:, :, :m].contiguous(), bits)
        q = torch.randn((B, Hq, 128), device="cuda", generator=g).half()
        out = torch.empty((B, Hq, 128), dtype=torch.float16, device="cuda")
        k1, v1 = kbuf[:, :, :1].contiguous(), vbuf[:, :, :1].contiguous()
        nbytes = [cache.kvq_cache_describe(layer)[1] for layer in range(L)]
        # groups of equal blocks; a train sweeps the blocks of one group several times between one pair of events
        groups = {}
        for layer, tiers in enumerate(layer_tiers):
            groups.setdefault(tiers[0][1] if w.layer_bits is not None else 0, []).append(layer)
        sweeps = 24 // max(len(v) for v in groups.values())
        best = {k: 1e9 for k in groups}
        for _ in range(400 // L):                # the device reaches its sustained clocks only after some tens of ms of work
            for layer in range(L):
                cache.kvq_decode_attention(layer, q, out)
        for rep in range(4):                     # every launch appends one token to its block (64 spare tokens per block)
            for key, layers in groups.items():
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                for layer in layers * 2:         # untimed lead-in: the timed launches are queued behind running work
                    cache.kvq_decode_attention(layer, q, out)
                e0.record()
                for _ in range(sweeps):
                    for layer in layers:
                        cache.kvq_append_decode_attention(layer, k1, v1, q, out)
                e1.record()
                torch.cuda.synchronize()
                if rep:
                    best[key] = min(best[key], e0.elapsed_time(e1) / (sweeps * len(layers)))
        if w.layer_bits is None:
            ms, bytes_launch = float(best[0]), float(np.mean(nbytes))
            entry = {}
        else:
            counts = {b: w.layer_bits.count(b) for b in (2, 4, 8)}
            by_bits = {b: (float(best[b]), float(np.mean([nbytes[i] for i in groups[b]]))) for b in (2, 4, 8)}
            tot = sum(counts.values())
            ms = sum(counts[b] * by_bits[b][0] for b in counts) / tot
            bytes_launch = sum(counts[b] * by_bits[b][1] for b in counts) / tot
            entry = {"by_bulk_width": {f"{b}bit": {"us_per_launch": round(by_bits[b][0] * 1e3, 2),
                                                   "GBps": round(by_bits[b][1] / by_bits[b][0] / 1e6, 1),
                                                   "frac": round(by_bits[b][1] / by_bits[b][0] / 1e6 / HBM_PEAK_GBPS, 4),
                                                   "blocks_of_48": counts[b]} for b in (2, 4, 8)},
                     "mean": "weighted by the workload's draw of bulk widths over its 48 blocks"}
        entry.update({"us_per_launch": round(ms * 1e3, 2), "MB_per_launch": round(bytes_launch / 1e6, 1),
                      "GBps": round(bytes_launch / ms / 1e6, 1), "frac": round(bytes_launch / ms / 1e6 / HBM_PEAK_GBPS, 4),
                      "units": units, "blocks_resident": L})
        res[name] = entry
        cache.close()
        del arena, cache, kbuf, vbuf
        torch.cuda.empty_cache()
    return res


def cpu_baseline(w, KV, q_np, seconds_hint=6.0):
    """The oracle's attention (de-quantize + fp64 attention) on one sequence of one block of the same workload, timed
    twice: with the BLAS pool limited to one thread, and with the pool as the process finds it.  The oracle's loop is
    plain numpy: beyond the matrix products it runs on one core whatever the pool size."""
    from oracle import OracleCache, CacheConfig
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
    except Exception:                                   # pragma: no cover
        threadpool_info = threadpool_limits = None
    K, V = KV
    g = w.n_q_heads // w.n_kv_heads
    oc = OracleCache(CacheConfig(1, 1, w.n_q_heads, w.n_kv_heads, page_tokens=w.page_tokens, max_tokens=w.n_tokens),
                     [1 << 60], [2])
    t = 0
    for n, bits in w.tiers_of_layer(0):
        oc.append(0, K[:1, :, t:t + n], V[:1, :, t:t + n], bits)
        t += n

    def run(seconds):
        reps, t0 = 0, time.time()
        while True:
            oc.attention(0, q_np[:1])
            reps += 1
            if time.time() - t0 > seconds:
                break
        return (time.time() - t0) / reps, reps

    pool = 1
    if threadpool_info is not None:
        pool = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    try:
        nproc = len(os.sched_getaffinity(0))
    except AttributeError:                              # pragma: no cover
        nproc = os.cpu_count() or 1
    dt_all, reps_all = run(seconds_hint)
    single = None
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            dt_1, reps_1 = run(seconds_hint)
        single = {"value": round(w.n_tokens / dt_1, 1), "threads": 1, "repetitions": reps_1, "s_each": round(dt_1, 3)}
    return {"value": round(w.n_tokens / dt_all, 1), "unit": "KV tokens/s", "cores": int(min(pool, nproc)), "kind": "oracle",
            "nproc": int(nproc), "blas_pool_threads": int(pool),
            "all_threads": {"value": round(w.n_tokens / dt_all, 1), "threads": int(min(pool, nproc)),
                            "repetitions": reps_all, "s_each": round(dt_all, 3)},
            "single_thread": single,
            "sample": f"one sequence of one block ({w.n_kv_heads} KV heads x {w.n_tokens} tokens, {g} query heads each), "
                      f"numpy fp64 de-quantize + attention; value = the all-threads figure"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="32b", choices=["7b", "14b", "32b", "70b"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-requant", action="store_true")
    ap.add_argument("--no-workloads", action="store_true", help="skip the short trains on the other workloads")
    ap.add_argument("--separate-calls", action="store_true",
                    help="step = kvq_quantize_append + kvq_decode_attention (two launches) instead of the fused call")
    ap.add_argument("--fused-merge", type=int, default=None)
    ap.add_argument("--splits", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path needs no cross-GPU step); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import kvq_synth
    import paper_2505_18610_amd as kq
    kq.load_library()
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    w = kvq_synth.WORKLOADS[args.workload]
    B, Hkv, Hq, L = w.batch, w.n_kv_heads, w.n_q_heads, w.n_layers
    units = B * Hkv
    n_trains = 5   # timing trains after the timed steps; with the fused step each of them appends one more token
    steps_total = args.steps + args.warmup + (0 if args.separate_calls else n_trains)

    cache, arena, (k_tail, v_tail), gen_s, append_stats, KV = build_state(kq, torch, w, steps_total)
    if args.fused_merge is not None:
        cache.kvq_cache_set_option(kq.KVQ_OPT_FUSED_MERGE, args.fused_merge)
    if args.splits:
        cache.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, args.splits)
    q_np = kvq_synth.make_q(w.seed, 0, B, Hq, w.n_tokens - 1, rope_base=w.rope_base)
    q = torch.from_numpy(q_np).cuda()
    outs = [torch.empty((B, Hq, 128), dtype=torch.float16, device="cuda") for _ in range(L)]
    new_k = [k_tail[:, :, i:i + 1].contiguous() for i in range(steps_total)]
    new_v = [v_tail[:, :, i:i + 1].contiguous() for i in range(steps_total)]
    stream = torch.cuda.current_stream()

    def step(i, events=None):
        # HIP events bracket a rotating sample of the attention launches (every 16th block): recording an event
        # costs several microseconds of stream time, so timing every launch would distort the step itself
        for layer in range(L):
            timed = events is not None and (layer + i) % 16 == 0
            if args.separate_calls:
                cache.kvq_quantize_append(layer, new_k[i], new_v[i], 0, stream)
            if timed:
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record(stream)
            if args.separate_calls:
                cache.kvq_decode_attention(layer, q, outs[layer], 0.0, stream)
            else:   # the same step in one launch: the attention kernel writes the new token itself
                cache.kvq_append_decode_attention(layer, new_k[i], new_v[i], q, outs[layer], None, 0.0, stream)
            if timed:
                e1.record(stream)
                events.append((e0, e1))

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        step(i, events)
    t_issue = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    clocks = read_clock_state()  # outside the timed region, right behind it
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    _, _, T_end, _ = cache.kvq_cache_describe(0)
    T_mid = T_end - args.steps / 2.0
    kv_tokens_per_s = B * T_mid * L / (ms_per_step * 1e-3)

    # roofline of the dominant kernel (fused de-quantize + decode attention, with the one-token append in front
    # unless --separate-calls), one launch = one block.
    # An event pair around a single launch adds several microseconds of its own (the pair's packets sit between
    # kernels), so the launch duration is taken from trains: one event pair around a sweep of the step's own launch
    # over all blocks, back to back on the same stream, continuing the state the timed steps left (a train of the
    # fused step appends one more token per block).  The per-launch figure of the pairs inside the timed steps is
    # kept beside it.
    attn_ms_pairs = float(np.mean([a.elapsed_time(b) for a, b in events]))
    trains = []
    for rep in range(n_trains):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for layer in range(L):
            if args.separate_calls:
                cache.kvq_decode_attention(layer, q, outs[layer], 0.0, stream)
            else:
                i = args.warmup + args.steps + rep
                cache.kvq_append_decode_attention(layer, new_k[i], new_v[i], q, outs[layer], None, 0.0, stream)
        e1.record(stream)
        trains.append((e0, e1))
    torch.cuda.synchronize()
    train_ms = [a.elapsed_time(b) / L for a, b in trains[1:]]
    attn_ms = float(np.mean(train_ms))
    plain_ms = attn_ms
    if not args.separate_calls:   # the attention-only kernel (kvq_decode_attention) beside the step's fused one
        ptrains = []
        for rep in range(n_trains):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for layer in range(L):
                cache.kvq_decode_attention(layer, q, outs[layer], 0.0, stream)
            e1.record(stream)
            ptrains.append((e0, e1))
        torch.cuda.synchronize()
        plain_ms = float(np.mean([a.elapsed_time(b) for a, b in ptrains[1:]])) / L
    bytes_per_launch = 0
    for layer in range(L):
        segs, _, _, _ = cache.kvq_cache_describe(layer)
        bytes_per_launch += sum((t1_ - t0_) * units * kq.kvq_bytes_per_token_head(b) for t0_, t1_, b in segs)
    bytes_per_launch /= L
    achieved = bytes_per_launch / (attn_ms * 1e-3) / 1e9
    # HBM traffic per launch comes from two rocprofv3 --pmc runs of this script (see profiles/); the stored figure is
    # tied to the sources it was measured with and is reported only while they are unchanged
    traffic, traffic_note = None, "no counter run stored for these sources"
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload}.json")
    src_hash = library_source_sha16()
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        if tj.get("library_source_sha16") == src_hash:
            traffic = tj.get("attention_only_kernel", {}).get("hbm_bytes_per_launch") if args.separate_calls \
                else tj.get("hbm_bytes_per_launch")
            traffic_note = f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, sources {src_hash}"
        else:
            traffic_note = f"stored counters belong to sources {tj.get('library_source_sha16')}, these are {src_hash}"
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_note,
                "kernel": "kvq_attention_kernel" if args.separate_calls else "kvq_attention_append_kernel",
                "avg_launch_ms": round(attn_ms, 5),
                "min_launch_ms": round(float(np.min(train_ms)), 5), "median_launch_ms": round(float(np.median(train_ms)), 5),
                "timing": f"HIP events around trains of {L} back-to-back launches (one per block), {n_trains - 1} trains",
                "avg_launch_ms_event_pair_in_steps": round(attn_ms_pairs, 5),
                "algorithmic_bytes_per_launch": int(bytes_per_launch),
                "attention_only_kernel": {"kernel": "kvq_attention_kernel", "avg_launch_ms": round(plain_ms, 5),
                                          "achieved": round(bytes_per_launch / (plain_ms * 1e-3) / 1e9, 1),
                                          "frac": round(bytes_per_launch / (plain_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}}

    result = {
        "metric": "decode-attention KV tokens/s per GPU", "value": round(kv_tokens_per_s, 1), "unit": "KV tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{w.name}-shaped: {L} blocks, {Hq}q/{Hkv}kv heads, head_dim 128, batch {B}, "
                               f"{w.n_tokens} cached tokens, tiers (tokens,bits) {list(w.tiers_of_layer(0))}, group 32, "
                               f"page {w.page_tokens} tokens",
                   "step": "per block: append 1 token + decode attention" +
                           (" (two calls)" if args.separate_calls else " (kvq_append_decode_attention, one launch)"),
                   "layers_share_values": True},
        "hbm_GBps_whole_step": round(bytes_per_launch * L / (ms_per_step * 1e-3) / 1e9, 1),
        "hbm_frac_whole_step": round(bytes_per_launch * L / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": roofline,
        "host_issue_ms_per_step": round((t_issue - t0) * 1e3 / args.steps, 4),
        "append": append_stats,
    }
    del outs
    ceiling = measure_read_ceiling(kq, torch, cache)
    roofline["plain_read_kernel_GBps"] = ceiling
    roofline["frac_of_plain_read_kernel"] = round(achieved / ceiling, 4)
    if not args.no_workloads:
        cache.close()
        del cache, arena
        torch.cuda.empty_cache()
        wl = other_workloads(kq, torch, kvq_synth, skip=args.workload)
        wl[args.workload] = {"us_per_launch": round(attn_ms * 1e3, 2), "MB_per_launch": round(bytes_per_launch / 1e6, 1),
                             "GBps": round(achieved, 1), "frac": round(achieved / HBM_PEAK_GBPS, 4), "units": units,
                             "blocks_resident": L}
        result["workloads"] = wl
    if not args.no_requant:
        result["requant"] = measure_requant(kq, torch)
        result["bulk_append"] = measure_bulk_append(kq, torch)
        result["shift_strategies_mse"] = compare_shift_strategies(kq, torch, kvq_synth)
        result["reparam_effect"] = reparam_effect(kq, torch, kvq_synth)
        result["allocation"] = allocation_demo(kq, torch, kvq_synth)
        result["int16_tier"] = int16_tier(kq, torch, kvq_synth)
        result["ragged_batch"] = ragged_batch(kq, torch, kvq_synth)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, KV, q_np)
    result["setup_seconds"] = {"generate_inputs": round(gen_s, 1)}
    prop = torch.cuda.get_device_properties(0)
    result["device"] = {"name": prop.name, "compute_units": prop.multi_processor_count,
                        "hbm_GiB": round(prop.total_memory / 2 ** 30, 1)}
    result["device"]["clocks"] = clocks
    print(json.dumps(result))


if __name__ == "__main__":
    main()
