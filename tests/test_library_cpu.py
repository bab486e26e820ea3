"""CPU checks of libkvq: exported symbols, argument errors, and the host bookkeeping (accounting-only caches)
against the oracle's bookkeeping on the same operation sequences.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import kvq_synth
import paper_2505_18610_amd as kq
from oracle import (OracleCache, CacheConfig, BudgetError, StateError, POLICY_PAPER, POLICY_OLDEST_FIRST,
                    bytes_per_token_head, TIER16_INT16)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.skipif(not os.path.exists(kq.library_path()), reason="libkvq.so not built")


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "kvq.h")).read()
    declared = set(re.findall(r"\b(kvq_[a-z0-9_]+)\s*\(", header))
    assert declared == set(kq.exported_symbols())
    lib = ctypes.CDLL(kq.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_bytes_per_token_head_matches_oracle_and_paper_shapes():
    for b in (16, 8, 4, 2):
        for G in (32, 64, 128):
            for m in (0, 1):
                assert kq.kvq_bytes_per_token_head(b, 128, G, m) == bytes_per_token_head(b, 128, G, bool(m))
                assert kq.kvq_bytes_per_token_head(b, 128, G, m, 1) == bytes_per_token_head(b, 128, G, bool(m), True)
    assert kq.kvq_bytes_per_token_head(16, 128, 32, 1, 1) == 544
    assert kq.kvq_bytes_per_token_head(3) == 0


def test_invalid_configs_and_arguments():
    good = dict(n_layers=1, batch=1, n_q_heads=8, n_kv_heads=2, max_tokens=1024, page_tokens=128)
    for bad in (dict(head_dim=64), dict(group=16), dict(group=96), dict(page_tokens=48), dict(n_q_heads=7), dict(window=100),
                dict(n_sink=5), dict(policy=7), dict(n_q_heads=64, n_kv_heads=2)):
        cfg = kq.KvqConfig(**{**good, **bad})
        assert kq.kvq_arena_bytes(cfg, 0) == 0
        with pytest.raises(kq.KvqError) as e:
            kq.KvqCache(cfg, [1 << 30], [2], arena=None, arena_bytes=1 << 30)
        assert e.value.status == kq.KVQ_E_INVALID
    cfg = kq.KvqConfig(**good)
    with pytest.raises(kq.KvqError):
        kq.KvqCache(cfg, [1 << 30], [3], arena=None, arena_bytes=1 << 30)          # Fbit not a power of two
    with pytest.raises(kq.KvqError) as e:
        kq.KvqCache(cfg, [1 << 30], [2], arena=None, arena_bytes=1024)             # arena too small
    assert e.value.status == kq.KVQ_E_OOM
    c = kq.KvqCache(cfg, [1 << 30], [2], arena=None, arena_bytes=1 << 26)
    for call, status in ((lambda: c.kvq_quantize_append(1, None, None, n_new=1), kq.KVQ_E_INVALID),
                         (lambda: c.kvq_quantize_append(0, None, None, n_new=1, entry_bits=3), kq.KVQ_E_INVALID),
                         (lambda: c.kvq_quantize_append(0, None, None, n_new=2000), kq.KVQ_E_STATE),
                         (lambda: c.kvq_progressive_requant(0, segment=0), kq.KVQ_E_STATE)):
        with pytest.raises(kq.KvqError) as e:
            call()
        assert e.value.status == status
    c.kvq_quantize_append(0, None, None, n_new=40, entry_bits=8)
    with pytest.raises(kq.KvqError) as e:
        c.kvq_quantize_append(0, None, None, n_new=8, entry_bits=4)                # width change inside a page
    assert e.value.status == kq.KVQ_E_STATE
    assert c.kvq_cache_describe(0)[0] == [(0, 40, 8)]
    assert kq.kvq_status_string(kq.KVQ_E_OOM) != kq.kvq_status_string(kq.KVQ_OK)
    # one append call takes fewer than 2^23 tokens (the kernels address a unit's new rows with 32-bit byte offsets)
    big = kq.KvqCache(kq.KvqConfig(**{**good, "max_tokens": 1 << 24, "page_tokens": 1024}), [1 << 60], [2], arena=None,
                      arena_bytes=1 << 40)
    with pytest.raises(kq.KvqError) as e:
        big.kvq_quantize_append(0, None, None, n_new=1 << 23, entry_bits=2)
    assert e.value.status == kq.KVQ_E_INVALID
    big.kvq_quantize_append(0, None, None, n_new=(1 << 23) - 1, entry_bits=2)
    assert big.kvq_cache_describe(0)[2] == (1 << 23) - 1


def _pair(policy, P, W, sink, budget, fbit, meta=1, Tmax=4096, B=2, H=2, group=32, tier16=0):
    ocfg = CacheConfig(1, B, 2 * H, H, page_tokens=P, max_tokens=Tmax, window=W, n_sink=sink, policy=policy,
                       count_metadata_in_budget=meta, group=group, tier16=tier16)
    oc = OracleCache(ocfg, [budget], [fbit])
    cfg = kq.KvqConfig(1, B, 2 * H, H, Tmax, page_tokens=P, window=W, n_sink=sink, policy=policy,
                       count_metadata_in_budget=meta, group=group)
    gc = kq.KvqCache(cfg, [budget], [fbit], arena=None, arena_bytes=1 << 30)
    if tier16:
        gc.kvq_cache_set_option(kq.KVQ_OPT_TIER16, tier16)
    return oc, gc


def _same_state(oc, gc):
    segs, used, T, cur = gc.kvq_cache_describe(0)
    assert segs == oc.segments(0)
    assert used == oc.bytes_used(0)
    assert T == oc.layers[0].T
    assert cur == oc.current_bits(0)


@pytest.mark.parametrize("policy,W,sink,fbit,tier16", [(POLICY_PAPER, 0, 0, 2, 0), (POLICY_PAPER, 64, 32, 2, 0),
                                                       (POLICY_PAPER, 64, 0, 4, 0), (POLICY_OLDEST_FIRST, 32, 0, 2, 0),
                                                       (POLICY_OLDEST_FIRST, 0, 32, 4, 0),
                                                       (POLICY_PAPER, 64, 32, 2, TIER16_INT16),
                                                       (POLICY_PAPER, 0, 0, 4, TIER16_INT16),
                                                       (POLICY_OLDEST_FIRST, 32, 32, 2, TIER16_INT16)])
def test_bookkeeping_matches_oracle_on_random_decode_runs(policy, W, sink, fbit, tier16):
    P, B, H = 32, 2, 2
    rng = np.random.default_rng(hash((policy, W, sink, fbit)) % 2 ** 32)
    per16 = bytes_per_token_head(16, 128, 32, True, bool(tier16))
    budget = B * H * (500 * bytes_per_token_head(fbit, 128, 32, True) + (W + sink + 2 * P) * per16)
    oc, gc = _pair(policy, P, W, sink, budget, fbit, Tmax=1024, B=B, H=H, tier16=tier16)
    K, V = kvq_synth.make_kv(77, 0, B, H, 0, 1024, rope_base=None)
    t = 0
    exhausted = False
    while t < 1024 and not exhausted:
        n = int(rng.integers(1, 40))
        n = min(n, 1024 - t)
        try:
            oc.append(0, K[:, :, t:t + n], V[:, :, t:t + n])
            ok = True
        except BudgetError:
            ok = False
        if ok:
            gc.kvq_quantize_append(0, None, None, n_new=n)
            t += n
        else:
            with pytest.raises(kq.KvqError) as e:
                gc.kvq_quantize_append(0, None, None, n_new=n)
            assert e.value.status == kq.KVQ_E_BUDGET
            _same_state(oc, gc)
            try:
                done = oc.requant(0, reserve_tokens=n)
            except BudgetError:
                with pytest.raises(kq.KvqError) as e:
                    gc.kvq_progressive_requant(0, reserve_tokens=n)
                assert e.value.status == kq.KVQ_E_BUDGET
                exhausted = True
            else:
                assert gc.kvq_progressive_requant(0, reserve_tokens=n) == done
        _same_state(oc, gc)
    assert exhausted and t > 400


@pytest.mark.parametrize("group", [64, 128])
def test_bookkeeping_with_larger_groups(group):
    """Groups of 64 / 128 channels change the bytes per token-head (fewer scale / zero-point pairs), hence every
    budget decision; the paper's own setting is 128 (Sec. 4.1.2)."""
    P, B, H, fbit = 32, 2, 2, 2
    budget = B * H * (200 * bytes_per_token_head(fbit, 128, group, True) + P * 512)
    oc, gc = _pair(POLICY_PAPER, P, 0, 0, budget, fbit, Tmax=512, B=B, H=H, group=group)
    K, V = kvq_synth.make_kv(78, 0, B, H, 0, 512, rope_base=None)
    t, exhausted = 0, False
    while t < 512 and not exhausted:
        n = min(17, 512 - t)
        try:
            oc.append(0, K[:, :, t:t + n], V[:, :, t:t + n])
            gc.kvq_quantize_append(0, None, None, n_new=n)
            t += n
        except BudgetError:
            with pytest.raises(kq.KvqError):
                gc.kvq_quantize_append(0, None, None, n_new=n)
            try:
                done = oc.requant(0, reserve_tokens=n)
                assert gc.kvq_progressive_requant(0, reserve_tokens=n) == done
            except BudgetError:
                with pytest.raises(kq.KvqError):
                    gc.kvq_progressive_requant(0, reserve_tokens=n)
                exhausted = True
        _same_state(oc, gc)
    assert exhausted and 200 <= t < 512


def test_explicit_construction_and_segment_requant_match_oracle():
    oc, gc = _pair(POLICY_PAPER, 64, 0, 0, 1 << 40, 2, Tmax=2048, B=1, H=2)
    K, V = kvq_synth.make_kv(78, 0, 1, 2, 0, 2048, rope_base=None)
    t = 0
    for n, b in ((256, 2), (320, 4), (448, 8), (100, 16)):
        oc.append(0, K[:, :, t:t + n], V[:, :, t:t + n], b)
        gc.kvq_quantize_append(0, None, None, n_new=n, entry_bits=b)
        t += n
    _same_state(oc, gc)
    for seg in (3, 2, 1):
        assert gc.kvq_progressive_requant(0, segment=seg) == oc.requant(0, segment=seg)
        _same_state(oc, gc)
    with pytest.raises(StateError):
        oc.requant(0, segment=0)
    with pytest.raises(kq.KvqError) as e:
        gc.kvq_progressive_requant(0, segment=0)
    assert e.value.status == kq.KVQ_E_STATE


def test_arena_accounting_and_reuse():
    cfg = kq.KvqConfig(2, 1, 2, 1, 4096, page_tokens=128)
    need = kq.kvq_arena_bytes(cfg, 0)
    unit = 32 * 128 * 1
    c = kq.KvqCache(cfg, [1 << 40, 1 << 40], [2, 2], arena=None, arena_bytes=need + 3 * 16 * unit)
    free0 = c.kvq_cache_arena_free_bytes()
    assert free0 == 3 * 16 * unit
    for _ in range(3):
        c.kvq_quantize_append(0, None, None, n_new=128, entry_bits=16)
    with pytest.raises(kq.KvqError) as e:
        c.kvq_quantize_append(1, None, None, n_new=1, entry_bits=16)
    assert e.value.status == kq.KVQ_E_OOM and c.kvq_cache_describe(1)[2] == 0
    # shrinking needs room for the new block first: 16 -> 8 of one page cannot start with a full arena
    with pytest.raises(kq.KvqError) as e:
        c.kvq_progressive_requant(0, segment=0)
    assert e.value.status == kq.KVQ_E_OOM and c.kvq_cache_describe(0)[0] == [(0, 384, 16)]
    assert c.kvq_cache_arena_free_bytes() == 0


# ------------------------------------------------------------------ block-wise memory allocation (Sec. 3.2, Eq. 6)
def test_allocate_bits_matches_the_oracle_enumeration():
    """The library's exact solver against the oracle's enumeration of Eq. 6 on random instances (structured and
    unstructured costs, arbitrary and unit-multiple memory sizes, infeasible budgets), the hand-solved instance, and the
    Fbit / budget vectors it yields for kvq_cache_create."""
    from oracle import allocate_bits_bruteforce, allocate_bits_dp
    rng = np.random.default_rng(5)
    for trial in range(60):
        N, C = int(rng.integers(1, 8)), int(rng.integers(1, 5))
        mem = np.sort(rng.integers(1, 50, (N, C)), 1) * int(rng.choice([1, 7, 4096]))
        s = -np.sort(-rng.uniform(0, 10, (N, C)), 1) if trial % 4 else rng.uniform(0, 10, (N, C))
        budget = int(rng.integers(max(0, mem[:, 0].sum() - 3), mem[:, -1].sum() + 3))
        want = allocate_bits_bruteforce(s, mem, budget)
        if want[0] is None:
            with pytest.raises(kq.KvqError) as e:
                kq.kvq_allocate_bits(s, mem, budget)
            assert e.value.status == kq.KVQ_E_BUDGET
            continue
        ch, cost, m = kq.kvq_allocate_bits(s, mem, budget)
        assert cost == pytest.approx(want[1], rel=1e-12) and m == want[2] <= budget
        assert cost == pytest.approx(sum(s[i, c] for i, c in enumerate(ch))) and m == sum(mem[i, c] for i, c in enumerate(ch))
    s = [[9.0, 1.0], [5.0, 4.0], [7.0, 2.0]]
    assert kq.kvq_allocate_bits(s, [[1, 2]] * 3, 5) == ([1, 0, 1], 8.0, 5)
    # a 48-block instance (beyond enumeration) against the knapsack recurrence
    N, widths = 48, (2, 4, 8)
    T, units = 32768, 64
    mem = np.array([[T * units * bytes_per_token_head(b, 128, 32, True) for b in widths]] * N)
    s = np.stack([rng.uniform(1, 100, N) * f for f in (1.0, 0.22, 0.012)], 1)
    budget = int(mem[:, 1].sum())                                   # as much memory as uniform 4 bits
    ch, cost, m = kq.kvq_allocate_bits(s, mem, budget)
    want = allocate_bits_dp(s, mem, budget)
    assert cost == pytest.approx(want[1], rel=1e-12) and m <= budget
    assert cost < s[:, 1].sum()                                      # better than uniform 4 bits
    fbit = [widths[c] for c in ch]
    cfg = kq.KvqConfig(N, 8, 40, 8, T, page_tokens=256)
    cache = kq.KvqCache(cfg, [int(mem[i, c]) for i, c in enumerate(ch)], fbit, arena=None, arena_bytes=1 << 40)
    cache.close()
    for bad in (dict(s=[[float("nan")]], mem=[[1]]), dict(s=[[-1.0]], mem=[[1]])):
        with pytest.raises(kq.KvqError):
            kq.kvq_allocate_bits(bad["s"], bad["mem"], 10)


def test_tier16_option_only_on_empty_caches():
    cfg = kq.KvqConfig(2, 1, 2, 1, 1024, page_tokens=32)
    c = kq.KvqCache(cfg, [1 << 30] * 2, [2, 2], arena=None, arena_bytes=1 << 26)
    with pytest.raises(kq.KvqError) as e:
        c.kvq_cache_set_option(kq.KVQ_OPT_TIER16, 2)
    assert e.value.status == kq.KVQ_E_INVALID
    c.kvq_cache_set_option(kq.KVQ_OPT_TIER16, kq.KVQ_TIER16_INT16)
    c.kvq_quantize_append(1, None, None, n_new=40)
    assert c.kvq_cache_describe(1)[1] == 40 * 544
    with pytest.raises(kq.KvqError) as e:
        c.kvq_cache_set_option(kq.KVQ_OPT_TIER16, kq.KVQ_TIER16_FP16)
    assert e.value.status == kq.KVQ_E_STATE
    # 16 -> 8 of the whole run by segment, then the arena accounting: one 8-bit code block and one metadata block per page
    free0 = c.kvq_cache_arena_free_bytes()
    assert c.kvq_progressive_requant(1, segment=0) == 2 and c.kvq_cache_describe(1)[0] == [(0, 40, 8)]
    assert c.kvq_cache_arena_free_bytes() - free0 == 2 * 32 * 32 * 8      # each page gave back half of its code block


def test_batch_entry_points_reject_what_they_cannot_run():
    """Argument checks of the ragged-batch calls that need no GPU: accounting-only caches cannot attend, and a batch
    holds at most 64 caches."""
    cfg = kq.KvqConfig(1, 1, 2, 1, 256, page_tokens=32)
    caches = [kq.KvqCache(cfg, [1 << 30], [2], arena=None, arena_bytes=1 << 24) for _ in range(65)]
    for c in caches:
        c.kvq_quantize_append(0, None, None, n_new=5)
    fake = [1 << 20] * 65          # never dereferenced: the calls fail before any launch
    with pytest.raises(kq.KvqError) as e:
        kq.kvq_decode_attention_batch(caches[:2], 0, fake[:2], _FakeOuts(2))
    assert e.value.status == kq.KVQ_E_STATE
    with pytest.raises(kq.KvqError) as e:
        kq.kvq_decode_attention_batch(caches, 0, fake, _FakeOuts(65))
    assert e.value.status == kq.KVQ_E_INVALID
    with pytest.raises(kq.KvqError) as e:
        kq.kvq_append_decode_attention_batch(caches[:2], 3, fake[:2], fake[:2], fake[:2], _FakeOuts(2))
    assert e.value.status == kq.KVQ_E_INVALID                       # no such block
    assert all(c.kvq_cache_describe(0)[2] == 5 for c in caches[:2])  # nothing was appended


class _FakeOut(int):
    class _D:
        itemsize = 4
    dtype = _D()


def _FakeOuts(n):
    return [_FakeOut(1 << 21) for _ in range(n)]


def test_cache_reset_returns_every_page():
    cfg = kq.KvqConfig(2, 2, 4, 2, 1024, page_tokens=32, window=32)
    c = kq.KvqCache(cfg, [1 << 30] * 2, [2, 4], arena=None, arena_bytes=1 << 26)
    free0 = c.kvq_cache_arena_free_bytes()
    for layer in range(2):
        c.kvq_quantize_append(layer, None, None, n_new=300)
        c.kvq_progressive_requant(layer)
        c.kvq_quantize_append(layer, None, None, n_new=70, entry_bits=0)
    assert c.kvq_cache_arena_free_bytes() < free0
    c.kvq_cache_reset(1)
    assert c.kvq_cache_describe(1) == ([], 0, 0, 16) and c.kvq_cache_describe(0)[2] == 370
    c.kvq_cache_reset()
    assert c.kvq_cache_arena_free_bytes() == free0 and c.kvq_cache_describe(0) == ([], 0, 0, 16)
    c.kvq_quantize_append(0, None, None, n_new=40)           # usable again
    assert c.kvq_cache_describe(0)[0] == [(0, 40, 16)]
    with pytest.raises(kq.KvqError) as e:
        c.kvq_cache_reset(5)
    assert e.value.status == kq.KVQ_E_INVALID


def test_header_is_plain_c_and_the_library_links_from_c(tmp_path):
    """include/kvq.h compiles as C99 and as C++17, and a C program linked against libkvq.so runs the entry points that
    need no GPU: the byte accounting, the allocation solver (Sec. 3.2, Eq. 6) and an accounting-only cache."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no C compiler")
    src = tmp_path / "use_kvq.c"
    src.write_text(r'''
#include "kvq.h"
#include <stdio.h>
int main(void) {
    if (kvq_bytes_per_token_head(2, 128, 32, 1, 0) != 96) return 1;
    double s[4] = {4.0, 1.0, 3.0, 0.5};
    uint64_t mem[4] = {10, 20, 10, 20};
    int32_t choice[2];
    double total;
    uint64_t used;
    if (kvq_allocate_bits(2, 2, s, mem, 30, choice, &total, &used) != KVQ_OK) return 2;
    if (choice[0] != 1 || choice[1] != 0 || total != 4.0 || used != 30) return 3;
    kvq_config_t cfg = {1, 1, 8, 2, 128, 32, 1024, 0, 0, 128, KVQ_POLICY_PAPER, 1};
    uint64_t budget = 1u << 20;
    uint8_t fbit = 2;
    kvq_cache_t* c = 0;
    if (kvq_cache_create(&cfg, &budget, &fbit, 0, 1u << 26, &c) != KVQ_OK) return 4;
    if (kvq_quantize_append(c, 0, 0, 0, 100, 0, 0) != KVQ_OK) return 5;
    int32_t n = 0, tokens = 0, bits = 0;
    uint64_t bytes = 0;
    kvq_segment_info_t seg[2];
    if (kvq_cache_describe(c, 0, seg, 2, &n, &bytes, &tokens, &bits) != KVQ_OK) return 6;
    if (n != 1 || tokens != 100 || bits != 16 || bytes != 100u * 2u * 512u) return 7;
    if (kvq_decode_attention(c, 0, 0, 0, 1, 0.0f, 0) == KVQ_OK) return 8;   /* no arena: must refuse */
    kvq_cache_destroy(c);
    puts(kvq_status_string(KVQ_OK));
    return 0;
}
''')
    inc = os.path.join(ROOT, "include")
    libdir = os.path.dirname(kq.library_path())
    for cmd in (["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, "-x", "c", os.path.join(inc, "kvq.h")],
                ["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, "-x", "c++", os.path.join(inc, "kvq.h")]):
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
    exe = tmp_path / "use_kvq"
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-lkvq",
                        "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)


def test_segment_requant_refuses_to_strand_the_partly_filled_last_page():
    """Lowering a run that ends in the partly filled last page is refused when the policy appends at 16 bits (a page
    holds one width, so no token could follow); under policy PAPER without a window the block's width follows the
    page and the append goes on.  Library and oracle take the same decision."""
    for policy, W, refuse in ((POLICY_OLDEST_FIRST, 0, True), (POLICY_PAPER, 64, True), (POLICY_PAPER, 0, False)):
        oc, gc = _pair(policy, 64, W, 0, 1 << 40, 2, Tmax=1024, B=1, H=2)
        K, V = kvq_synth.make_kv(79, 0, 1, 2, 0, 200, rope_base=None)
        oc.append(0, K[:, :, :100], V[:, :, :100], 0)
        gc.kvq_quantize_append(0, None, None, n_new=100)
        _same_state(oc, gc)
        if refuse:
            with pytest.raises(StateError):
                oc.requant(0, segment=0)
            with pytest.raises(kq.KvqError) as e:
                gc.kvq_progressive_requant(0, segment=0)
            assert e.value.status == kq.KVQ_E_STATE
        else:
            assert gc.kvq_progressive_requant(0, segment=0) == oc.requant(0, segment=0) == 2
        _same_state(oc, gc)
        oc.append(0, K[:, :, 100:200], V[:, :, 100:200], 0)      # the block still takes tokens
        gc.kvq_quantize_append(0, None, None, n_new=100)
        _same_state(oc, gc)


def test_staging_ring_bookkeeping(tmp_path):
    """The pinned staging ring (csrc/kvq_ring.h) with a fake marker backend: offsets stay inside a segment and aligned,
    a marker is recorded whenever the write position leaves a segment, a segment is written again only after its
    marker has been waited for, and nothing is ever waited for that was not recorded."""
    import shutil
    import subprocess
    if not shutil.which("g++"):
        pytest.skip("no C++ compiler")
    src = tmp_path / "ring_test.cpp"
    src.write_text(r'''
#include "kvq_ring.h"
#include <cstdio>
#include <cstdlib>
#include <vector>
struct Fake {
    std::vector<int> log;           // +seg+1: record, -(seg+1): wait
    bool recorded[4] = {false, false, false, false};
    bool record(int s) { recorded[s] = true; log.push_back(s + 1); return true; }
    bool wait(int s) { if (!recorded[s]) { std::puts("wait without record"); std::exit(2); } recorded[s] = false; log.push_back(-(s + 1)); return true; }
};
int main() {
    KvqStagingRing<Fake, 4> ring;
    Fake be;
    ring.init(1024);
    if (ring.total_bytes() != 4096) return 3;
    if (ring.reserve(be, 0, 64) != -1 || ring.reserve(be, 1025, 64) != -1) return 4;   // empty / larger than a segment
    unsigned seed = 12345;
    long last_seg = 0, wraps = 0;
    bool live[4] = {true, false, false, false};   // segments holding data whose marker has not been waited for
    for (int i = 0; i < 20000; ++i) {
        seed = seed * 1664525u + 1013904223u;
        const unsigned long bytes = 1 + (seed >> 8) % 700;
        const unsigned long align = (i & 1) ? 256 : 64;
        const size_t before = be.log.size();
        const long at = (long)ring.reserve(be, bytes, align);
        if (at < 0 || at % (long)align) return 5;
        const long seg = at / 1024;
        if ((at + (long)bytes - 1) / 1024 != seg) return 6;          // never straddles segments
        if (seg != last_seg) {
            if (seg != (last_seg + 1) % 4) return 7;                   // segments are taken in order
            if (at % 1024 != 0) return 8;                              // and entered at their start
            // leaving last_seg recorded its marker first; entering `seg` waited for its own old marker if it had one
            if (be.log.size() < before + 1 || be.log[before] != last_seg + 1) return 9;
            if (live[seg]) { if (be.log.size() != before + 2 || be.log[before + 1] != -(seg + 1)) return 10; }
            else if (be.log.size() != before + 1) return 11;
            live[seg] = true;
            last_seg = seg;
            ++wraps;
        } else if (be.log.size() != before) return 12;                 // no marker traffic inside a segment
    }
    if (wraps < 1000 || ring.waits() != wraps - 3) return 13;          // every entry but the first three waited
    std::puts("ok");
    return 0;
}
''')
    exe = tmp_path / "ring_test"
    r = subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-O1", "-I", os.path.join(ROOT, "paper_2505_18610_amd", "csrc"),
                        str(src), "-o", str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout, r.stderr)


def test_append_that_finds_the_arena_full_changes_nothing():
    """KVQ_E_OOM of an append is found before anything changes, also when the blocks that are missing are those of the
    pages leaving the window in that call (policy PAPER with a window quantizes them behind the append, Sec. 4.1.2):
    the block is as it was and stays usable (no call on it returns KVQ_E_STATE); the append goes through once a
    halving has made room."""
    P, W = 64, 64
    cfg = kq.KvqConfig(1, 3, 8, 4, 8192, page_tokens=P, window=W, policy=POLICY_PAPER, count_metadata_in_budget=0)
    hit = 0
    for payload_pages in range(10, 34):
        payload = payload_pages * P * 12 * 512 // 2          # arenas that fill up at different points of the sequence
        gc = kq.KvqCache(cfg, [1 << 60], [2], arena=None, arena_bytes=kq.kvq_arena_bytes(cfg, payload))
        gc.kvq_quantize_append(0, None, None, n_new=3 * P)
        gc.kvq_progressive_requant(0)                         # 16 -> 8: pages leaving the window now go to 8 bits
        for step in range(400):
            before = gc.kvq_cache_describe(0)
            try:
                gc.kvq_quantize_append(0, None, None, n_new=P)
                continue
            except kq.KvqError as e:
                assert e.status == kq.KVQ_E_OOM, e.status
            hit += 1
            assert gc.kvq_cache_describe(0) == before
            if before[3] == 2:
                break
            try:                                              # still usable: a halving is carried out ...
                assert gc.kvq_progressive_requant(0) > 0
            except kq.KvqError as e:                          # ... unless its own destination blocks do not fit either
                assert e.status == kq.KVQ_E_OOM, e.status
                assert gc.kvq_cache_describe(0) == before
                break
            gc.kvq_quantize_append(0, None, None, n_new=P)    # and the same append now goes through
        gc.close()
    assert hit >= 24


@pytest.mark.parametrize("seed", range(40))
def test_bookkeeping_matches_oracle_on_random_call_sequences(seed):
    """Random configurations and random calls -- appends at the policy's and at explicit widths, halvings under the
    policy, lowerings of a named run, resets -- on an accounting-only cache and on the oracle's cache: after every call
    both are in the same state, and a call one of them refuses the other refuses for the same kind of reason."""
    rng = np.random.default_rng(1000 + seed)
    P = int(rng.choice([32, 64]))
    policy = int(rng.choice([POLICY_PAPER, POLICY_OLDEST_FIRST]))
    W, sink = P * int(rng.integers(0, 3)), P * int(rng.integers(0, 2))
    fbit = int(rng.choice([2, 4, 8]))
    tier16 = int(rng.choice([0, TIER16_INT16]))
    meta = int(rng.integers(0, 2))
    group = int(rng.choice([32, 64, 128]))
    Tmax = P * int(rng.integers(6, 20))
    per16 = bytes_per_token_head(16, 128, group, bool(meta), bool(tier16))
    budget = int(rng.integers(2 * P, Tmax)) * per16 // int(rng.choice([1, 2, 4]))
    oc, gc = _pair(policy, P, W, sink, budget, fbit, meta=meta, Tmax=Tmax, B=1, H=1, group=group, tier16=tier16)
    K, V = kvq_synth.make_kv(seed, 0, 1, 1, 0, Tmax, rope_base=None)

    def both(o_call, g_call):
        """Runs the call on both sides; returns the kind of outcome, which must agree."""
        try:
            o_res, o_kind = o_call(), "ok"
        except BudgetError:
            o_res, o_kind = None, kq.KVQ_E_BUDGET
        except StateError:
            o_res, o_kind = None, kq.KVQ_E_STATE
        try:
            g_res, g_kind = g_call(), "ok"
        except kq.KvqError as e:
            g_res, g_kind = None, e.status
        assert o_kind == g_kind, (o_kind, g_kind)
        if o_kind == "ok" and o_res is not None:
            assert o_res == g_res
        return o_kind

    for step in range(120):
        T = oc.layers[0].T
        what = int(rng.integers(0, 10))
        if what <= 5:
            n = int(rng.integers(1, 2 * P))
            eb = 0 if rng.integers(0, 4) else int(rng.choice([16, 8, 4, 2]))
            if T + n > Tmax:   # the oracle needs the rows it is handed to exist
                both(lambda: (_ for _ in ()).throw(StateError("max_tokens exceeded")),
                     lambda: gc.kvq_quantize_append(0, None, None, n_new=n, entry_bits=eb))
            else:
                both(lambda: oc.append(0, K[:, :, T:T + n], V[:, :, T:T + n], eb),
                     lambda: gc.kvq_quantize_append(0, None, None, n_new=n, entry_bits=eb))
        elif what <= 7:
            r = int(rng.integers(0, P))
            both(lambda: oc.requant(0, reserve_tokens=r), lambda: gc.kvq_progressive_requant(0, reserve_tokens=r))
        elif what == 8:
            sg = int(rng.integers(0, 5))
            both(lambda: oc.requant(0, segment=sg), lambda: gc.kvq_progressive_requant(0, segment=sg))
        elif rng.integers(0, 4) == 0:
            oc, _ = _pair(policy, P, W, sink, budget, fbit, meta=meta, Tmax=Tmax, B=1, H=1, group=group, tier16=tier16)
            gc.kvq_cache_reset(0)
        _same_state(oc, gc)
