"""Per-phase timeline of the decode-attention launch, from the measurement build of the library.

    python -m paper_2505_18610_amd.build --phase-stamps        # builds libkvq_stamps.so (on the CPU machine)
    python -m paper_2505_18610_amd.phase_table 32b 70b 14b-2   # on an MI355X; prints a markdown table per workload
    python paper_2505_18610_amd/phase_table.py --launch-only 14b-2   # 64 launches of the library proper and nothing
                                                                     # else: the program to put behind rocprofv3 --pmc

    python -m paper_2505_18610_amd.build --no-arithmetic       # builds libkvq_noarith.so
    python -m paper_2505_18610_amd.phase_table --floor 32b 70b 14b-2 14b-4 14b-8 7b
                                                               # the launch with and without its arithmetic

The measurement build records the device wall clock when thread 0 of every workgroup passes the points listed in
csrc/kvq_phase_stamps.h.  Launches run in back-to-back trains (as in bench.py); the stamps of the last launch of
several trains are read and averaged.  Beside them the script times the same trains with the library proper, whose
kernels carry no stamps.  A measurement aid: nothing in the library, the tests or bench.py depends on it.
"""
from __future__ import annotations

import ctypes
import importlib.util
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))

# one block's tiers (tokens, bits) and shape; the names are those of kvq_synth.WORKLOADS, "14b-<b>" = a 14B-shaped block
# whose bulk is b bits wide
SHAPES = {
    "32b": ([(16384, 2), (8192, 4), (8064, 8), (128, 16)], dict(B=4, Hq=40, Hkv=8, P=128)),
    "70b": ([(81920, 2), (40960, 4), (7168, 8), (1024, 16)], dict(B=1, Hq=64, Hkv=8, P=1024)),
    "7b": ([(32256, 4), (512, 16)], dict(B=16, Hq=28, Hkv=4, P=256)),
    "14b-2": ([(32256, 2), (512, 16)], dict(B=8, Hq=40, Hkv=8, P=256)),
    "14b-4": ([(32256, 4), (512, 16)], dict(B=8, Hq=40, Hkv=8, P=256)),
    "14b-8": ([(32256, 8), (512, 16)], dict(B=8, Hq=40, Hkv=8, P=256)),
}
STAMPS = (("entry", 0), ("inputs staged", 1), ("own range done (wavefront 0)", 2), ("eight wavefronts joined", 6),
          ("wavefront partials merged", 3), ("partial published, ticket drawn", 4), ("split partials merged", 5))


def _binding(lib_path, tag):
    spec = importlib.util.spec_from_file_location("kvq_binding_" + tag, os.path.join(HERE, "binding.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    m.library_path = lambda: lib_path
    return m


def _build_cache(kq, torch, tiers, B, Hq, Hkv, P, L, arena):
    T = sum(n for n, _ in tiers)
    units = B * Hkv
    cfg = kq.KvqConfig(L, B, Hq, Hkv, T, page_tokens=P)
    if arena is None:
        arena = torch.empty(kq.kvq_arena_bytes(cfg, L * T * units * 520 + (64 << 20)), dtype=torch.uint8, device="cuda")
    cache = kq.KvqCache(cfg, [1 << 60] * L, [2] * L, arena=arena)
    g = torch.Generator(device="cuda").manual_seed(1)
    chunk = 8192
    k = torch.randn((B, Hkv, chunk, 128), device="cuda", generator=g).half()
    v = torch.randn((B, Hkv, chunk, 128), device="cuda", generator=g).half()
    for layer in range(L):
        for n, bits in tiers:
            for t0 in range(0, n, chunk):
                m = min(chunk, n - t0)
                cache.kvq_quantize_append(layer, k[:, :, :m].contiguous(), v[:, :, :m].contiguous(), bits)
    q = torch.randn((B, Hq, 128), device="cuda", generator=g).half()
    out = torch.empty((B, Hq, 128), dtype=torch.float16, device="cuda")
    return cache, arena, q, out


def _train_us(torch, cache, q, out, L, sweeps=6, reps=5):
    best = 1e9
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(sweeps):
            for layer in range(L):
                cache.kvq_decode_attention(layer, q, out)
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) * 1e3 / (sweeps * L))
    return best


def launch_only(names, launches=64):
    """The library proper on blocks of the given shapes: warm-up, then `launches` attention launches per shape."""
    import torch
    kq_p = _binding(os.path.join(HERE, "libkvq.so"), "proper")
    L = 4
    for name in names:
        tiers, kw = SHAPES[name]
        cache, arena, q, out = _build_cache(kq_p, torch, tiers, L=L, arena=None, **kw)
        for i in range(200 + launches):
            cache.kvq_decode_attention(i % L, q, out)
        torch.cuda.synchronize()
        print(f"{name}: {200 + launches} launches of kvq_decode_attention, {cache.kvq_cache_describe(0)[1]} bytes per block", flush=True)
        cache.close()
        del cache, arena


def main(names):
    import torch
    stamps_lib = os.path.join(HERE, "libkvq_stamps.so")
    if not os.path.exists(stamps_lib):
        raise SystemExit("build the measurement variant first: python -m paper_2505_18610_amd.build --phase-stamps")
    kq_s = _binding(stamps_lib, "stamps")
    kq_p = _binding(os.path.join(HERE, "libkvq.so"), "proper")
    L, n_launches = 8, 24
    for name in names:
        tiers, kw = SHAPES[name]
        units = kw["B"] * kw["Hkv"]
        cache, arena, q, out = _build_cache(kq_p, torch, tiers, L=L, arena=None, **kw)
        for _ in range(40):                                   # sustained clocks
            for layer in range(L):
                cache.kvq_decode_attention(layer, q, out)
        t_proper = _train_us(torch, cache, q, out, L)
        nbytes = cache.kvq_cache_describe(0)[1]
        cache.close()
        cache, arena, q, out = _build_cache(kq_s, torch, tiers, L=L, arena=arena, **kw)
        t_stamped = _train_us(torch, cache, q, out, L)
        lib = kq_s.load_library()
        lib.kvq_phase_stamps_read.argtypes = [ctypes.c_void_p]
        rows = {label: [] for label, _ in STAMPS}
        per_wg = {"range (staged -> own range done)": [], "wait for the other wavefronts": [], "LDS merge": [],
                  "publish + ticket": [], "merge of the splits (last workgroup)": []}
        for rep in range(n_launches):
            for i in range(8 + rep % L):                      # a train; its last launch is the one read
                cache.kvq_decode_attention(i % L, q, out)
            torch.cuda.synchronize()
            buf = (ctypes.c_ulonglong * (1024 * 8))()
            assert lib.kvq_phase_stamps_read(buf) == 0
            a = np.frombuffer(buf, dtype=np.uint64).reshape(1024, 8).astype(np.int64)
            a = a[a[:, 0] > a[:, 0].max() - 100000]           # this launch's workgroups (others: stale rows of earlier shapes)
            wgs = a.shape[0]
            t0 = a[:, 0].min()
            us = (a - t0) / 100.0
            last = a[:, 5] > a[:, 0]                          # workgroups that merged their unit's splits in this launch
            for label, k in STAMPS:
                col = us[last, k] if k == 5 else us[:, k]
                rows[label].append((col.min(), col.mean(), col.max()))
            per_wg["range (staged -> own range done)"].append((us[:, 2] - us[:, 1]).mean())
            per_wg["wait for the other wavefronts"].append((us[:, 6] - us[:, 2]).mean())
            per_wg["LDS merge"].append((us[:, 3] - us[:, 6]).mean())
            per_wg["publish + ticket"].append((us[:, 4] - us[:, 3]).mean())
            per_wg["merge of the splits (last workgroup)"].append((us[last, 5] - us[last, 4]).mean())
        splits = wgs // units
        print(f"\n### {name}: {units} units x {splits} splits = {wgs} workgroups, {nbytes / 1e6:.1f} MB per launch\n")
        print(f"library proper: {t_proper:.2f} us per launch ({nbytes / t_proper / 1e3:.0f} GB/s); measurement build: "
              f"{t_stamped:.2f} us per launch; stamps of {n_launches} launches, each the last of a train, relative to "
              "the first workgroup's entry\n")
        print("| point a workgroup passes | earliest (us) | mean (us) | latest (us) |")
        print("|---|---|---|---|")
        for label, _ in STAMPS:
            r = np.array(rows[label])
            print(f"| {label} | {r[:, 0].mean():.2f} | {r[:, 1].mean():.2f} | {r[:, 2].mean():.2f} |")
        print("\n| phase, per workgroup | mean (us) |")
        print("|---|---|")
        for label, vals in per_wg.items():
            print(f"| {label} | {np.mean(vals):.2f} |")
        sys.stdout.flush()
        cache.close()
        del cache, arena


# split counts tried beside the library's own plan (0) in the floor table: 192 workgroups where the plan uses 256
FLOOR_SPLITS = {"32b": (0, 6), "14b-2": (0, 3)}
PLANNED_SPLITS = {"32b": 8, "70b": 32, "7b": 3, "14b-2": 4, "14b-4": 3, "14b-8": 3}  # what the library chooses (see main())


def floor(names):
    """The library proper against the build without arithmetic (libkvq_noarith.so: every tile loaded, none computed
    on; claims, join and merge of the splits as in the library), alternating on one arena; fastest of several trains."""
    import torch
    lib_n = os.path.join(HERE, "libkvq_noarith.so")
    if not os.path.exists(lib_n):
        raise SystemExit("build the measurement variant first: python -m paper_2505_18610_amd.build --no-arithmetic")
    kqs = (("library", _binding(os.path.join(HERE, "libkvq.so"), "proper")), ("no arithmetic", _binding(lib_n, "noarith")))
    L = 8
    print("| block | workgroups | MB per launch | library (us) | of 8 TB/s | no arithmetic (us) | of 8 TB/s | arithmetic costs (us) |")
    print("|---|---|---|---|---|---|---|---|")
    for name in names:
        tiers, kw = SHAPES[name]
        units = kw["B"] * kw["Hkv"]
        arena = None
        for splits in FLOOR_SPLITS.get(name, (0,)):
            best = {}
            for rnd in range(3):
                for tag, kq in kqs:
                    cache, arena, q, out = _build_cache(kq, torch, tiers, L=L, arena=arena, **kw)
                    if splits:
                        cache.kvq_cache_set_option(kq.KVQ_OPT_SPLITS, splits)
                    for _ in range(20 if rnd else 60):            # sustained clocks
                        for layer in range(L):
                            cache.kvq_decode_attention(layer, q, out)
                    best[tag] = min(best.get(tag, 1e9), _train_us(torch, cache, q, out, L))
                    nbytes = cache.kvq_cache_describe(0)[1]
                    cache.close()
            a, b = best["library"], best["no arithmetic"]
            wg = f"{units} x {splits or PLANNED_SPLITS[name]} = {units * (splits or PLANNED_SPLITS[name])}"
            print(f"| {name} | {wg} | {nbytes / 1e6:.1f} | {a:.2f} | {nbytes / a / 80e3:.1f} % | {b:.2f} | "
                  f"{nbytes / b / 80e3:.1f} % | {a - b:.2f} |", flush=True)
        del arena


if __name__ == "__main__":
    if "--floor" in sys.argv:
        floor([a for a in sys.argv[1:] if a != "--floor"] or ["32b"])
    elif "--launch-only" in sys.argv:
        launch_only([a for a in sys.argv[1:] if a != "--launch-only"] or ["32b"])
    else:
        main(sys.argv[1:] or ["32b"])
