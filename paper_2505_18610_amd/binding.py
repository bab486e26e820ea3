"""ctypes binding of include/kvq.h.  Function and method names follow the C entry points."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

KVQ_OK, KVQ_E_INVALID, KVQ_E_BUDGET, KVQ_E_OOM, KVQ_E_STATE, KVQ_E_HIP, KVQ_E_LIMIT = range(7)
KVQ_POLICY_PAPER, KVQ_POLICY_OLDEST_FIRST = 0, 1
KVQ_WHICH_K, KVQ_WHICH_V = 0, 1
KVQ_OPT_SPLITS, KVQ_OPT_FUSED_MERGE, KVQ_OPT_DETERMINISTIC = 0, 1, 2
KVQ_OPT_TILE_COST_2BIT, KVQ_OPT_TILE_COST_4BIT, KVQ_OPT_TILE_COST_8BIT, KVQ_OPT_TILE_COST_16BIT = 3, 4, 5, 6
KVQ_OPT_SHIFT_STRATEGY = 7
KVQ_SHIFT_EQUIVALENT, KVQ_SHIFT_DIRECT, KVQ_SHIFT_MODIFIED = 0, 1, 2
KVQ_OPT_TIER16 = 8
KVQ_TIER16_FP16, KVQ_TIER16_INT16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class KvqConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "batch", "n_q_heads", "n_kv_heads", "head_dim", "group", "max_tokens", "window",
        "n_sink", "page_tokens", "policy", "count_metadata_in_budget")]

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, max_tokens, page_tokens=128, window=0, n_sink=0,
                 policy=KVQ_POLICY_PAPER, count_metadata_in_budget=1, head_dim=128, group=32):
        super().__init__(n_layers, batch, n_q_heads, n_kv_heads, head_dim, group, max_tokens, window, n_sink,
                         page_tokens, policy, count_metadata_in_budget)


class _SegmentInfo(C.Structure):
    _fields_ = [("token_begin", C.c_int32), ("token_end", C.c_int32), ("bits", C.c_int32)]


class KvqError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {kvq_status_string(status)} (status {int(status)})")


def library_path() -> str:
    return os.path.join(_HERE, "libkvq.so")


_SIGNATURES = {
    "kvq_arena_bytes": (C.c_uint64, [C.POINTER(KvqConfig), C.c_uint64]),
    "kvq_bytes_per_token_head": (C.c_uint64, [C.c_int32] * 5),
    "kvq_cache_create": (C.c_int, [C.POINTER(KvqConfig), C.POINTER(C.c_uint64), C.POINTER(C.c_uint8), C.c_void_p,
                                   C.c_uint64, C.POINTER(C.c_void_p)]),
    "kvq_cache_destroy": (None, [C.c_void_p]),
    "kvq_quantize_append": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]),
    "kvq_quantize_append_rope": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                           C.c_void_p, C.c_void_p]),
    "kvq_progressive_requant": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_int32)]),
    "kvq_decode_attention": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_void_p]),
    "kvq_decode_attention_static": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_float,
                                              C.c_void_p]),
    "kvq_append_decode_attention": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_int32, C.c_float, C.c_void_p]),
    "kvq_decode_attention_batch": (C.c_int, [C.POINTER(C.c_void_p), C.c_int32, C.c_int32, C.POINTER(C.c_void_p),
                                             C.POINTER(C.c_void_p), C.c_int32, C.c_float, C.c_void_p]),
    "kvq_append_decode_attention_batch": (C.c_int, [C.POINTER(C.c_void_p), C.c_int32, C.c_int32, C.POINTER(C.c_void_p),
                                                    C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                                    C.POINTER(C.c_void_p), C.c_int32, C.c_float, C.c_void_p]),
    "kvq_cache_describe": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(_SegmentInfo), C.c_int32, C.POINTER(C.c_int32),
                                     C.POINTER(C.c_uint64), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "kvq_cache_export_segment": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p]),
    "kvq_cache_set_option": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32]),
    "kvq_cache_arena_free_bytes": (C.c_uint64, [C.c_void_p]),
    "kvq_cache_reset": (C.c_int, [C.c_void_p, C.c_int32]),
    "kvq_cache_set_reparam": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]),
    "kvq_calibrate_lambda": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p]),
    "kvq_cache_sensitivity": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.POINTER(C.c_double), C.c_void_p]),
    "kvq_allocate_bits": (C.c_int, [C.c_int32, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_uint64), C.c_uint64,
                                    C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_uint64)]),
    "kvq_cache_sq_error": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]),
    "kvq_stream_read_probe": (C.c_int, [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.c_void_p]),
    "kvq_status_string": (C.c_char_p, [C.c_int]),
}


def exported_symbols():
    """Names include/kvq.h declares; the CPU test-suite checks the library exports each of them."""
    return sorted(_SIGNATURES)


def load_library():
    """Loads libkvq.so from the package directory; raises if it has not been built (no fallback exists)."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2505_18610_amd.build` "
                               "(or __graft_entry__.build()); there is no fallback path")
        # PyTorch ships its own copy of the HIP runtime.  The library must use the same one (the arena, the tensors and
        # the streams it is handed belong to it), which the dynamic linker arranges only if torch is loaded first.
        import torch  # noqa: F401
        lib = C.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _LIB = lib
    return _LIB


def kvq_status_string(status) -> str:
    return load_library().kvq_status_string(int(status)).decode()


def kvq_arena_bytes(cfg: KvqConfig, payload_bytes: int) -> int:
    return int(load_library().kvq_arena_bytes(C.byref(cfg), int(payload_bytes)))


def kvq_allocate_bits(s, mem, budget):
    """Eq. 6: s, mem [n_blocks][n_choices] (nested sequences or arrays); returns (choices list, total s, total bytes)."""
    n, c = len(s), len(s[0])
    sa = (C.c_double * (n * c))(*[float(x) for row in s for x in row])
    ma = (C.c_uint64 * (n * c))(*[int(x) for row in mem for x in row])
    ch = (C.c_int32 * n)()
    ts, tm = C.c_double(), C.c_uint64()
    st = load_library().kvq_allocate_bits(n, c, sa, ma, int(budget), ch, C.byref(ts), C.byref(tm))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_allocate_bits")
    return list(ch), ts.value, tm.value


def kvq_calibrate_lambda(k_calib, alpha, lam_out, stream=None):
    """k_calib: fp16 device tensor [batch, n_kv_heads, n_tokens, 128]; lam_out: fp32 device tensor [n_kv_heads, 128]."""
    b, h, t, d = k_calib.shape
    assert d == 128 and tuple(lam_out.shape) == (h, 128)
    st = load_library().kvq_calibrate_lambda(_ptr(k_calib), b, h, t, float(alpha), _ptr(lam_out), _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_calibrate_lambda")


def _ptr_array(items):
    """Host array of device pointers (None entries become NULL)."""
    return (C.c_void_p * len(items))(*[_ptr(t) for t in items])


def kvq_decode_attention_batch(caches, layer, qs, outs, softmax_scale=0.0, stream=None):
    """Ragged batch: caches[i] (KvqCache) attends with qs[i] into outs[i]; all outs share one dtype."""
    n = len(caches)
    assert n == len(qs) == len(outs) and n > 0
    out_is_fp32 = 1 if outs[0].dtype.itemsize == 4 else 0
    assert all((o.dtype.itemsize == 4) == bool(out_is_fp32) for o in outs)
    handles = (C.c_void_p * n)(*[c.handle for c in caches])
    st = load_library().kvq_decode_attention_batch(handles, n, layer, _ptr_array(qs), _ptr_array(outs), out_is_fp32,
                                                   float(softmax_scale), _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_decode_attention_batch")


def kvq_append_decode_attention_batch(caches, layer, ks, vs, qs, outs, cos_sins=None, softmax_scale=0.0, stream=None):
    """Ragged batch decode step: one new token (ks[i], vs[i]) into caches[i], then attention, in one attention launch."""
    n = len(caches)
    assert n == len(ks) == len(vs) == len(qs) == len(outs) and n > 0
    out_is_fp32 = 1 if outs[0].dtype.itemsize == 4 else 0
    assert all((o.dtype.itemsize == 4) == bool(out_is_fp32) for o in outs)
    handles = (C.c_void_p * n)(*[c.handle for c in caches])
    cs = _ptr_array(cos_sins) if cos_sins is not None else None
    st = load_library().kvq_append_decode_attention_batch(handles, n, layer, _ptr_array(ks), _ptr_array(vs), cs,
                                                          _ptr_array(qs), _ptr_array(outs), out_is_fp32,
                                                          float(softmax_scale), _stream(stream))
    if st != KVQ_OK:
        raise KvqError(st, "kvq_append_decode_attention_batch")


def kvq_bytes_per_token_head(bits, head_dim=128, group=32, count_metadata=1, int16_tier=0) -> int:
    return int(load_library().kvq_bytes_per_token_head(bits, head_dim, group, count_metadata, int16_tier))


def _ptr(t):
    """Device pointer of a torch tensor (or a raw int / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous()
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class KvqCache:
    """Owns one kvq_cache_t.  `arena` is a torch uint8 CUDA tensor the caller keeps alive, or None for an
    accounting-only cache (then `arena_bytes` is the virtual capacity)."""

    def __init__(self, cfg: KvqConfig, block_budget_bytes, block_fbit, arena=None, arena_bytes=None):
        self.lib = load_library()
        self.cfg = cfg
        self.arena = arena
        n = cfg.n_layers
        budgets = (C.c_uint64 * n)(*[int(b) for b in block_budget_bytes])
        fbits = (C.c_uint8 * n)(*[int(b) for b in block_fbit])
        if arena is not None:
            assert arena.is_cuda and arena.dtype.itemsize == 1 and arena.is_contiguous()
            ptr, nbytes = arena.data_ptr(), arena.numel()
        else:
            ptr, nbytes = None, int(arena_bytes)
        h = C.c_void_p()
        st = self.lib.kvq_cache_create(C.byref(cfg), budgets, fbits, ptr, nbytes, C.byref(h))
        if st != KVQ_OK:
            raise KvqError(st, "kvq_cache_create")
        self.handle = h

    def close(self):
        if getattr(self, "handle", None):
            self.lib.kvq_cache_destroy(self.handle)
            self.handle = None

    __del__ = close

    def _check(self, st, where):
        if st != KVQ_OK:
            raise KvqError(st, where)

    def kvq_quantize_append(self, layer, k, v, entry_bits=0, stream=None, n_new=None):
        if n_new is None:
            n_new = k.shape[2]
        self._check(self.lib.kvq_quantize_append(self.handle, layer, _ptr(k), _ptr(v), n_new, entry_bits,
                                                 _stream(stream)), "kvq_quantize_append")

    def kvq_quantize_append_rope(self, layer, k, v, cos_sin, entry_bits=0, stream=None):
        """k: un-rotated keys; cos_sin: fp32 device tensor [n_new, 128] (cos 64 | sin 64 per new token)."""
        assert tuple(cos_sin.shape) == (k.shape[2], 128)
        self._check(self.lib.kvq_quantize_append_rope(self.handle, layer, _ptr(k), _ptr(v), k.shape[2], entry_bits,
                                                      _ptr(cos_sin), _stream(stream)), "kvq_quantize_append_rope")

    def kvq_progressive_requant(self, layer, segment=-1, reserve_tokens=0, stream=None) -> int:
        n = C.c_int32(0)
        st = self.lib.kvq_progressive_requant(self.handle, layer, segment, reserve_tokens, _stream(stream), C.byref(n))
        self._check(st, "kvq_progressive_requant")
        return n.value

    def kvq_decode_attention(self, layer, q, out, softmax_scale=0.0, stream=None):
        out_is_fp32 = 1 if out.dtype.itemsize == 4 else 0
        self._check(self.lib.kvq_decode_attention(self.handle, layer, _ptr(q), _ptr(out), out_is_fp32,
                                                  float(softmax_scale), _stream(stream)), "kvq_decode_attention")

    def kvq_decode_attention_static(self, layer, q, out, softmax_scale=0.0, stream=None):
        out_is_fp32 = 1 if out.dtype.itemsize == 4 else 0
        self._check(self.lib.kvq_decode_attention_static(self.handle, layer, _ptr(q), _ptr(out), out_is_fp32,
                                                         float(softmax_scale), _stream(stream)),
                    "kvq_decode_attention_static")

    def kvq_append_decode_attention(self, layer, k, v, q, out, cos_sin=None, softmax_scale=0.0, stream=None):
        out_is_fp32 = 1 if out.dtype.itemsize == 4 else 0
        self._check(self.lib.kvq_append_decode_attention(self.handle, layer, _ptr(k), _ptr(v), _ptr(cos_sin), _ptr(q),
                                                         _ptr(out), out_is_fp32, float(softmax_scale), _stream(stream)),
                    "kvq_append_decode_attention")

    def kvq_cache_describe(self, layer):
        """Returns (segments [(token_begin, token_end, bits)], bytes_used, n_tokens, current_bits)."""
        cap = 4096
        segs = (_SegmentInfo * cap)()
        n, used, T, cur = C.c_int32(), C.c_uint64(), C.c_int32(), C.c_int32()
        self._check(self.lib.kvq_cache_describe(self.handle, layer, segs, cap, C.byref(n), C.byref(used), C.byref(T),
                                                C.byref(cur)), "kvq_cache_describe")
        return ([(segs[i].token_begin, segs[i].token_end, segs[i].bits) for i in range(min(cap, n.value))],
                used.value, T.value, cur.value)

    def kvq_cache_export_segment(self, layer, segment, which, stream=None):
        """Returns (codes, scales, zeros) numpy arrays in the canonical format (scales/zeros None for raw fp16 runs)."""
        segs, _, _, _ = self.kvq_cache_describe(layer)
        t0, t1, b = segs[segment]
        c = self.cfg
        n = t1 - t0
        if b == 16 and not getattr(self, "_tier16", 0):
            codes = np.empty((c.batch, c.n_kv_heads, n, c.head_dim), np.float16)
            S = Z = None
            sp = zp = None
        else:
            codes = np.empty((c.batch, c.n_kv_heads, n, c.head_dim * b // 8), np.uint8)
            S = np.empty((c.batch, c.n_kv_heads, n, c.head_dim // c.group), np.float16)
            Z = np.empty_like(S)
            sp, zp = S.ctypes.data, Z.ctypes.data
        self._check(self.lib.kvq_cache_export_segment(self.handle, layer, segment, which, codes.ctypes.data, sp, zp,
                                                      _stream(stream)), "kvq_cache_export_segment")
        return codes, S, Z

    def kvq_cache_set_option(self, option, value):
        self._check(self.lib.kvq_cache_set_option(self.handle, option, value), "kvq_cache_set_option")
        if option == KVQ_OPT_TIER16:
            self._tier16 = value   # decides the shape of exported 16-bit runs

    def kvq_cache_set_reparam(self, layer, lam, stream=None):
        """lam: fp32 device tensor [n_kv_heads, 128], or None to switch the reparameterization off."""
        self._check(self.lib.kvq_cache_set_reparam(self.handle, layer, _ptr(lam) if lam is not None else None,
                                                   _stream(stream)), "kvq_cache_set_reparam")

    def kvq_cache_sq_error(self, layer, k_ref, v_ref, stream=None):
        """(sum (K_hat - K)^2, sum (V_hat - V)^2) of the block against fp16 device tensors [B, Hkv, T, 128]."""
        out = (C.c_double * 2)()
        self._check(self.lib.kvq_cache_sq_error(self.handle, layer, _ptr(k_ref), _ptr(v_ref), out, _stream(stream)),
                    "kvq_cache_sq_error")
        return float(out[0]), float(out[1])

    def kvq_cache_sensitivity(self, layer, k_ref, v_ref, gk=None, gv=None, stream=None):
        """(|| G_K * (K - K_hat) ||_1, || G_V * (V - V_hat) ||_1); gradients fp32 device tensors or None (ones)."""
        out = (C.c_double * 2)()
        self._check(self.lib.kvq_cache_sensitivity(self.handle, layer, _ptr(k_ref), _ptr(v_ref), _ptr(gk), _ptr(gv), out,
                                                   _stream(stream)), "kvq_cache_sensitivity")
        return float(out[0]), float(out[1])

    def kvq_stream_read_probe(self, buf, n_workgroups, stream=None):
        self._check(self.lib.kvq_stream_read_probe(self.handle, _ptr(buf), buf.numel() * buf.element_size(), n_workgroups,
                                                   _stream(stream)), "kvq_stream_read_probe")

    def kvq_cache_reset(self, layer=-1):
        self._check(self.lib.kvq_cache_reset(self.handle, layer), "kvq_cache_reset")

    def kvq_cache_arena_free_bytes(self) -> int:
        return int(self.lib.kvq_cache_arena_free_bytes(self.handle))
