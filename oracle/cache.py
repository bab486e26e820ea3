"""Progressive-quantization KV cache of the oracle: storage, bookkeeping, policies (test infrastructure).

Follows Sec. 3.1: every transformer block has a final bit-width Fbit and a byte budget;
tokens are stored at 16 bits first; when the budget would be exceeded the bit-width of
the existing cache is halved (16 -> 8 -> 4 -> 2, never below Fbit).  The first n_sink and
the most recent `window` tokens stay at 16 bits (Sec. 4.1.2).  Bookkeeping is per page of
`page_tokens` tokens; K and V of a page always share one width (Table 2, K-V columns).
"""
from __future__ import annotations

import dataclasses
import numpy as np

from .quantizer import (quantize, dequantize, pack_codes, shrink_step, SHIFT_EQUIVALENT,
                        bytes_per_token_head, reparam_keys, reparam_queries)
from .attention import decode_attention_fp64

POLICY_PAPER = 0
POLICY_OLDEST_FIRST = 1
TIER16_FP16 = 0    # 16-bit tokens are the raw fp16 values
TIER16_INT16 = 1   # 16-bit tokens are 16-bit integer codes with (S, Z) per group: the INT16 format of Sec. 4.1.2


class BudgetError(Exception):
    """The operation would exceed the block's byte budget, or no further shrinking is allowed."""


class StateError(Exception):
    """The operation does not fit the cache's current state (e.g. width change inside a page)."""


@dataclasses.dataclass
class CacheConfig:
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    group: int = 32
    max_tokens: int = 32768
    window: int = 0
    n_sink: int = 0
    page_tokens: int = 128
    policy: int = POLICY_PAPER
    count_metadata_in_budget: int = 1
    shift_strategy: int = SHIFT_EQUIVALENT   # how 2b -> b steps treat codes, S and Z (Sec. 4.3.1)
    tier16: int = TIER16_FP16                # what a 16-bit token is; INT16 makes 16 -> 8 a step of Eq. 3 too


class _Page:
    def __init__(self, bits):
        self.bits = bits
        self.n = 0
        self.k = self.v = None                     # 16-bit, fp16 tier: fp16 [B,H,n,D]
        self.kc = self.ks = self.kz = None         # quantized: codes uint8 (uint16 in the INT16 tier) [B,H,n,D], S/Z fp16 [B,H,n,D/G]
        self.vc = self.vs = self.vz = None


class _Layer:
    def __init__(self, budget, fbit):
        self.budget, self.fbit = int(budget), int(fbit)
        self.T = 0
        self.pages: list[_Page] = []


def _cat(a, b):
    return b.copy() if a is None else np.concatenate([a, b], axis=2)


class OracleCache:
    def __init__(self, cfg: CacheConfig, block_budget_bytes, block_fbit):
        assert cfg.page_tokens % 32 == 0 and cfg.window % cfg.page_tokens == 0 and cfg.n_sink % cfg.page_tokens == 0
        assert all(f in (2, 4, 8, 16) for f in block_fbit)
        self.cfg = cfg
        self.layers = [_Layer(b, f) for b, f in zip(block_budget_bytes, block_fbit)]
        self.lam = [None] * len(self.layers)   # per block: fp32 [n_kv_heads, D] reparameterization factors or None

    def set_reparam(self, layer, lam):
        """Channel-wise reparameterization of one block (Sec. 3.3, Eq. 7): from now on its keys are stored as
        K Lambda^{-1} (all widths) and its queries are used as Q Lambda.  Only on an empty block."""
        if self.layers[layer].T != 0:
            raise StateError("reparameterization factors must be set before the first append")
        if lam is not None:
            lam = np.asarray(lam)
            assert lam.dtype == np.float32 and lam.shape == (self.cfg.n_kv_heads, self.cfg.head_dim)
            assert np.all(np.isfinite(lam)) and np.all(lam > 0)
        self.lam[layer] = lam

    # ---------------------------------------------------------------- bookkeeping
    def _bpth(self, bits):
        c = self.cfg
        return bytes_per_token_head(bits, c.head_dim, c.group, bool(c.count_metadata_in_budget),
                                    c.tier16 == TIER16_INT16)

    def bytes_used(self, layer):
        c = self.cfg
        return sum(p.n * c.batch * c.n_kv_heads * self._bpth(p.bits) for p in self.layers[layer].pages)

    def current_bits(self, layer):
        """Width of the block's bulk: the smallest width among pages after the sink (16 if none)."""
        P = self.cfg.page_tokens
        bits = [p.bits for i, p in enumerate(self.layers[layer].pages) if i >= self.cfg.n_sink // P]
        return min(bits) if bits else 16

    def _protected(self, L, i):
        """Sink pages and pages overlapping the most recent `window` tokens are never lowered."""
        c = self.cfg
        P = c.page_tokens
        if i < c.n_sink // P:
            return True
        return c.window > 0 and (i + 1) * P > L.T - c.window

    def segments(self, layer):
        """Maximal runs of consecutive pages with equal width: [(token_begin, token_end, bits)]."""
        L, P = self.layers[layer], self.cfg.page_tokens
        out = []
        for i, p in enumerate(L.pages):
            t0, t1 = i * P, i * P + p.n
            if out and out[-1][2] == p.bits:
                out[-1] = (out[-1][0], t1, p.bits)
            else:
                out.append((t0, t1, p.bits))
        return out

    # ---------------------------------------------------------------- append
    def _entry_bits(self, layer, entry_bits):
        c = self.cfg
        if entry_bits:
            return entry_bits
        if c.policy == POLICY_OLDEST_FIRST or c.window > 0:
            return 16
        return self.current_bits(layer)

    def _plan_append(self, layer, n_new, entry_bits):
        """Bookkeeping of an append of n_new tokens, without touching the cache: (entry width, pages evicted from
        the window, width they go to).  Raises StateError / BudgetError exactly where append would."""
        c, L, P = self.cfg, self.layers[layer], self.cfg.page_tokens
        assert entry_bits in (0, 2, 4, 8, 16)
        if L.T + n_new > c.max_tokens:
            raise StateError("max_tokens exceeded")
        e = self._entry_bits(layer, entry_bits)
        if L.T % P != 0 and L.pages[-1].bits != e:
            raise StateError("width change inside a page")
        evict = (entry_bits == 0 and c.policy == POLICY_PAPER and c.window > 0)
        bits = [p.bits for p in L.pages]
        cnt = [p.n for p in L.pages]
        T = L.T
        left = n_new
        while left:
            if T % P == 0:
                bits.append(e); cnt.append(0)
            take = min(left, P - cnt[-1])
            cnt[-1] += take; T += take; left -= take
        evicted, bcur = [], 16
        if evict:
            bcur = min([b for i, b in enumerate(bits) if i >= c.n_sink // P] or [16])
            if bcur < 16:
                while True:
                    i = self._tail16_start(bits, c.n_sink // P)
                    if T - i * P >= c.window + P:
                        bits[i] = bcur; evicted.append(i)
                    else:
                        break
        used = sum(n * c.batch * c.n_kv_heads * self._bpth(b) for n, b in zip(cnt, bits))
        if used > L.budget:
            raise BudgetError("append exceeds block budget")
        return e, evicted, bcur

    def append(self, layer, k, v, entry_bits=0):
        """Append n_new tokens (k, v fp16 [B, Hkv, n_new, D], keys already rotated).

        entry_bits 0 = the policy's entry width; 16/8/4/2 = store at that width (state
        construction).  Raises BudgetError, leaving the cache unchanged, if the block's
        bytes after the append (and after the window evictions it causes) exceed the budget.
        """
        c, L, P = self.cfg, self.layers[layer], self.cfg.page_tokens
        n_new = k.shape[2]
        assert k.dtype == np.float16 and v.dtype == np.float16 and k.shape == v.shape
        assert k.shape == (c.batch, c.n_kv_heads, n_new, c.head_dim)
        if n_new == 0:
            assert entry_bits in (0, 2, 4, 8, 16)
            return
        e, evicted, bcur = self._plan_append(layer, n_new, entry_bits)
        if self.lam[layer] is not None:
            k = reparam_keys(k, self.lam[layer])
        off = 0
        while off < n_new:
            if L.T % P == 0:
                L.pages.append(_Page(e))
            pg = L.pages[-1]
            take = min(n_new - off, P - pg.n)
            self._store(pg, k[:, :, off:off + take], v[:, :, off:off + take])
            L.T += take; off += take
        for i in evicted:
            self._lower_page(L.pages[i], bcur)

    @staticmethod
    def _tail16_start(bits, first):
        """Index of the first page of the trailing run of 16-bit pages (not before page `first`)."""
        i = len(bits)
        while i > first and bits[i - 1] == 16:
            i -= 1
        return i

    def _store(self, pg, k, v):
        G = self.cfg.group
        if pg.bits == 16 and self.cfg.tier16 == TIER16_FP16:
            pg.k, pg.v = _cat(pg.k, k), _cat(pg.v, v)
        else:
            kc, ks, kz = quantize(k, pg.bits, G)
            vc, vs, vz = quantize(v, pg.bits, G)
            pg.kc, pg.ks, pg.kz = _cat(pg.kc, kc), _cat(pg.ks, ks), _cat(pg.kz, kz)
            pg.vc, pg.vs, pg.vz = _cat(pg.vc, vc), _cat(pg.vs, vs), _cat(pg.vz, vz)
        pg.n += k.shape[2]

    # ---------------------------------------------------------------- shrinking
    def _lower_page(self, pg, target_bits):
        """Lower one page to target_bits.

        From 16 bits: direct quantization of the stored fp16 values (Eq. 1-2); by the
        appendix theorem this is what an integer 16-bit tier followed by Eq. 3 would give.
        From 2b to b bits: Eq. 3 on the codes, S_b = (2^b + 1) S_2b, Z unchanged (or one of the two
        ablation strategies of Sec. 4.3.1 when the configuration asks for it).  A page of the integer 16-bit
        tier goes down the same way, one halving at a time (16 -> 8 -> ... -> target_bits).
        """
        G = self.cfg.group
        if pg.bits == 16 and self.cfg.tier16 == TIER16_FP16:
            pg.kc, pg.ks, pg.kz = quantize(pg.k, target_bits, G)
            pg.vc, pg.vs, pg.vz = quantize(pg.v, target_bits, G)
            pg.k = pg.v = None
        else:
            assert target_bits * 2 == pg.bits or (pg.bits == 16 and target_bits in (8, 4, 2))
            b = pg.bits
            while b > target_bits:
                b //= 2
                pg.kc, pg.ks, pg.kz = shrink_step(pg.kc, pg.ks, pg.kz, b, self.cfg.shift_strategy)
                pg.vc, pg.vs, pg.vz = shrink_step(pg.vc, pg.vs, pg.vz, b, self.cfg.shift_strategy)
        pg.bits = target_bits

    def requant(self, layer, segment=-1, reserve_tokens=0):
        """One bit-width shrinking action; returns the number of pages re-quantized.

        segment >= 0: lower every page of that run (see segments()) one step.
        segment == -1, policy PAPER: the block's current width b_cur is halved: every
        unprotected page at b_cur goes to b_cur/2.  BudgetError if b_cur is already Fbit.
        segment == -1, policy OLDEST_FIRST: while bytes_used plus reserve_tokens 16-bit
        tokens exceed the budget, lower the oldest complete unprotected page whose width
        is above Fbit by one step.  BudgetError when no such page is left.
        """
        c, L, P = self.cfg, self.layers[layer], self.cfg.page_tokens
        if segment >= 0:
            segs = self.segments(layer)
            if segment >= len(segs):
                raise StateError("no such segment")
            t0, t1, b = segs[segment]
            if b == 2:
                raise StateError("already at 2 bits")
            if t1 == L.T and L.T % P != 0 and (c.policy == POLICY_OLDEST_FIRST or c.window > 0):
                # the run ends in the partly filled last page and the policy appends at 16 bits: lowered, that
                # page could take no further token (a page holds one width)
                raise StateError("run ends in the partly filled last page")
            idx = range(t0 // P, (t1 + P - 1) // P)
            for i in idx:
                self._lower_page(L.pages[i], b // 2)
            return len(idx)
        if c.policy == POLICY_PAPER:
            bcur = self.current_bits(layer)
            if bcur <= L.fbit:
                raise BudgetError("block already at Fbit")
            idx = [i for i, p in enumerate(L.pages) if p.bits == bcur and not self._protected(L, i)]
            if not idx:
                raise BudgetError("nothing to shrink")
            for i in idx:
                self._lower_page(L.pages[i], bcur // 2)
            return len(idx)
        steps = 0
        need = reserve_tokens * c.batch * c.n_kv_heads * self._bpth(16)
        while self.bytes_used(layer) + need > L.budget:
            cand = [i for i, p in enumerate(L.pages)
                    if p.bits > L.fbit and p.n == P and (i + 1) * P <= L.T - c.window and i >= c.n_sink // P]
            if not cand:
                raise BudgetError("no page left to shrink")
            pg = L.pages[cand[0]]
            self._lower_page(pg, pg.bits // 2)
            steps += 1
        return steps

    # ---------------------------------------------------------------- read-out
    def dequantized(self, layer):
        """K_hat, V_hat fp64 [B, Hkv, T, D] in token order."""
        G = self.cfg.group
        ks, vs = [], []
        for p in self.layers[layer].pages:
            if p.k is not None:
                ks.append(p.k.astype(np.float64)); vs.append(p.v.astype(np.float64))
            else:
                ks.append(dequantize(p.kc, p.ks, p.kz, G)); vs.append(dequantize(p.vc, p.vs, p.vz, G))
        return np.concatenate(ks, 2), np.concatenate(vs, 2)

    def reconstruction_sq_error(self, layer, K, V):
        """(sum over all cached elements of (K_hat - K)^2, the same for V) in fp64: how far the de-quantized cache
        is from the fp16 tensors K, V [B, H, T, D] it was built from (the measure used to compare the bit-width
        shrinking strategies of Sec. 4.3.1 without a model)."""
        Kh, Vh = self.dequantized(layer)
        T = Kh.shape[2]
        dk = Kh - K[:, :, :T].astype(np.float64)
        dv = Vh - V[:, :, :T].astype(np.float64)
        return float(np.sum(dk * dk)), float(np.sum(dv * dv))

    def attention(self, layer, q, scale=None):
        if self.lam[layer] is not None:
            q = reparam_queries(q, self.lam[layer], self.cfg.n_kv_heads)
        K, V = self.dequantized(layer)
        return decode_attention_fp64(q, K, V, scale)

    def export_segment(self, layer, segment, which):
        """Canonical export of one run.  16 bits, fp16 tier: (fp16 values [B,H,n,D], None, None).
        Quantized (and 16 bits of the INT16 tier): (packed codes uint8 [B,H,n,D*b/8], S fp16 [B,H,n,D/G],
        Z fp16 [B,H,n,D/G])."""
        P = self.cfg.page_tokens
        t0, t1, b = self.segments(layer)[segment]
        pages = self.layers[layer].pages[t0 // P:(t1 + P - 1) // P]
        if b == 16 and self.cfg.tier16 == TIER16_FP16:
            return np.concatenate([p.k if which == "K" else p.v for p in pages], 2), None, None
        pre = "k" if which == "K" else "v"
        codes = np.concatenate([getattr(p, pre + "c") for p in pages], 2)
        S = np.concatenate([getattr(p, pre + "s") for p in pages], 2)
        Z = np.concatenate([getattr(p, pre + "z") for p in pages], 2)
        return pack_codes(codes, b), S, Z


def decode_step_batch(caches, layer, ks, vs, qs, scale=None):
    """One decode step of block `layer` for a ragged batch: sequence (group) i has its own cache caches[i] -- its own
    length, widths and budget -- receives one new token ks[i], vs[i] (fp16 [B_i, Hkv, 1, D]) and attends with qs[i]
    (fp16 [B_i, Hq, D]) over its own cache only.  All or nothing: if any cache cannot take its token (BudgetError,
    StateError) the error is raised before any cache has changed.  Returns the list of fp64 outputs [B_i, Hq, D]."""
    assert len(caches) == len(ks) == len(vs) == len(qs)
    for c in caches:
        c._plan_append(layer, 1, 0)
    for c, k, v in zip(caches, ks, vs):
        c.append(layer, k, v)
    return [c.attention(layer, q, scale) for c, q in zip(caches, qs)]
