// Device code of the quantizers shared by the append, requantization and attention kernels (gfx950): Eq. 1-2 by
// "owner" lanes, the way codes travel through LDS into the tile layout of kvq_layout.h, and the append of new tokens
// into a tile of the integer 16-bit tier.
#ifndef KVQ_QUANT_DEV_H
#define KVQ_QUANT_DEV_H

#include "kvq_internal.h"
#include "kvq_append16.h"

namespace kvq_q {

using kvq_dev::u32x4;
using kvq_dev::h2f;
using kvq_dev::f2h_rn;
using kvq_dev::load_key8;

// (S, Z) of one group from its min and max (both exact fp16 values held as float), Eq. 2.
__device__ inline void group_params(float mn, float mx, int levels, uint16_t* S, uint16_t* Z, float* Sf) {
    float s32 = (mx - mn) / (float)levels;  // one fp32 subtract, one correctly rounded fp32 divide
    *S = f2h_rn(s32);
    *Z = f2h_rn(mn);
    *Sf = h2f(*S);
}
// Eq. 1 with the stored scale; a zero scale maps the whole group to code 0.
__device__ inline uint32_t code_of(float x, float mn, float Sf, int levels) {
    if (Sf == 0.0f) return 0u;
    float r = rintf((x - mn) / Sf);
    r = fminf(fmaxf(r, 0.0f), (float)levels);
    return (uint32_t)r;
}

template <int B>
__device__ inline uint32_t v_token_mask(uint32_t kb, int dw) {
    constexpr int per = 32 / B;  // slots per dword
    constexpr uint32_t field = (B == 32) ? 0xffffffffu : ((1u << B) - 1u);
    uint32_t m = 0;
#pragma unroll
    for (int e = 0; e < per; ++e) {
        int slot = dw * per + e;
        int tok = slot & 7;
        if ((kb >> tok) & 1u) m |= field << (e * B);
    }
    return m;
}

template <int B>
__device__ inline void store_chunks(uint8_t* tile, int lane, const uint32_t (&str)[2 * B]) {
#pragma unroll
    for (int c = 0; c < B / 2; ++c) {
        u32x4 v = {str[4 * c], str[4 * c + 1], str[4 * c + 2], str[4 * c + 3]};
        *reinterpret_cast<u32x4*>(tile + (c * 64 + lane) * 16) = v;
    }
}
template <int B>
__device__ inline void load_chunks(const uint8_t* tile, int lane, uint32_t (&str)[2 * B]) {
#pragma unroll
    for (int c = 0; c < B / 2; ++c) {
        u32x4 v = *reinterpret_cast<const u32x4*>(tile + (c * 64 + lane) * 16);
        str[4 * c] = v.x; str[4 * c + 1] = v.y; str[4 * c + 2] = v.z; str[4 * c + 3] = v.w;
    }
}
// Streaming variants for the page-at-a-time kernels, which read and write every byte exactly once.
template <int B>
__device__ inline void load_chunks_stream(const uint8_t* tile, int lane, uint32_t (&str)[2 * B]) {
#pragma unroll
    for (int c = 0; c < B / 2; ++c) {
        u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tile + (c * 64 + lane) * 16));
        str[4 * c] = v.x; str[4 * c + 1] = v.y; str[4 * c + 2] = v.z; str[4 * c + 3] = v.w;
    }
}
template <int B>
__device__ inline void store_chunks_stream(uint8_t* tile, int lane, const uint32_t (&str)[2 * B]) {
#pragma unroll
    for (int c = 0; c < B / 2; ++c) {
        u32x4 v = {str[4 * c], str[4 * c + 1], str[4 * c + 2], str[4 * c + 3]};
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(tile + (c * 64 + lane) * 16));
    }
}

// ------------------------------------------------------------------------------ row-owner quantizer core
// Quantized widths are produced by "owner" lanes: in each of two passes over a 32-token tile, lane l owns the
// group (token 16*pass + l/4, channels 32*(l%4) .. +31): 64 contiguous bytes, so the minimum and maximum need
// no cross-lane traffic.  The owner writes its 32 codes as bytes to LDS -- [token][channel] for a K tile,
// [channel][token] for a V tile -- from where every lane gathers the slots of the tile layout with 8-byte reads.
typedef _Float16 half2v __attribute__((ext_vector_type(2)));

__device__ inline uint32_t pk_min_u(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(half2v, a), __builtin_bit_cast(half2v, b)));
}
__device__ inline uint32_t pk_max_u(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(half2v, a), __builtin_bit_cast(half2v, b)));
}

// x - mn for the fp16 value in the low (hi = 0) or high (hi = 1) half of w, in one instruction: x * 1.0 - mn with
// the single rounding of a fused multiply-add, which is the rounding of the fp32 subtraction (the conversion of
// x to fp32 is exact), instead of a conversion followed by a subtraction.
__device__ inline float half_minus(uint32_t w, int hi, float mn) {
    float r;
    if (hi) asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w), "v"(mn));
    else asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w), "v"(mn));
    return r;
}

#define KVQ_LDS_CODES_K 4096                       // K: [32 tokens][128 channels] code bytes
#define KVQ_LDS_VGRP (32 * 32 + 16)                // V: per group [32 channels][32 tokens] code bytes, skewed
#define KVQ_LDS_CODES (4 * KVQ_LDS_VGRP)           // room for either arrangement

// Eq. 1-2 for the 32 fp16 values in w[16] (two per dword).  codes[e] receives the code of element e as a float.
// Fast path: a reciprocal multiply, with the IEEE division the definition asks for only where the product lies too
// close to a half-integer to decide the rounding (see the bound in the body).
// gspan = G / 32: a quantization group of G = 64 or 128 channels spans 2 or 4 neighbouring owner lanes (the
// owners of one token's four 32-channel runs are lanes 4k .. 4k+3), which then share min, max and so (S, Z).
template <int B>
__device__ inline void quantize_owner(const uint32_t (&w)[16], float (&codes)[32], uint16_t* S, uint16_t* Z,
                                      int gspan) {
    constexpr int levels = (1 << B) - 1;
    uint32_t mn2 = pk_min_u(w[0], w[1]), mx2 = pk_max_u(w[0], w[1]);  // (no plain copy of a loaded register: the copy
#pragma unroll                                                        //  would be placed, with a full wait, beside the load)
    for (int k = 2; k < 16; ++k) { mn2 = pk_min_u(mn2, w[k]); mx2 = pk_max_u(mx2, w[k]); }
    float mn = fminf(h2f((uint16_t)(mn2 & 0xffff)), h2f((uint16_t)(mn2 >> 16)));
    float mx = fmaxf(h2f((uint16_t)(mx2 & 0xffff)), h2f((uint16_t)(mx2 >> 16)));
    if (gspan >= 2) { mn = fminf(mn, __shfl_xor(mn, 1)); mx = fmaxf(mx, __shfl_xor(mx, 1)); }
    if (gspan >= 4) { mn = fminf(mn, __shfl_xor(mn, 2)); mx = fmaxf(mx, __shfl_xor(mx, 2)); }
    float Sf;
    group_params(mn, mx, levels, S, Z, &Sf);
    if constexpr (B == 16) {  // codes up to 65535: the reciprocal shortcut is not accurate enough, divide
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const float x = h2f((uint16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffff)));
            codes[e] = (float)code_of(x, mn, Sf, levels);
        }
        return;
    }
    // Reciprocal: the hardware's (1 ulp) refined by one Newton step, relative error below 2^-24 (1 + 2^-22).  Then
    // t = (x - Z) * rcp is within 2^-23 of the true quotient, relatively, and the correctly rounded fp32 quotient the
    // definition asks for within 2^-24: the two differ by less than 1.8e-7 * (levels + 1), and rint(t) is the
    // required code unless t lies that close to a half-integer (eps below adds a margin of 1.4).  Only then is the
    // IEEE division carried out, and only for the elements concerned.
    float rcp = 0.0f;
    if (Sf != 0.0f) {
        const float r0 = __builtin_amdgcn_rcpf(Sf);
        rcp = fmaf(r0, fmaf(-Sf, r0, 1.0f), r0);
    }
    constexpr float near_half = 0.5f - 2.5e-7f * (float)(levels + 1);
    // No element's quotient exceeds that of the group maximum (x <= mx and every step is monotone), so the clamp to
    // the top level is decided once per group instead of once per element; a group that needs it (S rounded down
    // to a subnormal fp16) takes the division path below, which clamps.
    const bool over = rintf((mx - mn) * rcp) > (float)levels;
    float worst = 0.0f;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const float t = half_minus(w[e >> 1], e & 1, mn) * rcp;
        const float r = rintf(t);
        worst = fmaxf(worst, fabsf(t - r));
        codes[e] = r;
    }
    if (__any(worst > near_half || over)) {
        asm volatile("" ::: "memory");  // keep this a branch
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const float x = h2f((uint16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffff)));
            const float t = (x - mn) * rcp;
            if (over || fabsf(t - rintf(t)) > near_half) codes[e] = (float)code_of(x, mn, Sf, levels);
        }
    }
}

// Owner -> LDS.  tl = token in tile, grp = channel group, which = 0 K / 1 V.
__device__ inline void scatter_codes(uint8_t* lds, int which, int tl, int grp, const float (&codes)[32]) {
    if (!which) {
        uint32_t d[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            uint32_t v = __builtin_amdgcn_cvt_pk_u8_f32(codes[4 * k], 0u, 0u);
            v = __builtin_amdgcn_cvt_pk_u8_f32(codes[4 * k + 1], 1u, v);
            v = __builtin_amdgcn_cvt_pk_u8_f32(codes[4 * k + 2], 2u, v);
            d[k] = __builtin_amdgcn_cvt_pk_u8_f32(codes[4 * k + 3], 3u, v);
        }
        u32x4* dst = reinterpret_cast<u32x4*>(lds + tl * 128 + grp * 32);
        dst[0] = u32x4{d[0], d[1], d[2], d[3]};
        dst[1] = u32x4{d[4], d[5], d[6], d[7]};
    } else {
        uint8_t* dst = lds + grp * KVQ_LDS_VGRP + tl;
#pragma unroll
        for (int c = 0; c < 32; ++c) dst[c * 32] = (uint8_t)(uint32_t)codes[c];
    }
}

// 8 code bytes (b0 in the low byte of w0) -> 8 codes of B bits, packed little-endian into the low 8*B bits.
template <int B>
__device__ inline void pack8(uint32_t w0, uint32_t w1, uint32_t* lo, uint32_t* hi) {
    if constexpr (B == 8) {
        *lo = w0; *hi = w1;
    } else if constexpr (B == 4) {
        uint32_t x = w0 | (w0 >> 4), y = w1 | (w1 >> 4);
        *lo = __builtin_amdgcn_perm(y, x, 0x06040200u);
        *hi = 0u;
    } else {
        uint32_t x = w0 | (w0 >> 6), y = w1 | (w1 >> 6);
        x |= x >> 12; y |= y >> 12;
        *lo = __builtin_amdgcn_perm(y, x, 0x0c0c0400u);
        *hi = 0u;
    }
}

// LDS -> the lane's packed string of the tile layout.
template <int B>
__device__ inline void gather_string(const uint8_t* lds, int which, int lane, uint32_t (&str)[2 * B]) {
    const int j = lane >> 4, n = lane & 15;
#pragma unroll
    for (int d = 0; d < 2 * B; ++d) str[d] = 0u;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const uint8_t* src;
        if (!which) {
            const int sub = p >> 2, grp = p & 3;
            const int t = 8 * (n >> 2) + 4 * sub + (n & 3);
            src = lds + t * 128 + grp * 32 + 8 * j;
        } else {
            const int ch = 16 * p + n;  // piece p = channel block nt
            src = lds + (ch >> 5) * KVQ_LDS_VGRP + (ch & 31) * 32 + 8 * j;
        }
        const uint32_t w0 = reinterpret_cast<const uint32_t*>(src)[0], w1 = reinterpret_cast<const uint32_t*>(src)[1];
        uint32_t lo, hi;
        pack8<B>(w0, w1, &lo, &hi);
        if constexpr (B == 8) { str[2 * p] = lo; str[2 * p + 1] = hi; }
        else if constexpr (B == 4) { str[p] = lo; }
        else { str[p >> 1] |= lo << (16 * (p & 1)); }
    }
}

__device__ inline void wave_sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The attention kernel multiplies probabilities (<= 1) by up to 64 and by the V scale in fp16; a cache that ever
// holds a V scale of 256 or more (a value range no attention layer produces) is marked and takes the kernel's
// overflow-proof path instead.
__device__ inline void note_large_v_scale(uint32_t* flags, int which, uint16_t S) {
    if (which && h2f(S) >= 256.0f) atomicOr(flags, 1u);
}

// Owner lanes write the (S, Z) of their group straight to the tile's metadata.
__device__ inline void store_meta_owner(uint8_t* meta, int which, int tl, int grp, uint16_t S, uint16_t Z) {
    uint16_t* ms = reinterpret_cast<uint16_t*>(meta + (which ? 512 : 0));
    uint16_t* mz = reinterpret_cast<uint16_t*>(meta + (which ? 768 : 256));
    const int idx = which ? kvq_vmeta_index(tl, grp) : tl * 4 + grp;
    ms[idx] = S;
    mz[idx] = Z;
}

// ------------------------------------------------------------------------------------------------ append
// Descriptors of the (at most two) pages a short append touches ride in the kernel arguments, which saves the
// dependent read of the device page table; longer appends look the table up.
struct KvqAppendPages {
    KvqPageDesc d[2];
    int first_page;  // -1: use the table
};
// (The offsets are pinned to scalar registers inside each branch: left alone, the two branches are merged into one
//  load through a selected pointer, which can only be a flat load, and while a flat load is pending every wait for a
//  global load becomes a wait for all of them.)
__device__ inline KvqPageDesc append_desc(const KvqPageDesc* table, const KvqAppendPages& ap, int page) {
    KvqPageDesc r;
    r.bits = 0u;
    r.int16 = 0u;
    if (ap.first_page < 0) {
        r.code_off256 = table[page].code_off256;
        r.meta_off256 = table[page].meta_off256;
        asm volatile("" : "+s"(r.code_off256), "+s"(r.meta_off256));
    } else {
        const bool first = page == ap.first_page;
        r.code_off256 = first ? ap.d[0].code_off256 : ap.d[1].code_off256;
        r.meta_off256 = first ? ap.d[0].meta_off256 : ap.d[1].meta_off256;
        asm volatile("" : "+s"(r.code_off256), "+s"(r.meta_off256));
    }
    return r;
}

// Appends the tokens [t_old, t_new) that fall into one tile of the integer 16-bit tier to its K (which = 0) or V (1)
// string: Eq. 1-2 with 2^16 - 1 levels by the owner lanes; the high and the low bytes of the codes then travel through
// LDS into the tile's two byte planes like two 8-bit tiles.  A tile that already holds tokens gets the bytes of the new
// tokens only (the append that started the tile has zeroed the slots and the metadata of the tokens to come); a new
// tile is written whole.  One wavefront.
//   code: the string (its high-byte plane; the low-byte plane follows), meta: the tile's metadata,
//   in: fp16 rows [t_new - t_old][128] of this (sequence, KV head), tok0: first token of the tile,
//   rope: [t_new - t_old][128] cos | sin rows or null, rinv: [n_kv_heads][128] reciprocal reparameterization factors or
//   null, head: this unit's KV head,
//   lds: scratch of this wavefront alone.
__device__ __forceinline__ void append_i16_string(uint8_t (&lds)[2][KVQ_LDS_CODES], uint8_t* __restrict__ code,
                                         uint8_t* __restrict__ meta, const uint16_t* __restrict__ in, int which, int tok0,
                                         int t_old, int t_new, int gspan, const float* __restrict__ rope,
                                         const float* __restrict__ rinv, int head, int lane) {
    const int j = lane >> 4, n = lane & 15;
    const int grp = lane & 3;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int tl = 16 * pass + (lane >> 2);
        const int tok = tok0 + tl;
        const bool isnew = tok >= t_old && tok < t_new;
        uint32_t w[16];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (isnew) {
                const uint16_t* row = in + (uint64_t)(tok - t_old) * KVQ_D;
                if (which) v = *reinterpret_cast<const u32x4*>(row + 32 * grp + 8 * c);
                else v = load_key8(row, 32 * grp + 8 * c, rope ? rope + (uint64_t)(tok - t_old) * KVQ_D : nullptr,
                                   rinv ? rinv + head * KVQ_D : nullptr);
            }
            w[4 * c] = v.x; w[4 * c + 1] = v.y; w[4 * c + 2] = v.z; w[4 * c + 3] = v.w;
        }
        float codes[32], lo[32];
        uint16_t S, Z;
        quantize_owner<16>(w, codes, &S, &Z, gspan);
#pragma unroll
        for (int e = 0; e < 32; ++e) {  // exact: integers below 2^16
            const float hi = floorf(codes[e] * 0.00390625f);
            lo[e] = codes[e] - 256.0f * hi;
            codes[e] = hi;
        }
        scatter_codes(lds[0], which, tl, grp, codes);
        scatter_codes(lds[1], which, tl, grp, lo);
        if (tok >= t_old) store_meta_owner(meta, which, tl, grp, S, Z);
    }
    wave_sync_lds();
    const bool has_old = tok0 < t_old;  // then only the bytes of the new tokens are stored: nothing is read back
#pragma unroll
    for (int plane = 0; plane < 2; ++plane) {
        uint32_t str[16];
        gather_string<8>(lds[plane], which, lane, str);
        uint8_t* dst = code + plane * (512u * 8);
        if (!has_old) {
            store_chunks<8>(dst, lane, str);
        } else if (!which) {  // K: dwords 8 sub .. 8 sub + 7 of a lane are one token
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const int tok = tok0 + 8 * (n >> 2) + 4 * sub + (n & 3);
                if (tok >= t_old && tok < t_new) {
#pragma unroll
                    for (int c = 2 * sub; c < 2 * sub + 2; ++c)
                        *reinterpret_cast<u32x4*>(dst + (c * 64 + lane) * 16) =
                            u32x4{str[4 * c], str[4 * c + 1], str[4 * c + 2], str[4 * c + 3]};
                }
            }
        } else {              // V: slot 4 d + e of a lane is token 8 j + ((4 d + e) & 7)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int tok = tok0 + 8 * j + i;
                if (tok >= t_old && tok < t_new) {
#pragma unroll
                    for (int d = (i >> 2); d < 16; d += 2)
                        dst[((d >> 2) * 64 + lane) * 16 + (d & 3) * 4 + (i & 3)] = (uint8_t)(str[d] >> (8 * (i & 3)));
                }
            }
        }
    }
}

}  // namespace kvq_q

#endif
