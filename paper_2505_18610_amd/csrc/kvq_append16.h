// Device code shared by the append kernel and the attention kernel: writing new fp16 tokens into a tile of the
// 16-bit tier (raw values in the tile layout of kvq_layout.h), with the optional rotary embedding (Sec. 3.3, Eq. 9)
// and channel-wise reparameterization (Sec. 3.3, Eq. 7) of the keys on the way.
#ifndef KVQ_APPEND16_H
#define KVQ_APPEND16_H

#include <hip/hip_runtime.h>
#include "kvq_layout.h"

namespace kvq_dev {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline float h2f(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ inline uint16_t f2h_rn(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }  // RNE

// K Lambda^{-1} of Eq. 7 on 8 consecutive channels (4 dwords of fp16 pairs): fp32 product with the channel's
// reciprocal factor, rounded to nearest-even into fp16.
// The product is rounded to fp32 first and to fp16 second, as two separate IEEE operations: the empty asm keeps the
// compiler from fusing them into a mixed-precision instruction that rounds the exact product once (1 fp16 ulp apart
// in about one element of 10^4).
__device__ inline uint32_t scale_pair(uint32_t w, float r_lo, float r_hi) {
    float lo = h2f((uint16_t)(w & 0xffff)) * r_lo, hi = h2f((uint16_t)(w >> 16)) * r_hi;
    asm volatile("" : "+v"(lo), "+v"(hi));
    return (uint32_t)f2h_rn(lo) | ((uint32_t)f2h_rn(hi) << 16);
}
__device__ inline u32x4 scale_keys8(u32x4 v, const float* rinv) {
    const float4 r0 = *reinterpret_cast<const float4*>(rinv), r1 = *reinterpret_cast<const float4*>(rinv + 4);
    return u32x4{scale_pair(v.x, r0.x, r0.y), scale_pair(v.y, r0.z, r0.w), scale_pair(v.z, r1.x, r1.y),
                 scale_pair(v.w, r1.z, r1.w)};
}

// Rotary embedding (Sec. 3.3, Eq. 9) of 8 consecutive channels ch0 .. ch0+7 of one token: own = these channels,
// partner = the channels ch0 +- 64 of the same token, cs = the token's table row [cos 64 | sin 64] (fp32).
//   lower half (ch < 64):  own * cos - partner * sin        upper half:  own * cos + partner * sin
// Every product and the sum are separate fp32 operations (the empty asm keeps them from being contracted or
// fused with the conversion); the result is rounded to fp16.
__device__ inline u32x4 rope8(u32x4 own, u32x4 partner, const float* cs, int ch0) {
    const int i0 = ch0 & 63;
    const bool upper = ch0 >= 64;
    const uint32_t* o = reinterpret_cast<const uint32_t*>(&own);
    const uint32_t* p = reinterpret_cast<const uint32_t*>(&partner);
    u32x4 out;
    uint32_t* r = reinterpret_cast<uint32_t*>(&out);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float res[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float c = cs[i0 + 2 * e + h], sn = cs[64 + i0 + 2 * e + h];
            float p1 = h2f((uint16_t)(o[e] >> (16 * h))) * c, p2 = h2f((uint16_t)(p[e] >> (16 * h))) * sn;
            asm volatile("" : "+v"(p1), "+v"(p2));
            float sum = upper ? p1 + p2 : p1 - p2;
            asm volatile("" : "+v"(sum));
            res[h] = sum;
        }
        r[e] = (uint32_t)f2h_rn(res[0]) | ((uint32_t)f2h_rn(res[1]) << 16);
    }
    return out;
}

// The new keys' 8 channels ch0.. of the row at `row` (fp16 [128]), rotated and scaled as configured.
__device__ inline u32x4 load_key8(const uint16_t* row, int ch0, const float* rope_row, const float* rinv_head) {
    u32x4 v = *reinterpret_cast<const u32x4*>(row + ch0);
    if (rope_row) v = rope8(v, *reinterpret_cast<const u32x4*>(row + (ch0 ^ 64)), rope_row, ch0);
    if (rinv_head) v = scale_keys8(v, rinv_head + ch0);
    return v;
}

// One wavefront writes the tokens [t_old, t_new) that fall into one K (which = 0) or V (which = 1) tile of a
// 16-bit page.  code: the tile; in: the unit's new rows, fp16 [t_new - t_old][128]; tok0: the tile's first token.
// A tile that holds no older token is written in full (slots of tokens that are not there yet are zero, so
// partially filled tiles stay well defined); otherwise only the new tokens' elements are stored - whole 16-byte
// chunks for K, single fp16 values for V.  rope: table of the new tokens, fp32 [t_new - t_old][128], or null;
// rinv_head: the 128 reciprocal reparameterization factors of this KV head, or null (keys only).
// STREAM: a tile written in full goes out with streaming stores (bulk appends: the tile is read much later; not for a
// caller that reads the tile back at once).
template <bool STREAM = false>
__device__ inline void append16_tile(uint8_t* code, const uint16_t* in, int which, int tok0, int t_old, int t_new,
                                     int lane, const float* rope, const float* rinv_head) {
    const int j = lane >> 4, n = lane & 15;
    const bool has_old = tok0 < t_old;
    uint16_t raw[64];
    if (!which) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int tok = tok0 + 8 * (n >> 2) + 4 * sub + (n & 3);
            const bool isnew = tok >= t_old && tok < t_new;
#pragma unroll
            for (int grp = 0; grp < 4; ++grp) {
                u32x4 v = {0u, 0u, 0u, 0u};
                if (isnew)
                    v = load_key8(in + (uint64_t)(tok - t_old) * KVQ_D, 32 * grp + 8 * j,
                                  rope ? rope + (uint64_t)(tok - t_old) * KVQ_D : nullptr, rinv_head);
                const int s0 = (sub * 4 + grp) * 8;
                raw[s0 + 0] = v.x & 0xffff; raw[s0 + 1] = v.x >> 16;
                raw[s0 + 2] = v.y & 0xffff; raw[s0 + 3] = v.y >> 16;
                raw[s0 + 4] = v.z & 0xffff; raw[s0 + 5] = v.z >> 16;
                raw[s0 + 6] = v.w & 0xffff; raw[s0 + 7] = v.w >> 16;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int tok = tok0 + 8 * j + i;
            const bool isnew = tok >= t_old && tok < t_new;
#pragma unroll
            for (int nt = 0; nt < 8; ++nt)
                raw[nt * 8 + i] = isnew ? in[(uint64_t)(tok - t_old) * KVQ_D + 16 * nt + n] : (uint16_t)0;
        }
    }
    if (has_old) {
        if (!which) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const int tok = tok0 + 8 * (n >> 2) + 4 * sub + (n & 3);
                if (tok >= t_old && tok < t_new) {
#pragma unroll
                    for (int c = 4 * sub; c < 4 * sub + 4; ++c)
                        *reinterpret_cast<u32x4*>(code + (c * 64 + lane) * 16) =
                            u32x4{(uint32_t)raw[8 * c] | ((uint32_t)raw[8 * c + 1] << 16),
                                  (uint32_t)raw[8 * c + 2] | ((uint32_t)raw[8 * c + 3] << 16),
                                  (uint32_t)raw[8 * c + 4] | ((uint32_t)raw[8 * c + 5] << 16),
                                  (uint32_t)raw[8 * c + 6] | ((uint32_t)raw[8 * c + 7] << 16)};
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int tok = tok0 + 8 * j + i;
                if (tok >= t_old && tok < t_new) {
#pragma unroll
                    for (int nt = 0; nt < 8; ++nt) {
                        const int slot = nt * 8 + i;  // 2 bytes at string offset 2 * slot
                        *reinterpret_cast<uint16_t*>(code + kvq_tile_byte(lane, 2u * slot)) = raw[slot];
                    }
                }
            }
        }
        return;
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const u32x4 v = {(uint32_t)raw[8 * c] | ((uint32_t)raw[8 * c + 1] << 16),
                         (uint32_t)raw[8 * c + 2] | ((uint32_t)raw[8 * c + 3] << 16),
                         (uint32_t)raw[8 * c + 4] | ((uint32_t)raw[8 * c + 5] << 16),
                         (uint32_t)raw[8 * c + 6] | ((uint32_t)raw[8 * c + 7] << 16)};
        if (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(code + (c * 64 + lane) * 16));
        else *reinterpret_cast<u32x4*>(code + (c * 64 + lane) * 16) = v;
    }
}

// A V tile of a 16-bit page whose tokens are all new, written by one wavefront through LDS: the rows are read with
// 16-byte loads (a wavefront instruction covers one contiguous KiB of the input), parked as [token][channel] in LDS
// and picked up in the tile layout (lane (j, n): tokens 8j .. 8j+7 of channels 16 nt + n), where the plain path reads
// the same 4,096 values with two-byte loads; streaming stores, as the tile is read much later.  Rows are rotated by 32 bytes per 8 tokens so that the four lane
// quarters, which read rows 8 apart, use different banks.  lds: 8 KiB of this wavefront alone, 16-byte aligned.
__device__ inline void append16_v_tile_lds(uint8_t* code, const uint16_t* in, int tok0, int t_old, int t_new, int lane,
                                           uint8_t* lds) {
    const int j = lane >> 4, n = lane & 15;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int chunk = c * 64 + lane, tl = chunk >> 4, ch8 = chunk & 15;
        const int tok = tok0 + tl;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (tok < t_new) v = *reinterpret_cast<const u32x4*>(in + (uint64_t)(tok - t_old) * KVQ_D + 8 * ch8);
        *reinterpret_cast<u32x4*>(lds + tl * 256 + ((ch8 * 16 + 32 * (tl >> 3)) & 255)) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int c = 0; c < 8; ++c) {  // chunk c of the lane's string = channel block nt = c, tokens 8j + 0..7
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int r0 = 8 * j + 2 * e, r1 = r0 + 1;      // same group of 8 rows: same rotation
            const int col = ((16 * c + n) * 2 + 32 * j) & 255;
            const uint32_t lo = *reinterpret_cast<const uint16_t*>(lds + r0 * 256 + col);
            const uint32_t hi = *reinterpret_cast<const uint16_t*>(lds + r1 * 256 + col);
            w[e] = lo | (hi << 16);
        }
        __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4*>(code + (c * 64 + lane) * 16));
    }
}

}  // namespace kvq_dev

#endif
