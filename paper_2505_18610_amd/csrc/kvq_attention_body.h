// Fused de-quantize + single-token GQA decode attention over the mixed-width paged cache (gfx950).
//
// One workgroup (8 wavefronts, one per compute unit) handles one (sequence, KV head) unit and one cost-balanced
// range of 32-token tiles; its wavefronts claim two-tile chunks of the range from a counter in LDS, stream
// them with 16-byte non-temporal loads and keep their own online-softmax state.  Both contractions run on the
// matrix cores with the g <= 16 query heads of the unit as the 16-wide N dimension:
//   scores^T[token, head] = sum_grp S[token,grp] * (codes[token, grp-channels] . q[head, grp-channels])
//                           + sum_grp Z[token,grp] * sum(q[head, grp-channels])
//   out^T[channel, head] += sum_token codes[token, channel] * (p[token, head] * S_v[token, grp(channel)])
//                           + sum_token Z_v[token, grp(channel)] * p[token, head]
// Integer codes are exact in fp16, so scales and zero points never touch individual elements: they are
// applied to per-group partial sums (K) or folded into the probabilities (V), and the zero-point sums and
// the softmax denominator come out of one extra MFMA each.  Wavefront partials are merged through LDS,
// split partials through global memory (a second small kernel, or the last-arriving workgroup).
//
// This header holds the whole device code; the kernels that instantiate it are in kvq_attention.hip (one cache) and
// kvq_attention_batch.hip (ragged batch).
#ifndef KVQ_ATTENTION_BODY_H
#define KVQ_ATTENTION_BODY_H

#include "kvq_internal.h"
#include "kvq_append16.h"
#ifdef KVQ_WITH_I16_APPEND
#include "kvq_quant_dev.h"
#endif

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define KVQ_MAGIC 0x64006400u  // two fp16 1024.0: OR-ing a small integer into the mantissa gives 1024 + c

__device__ inline half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    u32x4 v = {a, b, c, d};
    return __builtin_bit_cast(half8, v);
}
__device__ inline uint32_t pk_fma(uint32_t x, float mul, float add) {
    half2v h = __builtin_bit_cast(half2v, x);
    half2v m = {(_Float16)mul, (_Float16)mul};
    half2v a = {(_Float16)add, (_Float16)add};
    h = h * m + a;
    return __builtin_bit_cast(uint32_t, h);
}
__device__ inline uint32_t pk_add(uint32_t x, float add) {
    half2v h = __builtin_bit_cast(half2v, x);
    half2v a = {(_Float16)add, (_Float16)add};
    h = h + a;
    return __builtin_bit_cast(uint32_t, h);
}
__device__ inline uint32_t pk_mul(uint32_t x, uint32_t y) {
    half2v h = __builtin_bit_cast(half2v, x) * __builtin_bit_cast(half2v, y);
    return __builtin_bit_cast(uint32_t, h);
}
__device__ inline float mixf(uint32_t packed, int hi) {  // fp16 half of a dword as float (folds into v_fma_mix)
    half2v h = __builtin_bit_cast(half2v, packed);
    return (float)(hi ? h.y : h.x);
}

// (x & mask) | magic in one VALU op; gfx9 VOP3 takes no literals and one scalar operand, so the mask rides in
// an SGPR and the magic constant in a VGPR.
__device__ inline uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask), "v"(magic));
    return r;
}

// Piece p (8 consecutive slots) of a lane's packed string -> 8 exact fp16 integers in MFMA operand order:
// operand register v holds slots v (low half) and v+4 (high half).
template <int B>
__device__ inline half8 dq_piece(const uint32_t* w, int p) {
    uint32_t r0, r1, r2, r3;
    const uint32_t magic = KVQ_MAGIC;
    if constexpr (B == 8) {
        uint32_t w0 = w[2 * p], w1 = w[2 * p + 1];
        r0 = pk_add(__builtin_amdgcn_perm(w1, w0, 0x0c040c00u) | KVQ_MAGIC, -1024.f);
        r1 = pk_add(__builtin_amdgcn_perm(w1, w0, 0x0c050c01u) | KVQ_MAGIC, -1024.f);
        r2 = pk_add(__builtin_amdgcn_perm(w1, w0, 0x0c060c02u) | KVQ_MAGIC, -1024.f);
        r3 = pk_add(__builtin_amdgcn_perm(w1, w0, 0x0c070c03u) | KVQ_MAGIC, -1024.f);
    } else if constexpr (B == 4) {
        uint32_t x = w[p], y = x >> 8;
        r0 = pk_add(and_or(x, 0x000f000fu, magic), -1024.f);
        r1 = pk_fma(and_or(x, 0x00f000f0u, magic), 0.0625f, -64.f);
        r2 = pk_add(and_or(y, 0x000f000fu, magic), -1024.f);
        r3 = pk_fma(and_or(y, 0x00f000f0u, magic), 0.0625f, -64.f);
    } else {  // B == 2: 16 bits of dword p/2
        uint32_t x = w[p >> 1];
        uint32_t t = (p & 1) ? __builtin_amdgcn_perm(0u, x, 0x0c030c02u) : __builtin_amdgcn_perm(0u, x, 0x0c010c00u);
        r0 = pk_add(and_or(t, 0x00030003u, magic), -1024.f);
        r1 = pk_fma(and_or(t, 0x000c000cu, magic), 0.25f, -256.f);
        r2 = pk_fma(and_or(t, 0x00300030u, magic), 0.0625f, -64.f);
        r3 = pk_fma(and_or(t, 0x00c000c0u, magic), 0.015625f, -16.f);
    }
    return as_half8(r0, r1, r2, r3);
}

// The same piece as fp16 *denormals*: the code bits are left where they are in the mantissa, so register v
// holds c * 2^(pos_v - 24) with pos_v = 0 (8 bit), {0,4,0,4}[v] (4 bit), 2v (2 bit).  The matrix cores take
// denormal inputs exactly; the K product compensates with a query operand pre-scaled by 2^-pos_v and one
// multiplication of the per-token sum by 2^24.  One VALU op per two codes.
template <int B>
__device__ inline half8 dq_piece_denorm(const uint32_t* w, int p) {
    uint32_t r0, r1, r2, r3;
    if constexpr (B == 8) {
        uint32_t w0 = w[2 * p], w1 = w[2 * p + 1];
        r0 = __builtin_amdgcn_perm(w1, w0, 0x0c040c00u);
        r1 = __builtin_amdgcn_perm(w1, w0, 0x0c050c01u);
        r2 = __builtin_amdgcn_perm(w1, w0, 0x0c060c02u);
        r3 = __builtin_amdgcn_perm(w1, w0, 0x0c070c03u);
    } else if constexpr (B == 4) {
        uint32_t x = w[p], y = x >> 8;
        r0 = x & 0x000f000fu;
        r1 = x & 0x00f000f0u;
        r2 = y & 0x000f000fu;
        r3 = y & 0x00f000f0u;
    } else {
        uint32_t x = w[p >> 1];
        uint32_t t = (p & 1) ? __builtin_amdgcn_perm(0u, x, 0x0c030c02u) : __builtin_amdgcn_perm(0u, x, 0x0c010c00u);
        r0 = t & 0x00030003u;
        r1 = t & 0x000c000cu;
        r2 = t & 0x00300030u;
        r3 = t & 0x00c000c0u;
    }
    return as_half8(r0, r1, r2, r3);
}

// Width tag 17 stands for a tile of the integer 16-bit tier: 16 bits per code, held as a high-byte and a low-byte
// plane of 8-bit strings, with metadata.  (A template tag only: page descriptors say 16 for both kinds, and a
// cache has one kind.)
#define KVQ_I16 17
template <int B> constexpr int code_bits() { return B == KVQ_I16 ? 16 : B; }
template <int B> constexpr bool has_meta() { return B != 16; }
template <int B> constexpr int q_class() { return B == KVQ_I16 ? 8 : B; }  // arrangement of the query operands

// Piece p of a low-byte plane as exact fp16 fractions c / 256 (the high bytes enter as the integers c).
__device__ inline half8 dq_piece_frac(const uint32_t* w, int p) {
    const uint32_t w0 = w[2 * p], w1 = w[2 * p + 1];
    const uint32_t r0 = pk_fma(__builtin_amdgcn_perm(w1, w0, 0x0c040c00u) | KVQ_MAGIC, 0.00390625f, -4.f);
    const uint32_t r1 = pk_fma(__builtin_amdgcn_perm(w1, w0, 0x0c050c01u) | KVQ_MAGIC, 0.00390625f, -4.f);
    const uint32_t r2 = pk_fma(__builtin_amdgcn_perm(w1, w0, 0x0c060c02u) | KVQ_MAGIC, 0.00390625f, -4.f);
    const uint32_t r3 = pk_fma(__builtin_amdgcn_perm(w1, w0, 0x0c070c03u) | KVQ_MAGIC, 0.00390625f, -4.f);
    return as_half8(r0, r1, r2, r3);
}

// The cache is read exactly once per launch: streaming (non-temporal) loads, which measurably raise the HBM
// rate of a pure read of this size.
__device__ inline u32x4 load_stream16(const uint8_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

// tile: wavefront-uniform address (scalar registers); lane_off = 16 * lane, computed once per kernel.  Written
// this way the loads need no per-load address registers (scalar base + one loop-invariant offset register).
template <int NDW>
__device__ inline void load_string(const uint8_t* tile, uint32_t lane_off, uint32_t (&w)[NDW]) {
#pragma unroll
    for (int c = 0; c < NDW / 4; ++c) {
        u32x4 v = load_stream16(tile + lane_off + c * 1024);
        w[4 * c] = v.x; w[4 * c + 1] = v.y; w[4 * c + 2] = v.z; w[4 * c + 3] = v.w;
    }
}

// Measurement build without arithmetic (python -m paper_2505_18610_amd.build --no-arithmetic): every load of a tile is
// issued and waited for as in the library, claims, descriptors, the join and the merge of the splits run as they do,
// but no tile is computed on.  Its launch time is the floor that the launch structure and memory leave to any
// arithmetic; its results are meaningless.  Nothing but paper_2505_18610_amd/phase_table.py --floor loads it.
#ifdef KVQ_NO_ARITHMETIC
template <int N>
__device__ inline void keep_loaded(const uint32_t (&w)[N]) {
#pragma unroll
    for (int e = 0; e < N; ++e) asm volatile("" :: "v"(w[e]));
}
__device__ inline void keep_loaded(const u32x4& v) { asm volatile("" :: "v"(v.x), "v"(v.y), "v"(v.z), "v"(v.w)); }
#endif

struct WaveState {
    float4v o[8];   // out^T accumulators: o[nt][i] = channel 16nt + 4j + i of head n (lane = 16j + n)
    float4v zl;     // quarter 0: zero-point sums of V groups 0..3; quarter 1, element 0: softmax denominator
    float m;        // running maximum of head n in log2 units (equal in the four quarters)
    int oexp;       // the accumulators o[] hold the true sums times 2^oexp (denormal V code operands, see below)
    int safe_v;     // 1: some V scale of this cache is large; use the overflow-proof V path
};

// query operands of one lane: [grp][4 dwords]
struct QOps {
    uint32_t q[4][4];
    uint32_t qsum[2];  // per-group sums of q (times the softmax scale), fp16 hi parts in lane quarter 0, lo parts in
                       // quarter 1, zero elsewhere: B operand of the K=16 MFMA that adds the zero-point term
    int cls;           // width the operands are arranged for: 16 natural k-slot order; 8/4/2 the (v, v+4)
                       // pairing, pre-scaled by 2^-pos_v of that width's denormal code operands
    int have_qsum;
};

__device__ inline uint32_t pack_rn(float a, float b) {  // two floats -> packed fp16, round to nearest even
    half2v h = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(uint32_t, h);
}

__device__ inline void load_q_ops(QOps& Q, const _Float16* q_lds, int lane, int cls, float scale_log2) {
    const int j = lane >> 4, n = lane & 15;
    const _Float16* row = q_lds + n * KVQ_D;
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
        const _Float16* p = row + 32 * grp + 8 * j;
        float sum = 0.f;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            _Float16 lo = (cls == 16) ? p[2 * v] : p[v];
            _Float16 hi = (cls == 16) ? p[2 * v + 1] : p[v + 4];
            sum += (float)lo + (float)hi;
            float f = 1.0f;
            if (cls == 4) f = (v & 1) ? 0.0625f : 1.0f;
            if (cls == 2) f = (v == 0) ? 1.0f : (v == 1) ? 0.25f : (v == 2) ? 0.0625f : 0.015625f;
            half2v h = {lo, hi};
            half2v fs = {(_Float16)f, (_Float16)f};
            h = h * fs;  // exact: a power of two (tiny |q| may round in the denormal range)
            Q.q[grp][v] = __builtin_bit_cast(uint32_t, h);
        }
        if (!Q.have_qsum) {  // sum of q over the group's 32 channels: 8 here, the rest in the other quarters
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            sum *= scale_log2;  // the zero-point term then needs no scaling after its MFMA
            _Float16 h = (_Float16)sum;
            _Float16 l = (_Float16)(sum - (float)h);
            uint32_t hb = __builtin_bit_cast(uint16_t, h), lb = __builtin_bit_cast(uint16_t, l);
            uint32_t mine = (j == 0) ? hb : (j == 1) ? lb : 0u;
            if (grp & 1) Q.qsum[grp >> 1] |= mine << 16;
            else Q.qsum[grp >> 1] = mine;
        }
    }
    Q.have_qsum = 1;
    Q.cls = cls;
}

__device__ inline float4v mfma(half8 a, half8 b, float4v c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Registers of one pipeline stage: TPI tiles in flight, each the lane's packed K and V strings and its
// 16-byte share of the tile's metadata.
template <int B, int TPI>
struct Stage {
    uint32_t kw[TPI][2 * B];
    uint32_t vw[TPI][2 * B];
    u32x4 meta[TPI];
    int tok0[TPI];  // first token of each tile (a huge value marks a slot that only pads the stage)
};

#define KVQ_ATTN_THREADS 512
#define KVQ_ATTN_WAVES 8
#define KVQ_PAD_TOK0 0x3fffff00
#ifndef KVQ_RING_SINGLE
#define KVQ_RING_SINGLE 2  // register stages of the single-tile pipelines of the narrow widths
#endif
#ifndef KVQ_SKIP_PAD
#define KVQ_SKIP_PAD 0
#endif
#ifndef KVQ_TAIL_SINGLES
#define KVQ_TAIL_SINGLES 16  // tiles at the end of a workgroup's range that are claimed one at a time
#endif
#ifndef KVQ_RING_2BIT
#define KVQ_RING_2BIT 2   // register stages of the 2-bit pipeline (one less is in flight)
#endif
#ifndef KVQ_RING_4BIT
#define KVQ_RING_4BIT 2
#endif
#define KVQ_WAVE_LDS_CONST (2 * KVQ_META_TILE_BYTES)  // 16 bytes of fp16 ones, then 16 bytes of zeros
#define KVQ_WAVE_LDS_BYTES (2 * KVQ_META_TILE_BYTES + 32)

// K half: scores^T (scaled to log2 units) of the 32 tokens of one tile for the 16 head columns.
// meta_lds: this tile's 1 KiB metadata, already redistributed through LDS.
template <int B>
__device__ inline void scores_tile(const QOps& Q, const uint32_t (&kw)[2 * code_bits<B>()], const uint8_t* meta_lds,
                                   float scale_log2, int lane, float (&s)[2][4]) {
    const int j = lane >> 4, n = lane & 15;
    const float4v zero4 = {0.f, 0.f, 0.f, 0.f};
    if constexpr (B == 16) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            float4v acc = zero4;
#pragma unroll
            for (int grp = 0; grp < 4; ++grp) {
                int p = sub * 4 + grp;
                half8 a = as_half8(kw[4 * p], kw[4 * p + 1], kw[4 * p + 2], kw[4 * p + 3]);
                half8 b = as_half8(Q.q[grp][0], Q.q[grp][1], Q.q[grp][2], Q.q[grp][3]);
                acc = mfma(a, b, acc);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) s[sub][i] = acc[i] * scale_log2;
        }
    } else {
        // scales of the 8 tokens whose scores this lane quarter receives: tokens 8j .. 8j+7, 4 groups each
        uint32_t ks[16];
        const u32x4* ksp = reinterpret_cast<const u32x4*>(meta_lds + j * 64);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            u32x4 v = ksp[c];
            ks[4 * c] = v.x; ks[4 * c + 1] = v.y; ks[4 * c + 2] = v.z; ks[4 * c + 3] = v.w;
        }
        const u32x2 qs2 = {Q.qsum[0], Q.qsum[1]};
        const half4 qs = __builtin_bit_cast(half4, qs2);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            // zero points of the token this lane supplies as an A row: token 8*(n/4) + 4*sub + n%4
            int t = 8 * (n >> 2) + 4 * sub + (n & 3);
            u32x2 kz = *reinterpret_cast<const u32x2*>(meta_lds + 256 + t * 8);
            float4v zacc = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(half4, kz), qs, zero4, 0, 0, 0);
            float4v acc = zero4;
#pragma unroll
            for (int grp = 0; grp < 4; ++grp) {
                half8 b = as_half8(Q.q[grp][0], Q.q[grp][1], Q.q[grp][2], Q.q[grp][3]);
                float4v part;
                if constexpr (B == KVQ_I16)  // (c_hi + c_lo / 256) . q: both planes are exact fp16 operands
                    part = mfma(dq_piece_frac(kw + 16, sub * 4 + grp), b, mfma(dq_piece<8>(kw, sub * 4 + grp), b, zero4));
                else
                    part = mfma(dq_piece_denorm<B>(kw, sub * 4 + grp), b, zero4);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int tk = 4 * sub + i;  // token 8j + tk: dwords 2*tk, 2*tk+1 hold its four scales
                    float sc = mixf(ks[2 * tk + (grp >> 1)], grp & 1);
                    acc[i] = fmaf(sc, part[i], acc[i]);
                }
            }
            // 8, 4, 2 bits: the code operands were denormals, 2^24 restores the sum of S * (c . q); integer 16-bit
            // tier: the operands were codes / 256
            const float restore = B == KVQ_I16 ? 256.0f : 16777216.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i) s[sub][i] = fmaf(acc[i], scale_log2 * restore, zacc[i]);
        }
    }
}

// Exponent of the accumulators while tiles of width B are added with denormal code operands: the codes enter
// the matrix cores as c * 2^(pos - 24) and the probabilities are scaled up by 2^(posmax - pos), so every product
// carries 2^(posmax - 24).  posmax = 6 / 4 / 0 for 2 / 4 / 8 bits; raw fp16 tiles and the overflow-proof path
// add true values.
template <int B>
__device__ inline int v_exponent(int safe_v) {
    if (B == 16 || B == KVQ_I16 || safe_v) return 0;
    return B == 2 ? 6 - 24 : B == 4 ? 4 - 24 : -24;
}
__device__ inline void set_accumulator_exponent(WaveState& st, int e) {
    if (st.oexp == e) return;
    const float f = __builtin_ldexpf(1.0f, e - st.oexp);  // exact power of two
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) st.o[nt] *= f;
    st.oexp = e;
}

// V half: out^T += V^T p^T with the probabilities `pop` (MFMA B operand) of the same tile.
// Fast path: V codes as fp16 denormals (one VALU op per two codes); the probabilities absorb the per-register
// position factor (exact powers of two, p <= 1) before they are multiplied by the V scales.  p * 64 * S_v must
// stay below the fp16 maximum: caches whose quantizer ever produced a V scale >= 256 take the other path, which
// builds exact fp16 integers from the codes instead (two ops per two codes) and adds true values.
template <int B, bool SAFE>
__device__ inline void accumulate_tile(WaveState& st, const uint32_t (&vw)[2 * code_bits<B>()], const uint8_t* meta_lds,
                                       const uint8_t* const_lds, const uint32_t (&pop)[4], int lane) {
    const int j = lane >> 4, n = lane & 15;
    const half8 pb = as_half8(pop[0], pop[1], pop[2], pop[3]);
    if constexpr (B == 16) {
        const uint32_t ones = (n == 4) ? 0x3c003c00u : 0u;  // row 4 of the extra MFMA sums p (denominator)
        st.zl = mfma(as_half8(ones, ones, ones, ones), pb, st.zl);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
            half8 a = as_half8(vw[4 * nt], vw[4 * nt + 1], vw[4 * nt + 2], vw[4 * nt + 3]);
            st.o[nt] = mfma(a, pb, st.o[nt]);
        }
    } else {
        // rows 0..3 of the extra MFMA: zero points of V group n over the 8 tokens of this quarter; row 4: ones;
        // other rows: zeros (both constants sit behind the wavefront's metadata area)
        const uint8_t* zsrc = (n < 4) ? meta_lds + 768 + n * 64 + j * 16 : const_lds + (n == 4 ? 0 : 16);
        u32x4 zv = *reinterpret_cast<const u32x4*>(zsrc);
        st.zl = mfma(as_half8(zv.x, zv.y, zv.z, zv.w), pb, st.zl);
        if constexpr (B == KVQ_I16) {
            // true values: (c_hi + c_lo / 256) * (p * 256 S_v); 256 S_v is exact and at most 512
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x4 sv = *reinterpret_cast<const u32x4*>(meta_lds + 512 + g * 64 + j * 16);
                const uint32_t k256 = 0x5c005c00u;  // two fp16 256.0
                half8 pg = as_half8(pk_mul(pop[0], pk_mul(sv.x, k256)), pk_mul(pop[1], pk_mul(sv.y, k256)),
                                    pk_mul(pop[2], pk_mul(sv.z, k256)), pk_mul(pop[3], pk_mul(sv.w, k256)));
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    int nt = 2 * g + h;
                    st.o[nt] = mfma(dq_piece<8>(vw, nt), pg, st.o[nt]);
                    st.o[nt] = mfma(dq_piece_frac(vw + 16, nt), pg, st.o[nt]);
                }
            }
        } else if constexpr (SAFE) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x4 sv = *reinterpret_cast<const u32x4*>(meta_lds + 512 + g * 64 + j * 16);
                half8 pg = as_half8(pk_mul(pop[0], sv.x), pk_mul(pop[1], sv.y), pk_mul(pop[2], sv.z),
                                    pk_mul(pop[3], sv.w));
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    int nt = 2 * g + h;
                    st.o[nt] = mfma(dq_piece<B>(vw, nt), pg, st.o[nt]);
                }
            }
        } else {
            uint32_t pf[4];  // probabilities times 2^(posmax - pos) of the operand register they meet
            if constexpr (B == 2) {
                pf[0] = pk_fma(pop[0], 64.f, 0.f); pf[1] = pk_fma(pop[1], 16.f, 0.f);
                pf[2] = pk_fma(pop[2], 4.f, 0.f); pf[3] = pop[3];
            } else if constexpr (B == 4) {
                pf[0] = pk_fma(pop[0], 16.f, 0.f); pf[1] = pop[1];
                pf[2] = pk_fma(pop[2], 16.f, 0.f); pf[3] = pop[3];
            } else {
                pf[0] = pop[0]; pf[1] = pop[1]; pf[2] = pop[2]; pf[3] = pop[3];
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x4 sv = *reinterpret_cast<const u32x4*>(meta_lds + 512 + g * 64 + j * 16);
                half8 pg = as_half8(pk_mul(pf[0], sv.x), pk_mul(pf[1], sv.y), pk_mul(pf[2], sv.z),
                                    pk_mul(pf[3], sv.w));
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    int nt = 2 * g + h;
                    st.o[nt] = mfma(dq_piece_denorm<B>(vw, nt), pg, st.o[nt]);
                }
            }
        }
    }
}

// Online softmax over the TPI*32 scores of a stage (log2 domain).  The running maximum st.m is equal in the
// four lane quarters of a head column; the cross-quarter reduction and the rescaling of the accumulators run
// only when some lane sees a score above it, which becomes rare after the first tiles.
template <int B, int TPI>
__device__ inline void softmax_stage(WaveState& st, float (&s)[TPI][2][4], const int (&tok0)[TPI], int n_tokens,
                                     int lane, uint32_t (&pop)[TPI][4]) {
    const int j = lane >> 4;
    bool ragged = false;
#pragma unroll
    for (int k = 0; k < TPI; ++k) ragged |= (tok0[k] + KVQ_TILE_TOKENS > n_tokens);
    if (ragged) {  // last tile of the cache, or a slot that only pads the stage
        asm volatile("" ::: "memory");  // keep this a branch: the selects must not run for every tile
#pragma unroll
        for (int k = 0; k < TPI; ++k)
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (tok0[k] + 8 * j + 4 * sub + i >= n_tokens) s[k][sub][i] = -INFINITY;
    }
    float lmax = -INFINITY;
#pragma unroll
    for (int k = 0; k < TPI; ++k)
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 4; ++i) lmax = fmaxf(lmax, s[k][sub][i]);
    if (__any(lmax > st.m)) {
        float tmax = fmaxf(lmax, __shfl_xor(lmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        // the exact maximum is the reference point: the dominant token then has p = 1 and p * S_v is exact
        float m_new = fmaxf(st.m, tmax);
        float alpha = (st.m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m - m_new);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) st.o[nt] *= alpha;
        st.zl *= alpha;
        st.m = m_new;
    }
#pragma unroll
    for (int k = 0; k < TPI; ++k) {
        float p[2][4];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 4; ++i) p[sub][i] = __builtin_amdgcn_exp2f(s[k][sub][i] - st.m);
        if constexpr (B == 16) {  // natural order: slots 0..3 = sub 0, slots 4..7 = sub 1
            pop[k][0] = pack_rn(p[0][0], p[0][1]);
            pop[k][1] = pack_rn(p[0][2], p[0][3]);
            pop[k][2] = pack_rn(p[1][0], p[1][1]);
            pop[k][3] = pack_rn(p[1][2], p[1][3]);
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                pop[k][v] = pack_rn(p[0][v], p[1][v]);
        }
    }
}

__device__ inline void wave_lds_sync() {  // orders LDS traffic between the lanes of one wavefront
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// All TPI tiles of one stage: K products, one joint softmax, V products.
template <int B, int TPI, bool SAFE>
__device__ inline void compute_stage(WaveState& st, const QOps& Q, const Stage<B, TPI>& sg, uint8_t* meta_lds,
                                     int n_tokens, float scale_log2, int lane) {
#ifdef KVQ_NO_ARITHMETIC
#pragma unroll
    for (int k = 0; k < TPI; ++k) {
        keep_loaded(sg.kw[k]);
        keep_loaded(sg.vw[k]);
        keep_loaded(sg.meta[k]);
    }
    return;
#endif
    if constexpr (B < 16) {
#pragma unroll
        for (int k = 0; k < TPI; ++k)
            *reinterpret_cast<u32x4*>(meta_lds + k * KVQ_META_TILE_BYTES + lane * 16) = sg.meta[k];
        wave_lds_sync();
    }
    float s[TPI][2][4];
#pragma unroll
    for (int k = 0; k < TPI; ++k) {
        // a slot that only pads the stage (wavefront-uniform) costs no arithmetic: its scores are masked anyway
        if (k == 0 || !KVQ_SKIP_PAD || sg.tok0[k] != KVQ_PAD_TOK0) {
            scores_tile<B>(Q, sg.kw[k], meta_lds + k * KVQ_META_TILE_BYTES, scale_log2, lane, s[k]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) s[k][e >> 2][e & 3] = -INFINITY;
        }
    }
    uint32_t pop[TPI][4];
    softmax_stage<B, TPI>(st, s, sg.tok0, n_tokens, lane, pop);
#pragma unroll
    for (int k = 0; k < TPI; ++k)
        if (k == 0 || !KVQ_SKIP_PAD || sg.tok0[k] != KVQ_PAD_TOK0)
            accumulate_tile<B, SAFE>(st, sg.vw[k], meta_lds + k * KVQ_META_TILE_BYTES, meta_lds + KVQ_WAVE_LDS_CONST, pop[k], lane);
    if constexpr (B < 16) wave_lds_sync();
}

// A claimed chunk, resolved to addresses; every member is wavefront-uniform (scalar registers).
struct Claim {
    int tile;             // first tile
    int nt;               // tiles (1 or 2), adjacent in one page
    uint32_t bits;        // width of the page; 0: nothing left in this window
    const uint8_t* code;  // K string of the first tile; its V string follows, then the next tile's pair
    const uint8_t* meta;  // metadata of the first tile; the next tile's follows
};

// What a wavefront needs to find and claim work inside its workgroup's tile range.  The range is cut into
// chunks of two consecutive tiles (one when pages hold an odd number of tiles, and at the end of the range); the 8 wavefronts of the
// workgroup claim chunks from a counter in LDS, so wavefronts that get more issue slots simply do more chunks.
//   next      - resolved claim, the chunk whose loads are issued next
//   claim_v   - result of the claim after it (LDS atomic in flight while a stage is computed)
//   desc_v    - descriptor read of a claimed chunk, chunk index in desc_chunk
struct RunCtx {
    const uint8_t* arena;
    const u32x4* desc_lds;   // descriptors of pages page0 .. of the current descriptor window
    unsigned* claim_ctr;     // LDS: next unclaimed chunk
    int page0;
    int tpp;
    uint32_t tpp_magic;      // ceil(2^32 / tpp): tile / tpp = mulhi(tile, magic) for tile < 2^22, tpp <= 2^10
    int unit;
    int n_tokens;
    int lo, hi;              // tile range of the current descriptor window
    int n_pairs;             // chunks 0 .. n_pairs - 1 hold two tiles, the chunks after them one
    int n_chunks;
    int next_static;         // >= 0: deterministic mode, this wavefront takes chunks next_static, + static_stride, ...
    int static_stride;
    float scale_log2;
    uint32_t lane_off;       // 16 * lane
    Claim next;
    int desc_chunk;
    u32x4 desc_v;
    int claim_v;
};

__device__ inline void start_claim(RunCtx& c) {
    if (c.next_static >= 0) {
        c.claim_v = c.next_static;
        c.next_static = __builtin_amdgcn_readfirstlane(c.next_static + c.static_stride);  // provably uniform
        return;
    }
    int v = 0;
    if ((threadIdx.x & 63) == 0) v = (int)__hip_atomic_fetch_add(c.claim_ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    c.claim_v = v;
}
__device__ inline int finish_claim(const RunCtx& c) { return __builtin_amdgcn_readfirstlane(c.claim_v); }

__device__ inline int page_of_tile(const RunCtx& c, int tile) {
    return c.tpp == 1 ? tile : (int)__umulhi((uint32_t)tile, c.tpp_magic);
}
__device__ inline void start_desc(RunCtx& c, int chunk) {
    chunk = __builtin_amdgcn_readfirstlane(chunk);
    c.desc_chunk = chunk;
    const int cc = max(0, min(chunk, c.n_chunks - 1));  // past the end: any valid slot, ignored later
    const int tile = c.lo + cc + min(cc, c.n_pairs);
    c.desc_v = c.desc_lds[page_of_tile(c, tile) - c.page0];
}
__device__ inline Claim finish_desc(const RunCtx& c) {
    Claim r;
    const int chunk = c.desc_chunk;
    r.tile = c.lo + chunk + min(chunk, c.n_pairs);
    r.nt = min(chunk < c.n_pairs ? 2 : 1, c.hi - r.tile);
    const uint32_t code_off = __builtin_amdgcn_readfirstlane(c.desc_v.x);
    const uint32_t meta_off = __builtin_amdgcn_readfirstlane(c.desc_v.y);
    const uint32_t bits = __builtin_amdgcn_readfirstlane(c.desc_v.z);
    r.bits = chunk < c.n_chunks ? bits : 0u;
    const int page = page_of_tile(c, r.tile), tip = r.tile - page * c.tpp;
    const uint64_t tslot = (uint64_t)c.unit * c.tpp + tip;
    r.code = c.arena + (uint64_t)code_off * 256u + tslot * (1024u * bits);
    r.meta = c.arena + (uint64_t)meta_off * 256u + tslot * KVQ_META_TILE_BYTES;
    return r;
}
// Claims the next chunk; between begin and end there should be a stage's worth of arithmetic, which hides the
// LDS atomic (the descriptor read that follows it is short).  A wavefront commits itself to one chunk beyond the
// ones in flight, not more: chunks claimed early are chunks nobody else can take when the range runs out.
__device__ inline void advance_begin(RunCtx& c) { start_claim(c); }
__device__ inline void advance_end(RunCtx& c) {
    start_desc(c, finish_claim(c));
    c.next = finish_desc(c);
}

// Issue every global load of one stage (nothing waits here): the tiles of one chunk; slots the chunk does not
// fill re-read its first tile and are masked out by their tok0.
template <int B, int TPI>
__device__ inline void issue_stage(Stage<B, TPI>& sg, const RunCtx& c, const Claim& cl) {
#pragma unroll
    for (int k = 0; k < TPI; ++k) {
        const bool real = k < cl.nt;
        const uint8_t* code = cl.code + (real ? k : 0) * (1024u * B);
        const uint8_t* meta = cl.meta + (real ? k : 0) * KVQ_META_TILE_BYTES;
        load_string<2 * B>(code, c.lane_off, sg.kw[k]);
        load_string<2 * B>(code + 512u * B, c.lane_off, sg.vw[k]);
        if constexpr (B < 16) sg.meta[k] = load_stream16(meta + c.lane_off);
        sg.tok0[k] = real ? (cl.tile + k) * KVQ_TILE_TOKENS : KVQ_PAD_TOK0;
    }
}

// Process the resolved claim c.next (width B) and keep claiming and processing chunks while they have the same
// width, software-pipelined: the loads of the following chunks are in flight while the current one is computed.
// Returns with c.next = the first claimed chunk that was not processed (another width, or bits 0 = nothing left).
//
// The steady-state path contains no load that is issued conditionally: the wait counts in front of a stage's
// first use are then exactly "everything issued after it may still be in flight".  (A load under a condition
// would make the compiler wait for the stricter of the two paths, i.e. drain the prefetch every time.)  The
// end of a run therefore has code of its own.
template <int B, int TPI, int N, bool SAFE>
__device__ inline void run_chunks(WaveState& st, QOps& Q, const _Float16* q_lds, RunCtx& c, uint8_t* meta_lds,
                                  int lane) {
    // Values a path derives from the lane index (LDS addresses, operand selectors) would otherwise be hoisted out of the
    // caller's loop over runs, for all widths at once, and held in registers the kernel does not have.
    asm volatile("" : "+v"(lane));
    set_accumulator_exponent(st, v_exponent<B>(SAFE));
    if constexpr (B >= 8) {
        // wide tiles (8 and 16 KiB, the latter raw fp16 or integer byte planes): one register stage, tile by tile, K and V staggered (V loads fly during
        // the K product, the next tile's K and metadata loads during the V product)
        constexpr int W = code_bits<B>();
        uint32_t kw[2 * W], vw[2 * W];
        u32x4 mreg = {0u, 0u, 0u, 0u};
        Claim cur = c.next;
        int k = 0;
        load_string<2 * W>(cur.code, c.lane_off, kw);
        if constexpr (has_meta<B>()) mreg = load_stream16(cur.meta + c.lane_off);
        load_string<2 * W>(cur.code + 512u * W, c.lane_off, vw);
        // the query operands are arranged afresh at the start of every run, also when the last run had the same
        // arrangement: carried from run to run they would occupy 16 registers across the dispatch in between
        load_q_ops(Q, q_lds, lane, q_class<B>(), c.scale_log2);
        for (;;) {
            float s[1][2][4];
            uint32_t pop[1][4];
            const int tok0[1] = {(cur.tile + k) * KVQ_TILE_TOKENS};
#ifdef KVQ_NO_ARITHMETIC
            keep_loaded(kw);
            keep_loaded(mreg);
            s[0][0][0] = 0.f;
#else
            if constexpr (has_meta<B>()) {
                *reinterpret_cast<u32x4*>(meta_lds + lane * 16) = mreg;
                wave_lds_sync();
            }
            scores_tile<B>(Q, kw, meta_lds, c.scale_log2, lane, s[0]);
#endif
            const uint8_t *code, *meta;
            bool more;
            if (k + 1 < cur.nt) {  // next tile of the same chunk
                ++k;
                code = cur.code + k * (1024u * W);
                meta = cur.meta + k * KVQ_META_TILE_BYTES;
                more = true;
            } else {  // a wide tile takes long enough to claim its successor only now
                advance_begin(c);
                advance_end(c);
                more = c.next.bits == (uint32_t)W;
                if (more) { cur = c.next; k = 0; code = cur.code; meta = cur.meta; }
            }
#ifdef KVQ_NO_ARITHMETIC
            if (!more) { keep_loaded(vw); return; }
            load_string<2 * W>(code, c.lane_off, kw);
            if constexpr (has_meta<B>()) mreg = load_stream16(meta + c.lane_off);
            keep_loaded(vw);
            load_string<2 * W>(code + 512u * W, c.lane_off, vw);
#else
            if (!more) {  // last tile of the run
                softmax_stage<B, 1>(st, s, tok0, c.n_tokens, lane, pop);
                accumulate_tile<B, SAFE>(st, vw, meta_lds, meta_lds + KVQ_WAVE_LDS_CONST, pop[0], lane);
                if constexpr (has_meta<B>()) wave_lds_sync();
                return;
            }
            load_string<2 * W>(code, c.lane_off, kw);
            if constexpr (has_meta<B>()) mreg = load_stream16(meta + c.lane_off);
            softmax_stage<B, 1>(st, s, tok0, c.n_tokens, lane, pop);
            accumulate_tile<B, SAFE>(st, vw, meta_lds, meta_lds + KVQ_WAVE_LDS_CONST, pop[0], lane);
            if constexpr (has_meta<B>()) wave_lds_sync();
            load_string<2 * W>(code + 512u * W, c.lane_off, vw);
#endif
        }
    } else {
        // narrow tiles: a ring of N register stages of TPI tiles each, N - 1 of them in flight
        Stage<B, TPI> sg[N];
        issue_stage<B, TPI>(sg[0], c, c.next);
        advance_begin(c);
        load_q_ops(Q, q_lds, lane, B, c.scale_log2);  // afresh in every run, see above
        advance_end(c);
        int n_live = 1, head = 0;
        // (the run is left by jumps, not by flags: a flag-guarded chain of steps would give the control-flow
        //  graph paths from a step straight back to itself, and the wait counts are derived from that graph)
#pragma unroll
        for (int i = 1; i + 1 < N; ++i) {  // fill the ring
            if (c.next.bits != B || c.next.nt != TPI) goto drain;
            issue_stage<B, TPI>(sg[i], c, c.next);
            n_live = i + 1;
            advance_begin(c);
            advance_end(c);
        }
        for (;;) {
#pragma unroll
            for (int k = 0; k < N; ++k) {
                if (c.next.bits != B || c.next.nt != TPI) { head = k; goto drain; }
                issue_stage<B, TPI>(sg[(k + N - 1) % N], c, c.next);
                advance_begin(c);
                compute_stage<B, TPI, SAFE>(st, Q, sg[k], meta_lds, c.n_tokens, c.scale_log2, lane);
                advance_end(c);
            }
        }
    drain:
        // end of the run: the stages still in flight are sg[head], sg[head + 1], ... (n_live of them); bring
        // them to the front and compute them in order
#pragma unroll
        for (int h = 1; h < N; ++h) {
            if (head == h) {
                Stage<B, TPI> tmp[N - 1];
#pragma unroll
                for (int i = 0; i + 1 < N; ++i) tmp[i] = sg[(h + i) % N];
#pragma unroll
                for (int i = 0; i + 1 < N; ++i) sg[i] = tmp[i];
            }
        }
#pragma unroll
        for (int i = 0; i + 1 < N; ++i)
            if (i < n_live) compute_stage<B, TPI, SAFE>(st, Q, sg[i], meta_lds, c.n_tokens, c.scale_log2, lane);
    }
}

// Device-scope (all XCDs) relaxed accesses: they go through to memory instead of living in one XCD's L2, so
// split partials can be handed to the merging workgroup without whole-cache write-backs or invalidations.
__device__ inline void store_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float load_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline float2v load_pair(const float* p, bool agent) {  // 8 bytes at p (8-byte aligned)
    if (agent) {
        const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
        return float2v{__uint_as_float((uint32_t)u), __uint_as_float((uint32_t)(u >> 32))};
    }
    return *reinterpret_cast<const float2v*>(p);
}

#define KVQ_DESC_CACHE 256  // page descriptors staged in LDS per chunk of the split's range
#define KVQ_OPAD 132  // padded row of the LDS reduction slab (floats)


// LDS of one workgroup.
struct AttnShared {
    __attribute__((aligned(16))) _Float16 q[16 * KVQ_D];
    float red_o[KVQ_ATTN_WAVES][16 * KVQ_OPAD];  // partial outputs of the eight wavefronts
    float red_m[KVQ_ATTN_WAVES][16];
    float red_l[KVQ_ATTN_WAVES][16];
    int is_last;
    unsigned claim_ctr;
    u32x4 desc[KVQ_DESC_CACHE];
    __attribute__((aligned(16))) uint8_t meta[KVQ_ATTN_WAVES * KVQ_WAVE_LDS_BYTES];
};


// Phase stamps: hooks of the measurement build (python -m paper_2505_18610_amd.build --phase-stamps), which records
// when a workgroup passes the points marked below; the library proper compiles them to nothing.
#ifdef KVQ_PHASE_STAMPS
#include "kvq_phase_stamps.h"
#else
#define KVQ_STAMP(k) do { } while (0)
#define KVQ_STAMP_ID() do { } while (0)
#endif
#define KVQ_MERGE_LDS_FLOATS (KVQ_MAX_SPLITS * 16 * 3 + 16 + (KVQ_ATTN_THREADS / 32) * 32 * 4)

// Merge of the split partials of one unit by a workgroup of KVQ_ATTN_THREADS threads.  Threads work in 16 slots
// of 32 (one head, 4 channels per thread); with fewer than 16 heads the splits of a head are dealt to several
// slot groups.  Every global load is issued before the first one is waited for, so the merge costs one memory
// round trip, three barriers and the store.  Per split the partials hold (max, sum) pairs per head and the
// un-normalised output rows.  lds: KVQ_MERGE_LDS_FLOATS floats.  Call it with the whole workgroup.
template <bool AGENT>
__device__ inline void merge_splits(const KvqAttnParams& P, int unit, int tid, float* lds) {
    const int g = P.gqa, ns = P.n_splits;
    const int b = unit / P.n_kv_heads, hk = unit - b * P.n_kv_heads;
    const float* po = P.part_o + (size_t)unit * ns * 16 * KVQ_D;
    const float* pml = P.part_ml + (size_t)unit * ns * 32;
    float* ml_lds = lds;                               // [split][16] (m, l)
    float* f_lds = lds + KVQ_MAX_SPLITS * 32;          // [split][16] weight of the split in the merged sum
    float* invl_lds = f_lds + KVQ_MAX_SPLITS * 16;     // [16]
    float* rec_lds = invl_lds + 16;                    // [slot][32][4]
    const int slots = KVQ_ATTN_THREADS >> 5;           // 16 >= g
    const int G = max(1, min(slots / g, ns));          // slot groups sharing the splits of one head
    const int slot = tid >> 5, d4 = tid & 31;
    const int sgi = slot / g, head = slot - sgi * g;
    const bool active = sgi < G;
    // ---- every load of the first round: (m, l) pairs, then this thread's share of the partial outputs
    float2v mlr[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = tid + k * KVQ_ATTN_THREADS;      // pair index: split * g + head
        mlr[k] = float2v{-INFINITY, 0.f};
        if (e < ns * g) { const int sp = e / g, h = e - sp * g; mlr[k] = load_pair(pml + sp * 32 + 2 * h, AGENT); }
    }
    // The unit's partial outputs as a buffer of ns splits: 16-byte loads (half the load instructions of 8-byte pairs,
    // and their issue is what the merge of many splits waits for), no branch -- a split index beyond ns is out of
    // range and reads zeros, and so does an idle thread, whose offset is put out of range.  AGENT: device-scope
    // loads (sc1), as the 8-byte atomic loads of the (m, l) pairs are.
    const __amdgpu_buffer_rsrc_t slab =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(po), 0, ns * 16 * KVQ_D * (int)sizeof(float), 0x00020000);
    // A load instruction costs its issue slots whether or not it is in range, so with few splits per slot group
    // only the first four are issued.
    const bool many = ns > 4 * G;
    float4v v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int sp = sgi + k * G;
        const uint32_t off = active ? (uint32_t)((sp * 16 + head) * KVQ_D + 4 * d4) * 4u : 0x80000000u;
        v[k] = float4v{0.f, 0.f, 0.f, 0.f};
        if (k < 4 || many)
            v[k] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(slab, (int)off, 0, AGENT ? 16 : 0));
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int e = tid + k * KVQ_ATTN_THREADS;
        if (e < ns * g) { const int sp = e / g, h = e - sp * g; ml_lds[(sp * 16 + h) * 2] = mlr[k][0]; ml_lds[(sp * 16 + h) * 2 + 1] = mlr[k][1]; }
    }
    __syncthreads();
    // ---- per head (slot = head, 32 lanes over the splits): common maximum, weights, denominator
    if (slot < g) {
        float m = -INFINITY;
        for (int sp = d4; sp < ns; sp += 32) m = fmaxf(m, ml_lds[(sp * 16 + slot) * 2]);
#pragma unroll
        for (int o = 1; o < 32; o <<= 1) m = fmaxf(m, __shfl_xor(m, o));
        float l = 0.f;
        for (int sp = d4; sp < ns; sp += 32) {
            const float ms = ml_lds[(sp * 16 + slot) * 2];
            const float f = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - m);
            f_lds[sp * 16 + slot] = f;
            l += ml_lds[(sp * 16 + slot) * 2 + 1] * f;
        }
        // fixed-order tree: the same for both merge variants and from launch to launch
#pragma unroll
        for (int o = 1; o < 32; o <<= 1) l += __shfl_xor(l, o);
        if (d4 == 0) invl_lds[slot] = 1.0f / l;
    }
    __syncthreads();
    // ---- weighted sum of this thread's splits (further rounds only beyond 16 * G splits)
    float4v acc = {0.f, 0.f, 0.f, 0.f};
    if (active) {
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const int sp = sgi + k * G;
            if (sp < ns) {
                const float f = f_lds[sp * 16 + head];
                acc += v[k] * f;
            }
        }
        for (int sp = sgi + 16 * G; sp < ns; sp += G) {
            const float* src = po + ((size_t)sp * 16 + head) * KVQ_D + 4 * d4;
            const float2v a = load_pair(src, AGENT), c2 = load_pair(src + 2, AGENT);
            acc += float4v{a[0], a[1], c2[0], c2[1]} * f_lds[sp * 16 + head];
        }
    }
    if (G > 1) {  // combine the slot groups in a fixed order
        if (active && sgi > 0) *reinterpret_cast<float4v*>(rec_lds + (size_t)(slot * 32 + d4) * 4) = acc;
        __syncthreads();
        if (active && sgi == 0)
            for (int k = 1; k < G; ++k) acc += *reinterpret_cast<const float4v*>(rec_lds + (size_t)((k * g + head) * 32 + d4) * 4);
    }
    if (active && sgi == 0) {
        const float inv = invl_lds[head];
        const size_t oi = ((size_t)b * P.n_q_heads + hk * g + head) * KVQ_D + 4 * d4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float r = acc[i] * inv;
            if (P.out_fp32) static_cast<float*>(P.out)[oi + i] = r;
            else static_cast<_Float16*>(P.out)[oi + i] = (_Float16)r;
        }
    }
}

static_assert(KVQ_ATTN_WAVES * 16 * KVQ_OPAD >= KVQ_MERGE_LDS_FLOATS, "the wavefront slab doubles as scratch of the split merge");

// End of a workgroup's range: merge of its eight wavefront partials through LDS, then either the output (one split),
// the partial for the separate merge kernel, or the fused merge of the unit's split partials.
__device__ __forceinline__ void finish_workgroup(const KvqAttnParams& P, AttnShared& sh, WaveState& st, int split, int unit) {
    // the thread index is taken afresh, opaque to the compiler: nothing derived from it stays in a register across
    // the streaming loop for the sake of this epilogue
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane >> 4, n = lane & 15;
    const int g = P.gqa, ns = P.n_splits;
    const int b = unit / P.n_kv_heads, hk = unit - b * P.n_kv_heads;
    float (*const red_o)[16 * KVQ_OPAD] = sh.red_o;

    set_accumulator_exponent(st, 0);
    // ---- wavefront epilogue: add the zero-point term, fetch the denominator, leave the partial in LDS
    const float l_w = __shfl(st.zl[0], 16 + n);
    {
        const float z0 = __shfl(st.zl[0], n), z1 = __shfl(st.zl[1], n), z2 = __shfl(st.zl[2], n), z3 = __shfl(st.zl[3], n);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            st.o[0][i] += z0; st.o[1][i] += z0;
            st.o[2][i] += z1; st.o[3][i] += z1;
            st.o[4][i] += z2; st.o[5][i] += z2;
            st.o[6][i] += z3; st.o[7][i] += z3;
        }
    }
    if (j == 0) { sh.red_m[wave][n] = st.m; sh.red_l[wave][n] = l_w; }
    if (n < g) {
#pragma unroll
        for (int nt = 0; nt < 8; ++nt)
            *reinterpret_cast<float4v*>(&red_o[wave][n * KVQ_OPAD + 16 * nt + 4 * j]) = st.o[nt];
    }
    __syncthreads();  // the eight wavefronts of the workgroup have joined
    KVQ_STAMP(6);

    const bool direct = (ns == 1);
    const bool fused = !direct && P.fused_merge;

    // ---- merge the eight wavefront partials: thread t takes the pairs of elements t, t + 512 of the
    // [head][64 channel pairs] block; common maximum, weights and a fixed-order sum, one pass over LDS
    const int n_pairs = g * (KVQ_D / 2);
    float2v acc[2], ml[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int pr = tid + r * KVQ_ATTN_THREADS;
        acc[r] = float2v{0.f, 0.f};
        ml[r] = float2v{-INFINITY, 0.f};
        if (pr < n_pairs) {
            const int head = pr >> 6, d = 2 * (pr & 63);
            float M = -INFINITY;
            for (int w = 0; w < KVQ_ATTN_WAVES; ++w) M = fmaxf(M, sh.red_m[w][head]);
            float2v a = {0.f, 0.f};
            float L = 0.f;
            for (int w = 0; w < KVQ_ATTN_WAVES; ++w) {
                const float mw = sh.red_m[w][head];
                const float f = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - M);
                const float2v o2 = *reinterpret_cast<const float2v*>(&red_o[w][head * KVQ_OPAD + d]);
                a[0] = fmaf(o2[0], f, a[0]);
                a[1] = fmaf(o2[1], f, a[1]);
                L = fmaf(sh.red_l[w][head], f, L);
            }
            acc[r] = a;
            ml[r] = float2v{M, L};
        }
    }
    KVQ_STAMP(3);
    float* po = P.part_o + ((size_t)unit * ns + split) * 16 * KVQ_D;
    float* pml = P.part_ml + ((size_t)unit * ns + split) * 32;
    if (!fused) {
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int pr = tid + r * KVQ_ATTN_THREADS;
            if (pr >= n_pairs) continue;
            const int head = pr >> 6, d = 2 * (pr & 63);
            if (direct) {
                const float inv = 1.0f / ml[r][1];
                const float r0 = acc[r][0] * inv, r1 = acc[r][1] * inv;
                const size_t oi = ((size_t)b * P.n_q_heads + hk * g + head) * KVQ_D + d;
                if (P.out_fp32) *reinterpret_cast<float2v*>(static_cast<float*>(P.out) + oi) = float2v{r0, r1};
                else *reinterpret_cast<half2v*>(static_cast<_Float16*>(P.out) + oi) = half2v{(_Float16)r0, (_Float16)r1};
            } else {  // the merge kernel that follows reads these
                *reinterpret_cast<float2v*>(po + 2 * pr) = acc[r];
                if (d == 0) *reinterpret_cast<float2v*>(pml + 2 * head) = ml[r];
            }
        }
        return;
    }

    // ---- fused merge of the split partials: every workgroup publishes its partial with device-scope stores, waits
    // until they have been performed, and one thread bumps the unit's arrival counter (device-scope atomic); the
    // workgroup that draws the last ticket reads all partials back with device-scope loads and writes the output.
    // The counter is left at zero for the next launch.
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int pr = tid + r * KVQ_ATTN_THREADS;
        if (pr >= n_pairs) continue;
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(po + 2 * pr), __builtin_bit_cast(unsigned long long, acc[r]),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((pr & 63) == 0)
            __hip_atomic_store(reinterpret_cast<unsigned long long*>(pml + 2 * (pr >> 6)),
                               __builtin_bit_cast(unsigned long long, ml[r]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    int& is_last = sh.is_last;
    if (tid == 0) {
        const uint32_t old = __hip_atomic_fetch_add(&P.counters[unit], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        is_last = (old == (uint32_t)ns - 1u) ? 1 : 0;
    }
    __syncthreads();
    KVQ_STAMP(4);
    if (!is_last) return;
    merge_splits<true>(P, unit, tid, &sh.red_o[0][0]);
    if (tid == 0) __hip_atomic_store(&P.counters[unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    KVQ_STAMP(5);
}

// The whole kernel for one of the two V paths (SAFE: overflow-proof, see accumulate_tile) and one of the two kinds
// of 16-bit tier (I16: integer codes in byte planes; else raw fp16, which is also the kind a one-token append can
// be fused into).  A cache has one kind only, so each kernel carries the code of one.
// BATCH: the workgroup's (split, unit) come from the caller (ragged batch); else they are the workgroup's grid indices,
// read where they are needed (handing them in as values costs the single-cache kernels scalar registers they lack).
// APPEND: the kernel can carry out a one-token append into the raw fp16 tier (P.app_t_old >= 0) before it attends.
template <bool SAFE, bool I16, bool BATCH = false, bool APPEND = !I16>
__device__ __forceinline__ void attention_body(const KvqAttnParams& P, AttnShared& sh, const int split_in = 0,
                                               const int unit_in = 0) {
    const int split = BATCH ? split_in : (int)blockIdx.x, unit = BATCH ? unit_in : (int)blockIdx.y;
    _Float16* const q_lds = sh.q;
    unsigned& claim_ctr = sh.claim_ctr;
    u32x4* const desc_lds = sh.desc;
    uint8_t* const meta_lds = sh.meta;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = P.gqa;
    const int b = unit / P.n_kv_heads, hk = unit - b * P.n_kv_heads;

    KVQ_STAMP(0);
    KVQ_STAMP_ID();
    const int tpp = P.tiles_per_page;
    const int t_begin = P.split_begin[split], t_end = P.split_begin[split + 1];
    const int p_first = t_begin / tpp, p_last = (t_end + tpp - 1) / tpp;  // pages touched: [p_first, p_last)
    // stage q (heads beyond g are zero) and the first window of page descriptors with one round trip
    if (tid < 256) {
        const int head = tid >> 4, c16 = tid & 15;
        u32x4 qv = {0u, 0u, 0u, 0u};
        if (head < g) {
            qv = *reinterpret_cast<const u32x4*>(static_cast<const _Float16*>(P.q) +
                                                 ((size_t)b * P.n_q_heads + hk * g + head) * KVQ_D + c16 * 8);
            if (P.lambda) {  // Q Lambda of the channel-wise reparameterization (Sec. 3.3, Eq. 7): fp32 product, RNE to fp16
                const float* lam = P.lambda + hk * KVQ_D + c16 * 8;
                uint32_t* qw = reinterpret_cast<uint32_t*>(&qv);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const _Float16 lo = __builtin_bit_cast(_Float16, (uint16_t)(qw[e] & 0xffff));
                    const _Float16 hi = __builtin_bit_cast(_Float16, (uint16_t)(qw[e] >> 16));
                    float plo = (float)lo * lam[2 * e], phi = (float)hi * lam[2 * e + 1];
                    asm volatile("" : "+v"(plo), "+v"(phi));  // two roundings (fp32, then fp16), never a fused one
                    const _Float16 nlo = (_Float16)plo, nhi = (_Float16)phi;
                    qw[e] = (uint32_t)__builtin_bit_cast(uint16_t, nlo) | ((uint32_t)__builtin_bit_cast(uint16_t, nhi) << 16);
                }
            }
        }
        u32x4 dv = {0u, 0u, 0u, 0u};
        if (tid < min(KVQ_DESC_CACHE, p_last - p_first)) dv = reinterpret_cast<const u32x4*>(P.table)[p_first + tid];
        *reinterpret_cast<u32x4*>(&q_lds[head * KVQ_D + c16 * 8]) = qv;
        desc_lds[tid] = dv;
    }
    // A one-token append fused into this launch: the workgroup whose range ends with the new token's tile writes
    // the token.  Its wavefront 0 does that after the staging barrier, waits until the stores have reached L2 and
    // takes the chunk that holds the tile as its first one (nobody else can claim it); the other seven wavefronts
    // start on the rest of the range meanwhile.
    const int tile_new = (APPEND && P.app_t_old >= 0) ? P.app_t_old / KVQ_TILE_TOKENS : -1;
    const bool appends = APPEND && tile_new >= t_begin && tile_new < t_end;
    const bool one_window = p_last - p_first <= KVQ_DESC_CACHE;
    // the first chunk of every wavefront is fixed (see below); the counter starts behind them
    if (tid == 0) claim_ctr = (appends && one_window) ? KVQ_ATTN_WAVES - 1 : KVQ_ATTN_WAVES;
    __syncthreads();
    if (APPEND && appends && wave == 0) {
        const int tip = tile_new - (tile_new / tpp) * tpp;
        const uint64_t tslot = (uint64_t)unit * tpp + tip;
        uint8_t* code = const_cast<uint8_t*>(P.arena) + (uint64_t)P.app_desc.code_off256 * 256u + tslot * 2 * (512u * 16);
        const uint16_t* in_k = static_cast<const uint16_t*>(P.app_k) + (size_t)unit * KVQ_D;
        const uint16_t* in_v = static_cast<const uint16_t*>(P.app_v) + (size_t)unit * KVQ_D;
#ifdef KVQ_WITH_I16_APPEND
        if constexpr (I16) {  // integer tier: the token is quantized (Eq. 1-2, 2^16 - 1 levels); the reduction slab is free
            uint8_t* meta = const_cast<uint8_t*>(P.arena) + (uint64_t)P.app_desc.meta_off256 * 256u + tslot * KVQ_META_TILE_BYTES;
            auto& lds = *reinterpret_cast<uint8_t (*)[2][KVQ_LDS_CODES]>(&sh.red_o[0][0]);
            kvq_q::append_i16_string(lds, code, meta, in_k, 0, tile_new * KVQ_TILE_TOKENS, P.app_t_old, P.app_t_old + 1,
                                     P.app_gspan, P.app_rope, P.app_rinv, hk, lane);
            kvq_q::wave_sync_lds();
            kvq_q::append_i16_string(lds, code + 512u * 16, meta, in_v, 1, tile_new * KVQ_TILE_TOKENS, P.app_t_old,
                                     P.app_t_old + 1, P.app_gspan, nullptr, nullptr, 0, lane);
        } else
#endif
        {
            kvq_dev::append16_tile(code, in_k, 0, tile_new * KVQ_TILE_TOKENS, P.app_t_old, P.app_t_old + 1, lane, P.app_rope,
                                   P.app_rinv ? P.app_rinv + hk * KVQ_D : nullptr);
            kvq_dev::append16_tile(code + 512u * 16, in_v, 1, tile_new * KVQ_TILE_TOKENS, P.app_t_old, P.app_t_old + 1, lane,
                                   nullptr, nullptr);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    KVQ_STAMP(1);
    QOps Q;
    Q.cls = -1;
    Q.have_qsum = 0;
    Q.qsum[0] = Q.qsum[1] = 0u;

    WaveState st;
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) st.o[nt] = float4v{0.f, 0.f, 0.f, 0.f};
    st.zl = float4v{0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.oexp = 0;
    st.safe_v = SAFE ? 1 : 0;

    RunCtx ctx;
    ctx.arena = P.arena; ctx.desc_lds = desc_lds; ctx.claim_ctr = &claim_ctr; ctx.tpp = tpp; ctx.unit = unit;
    ctx.tpp_magic = P.tpp_magic;
    ctx.n_tokens = P.n_tokens; ctx.scale_log2 = P.scale_log2;
    ctx.lane_off = (uint32_t)lane * 16u;
    uint8_t* my_meta = meta_lds + wave * KVQ_WAVE_LDS_BYTES;
    if (lane < 8) reinterpret_cast<uint32_t*>(my_meta + KVQ_WAVE_LDS_CONST)[lane] = lane < 4 ? 0x3c003c00u : 0u;
    for (int pc = p_first; pc < p_last; pc += KVQ_DESC_CACHE) {
        const int pn = min(KVQ_DESC_CACHE, p_last - pc);
        const bool reserve = appends && pc + KVQ_DESC_CACHE >= p_last;  // the window that ends with the new tile
        if (pc != p_first) {  // further descriptor windows of a very long range
            __syncthreads();
            if (tid < pn) desc_lds[tid] = reinterpret_cast<const u32x4*>(P.table)[pc + tid];
            if (tid == 0) claim_ctr = reserve ? KVQ_ATTN_WAVES - 1 : KVQ_ATTN_WAVES;
            __syncthreads();
        }
        ctx.page0 = pc;
        ctx.lo = max(t_begin, pc * tpp);
        ctx.hi = min(t_end, (pc + pn) * tpp);
        // Chunks of two tiles (one when pages hold an odd number of tiles), except at the end of the range: its last
        // KVQ_TAIL_SINGLES tiles are claimed one by one, so that the wavefronts run out of work at nearly the same time.
        const int n_t = ctx.hi - ctx.lo;
        if (n_t <= 0) continue;
        const int singles = (tpp & 1) ? n_t : (pc + KVQ_DESC_CACHE >= p_last ? min(KVQ_TAIL_SINGLES, n_t) : 0);
        ctx.n_pairs = (n_t - singles) >> 1;
        const int n_all = n_t - ctx.n_pairs;
        // The first chunk of every wavefront is fixed, from then on chunks are claimed one at a time.  Normally it
        // is the wavefront's own index.  With a fused append the last chunk is kept out of the claimable range:
        // wavefront 0 starts with it, wavefronts 1..7 with chunks 0..6.
        int first;
        if (!reserve) {
            ctx.n_chunks = n_all;
            first = wave;
            ctx.static_stride = KVQ_ATTN_WAVES;
            ctx.next_static = P.deterministic ? wave + KVQ_ATTN_WAVES : -1;
            start_desc(ctx, first);
        } else {
            ctx.static_stride = KVQ_ATTN_WAVES - 1;
            if (wave == 0) {
                first = n_all - 1;
                ctx.next_static = P.deterministic ? 0x3fffff00 : -1;  // deterministic mode: nothing after it
                ctx.n_chunks = n_all;
                start_desc(ctx, first);
            } else {
                first = wave - 1;
                ctx.next_static = P.deterministic ? wave - 1 + (KVQ_ATTN_WAVES - 1) : -1;
                ctx.n_chunks = n_all - 1;
                start_desc(ctx, first);
            }
        }
        ctx.next = finish_desc(ctx);
        ctx.n_chunks = reserve ? n_all - 1 : n_all;
        while (ctx.next.bits != 0u) {
            switch (ctx.next.bits) {
                case 16:
                    if constexpr (I16) run_chunks<KVQ_I16, 1, 2, false>(st, Q, q_lds, ctx, my_meta, lane);
                    else run_chunks<16, 1, 2, false>(st, Q, q_lds, ctx, my_meta, lane);
                    break;
                case 8: run_chunks<8, 1, 2, SAFE>(st, Q, q_lds, ctx, my_meta, lane); break;
                case 4:
                    if (ctx.next.nt == 2) run_chunks<4, 2, KVQ_RING_4BIT, SAFE>(st, Q, q_lds, ctx, my_meta, lane);
                    else run_chunks<4, 1, KVQ_RING_SINGLE, SAFE>(st, Q, q_lds, ctx, my_meta, lane);
                    break;
                default:
                    if (ctx.next.nt == 2) run_chunks<2, 2, KVQ_RING_2BIT, SAFE>(st, Q, q_lds, ctx, my_meta, lane);
                    else run_chunks<2, 1, KVQ_RING_SINGLE, SAFE>(st, Q, q_lds, ctx, my_meta, lane);
                    break;
            }
        }
    }

    KVQ_STAMP(2);
    finish_workgroup(P, sh, st, split, unit);
}

}  // namespace

#endif
