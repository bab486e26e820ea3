// Fused de-quantize + single-token GQA decode attention over the mixed-width paged cache (gfx950).
//
// One workgroup (4 wavefronts) handles one (sequence, KV head) unit and one byte-balanced range of 32-token
// tiles; each wavefront streams every fourth tile of the range with 16-byte loads and keeps its own
// online-softmax state.  Both contractions run on the matrix cores with the g <= 16 query heads of the unit
// as the 16-wide N dimension:
//   scores^T[token, head] = sum_grp S[token,grp] * (codes[token, grp-channels] . q[head, grp-channels])
//                           + sum_grp Z[token,grp] * sum(q[head, grp-channels])
//   out^T[channel, head] += sum_token codes[token, channel] * (p[token, head] * S_v[token, grp(channel)])
//                           + sum_token Z_v[token, grp(channel)] * p[token, head]
// Integer codes are exact in fp16, so scales and zero points never touch individual elements: they are
// applied to per-group partial sums (K) or folded into the probabilities (V), and the zero-point sums and
// the softmax denominator come out of one extra MFMA each.  Wavefront partials are merged through LDS,
// split partials through global memory (a second small kernel, or the last-arriving workgroup).
#include "kvq_internal.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));
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

template <int NDW>
__device__ inline void load_string(const uint8_t* tile, int lane, uint32_t (&w)[NDW]) {
#pragma unroll
    for (int c = 0; c < NDW / 4; ++c) {
        u32x4 v = *reinterpret_cast<const u32x4*>(tile + (c * 64 + lane) * 16);
        w[4 * c] = v.x; w[4 * c + 1] = v.y; w[4 * c + 2] = v.z; w[4 * c + 3] = v.w;
    }
}

struct WaveState {
    float4v o[8];   // out^T accumulators: o[nt][i] = channel 16nt + 4j + i of head n (lane = 16j + n)
    float4v zl;     // quarter 0: zero-point sums of V groups 0..3; quarter 1, element 0: softmax denominator
    float m;        // running maximum of head n in log2 units (equal in the four quarters)
};

// query operands of one lane: [grp][4 dwords]
struct QOps {
    uint32_t q[4][4];
    uint32_t qsum[4];  // quarter 0: hi/lo fp16 split of the per-group sums of q; other quarters: zero
    int natural;       // 1: k-slot order of the 16-bit tier, 0: the (v, v+4) pairing of the quantized tiers
};

__device__ inline void load_q_ops(QOps& Q, const _Float16* q_lds, int lane, int natural) {
    const int j = lane >> 4, n = lane & 15;
    const uint16_t* row = reinterpret_cast<const uint16_t*>(q_lds) + n * KVQ_D;
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
        const uint16_t* p = row + 32 * grp + 8 * j;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            uint32_t lo = natural ? p[2 * v] : p[v];
            uint32_t hi = natural ? p[2 * v + 1] : p[v + 4];
            Q.q[grp][v] = lo | (hi << 16);
        }
    }
    Q.natural = natural;
}

__device__ inline float4v mfma(half8 a, half8 b, float4v c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Registers of one tile in flight: the lane's packed K and V strings and its 16-byte share of the metadata.
template <int B>
struct Stage {
    uint32_t kw[2 * B];
    uint32_t vw[2 * B];
    u32x4 meta;
};

// Issue every global load of one tile (nothing waits here).
template <int B>
__device__ inline void issue_tile(Stage<B>& sg, const uint8_t* __restrict__ code, const uint8_t* __restrict__ meta,
                                  int lane) {
    load_string<2 * B>(code, lane, sg.kw);
    load_string<2 * B>(code + 512u * B, lane, sg.vw);
    if constexpr (B < 16) sg.meta = *reinterpret_cast<const u32x4*>(meta + lane * 16);
}

// One 32-token tile of width B from registers.  meta_lds: this wavefront's 1 KiB staging area, through which
// the metadata is redistributed (each lane needs the scales of the 8 tokens of its quarter).
// tok0 = first token of the tile, n_tokens = cache length (tokens beyond it are masked).
template <int B>
__device__ inline void compute_k(WaveState& st, const QOps& Q, const uint32_t (&kw)[2 * B], const u32x4& meta_regs,
                                 uint8_t* meta_lds, int tok0, int n_tokens, float scale_log2, int lane,
                                 uint32_t (&pop)[4]) {
    const int j = lane >> 4, n = lane & 15;
    const float4v zero4 = {0.f, 0.f, 0.f, 0.f};
    float s[2][4];

    if constexpr (B < 16) {
        *reinterpret_cast<u32x4*>(meta_lds + lane * 16) = meta_regs;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }

    // ---- K: scores^T for the 32 tokens x 16 heads
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
            for (int i = 0; i < 4; ++i) s[sub][i] = acc[i];
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
        half8 qs = as_half8(Q.qsum[0], Q.qsum[1], Q.qsum[2], Q.qsum[3]);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            // zero points of the token this lane supplies as an A row: token 8*(n/4) + 4*sub + n%4
            int t = 8 * (n >> 2) + 4 * sub + (n & 3);
            u32x2 kz = *reinterpret_cast<const u32x2*>(meta_lds + 256 + t * 8);
            float4v acc = mfma(as_half8(kz.x, kz.y, kz.x, kz.y), qs, zero4);
#pragma unroll
            for (int grp = 0; grp < 4; ++grp) {
                half8 a = dq_piece<B>(kw, sub * 4 + grp);
                half8 b = as_half8(Q.q[grp][0], Q.q[grp][1], Q.q[grp][2], Q.q[grp][3]);
                float4v part = mfma(a, b, zero4);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int tk = 4 * sub + i;  // token 8j + tk: dwords 2*tk, 2*tk+1 hold its four scales
                    float sc = mixf(ks[2 * tk + (grp >> 1)], grp & 1);
                    acc[i] = fmaf(sc, part[i], acc[i]);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) s[sub][i] = acc[i];
        }
    }

    // ---- online softmax (log2 domain)
    float tmax = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s[sub][i] *= scale_log2;
            tmax = fmaxf(tmax, s[sub][i]);
        }
    if (tok0 + KVQ_TILE_TOKENS > n_tokens) {  // ragged last tile only
        tmax = -INFINITY;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (tok0 + 8 * j + 4 * sub + i >= n_tokens) s[sub][i] = -INFINITY;
                tmax = fmaxf(tmax, s[sub][i]);
            }
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    float m_new = fmaxf(st.m, tmax);
    if (__any(m_new > st.m)) {
        float alpha = (st.m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m - m_new);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) st.o[nt] *= alpha;
        st.zl *= alpha;
        st.m = m_new;
    }
    {
        float p[2][4];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 4; ++i) p[sub][i] = __builtin_amdgcn_exp2f(s[sub][i] - st.m);
        if constexpr (B == 16) {  // natural order: slots 0..3 = sub 0, slots 4..7 = sub 1
            pop[0] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p[0][0], p[0][1]));
            pop[1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p[0][2], p[0][3]));
            pop[2] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p[1][0], p[1][1]));
            pop[3] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p[1][2], p[1][3]));
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v)
                pop[v] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p[0][v], p[1][v]));
        }
    }
}

// V half of a tile: out^T += V^T p^T with the probabilities `pop` compute_k produced for the same tile.
template <int B>
__device__ inline void compute_v(WaveState& st, const uint32_t (&vw)[2 * B], const uint8_t* meta_lds,
                                 const uint32_t (&pop)[4], int lane) {
    const int j = lane >> 4, n = lane & 15;
    const half8 pb = as_half8(pop[0], pop[1], pop[2], pop[3]);
    const uint32_t ones = (n == 4) ? 0x3c003c00u : 0u;  // row 4 of the extra MFMA sums p (denominator)
    if constexpr (B == 16) {
        st.zl = mfma(as_half8(ones, ones, ones, ones), pb, st.zl);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) {
            half8 a = as_half8(vw[4 * nt], vw[4 * nt + 1], vw[4 * nt + 2], vw[4 * nt + 3]);
            st.o[nt] = mfma(a, pb, st.o[nt]);
        }
    } else {
        // rows 0..3 of the extra MFMA: zero points of V group n over the 8 tokens of this quarter
        u32x4 zv = *reinterpret_cast<const u32x4*>(meta_lds + 768 + (n & 3) * 64 + j * 16);
        if (n >= 4) { zv.x = ones; zv.y = ones; zv.z = ones; zv.w = ones; }
        st.zl = mfma(as_half8(zv.x, zv.y, zv.z, zv.w), pb, st.zl);
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
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

template <int B>
__device__ inline void compute_tile(WaveState& st, const QOps& Q, const Stage<B>& sg, uint8_t* meta_lds, int tok0,
                                    int n_tokens, float scale_log2, int lane) {
    uint32_t pop[4];
    compute_k<B>(st, Q, sg.kw, sg.meta, meta_lds, tok0, n_tokens, scale_log2, lane, pop);
    compute_v<B>(st, sg.vw, meta_lds, pop, lane);
}

struct RunCtx {
    const uint8_t* arena;
    const u32x4* desc_lds;   // descriptors of pages page0 .. of the current chunk
    int page0;
    int tpp;
    int unit;
    int n_tokens;
    float scale_log2;
};

template <int B>
__device__ inline void tile_addr(const RunCtx& c, int tile, const uint8_t** code, const uint8_t** meta) {
    const int page = tile / c.tpp, tip = tile - page * c.tpp;
    const u32x4 d = c.desc_lds[page - c.page0];
    const uint32_t code_off = __builtin_amdgcn_readfirstlane(d.x);
    const uint32_t meta_off = __builtin_amdgcn_readfirstlane(d.y);
    const uint64_t tslot = (uint64_t)c.unit * c.tpp + tip;
    *code = c.arena + (uint64_t)code_off * 256u + tslot * 2 * (512u * B);
    *meta = c.arena + (uint64_t)meta_off * 256u + tslot * KVQ_META_TILE_BYTES;
}

// This wavefront's tiles first, first+4, ... < end, all of width B, software-pipelined: the loads of the next
// tile are in flight while the current one is computed (two register stages, ping-pong).
template <int B>
__device__ inline void run_tiles(WaveState& st, const QOps& Q, const RunCtx& c, int first, int end,
                                 uint8_t* meta_lds, int lane) {
    if (first >= end) return;
    if constexpr (B == 16) {
        // raw fp16 tiles are 16 KiB: one register stage, K and V staggered (V loads fly during the K product,
        // the next tile's K loads during the V product)
        uint32_t kw[32], vw[32];
        const u32x4 nometa = {0u, 0u, 0u, 0u};
        const uint8_t *code, *meta;
        tile_addr<16>(c, first, &code, &meta);
        load_string<32>(code, lane, kw);
        load_string<32>(code + 512u * 16, lane, vw);
        for (int t = first; t < end; t += 4) {
            uint32_t pop[4];
            compute_k<16>(st, Q, kw, nometa, meta_lds, t * KVQ_TILE_TOKENS, c.n_tokens, c.scale_log2, lane, pop);
            const bool more = t + 4 < end;
            if (more) {
                tile_addr<16>(c, t + 4, &code, &meta);
                load_string<32>(code, lane, kw);
            }
            compute_v<16>(st, vw, meta_lds, pop, lane);
            if (more) load_string<32>(code + 512u * 16, lane, vw);
        }
        return;
    }
    Stage<B> s0, s1;
    const uint8_t *code, *meta;
    tile_addr<B>(c, first, &code, &meta);
    issue_tile<B>(s0, code, meta, lane);
    int t = first;
    for (;;) {
        const int t1 = t + 4;
        const bool has1 = t1 < end;
        if (has1) {
            tile_addr<B>(c, t1, &code, &meta);
            issue_tile<B>(s1, code, meta, lane);
        }
        compute_tile<B>(st, Q, s0, meta_lds, t * KVQ_TILE_TOKENS, c.n_tokens, c.scale_log2, lane);
        if (!has1) break;
        const int t2 = t1 + 4;
        const bool has2 = t2 < end;
        if (has2) {
            tile_addr<B>(c, t2, &code, &meta);
            issue_tile<B>(s0, code, meta, lane);
        }
        compute_tile<B>(st, Q, s1, meta_lds, t1 * KVQ_TILE_TOKENS, c.n_tokens, c.scale_log2, lane);
        if (!has2) break;
        t = t2;
    }
}

// Merge of split partials: thread `tid` of `nthreads` produces out[head][d] for its share of (head, d).
__device__ inline void merge_splits(const KvqAttnParams& P, int unit, int tid, int nthreads) {
    const int g = P.gqa;
    const int b = unit / P.n_kv_heads, hk = unit - b * P.n_kv_heads;
    const float* po = P.part_o + (size_t)unit * P.n_splits * 16 * KVQ_D;
    const float* pml = P.part_ml + (size_t)unit * P.n_splits * 32;
    for (int e = tid; e < g * KVQ_D; e += nthreads) {
        int head = e >> 7, d = e & 127;
        float M = -INFINITY;
        for (int sp = 0; sp < P.n_splits; ++sp) M = fmaxf(M, pml[sp * 32 + head]);
        float L = 0.f, acc = 0.f;
        for (int sp = 0; sp < P.n_splits; ++sp) {
            float ms = pml[sp * 32 + head];
            float f = (ms == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms - M);
            L += pml[sp * 32 + 16 + head] * f;
            acc += po[((size_t)sp * 16 + head) * KVQ_D + d] * f;
        }
        float r = acc / L;
        size_t oi = ((size_t)b * P.n_q_heads + hk * g + head) * KVQ_D + d;
        if (P.out_fp32) static_cast<float*>(P.out)[oi] = r;
        else static_cast<_Float16*>(P.out)[oi] = (_Float16)r;
    }
}

#define KVQ_DESC_CACHE 256  // page descriptors staged in LDS per chunk of the split's range
#define KVQ_OPAD 132  // padded row of the LDS reduction slab (floats)

__global__ __launch_bounds__(256, 2) void kvq_attention_kernel(const KvqAttnParams P) {
    __shared__ _Float16 q_lds[16 * KVQ_D];
    __shared__ float qsum_lds[16 * 4];
    __shared__ float red_o[4][16 * KVQ_OPAD];
    __shared__ float red_m[4][16];
    __shared__ float red_l[4][16];
    __shared__ int is_last;
    __shared__ u32x4 desc_lds[KVQ_DESC_CACHE];
    __shared__ __attribute__((aligned(16))) uint8_t meta_lds[4 * KVQ_META_TILE_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane >> 4, n = lane & 15;
    const int split = blockIdx.x, unit = blockIdx.y;
    const int g = P.gqa;
    const int b = unit / P.n_kv_heads, hk = unit - b * P.n_kv_heads;

    // stage q (heads beyond g are zero) and its per-group sums
    {
        const _Float16* qg = static_cast<const _Float16*>(P.q) + ((size_t)b * P.n_q_heads + hk * g) * KVQ_D;
        for (int e = tid; e < 16 * KVQ_D; e += 256) q_lds[e] = (e < g * KVQ_D) ? qg[e] : (_Float16)0.f;
        __syncthreads();
        if (tid < 64) {
            int head = tid >> 2, grp = tid & 3;
            float sum = 0.f;
            for (int d = 0; d < 32; ++d) sum += (float)q_lds[head * KVQ_D + grp * 32 + d];
            qsum_lds[tid] = sum;
        }
        __syncthreads();
    }
    QOps Q;
    {
        uint16_t hi[4], lo[4];
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            float sum = qsum_lds[n * 4 + grp];
            _Float16 h = (_Float16)sum;
            _Float16 l = (_Float16)(sum - (float)h);
            hi[grp] = __builtin_bit_cast(uint16_t, h);
            lo[grp] = __builtin_bit_cast(uint16_t, l);
        }
        bool q0 = (j == 0);
        Q.qsum[0] = q0 ? ((uint32_t)hi[0] | ((uint32_t)hi[1] << 16)) : 0u;
        Q.qsum[1] = q0 ? ((uint32_t)hi[2] | ((uint32_t)hi[3] << 16)) : 0u;
        Q.qsum[2] = q0 ? ((uint32_t)lo[0] | ((uint32_t)lo[1] << 16)) : 0u;
        Q.qsum[3] = q0 ? ((uint32_t)lo[2] | ((uint32_t)lo[3] << 16)) : 0u;
        Q.natural = -1;
    }

    WaveState st;
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) st.o[nt] = float4v{0.f, 0.f, 0.f, 0.f};
    st.zl = float4v{0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;

    const int tpp = P.tiles_per_page;
    const int t_begin = P.split_begin[split], t_end = P.split_begin[split + 1];
    RunCtx ctx;
    ctx.arena = P.arena; ctx.desc_lds = desc_lds; ctx.tpp = tpp; ctx.unit = unit;
    ctx.n_tokens = P.n_tokens; ctx.scale_log2 = P.scale_log2;
    uint8_t* my_meta = meta_lds + wave * KVQ_META_TILE_BYTES;
    const int p_first = t_begin / tpp, p_last = (t_end + tpp - 1) / tpp;  // pages touched: [p_first, p_last)
    for (int pc = p_first; pc < p_last; pc += KVQ_DESC_CACHE) {
        const int pn = min(KVQ_DESC_CACHE, p_last - pc);
        __syncthreads();
        for (int e = tid; e < pn; e += 256) desc_lds[e] = reinterpret_cast<const u32x4*>(P.table)[pc + e];
        __syncthreads();
        ctx.page0 = pc;
        const int lo = max(t_begin, pc * tpp), hi = min(t_end, (pc + pn) * tpp);
        // first tile of this wavefront in [lo, hi): tiles are dealt round-robin from t_begin
        int t = lo + ((t_begin + wave - lo) % 4 + 4) % 4;
        while (t < hi) {
            const int page = t / tpp;
            const int bits = __builtin_amdgcn_readfirstlane(desc_lds[page - pc].z);
            int pe = page + 1;
            while (pe < pc + pn && __builtin_amdgcn_readfirstlane(desc_lds[pe - pc].z) == bits) ++pe;
            const int rend = min(pe * tpp, hi);
            const int natural = (bits == 16);
            if (Q.natural != natural) load_q_ops(Q, q_lds, lane, natural);
            switch (bits) {
                case 16: run_tiles<16>(st, Q, ctx, t, rend, my_meta, lane); break;
                case 8: run_tiles<8>(st, Q, ctx, t, rend, my_meta, lane); break;
                case 4: run_tiles<4>(st, Q, ctx, t, rend, my_meta, lane); break;
                default: run_tiles<2>(st, Q, ctx, t, rend, my_meta, lane); break;
            }
            t += ((rend - t + 3) / 4) * 4;
        }
    }

    // ---- wavefront epilogue: add the zero-point term, fetch the denominator
    float l_w = __shfl(st.zl[0], 16 + n);
    {
        float z0 = __shfl(st.zl[0], n), z1 = __shfl(st.zl[1], n), z2 = __shfl(st.zl[2], n), z3 = __shfl(st.zl[3], n);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            st.o[0][i] += z0; st.o[1][i] += z0;
            st.o[2][i] += z1; st.o[3][i] += z1;
            st.o[4][i] += z2; st.o[5][i] += z2;
            st.o[6][i] += z3; st.o[7][i] += z3;
        }
    }
    // ---- merge the four wavefronts through LDS
    if (j == 0) { red_m[wave][n] = st.m; }
    __syncthreads();
    float M = fmaxf(fmaxf(red_m[0][n], red_m[1][n]), fmaxf(red_m[2][n], red_m[3][n]));
    float f = (st.m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.m - M);
    if (j == 0) red_l[wave][n] = l_w * f;
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) {
        float4v v = st.o[nt] * f;
        *reinterpret_cast<float4v*>(&red_o[wave][n * KVQ_OPAD + 16 * nt + 4 * j]) = v;
    }
    __syncthreads();

    const bool direct = (P.n_splits == 1);
    float* po = P.part_o + ((size_t)unit * P.n_splits + split) * 16 * KVQ_D;
    float* pml = P.part_ml + ((size_t)unit * P.n_splits + split) * 32;
    for (int e = tid; e < g * KVQ_D; e += 256) {
        int head = e >> 7, d = e & 127;
        int li = head * KVQ_OPAD + d;
        float acc = red_o[0][li] + red_o[1][li] + red_o[2][li] + red_o[3][li];
        if (direct) {
            float L = red_l[0][head] + red_l[1][head] + red_l[2][head] + red_l[3][head];
            float r = acc / L;
            size_t oi = ((size_t)b * P.n_q_heads + hk * g + head) * KVQ_D + d;
            if (P.out_fp32) static_cast<float*>(P.out)[oi] = r;
            else static_cast<_Float16*>(P.out)[oi] = (_Float16)r;
        } else {
            po[e] = acc;
        }
    }
    if (direct) return;
    if (tid < 16) {
        float Mh = fmaxf(fmaxf(red_m[0][tid], red_m[1][tid]), fmaxf(red_m[2][tid], red_m[3][tid]));
        pml[tid] = Mh;
        pml[16 + tid] = red_l[0][tid] + red_l[1][tid] + red_l[2][tid] + red_l[3][tid];
    }
    if (!P.fused_merge) return;

    // ---- fused merge: the last workgroup of the unit to arrive combines all split partials
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        uint32_t old = atomicAdd(&P.counters[unit], 1u);
        is_last = (old == (uint32_t)P.n_splits - 1u);
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    merge_splits(P, unit, tid, 256);
    if (tid == 0) P.counters[unit] = 0u;
}

__global__ __launch_bounds__(256) void kvq_merge_kernel(const KvqAttnParams P) {
    merge_splits(P, blockIdx.x, threadIdx.x, 256);
}

}  // namespace

hipError_t kvq_launch_attention(const KvqAttnParams& p, int units, hipStream_t s) {
    hipLaunchKernelGGL(kvq_attention_kernel, dim3(p.n_splits, units), dim3(256), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.n_splits > 1 && !p.fused_merge) {
        hipLaunchKernelGGL(kvq_merge_kernel, dim3(units), dim3(256), 0, s, p);
        e = hipGetLastError();
    }
    return e;
}
