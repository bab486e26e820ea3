// Quantize-on-append, fp16 -> b-bit page quantization and the Equivalent Right Shift kernels (gfx950).
//
// Quantizer: Sec. 2.2 Eq. 1-2 (asymmetric min-max per group of 32 channels of one token of one KV head).
// Shrinking: Sec. 3.1 Eq. 3 with S_b = (2^b + 1) S_2b and Z kept.
// All kernels work directly in the tile layout described in kvq_layout.h: one wavefront owns one tile and
// every lane quantizes the 64 slots it will later feed to the matrix cores.
#include "kvq_quant_dev.h"

namespace {

using namespace kvq_q;

// grid.x = 2 * (tiles touched) (even: K tile, odd: V tile), grid.y = (sequence, KV head) unit, 64 threads.
// Append into the 16-bit tier: the new rows are copied into the tile layout.
__global__ __launch_bounds__(64) void kvq_append16_kernel(uint8_t* __restrict__ arena,
                                                          const KvqPageDesc* __restrict__ table,
                                                          const uint16_t* __restrict__ k_in,
                                                          const uint16_t* __restrict__ v_in, int t_old,
                                                          int n_new, int tpp, int tile0, KvqAppendPages ap,
                                                          const float* __restrict__ rinv, int n_kv_heads,
                                                          const float* __restrict__ rope) {
    const int lane = threadIdx.x;
    const int which = blockIdx.x & 1;
    const int tile = tile0 + (blockIdx.x >> 1);
    const int unit = blockIdx.y;
    const int page = tile / tpp, tip = tile - page * tpp;
    const KvqPageDesc pd = append_desc(table, ap, page);
    const uint64_t tslot = (uint64_t)unit * tpp + tip;
    uint8_t* code = arena + (uint64_t)pd.code_off256 * 256u + (tslot * 2 + which) * (512u * 16);
    const uint16_t* in = (which ? v_in : k_in) + (uint64_t)unit * n_new * KVQ_D;
    if (which && tile * KVQ_TILE_TOKENS >= t_old) {  // a V tile made of new tokens only: through LDS (wavefront-uniform)
        __shared__ __attribute__((aligned(16))) uint8_t lds[32 * 256];
        kvq_dev::append16_v_tile_lds(code, in, tile * KVQ_TILE_TOKENS, t_old, t_old + n_new, lane, lds);
        return;
    }
    kvq_dev::append16_tile<true>(code, in, which, tile * KVQ_TILE_TOKENS, t_old, t_old + n_new, lane, which ? nullptr : rope,
                                 (rinv && !which) ? rinv + (unit % n_kv_heads) * KVQ_D : nullptr);
}

// Quantizing append (B = 8, 4, 2), built on the row-owner core: grid.x = ceil(n_strings / KVQ_APPEND_WG_WAVES) workgroups,
// n_strings = 2 * touched tiles (K and V string of each), grid.y = unit; one wavefront per string.
// PLAIN: keys arrive rotated and the block has no reparameterization (rope and rinv are null): the instantiation
// carries none of that code, which is the bulk of the general kernel's registers.
// Four wavefronts per workgroup, each with a (tile, K | V) string of its own and its own LDS: 1 to 2 % faster on bulk
// appends than one-wavefront workgroups (a quarter of the workgroups to dispatch); nothing is shared between them.
#define KVQ_APPEND_WG_WAVES 4
template <int B, bool PLAIN>
__global__ __launch_bounds__(64 * KVQ_APPEND_WG_WAVES) void kvq_append_q_kernel(uint8_t* __restrict__ arena,
                                                          const KvqPageDesc* __restrict__ table,
                                                          const uint16_t* __restrict__ k_in,
                                                          const uint16_t* __restrict__ v_in, int t_old,
                                                          int n_new, int tpp, int tile0, KvqAppendPages ap,
                                                          uint32_t* __restrict__ flags, int gspan,
                                                          const float* __restrict__ rinv, int n_kv_heads,
                                                          const float* __restrict__ rope, int n_strings) {
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[KVQ_APPEND_WG_WAVES][KVQ_LDS_CODES];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint8_t* const lds = lds_all[wave];
    const int lane = threadIdx.x & 63, j = lane >> 4, n = lane & 15;
    const int string = blockIdx.x * KVQ_APPEND_WG_WAVES + wave;  // (tile, K | V) of this wavefront
    if (string >= n_strings) return;
    const int which = string & 1;
    const int tile = tile0 + (string >> 1);
    const int unit = blockIdx.y;
    const int page = tile / tpp, tip = tile - page * tpp;
    const KvqPageDesc pd = append_desc(table, ap, page);
    const uint64_t tslot = (uint64_t)unit * tpp + tip;
    uint8_t* code = arena + (uint64_t)pd.code_off256 * 256u + (tslot * 2 + which) * (512u * B);
    uint8_t* meta = arena + (uint64_t)pd.meta_off256 * 256u + tslot * KVQ_META_TILE_BYTES;
    const int t_new = t_old + n_new, tok0 = tile * KVQ_TILE_TOKENS;
    const uint16_t* in = (which ? v_in : k_in) + (uint64_t)unit * n_new * KVQ_D;
    const int grp = lane & 3;
    // every load of the tile first (both passes: 8 x 16 bytes per lane in flight), then the arithmetic
    uint32_t w[2][16];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int tok = tok0 + 16 * pass + (lane >> 2);
        u32x4 v[4];
        if (PLAIN || which) {
            // Buffer loads with the unit's n_new rows as the buffer: a lane whose token is not new (before t_old or at
            // or after t_new) gets an offset beyond the buffer (n_new < 2^23 rows of 256 bytes end below 2^31) and
            // reads zeros, which is what such a token quantizes -- no branch around the loads.
            const __amdgpu_buffer_rsrc_t rows =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(in), 0, n_new * (KVQ_D * 2), 0x00020000);
            const uint32_t rel = (uint32_t)(tok - t_old);
            const uint32_t off = (rel < (uint32_t)n_new ? rel * (uint32_t)(KVQ_D * 2) : 0x80000000u) + 64u * grp;
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = __builtin_amdgcn_raw_buffer_load_b128(rows, (int)(off + 16u * c), 0, 0);
        } else {
            const bool isnew = tok >= t_old && tok < t_new;
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = u32x4{0u, 0u, 0u, 0u};
            if (isnew) {
                const uint16_t* row = in + (uint64_t)(tok - t_old) * KVQ_D;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    v[c] = load_key8(row, 32 * grp + 8 * c, rope ? rope + (uint64_t)(tok - t_old) * KVQ_D : nullptr,
                                     rinv ? rinv + (unit % n_kv_heads) * KVQ_D : nullptr);
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            w[pass][4 * c] = v[c].x; w[pass][4 * c + 1] = v[c].y; w[pass][4 * c + 2] = v[c].z; w[pass][4 * c + 3] = v[c].w;
        }
    }
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int tl = 16 * pass + (lane >> 2);
        const int tok = tok0 + tl;
        float codes[32];
        uint16_t S, Z;
        quantize_owner<B>(w[pass], codes, &S, &Z, gspan);  // tokens that are not new quantize zeros: codes 0, S = Z = 0
        note_large_v_scale(flags, which, S);
        scatter_codes(lds, which, tl, grp, codes);
        if (tok >= t_old) store_meta_owner(meta, which, tl, grp, S, Z);
    }
    wave_sync_lds();
    uint32_t str[2 * B];
    gather_string<B>(lds, which, lane, str);
    // stored tokens keep their bits
    uint32_t keep = 0;
    if (!which) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
            if (tok0 + 8 * (n >> 2) + 4 * sub + (n & 3) < t_old) keep |= 1u << sub;
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (tok0 + 8 * j + i < t_old) keep |= 1u << i;
    }
    if (tok0 < t_old) {  // (wavefront-uniform) the tile already holds tokens: it is rewritten step by step, plain stores
        if (keep) {
            uint32_t old[2 * B];
            load_chunks<B>(code, lane, old);
#pragma unroll
            for (int d = 0; d < 2 * B; ++d) {
                uint32_t m = which ? v_token_mask<B>(keep, d) : (((keep >> (d / B)) & 1u) ? 0xffffffffu : 0u);
                str[d] = (old[d] & m) | (str[d] & ~m);
            }
        }
        store_chunks<B>(code, lane, str);
        asm volatile("" ::: "memory");  // keeps the two kinds of store apart (merged, they would both be plain ones)
        return;
    }
    // a tile made of new tokens only is written once and read much later: streaming stores (with plain stores the
    // bulk appends run a quarter slower)
    store_chunks_stream<B>(code, lane, str);
}

// Append into the integer 16-bit tier: Eq. 1-2 with 2^16 - 1 levels by the same owner lanes; the high and the low
// bytes of the codes then travel through LDS and into the tile's two byte planes like two 8-bit tiles.
// (The same steps as kvq_q::append_i16_string, which the attention kernel uses for its fused one-token append, written
// out here: as a call of that function this kernel measured 15 % slower on bulk appends, forced inlining or not.)
__global__ __launch_bounds__(64) void kvq_append_i16_kernel(uint8_t* __restrict__ arena,
                                                            const KvqPageDesc* __restrict__ table,
                                                            const uint16_t* __restrict__ k_in,
                                                            const uint16_t* __restrict__ v_in, int t_old,
                                                            int n_new, int tpp, int tile0, KvqAppendPages ap,
                                                            int gspan, const float* __restrict__ rinv,
                                                            int n_kv_heads, const float* __restrict__ rope) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[2][KVQ_LDS_CODES];
    const int lane = threadIdx.x, j = lane >> 4, n = lane & 15;
    const int which = blockIdx.x & 1;
    const int tile = tile0 + (blockIdx.x >> 1);
    const int unit = blockIdx.y;
    const int page = tile / tpp, tip = tile - page * tpp;
    const KvqPageDesc pd = append_desc(table, ap, page);
    const uint64_t tslot = (uint64_t)unit * tpp + tip;
    uint8_t* code = arena + (uint64_t)pd.code_off256 * 256u + (tslot * 2 + which) * (512u * 16);
    uint8_t* meta = arena + (uint64_t)pd.meta_off256 * 256u + tslot * KVQ_META_TILE_BYTES;
    const int t_new = t_old + n_new, tok0 = tile * KVQ_TILE_TOKENS;
    const uint16_t* in = (which ? v_in : k_in) + (uint64_t)unit * n_new * KVQ_D;
    const int grp = lane & 3;
    // every load of the tile first, as in kvq_append_q_kernel: rows that need neither rotation nor reparameterization
    // come through range-checked buffer loads (a token that is not new reads zeros)
    const bool plain = which || (!rope && !rinv);  // wavefront-uniform
    uint32_t w[2][16];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int tok = tok0 + 16 * pass + (lane >> 2);
        u32x4 v[4];
        if (plain) {
            const __amdgpu_buffer_rsrc_t rows =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(in), 0, n_new * (KVQ_D * 2), 0x00020000);
            const uint32_t rel = (uint32_t)(tok - t_old);
            const uint32_t off = (rel < (uint32_t)n_new ? rel * (uint32_t)(KVQ_D * 2) : 0x80000000u) + 64u * grp;
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = __builtin_amdgcn_raw_buffer_load_b128(rows, (int)(off + 16u * c), 0, 0);
        } else {
            const bool isnew = tok >= t_old && tok < t_new;
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = u32x4{0u, 0u, 0u, 0u};
            if (isnew) {
                const uint16_t* row = in + (uint64_t)(tok - t_old) * KVQ_D;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    v[c] = load_key8(row, 32 * grp + 8 * c, rope ? rope + (uint64_t)(tok - t_old) * KVQ_D : nullptr,
                                     rinv ? rinv + (unit % n_kv_heads) * KVQ_D : nullptr);
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            w[pass][4 * c] = v[c].x; w[pass][4 * c + 1] = v[c].y; w[pass][4 * c + 2] = v[c].z; w[pass][4 * c + 3] = v[c].w;
        }
    }
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int tl = 16 * pass + (lane >> 2);
        const int tok = tok0 + tl;
        float codes[32], lo[32];
        uint16_t S, Z;
        quantize_owner<16>(w[pass], codes, &S, &Z, gspan);
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
    uint32_t keep = 0;  // stored tokens keep their bits
    if (!which) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
            if (tok0 + 8 * (n >> 2) + 4 * sub + (n & 3) < t_old) keep |= 1u << sub;
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (tok0 + 8 * j + i < t_old) keep |= 1u << i;
    }
#pragma unroll
    for (int plane = 0; plane < 2; ++plane) {
        uint32_t str[16];
        gather_string<8>(lds[plane], which, lane, str);
        uint8_t* dst = code + plane * (512u * 8);
        if (tok0 < t_old && keep) {
            uint32_t old[16];
            load_chunks<8>(dst, lane, old);
#pragma unroll
            for (int d = 0; d < 16; ++d) {
                uint32_t m = which ? v_token_mask<8>(keep, d) : (((keep >> (d / 8)) & 1u) ? 0xffffffffu : 0u);
                str[d] = (old[d] & m) | (str[d] & ~m);
            }
        }
        if (tok0 >= t_old) {
            store_chunks_stream<8>(dst, lane, str);
        } else {
            store_chunks<8>(dst, lane, str);
            asm volatile("" ::: "memory");  // keeps the two kinds of store apart
        }
    }
}

// ------------------------------------------------------------------------------------- fp16 page -> b bits
// grid.x = 2 * n_jobs * tiles_per_page, grid.y = unit, 64 threads.  Direct quantization (Eq. 1-2) of a page
// that still holds raw fp16 values: the tile is first laid out [token][channel] in LDS, then quantized by
// owner lanes exactly like an append.
template <int B>
__global__ __launch_bounds__(64) void kvq_quant16_kernel(uint8_t* __restrict__ arena,
                                                         const KvqRequantJob* __restrict__ jobs, int tpp,
                                                         uint32_t* __restrict__ flags, int gspan,
                                                         const KvqJobArgs ja) {
    // One LDS block: [pad | raw rows 0..15 | raw rows 16..31].  The codes of both passes go to the first KVQ_LDS_CODES bytes,
    // i.e. the pad and the rows of the first pass, which every lane has read by the time the first codes are written (the
    // LDS carries out a wavefront's instructions in order); the rows of the second pass are not touched.  8.1 KiB per
    // wavefront instead of 12.1: the LDS then admits 19 wavefronts per compute unit instead of 13 (16 -> 8: +7 %).
    __shared__ __attribute__((aligned(16))) uint8_t lds_block[(KVQ_LDS_CODES - 16 * 256) + 32 * 256];
    uint8_t* const lds = lds_block;
    uint8_t* const raw_lds = lds_block + (KVQ_LDS_CODES - 16 * 256);
    const int lane = threadIdx.x, j = lane >> 4, n = lane & 15;
    const int which = blockIdx.x & 1;
    const int idx = blockIdx.x >> 1;
    const int job = idx / tpp, tip = idx - job * tpp;
    const int unit = blockIdx.y;
    const KvqRequantJob jb = ja.n ? ja.jobs[job] : jobs[job];
    if (tip >= (int)jb.n_tiles) return;  // tiles of a partly filled page that hold no token yet (wavefront-uniform)
    const uint64_t tslot = (uint64_t)unit * tpp + tip;
    const uint8_t* src = arena + (uint64_t)jb.src_code_off256 * 256u + (tslot * 2 + which) * (512u * 16);
    uint8_t* dst = arena + (uint64_t)jb.dst_code_off256 * 256u + (tslot * 2 + which) * (512u * B);
    uint8_t* meta = arena + (uint64_t)jb.meta_off256 * 256u + tslot * KVQ_META_TILE_BYTES;
    {
        uint32_t in[32];
        load_chunks_stream<16>(src, lane, in);
        // LDS rows are tokens (256 bytes); the bytes of row r are rotated by 32 * (r / 8), so that the four lane
        // quarters, which write rows 8 apart, land in different banks
        if (!which) {
#pragma unroll
            for (int p = 0; p < 8; ++p) {  // piece (sub, grp): 8 consecutive channels of one token
                const int sub = p >> 2, g = p & 3;
                const int t = 8 * (n >> 2) + 4 * sub + (n & 3);
                *reinterpret_cast<u32x4*>(raw_lds + t * 256 + (((32 * g + 8 * j) * 2 + 32 * (t >> 3)) & 255)) =
                    u32x4{in[4 * p], in[4 * p + 1], in[4 * p + 2], in[4 * p + 3]};
            }
        } else {
#pragma unroll
            for (int d = 0; d < 32; ++d) {  // dword d = slots 2d, 2d+1 = tokens 8j + (2d%8), +1 of channel 16*(d/4)+n
                const int nt = d >> 2, i = (2 * d) & 7;
                const int col = ((16 * nt + n) * 2 + 32 * j) & 255;  // rows 8j + i and 8j + i + 1 share the rotation
                *reinterpret_cast<uint16_t*>(raw_lds + (8 * j + i) * 256 + col) = (uint16_t)(in[d] & 0xffff);
                *reinterpret_cast<uint16_t*>(raw_lds + (8 * j + i + 1) * 256 + col) = (uint16_t)(in[d] >> 16);
            }
        }
    }
    wave_sync_lds();
    const int grp = lane & 3;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int tl = 16 * pass + (lane >> 2);
        uint32_t w[16];
#pragma unroll
        for (int h = 0; h < 2; ++h) {  // the two 32-byte halves of the group's 64 bytes (the rotation may wrap between them)
            const u32x4* rp = reinterpret_cast<const u32x4*>(raw_lds + tl * 256 + ((grp * 64 + 32 * h + 32 * (tl >> 3)) & 255));
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                u32x4 v = rp[c];
                w[8 * h + 4 * c] = v.x; w[8 * h + 4 * c + 1] = v.y; w[8 * h + 4 * c + 2] = v.z; w[8 * h + 4 * c + 3] = v.w;
            }
        }
        float codes[32];
        uint16_t S, Z;
        quantize_owner<B>(w, codes, &S, &Z, gspan);
        note_large_v_scale(flags, which, S);
        scatter_codes(lds, which, tl, grp, codes);
        store_meta_owner(meta, which, tl, grp, S, Z);
    }
    wave_sync_lds();
    uint32_t str[2 * B];
    gather_string<B>(lds, which, lane, str);
    store_chunks_stream<B>(dst, lane, str);
}

// ------------------------------------------------------------------------------- Equivalent Right Shift
// Eq. 3 on packed codes, slot order preserved, several codes per 32-bit multiply (no carry can cross a field:
// 13*(15+2) < 2^8 and 241*(255+8) < 2^16).  From the integer 16-bit tier the product 65281 * (X + 128) needs all 32
// bits of an unsigned multiply (largest value 4,286,546,303), so that step takes one multiply per code.
__device__ inline uint32_t shrink_4_to_2(uint32_t w) {  // 8 nibbles -> 8 two-bit codes (16 bits)
    uint32_t e = w & 0x0f0f0f0fu, o = (w >> 4) & 0x0f0f0f0fu;
    e = (((e + 0x02020202u) * 13u) >> 6) & 0x03030303u;
    o = (((o + 0x02020202u) * 13u) >> 6) & 0x03030303u;
    uint32_t c = e | (o << 2);
    c = (c | (c >> 4)) & 0x00ff00ffu;
    return (c | (c >> 8)) & 0xffffu;
}
__device__ inline uint32_t shrink_16_to_8(uint32_t hi, uint32_t lo) {  // 4 high bytes, 4 low bytes -> 4 bytes
    uint32_t out = 0u;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t x = (((hi >> (8 * k)) & 0xffu) << 8) | ((lo >> (8 * k)) & 0xffu);
        out |= ((65281u * (x + 128u)) >> 24) << (8 * k);
    }
    return out;
}
__device__ inline uint32_t shrink_8_to_4(uint32_t w) {  // 4 bytes -> 4 nibbles (16 bits)
    uint32_t e = w & 0x00ff00ffu, o = (w >> 8) & 0x00ff00ffu;
    e = (((e + 0x00080008u) * 241u) >> 12) & 0x000f000fu;
    o = (((o + 0x00080008u) * 241u) >> 12) & 0x000f000fu;
    uint32_t c = e | (o << 4);
    return (c | (c >> 8)) & 0xffffu;
}

// The two other strategies of the ablation (Sec. 4.3.1) keep the upper B bits of every 2B-bit code.
__device__ inline uint32_t trunc_4_to_2(uint32_t w) {  // 8 nibbles -> their upper two bits, packed (16 bits)
    uint32_t e = (w >> 2) & 0x03030303u, o = (w >> 6) & 0x03030303u;
    uint32_t c = e | (o << 2);
    c = (c | (c >> 4)) & 0x00ff00ffu;
    return (c | (c >> 8)) & 0xffffu;
}
__device__ inline uint32_t trunc_8_to_4(uint32_t w) {  // 4 bytes -> their upper nibbles, packed (16 bits)
    uint32_t e = (w >> 4) & 0x000f000fu, o = (w >> 12) & 0x000f000fu;
    uint32_t c = e | (o << 4);
    return (c | (c >> 8)) & 0xffffu;
}

#define KVQ_SHIFT_EQUIVALENT_ 0
#define KVQ_SHIFT_DIRECT_ 1
#define KVQ_SHIFT_MODIFIED_ 2

// grid.x = n_jobs * tiles_per_page, grid.y = unit, 64 threads; one wavefront shrinks the K and the V tile of
// one (page, unit, tile) from 2B to B bits and rewrites its 256 scales (and, for the Modified strategy, zero
// points) in place.  B = 8 is the step out of the integer 16-bit tier.
//   STRAT 0, Equivalent Right Shift (Eq. 3):  codes by Eq. 3, S <- (2^B + 1) S, Z kept
//   STRAT 1, Direct Right Shift:              codes >> B,     S <- (2^B + 1) S, Z kept
//   STRAT 2, Modified Right Shift:            codes >> B,     S <- 2^B S,       Z <- Z + (2^B S - S) / 2
// Products and the sum are formed in fp32 (the products are exact) and rounded to nearest-even into fp16.
template <int B, int STRAT>
__global__ __launch_bounds__(64) void kvq_shrink_kernel(uint8_t* __restrict__ arena,
                                                        const KvqRequantJob* __restrict__ jobs, int tpp,
                                                        uint32_t* __restrict__ flags, const KvqJobArgs ja) {
    const int lane = threadIdx.x;
    const int job = blockIdx.x / tpp, tip = blockIdx.x - job * tpp;
    const int unit = blockIdx.y;
    const KvqRequantJob jb = ja.n ? ja.jobs[job] : jobs[job];
    if (tip >= (int)jb.n_tiles) return;  // tiles of a partly filled page that hold no token yet (wavefront-uniform)
    const uint64_t tslot = (uint64_t)unit * tpp + tip;
    const uint8_t* src = arena + (uint64_t)jb.src_code_off256 * 256u + tslot * 2 * (512u * 2 * B);
    uint8_t* dst = arena + (uint64_t)jb.dst_code_off256 * 256u + tslot * 2 * (512u * B);
    uint8_t* meta = arena + (uint64_t)jb.meta_off256 * 256u + tslot * KVQ_META_TILE_BYTES;
    // K scales at +0, K zero points at +256, V scales at +512, V zero points at +768: 64 dwords each, one
    // dword (two fp16) per lane, a zero point at the same index as its scale
    uint32_t sk = reinterpret_cast<const uint32_t*>(meta)[lane];
    uint32_t sv = reinterpret_cast<const uint32_t*>(meta + 512)[lane];
    uint32_t zk = 0u, zv = 0u;
    if constexpr (STRAT == KVQ_SHIFT_MODIFIED_) {
        zk = reinterpret_cast<const uint32_t*>(meta + 256)[lane];
        zv = reinterpret_cast<const uint32_t*>(meta + 768)[lane];
    }
#pragma unroll
    for (int kv = 0; kv < 2; ++kv) {
        uint32_t in[4 * B];
        load_chunks_stream<2 * B>(src + kv * (512u * 2 * B), lane, in);
        uint32_t out[2 * B];
#pragma unroll
        for (int d = 0; d < 2 * B; ++d) {
            if constexpr (B == 8) {  // source: high-byte plane in[0..15], low-byte plane in[16..31]
                if constexpr (STRAT == KVQ_SHIFT_EQUIVALENT_) out[d] = shrink_16_to_8(in[d], in[16 + d]);
                else out[d] = in[d];
            } else if constexpr (STRAT == KVQ_SHIFT_EQUIVALENT_) {
                if constexpr (B == 2) out[d] = shrink_4_to_2(in[2 * d]) | (shrink_4_to_2(in[2 * d + 1]) << 16);
                else out[d] = shrink_8_to_4(in[2 * d]) | (shrink_8_to_4(in[2 * d + 1]) << 16);
            } else {
                if constexpr (B == 2) out[d] = trunc_4_to_2(in[2 * d]) | (trunc_4_to_2(in[2 * d + 1]) << 16);
                else out[d] = trunc_8_to_4(in[2 * d]) | (trunc_8_to_4(in[2 * d + 1]) << 16);
            }
        }
        store_chunks_stream<B>(dst + kv * (512u * B), lane, out);
    }
    const float f = STRAT == KVQ_SHIFT_MODIFIED_ ? (float)(1 << B) : (float)((1 << B) + 1);
    uint32_t nk = 0u, nv = 0u, nzk = 0u, nzv = 0u;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float s_k = h2f((uint16_t)(sk >> (16 * h))), s_v = h2f((uint16_t)(sv >> (16 * h)));
        const float nk32 = s_k * f, nv32 = s_v * f;
        nk |= (uint32_t)f2h_rn(nk32) << (16 * h);
        nv |= (uint32_t)f2h_rn(nv32) << (16 * h);
        if constexpr (STRAT == KVQ_SHIFT_MODIFIED_) {
            const float hk = 0.5f * (nk32 - s_k), hv = 0.5f * (nv32 - s_v);  // exact
            nzk |= (uint32_t)f2h_rn(h2f((uint16_t)(zk >> (16 * h))) + hk) << (16 * h);
            nzv |= (uint32_t)f2h_rn(h2f((uint16_t)(zv >> (16 * h))) + hv) << (16 * h);
        }
    }
    reinterpret_cast<uint32_t*>(meta)[lane] = nk;
    reinterpret_cast<uint32_t*>(meta + 512)[lane] = nv;
    if constexpr (STRAT == KVQ_SHIFT_MODIFIED_) {
        reinterpret_cast<uint32_t*>(meta + 256)[lane] = nzk;
        reinterpret_cast<uint32_t*>(meta + 768)[lane] = nzv;
    }
    note_large_v_scale(flags, 1, (uint16_t)(nv & 0xffff));
    note_large_v_scale(flags, 1, (uint16_t)(nv >> 16));
}

// --------------------------------------------------------------------------------- reconstruction error
// grid.x = 2 * tiles (even: K tile, odd: V tile), grid.y = unit, 64 threads.  Over the tile's stored tokens, with
// x_hat = code * S + Z (or the raw value of a 16-bit tile) and x the reference fp16 tensor [unit][token][128]:
//   L1 = false: adds (x_hat - x)^2                       into err[0] (K) or err[1] (V)
//   L1 = true:  adds |g * (x_hat - x)| (g = 1 if no gradient tensor [unit][token][128] fp32 is given), the terms
//               of the sensitivity of Sec. 3.2, Eq. 5
// fp32 inside a tile, fp64 across tiles.
template <bool L1>
__global__ __launch_bounds__(64) void kvq_error_kernel(const uint8_t* __restrict__ arena,
                                                       const KvqPageDesc* __restrict__ table,
                                                       const uint16_t* __restrict__ k_ref,
                                                       const uint16_t* __restrict__ v_ref,
                                                       const float* __restrict__ gk, const float* __restrict__ gv,
                                                       int n_tokens, int tpp, double* __restrict__ err) {
    const int lane = threadIdx.x, j = lane >> 4, n = lane & 15;
    const int which = blockIdx.x & 1, tile = blockIdx.x >> 1, unit = blockIdx.y;
    const int page = tile / tpp, tip = tile - page * tpp;
    const KvqPageDesc pd = table[page];
    const int B = (int)pd.bits;
    const uint64_t tslot = (uint64_t)unit * tpp + tip;
    const uint8_t* code = arena + (uint64_t)pd.code_off256 * 256u + (tslot * 2 + which) * (512u * (uint32_t)B);
    const uint16_t* meta = reinterpret_cast<const uint16_t*>(arena + (uint64_t)pd.meta_off256 * 256u +
                                                             tslot * KVQ_META_TILE_BYTES);
    const uint64_t unit_base = (uint64_t)unit * n_tokens * KVQ_D;
    const uint16_t* ref = (which ? v_ref : k_ref) + unit_base;
    const float* grad = which ? gv : gk;
    const int tok0 = tile * KVQ_TILE_TOKENS;
    float acc = 0.f;
    for (int slot = 0; slot < 64; ++slot) {
        int t, d, g;
        if (!which) {
            const int p = slot >> 3, i = slot & 7, sub = p >> 2;
            g = p & 3;
            t = 8 * (n >> 2) + 4 * sub + (n & 3);
            d = 32 * g + 8 * j + i;
        } else {
            const int nt = slot >> 3, i = slot & 7;
            t = 8 * j + i;
            d = 16 * nt + n;
            g = d >> 5;
        }
        if (tok0 + t >= n_tokens) continue;
        const uint32_t bit = (uint32_t)slot * (uint32_t)B;
        const uint8_t* at = code + kvq_tile_byte(lane, bit >> 3);
        // x_hat - x = code * S + (Z - x): the difference of two fp16 numbers is exact in fp32 and the fused
        // multiply-add rounds once, so large codes times large scales lose nothing before the subtraction
        const uint64_t at_ref = (uint64_t)(tok0 + t) * KVQ_D + d;
        const float x = h2f(ref[at_ref]);
        const int mi = which ? 256 + kvq_vmeta_index(t, g) : t * 4 + g;
        float dx;
        if (B == 16 && pd.int16) {  // byte planes: slot s of the lane's high-byte string, then of its low-byte string
            const uint32_t c = ((uint32_t)code[kvq_tile_byte(lane, (uint32_t)slot)] << 8) |
                               (uint32_t)code[512u * 8 + kvq_tile_byte(lane, (uint32_t)slot)];
            dx = fmaf((float)c, h2f(meta[mi]), h2f(meta[mi + 128]) - x);
        } else if (B == 16) {
            dx = h2f(*reinterpret_cast<const uint16_t*>(at)) - x;
        } else {
            const uint32_t c = ((uint32_t)*at >> (bit & 7u)) & ((1u << B) - 1u);
            dx = fmaf((float)c, h2f(meta[mi]), h2f(meta[mi + 128]) - x);
        }
        if (L1) acc += fabsf(grad ? grad[unit_base + at_ref] * dx : dx);
        else acc += dx * dx;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) atomicAdd(&err[which], (double)acc);
}

// ------------------------------------------------------------------------ channel-wise reparameterization
// dst[0 .. n) = lambda, dst[n .. 2n) = 1 / lambda (one correctly rounded fp32 division per channel).
__global__ void kvq_reparam_store_kernel(const float* __restrict__ lambda, float* __restrict__ dst, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { const float l = lambda[i]; dst[i] = l; dst[n + i] = 1.0f / l; }
}
// Eq. 8, first half: acc[h][i] = max over sequences and tokens of |K|.  grid (n_kv_heads, slices), 128 threads
// (one channel each); acc holds float bit patterns of non-negative values, whose unsigned order is their order.
__global__ __launch_bounds__(128) void kvq_absmax_kernel(const uint16_t* __restrict__ k, int batch, int n_kv_heads,
                                                         int n_tokens, uint32_t* __restrict__ acc) {
    const int h = blockIdx.x, c = threadIdx.x;
    float m = 0.f;
    const long rows = (long)batch * n_tokens;
    for (long r = blockIdx.y; r < rows; r += gridDim.y) {
        const long bb = r / n_tokens, t = r - bb * n_tokens;
        m = fmaxf(m, fabsf(h2f(k[((bb * n_kv_heads + h) * n_tokens + t) * KVQ_D + c])));
    }
    atomicMax(&acc[h * KVQ_D + c], __float_as_uint(m));
}
// Eq. 8, second half, in place: lambda = max(absmax, floor)^alpha, pow in fp64, rounded to fp32.
__global__ void kvq_lambda_pow_kernel(float* __restrict__ lam, int n, float alpha, float floor_) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) lam[i] = (float)pow((double)fmaxf(lam[i], floor_), (double)alpha);
}

// Plain streaming read (16 bytes per lane, 4 non-temporal loads in flight): the practical HBM read ceiling of the device,
// against which the attention kernel's bandwidth is put next to the published peak.
__global__ __launch_bounds__(256) void kvq_stream_read_kernel(const u32x4* __restrict__ p, size_t n,
                                                              uint32_t* __restrict__ sink) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 3 * stride < n; i += 4 * stride) {
        u32x4 a = __builtin_nontemporal_load(p + i), b = __builtin_nontemporal_load(p + i + stride);
        u32x4 c = __builtin_nontemporal_load(p + i + 2 * stride), d = __builtin_nontemporal_load(p + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n; i += stride) acc ^= __builtin_nontemporal_load(p + i);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1u;  // practically never: keeps the loads alive
}

__global__ void kvq_fill_u32_kernel(uint32_t* dst, uint32_t value, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

}  // namespace

hipError_t kvq_launch_append(int bits, uint8_t* arena, const KvqPageDesc* table, const void* k_in,
                             const void* v_in, int t_old, int n_new, int tiles_per_page, int units,
                             const KvqPageDesc* first_two, int first_page, uint32_t* flags, int group,
                             const float* rinv, int n_kv_heads, const float* rope, bool int16, hipStream_t s) {
    const int gspan = group / KVQ_G;
    int tile0 = t_old / KVQ_TILE_TOKENS;
    int tile1 = (t_old + n_new + KVQ_TILE_TOKENS - 1) / KVQ_TILE_TOKENS;
    dim3 grid(2 * (tile1 - tile0), units), block(64);
    const int n_strings = 2 * (tile1 - tile0);
    const dim3 qgrid((n_strings + KVQ_APPEND_WG_WAVES - 1) / KVQ_APPEND_WG_WAVES, units), qblock(64 * KVQ_APPEND_WG_WAVES);
    const uint16_t* k = static_cast<const uint16_t*>(k_in);
    const uint16_t* v = static_cast<const uint16_t*>(v_in);
    KvqAppendPages ap;
    ap.first_page = first_two ? first_page : -1;
    ap.d[0] = first_two ? first_two[0] : KvqPageDesc{0, 0, 0, 0};
    ap.d[1] = first_two ? first_two[1] : KvqPageDesc{0, 0, 0, 0};
    switch (bits + (int16 && bits == 16 ? 1 : 0)) {
        case 17: hipLaunchKernelGGL(kvq_append_i16_kernel, grid, block, 0, s, arena, table, k, v, t_old, n_new, tiles_per_page, tile0, ap, gspan, rinv, n_kv_heads, rope); break;
        case 16: hipLaunchKernelGGL(kvq_append16_kernel, grid, block, 0, s, arena, table, k, v, t_old, n_new, tiles_per_page, tile0, ap, rinv, n_kv_heads, rope); break;
        case 8:
            if (!rinv && !rope) hipLaunchKernelGGL((kvq_append_q_kernel<8, true>), qgrid, qblock, 0, s, arena, table, k, v, t_old, n_new, tiles_per_page, tile0, ap, flags, gspan, rinv, n_kv_heads, rope, n_strings);
            else hipLaunchKernelGGL((kvq_append_q_kernel<8, false>), qgrid, qblock, 0, s, arena, table, k, v, t_old, n_new, tiles_per_page, tile0, ap, flags, gspan, rinv, n_kv_heads, rope, n_strings);
            break;
        case 4:
            if (!rinv && !rope) hipLaunchKernelGGL((kvq_append_q_kernel<4, true>), qgrid, qblock, 0, s, arena, table, k, v, t_old, n_new, tiles_per_page, tile0, ap, flags, gspan, rinv, n_kv_heads, rope, n_strings);
            else hipLaunchKernelGGL((kvq_append_q_kernel<4, false>), qgrid, qblock, 0, s, arena, table, k, v, t_old, n_new, tiles_per_page, tile0, ap, flags, gspan, rinv, n_kv_heads, rope, n_strings);
            break;
        case 2:
            if (!rinv && !rope) hipLaunchKernelGGL((kvq_append_q_kernel<2, true>), qgrid, qblock, 0, s, arena, table, k, v, t_old, n_new, tiles_per_page, tile0, ap, flags, gspan, rinv, n_kv_heads, rope, n_strings);
            else hipLaunchKernelGGL((kvq_append_q_kernel<2, false>), qgrid, qblock, 0, s, arena, table, k, v, t_old, n_new, tiles_per_page, tile0, ap, flags, gspan, rinv, n_kv_heads, rope, n_strings);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

static void fill_job_args(KvqJobArgs& ja, const KvqRequantJob* jobs_host, int n_jobs) {
    ja.n = (jobs_host && n_jobs <= KVQ_JOBS_BY_ARG) ? n_jobs : 0;
    ja.pad[0] = ja.pad[1] = ja.pad[2] = 0;
    for (int i = 0; i < ja.n; ++i) ja.jobs[i] = jobs_host[i];
}

// jobs_host != nullptr and n_jobs <= KVQ_JOBS_BY_ARG: the list travels in the kernel arguments and jobs_dev is
// not read; otherwise jobs_dev must already hold the list (in stream order).
hipError_t kvq_launch_shrink(int dst_bits, int strategy, uint8_t* arena, const KvqRequantJob* jobs_dev,
                             const KvqRequantJob* jobs_host, int n_jobs, int tiles_per_page, int units,
                             uint32_t* flags, hipStream_t s) {
    dim3 grid(n_jobs * tiles_per_page, units), block(64);
    KvqJobArgs ja;
    fill_job_args(ja, jobs_host, n_jobs);
#define KVQ_SHRINK_CASE(B_, S_) \
    hipLaunchKernelGGL((kvq_shrink_kernel<B_, S_>), grid, block, 0, s, arena, jobs_dev, tiles_per_page, flags, ja)
    switch (dst_bits * 4 + strategy) {
        case 8 * 4 + 0: KVQ_SHRINK_CASE(8, 0); break;
        case 8 * 4 + 1: KVQ_SHRINK_CASE(8, 1); break;
        case 8 * 4 + 2: KVQ_SHRINK_CASE(8, 2); break;
        case 4 * 4 + 0: KVQ_SHRINK_CASE(4, 0); break;
        case 4 * 4 + 1: KVQ_SHRINK_CASE(4, 1); break;
        case 4 * 4 + 2: KVQ_SHRINK_CASE(4, 2); break;
        case 2 * 4 + 0: KVQ_SHRINK_CASE(2, 0); break;
        case 2 * 4 + 1: KVQ_SHRINK_CASE(2, 1); break;
        case 2 * 4 + 2: KVQ_SHRINK_CASE(2, 2); break;
        default: return hipErrorInvalidValue;
    }
#undef KVQ_SHRINK_CASE
    return hipGetLastError();
}

hipError_t kvq_launch_error(bool l1, const uint8_t* arena, const KvqPageDesc* table, const void* k_ref,
                            const void* v_ref, const float* gk, const float* gv, int n_tokens, int tiles_per_page,
                            int units, double* err, hipStream_t s) {
    const int n_tiles = (n_tokens + KVQ_TILE_TOKENS - 1) / KVQ_TILE_TOKENS;
    const dim3 grid(2 * n_tiles, units), block(64);
    const uint16_t* k = static_cast<const uint16_t*>(k_ref);
    const uint16_t* v = static_cast<const uint16_t*>(v_ref);
    if (l1) hipLaunchKernelGGL(kvq_error_kernel<true>, grid, block, 0, s, arena, table, k, v, gk, gv, n_tokens, tiles_per_page, err);
    else hipLaunchKernelGGL(kvq_error_kernel<false>, grid, block, 0, s, arena, table, k, v, gk, gv, n_tokens, tiles_per_page, err);
    return hipGetLastError();
}

hipError_t kvq_launch_quant16(int dst_bits, uint8_t* arena, const KvqRequantJob* jobs_dev,
                              const KvqRequantJob* jobs_host, int n_jobs, int tiles_per_page, int units,
                              uint32_t* flags, int group, hipStream_t s) {
    dim3 grid(2 * n_jobs * tiles_per_page, units), block(64);
    KvqJobArgs ja;
    fill_job_args(ja, jobs_host, n_jobs);
    switch (dst_bits) {
        case 8: hipLaunchKernelGGL(kvq_quant16_kernel<8>, grid, block, 0, s, arena, jobs_dev, tiles_per_page, flags, group / KVQ_G, ja); break;
        case 4: hipLaunchKernelGGL(kvq_quant16_kernel<4>, grid, block, 0, s, arena, jobs_dev, tiles_per_page, flags, group / KVQ_G, ja); break;
        case 2: hipLaunchKernelGGL(kvq_quant16_kernel<2>, grid, block, 0, s, arena, jobs_dev, tiles_per_page, flags, group / KVQ_G, ja); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t kvq_launch_reparam_store(const float* lambda, float* dst, int n, hipStream_t s) {
    hipLaunchKernelGGL(kvq_reparam_store_kernel, dim3((n + 255) / 256), dim3(256), 0, s, lambda, dst, n);
    return hipGetLastError();
}

hipError_t kvq_launch_calibrate(const void* k, int batch, int n_kv_heads, int n_tokens, float alpha, float floor_,
                                float* lambda, hipStream_t s) {
    const int n = n_kv_heads * KVQ_D;
    hipLaunchKernelGGL(kvq_fill_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, reinterpret_cast<uint32_t*>(lambda), 0u, (size_t)n);
    const long rows = (long)batch * n_tokens;
    const int slices = (int)(rows < 1024 ? rows : 1024);
    hipLaunchKernelGGL(kvq_absmax_kernel, dim3(n_kv_heads, slices), dim3(128), 0, s, static_cast<const uint16_t*>(k),
                       batch, n_kv_heads, n_tokens, reinterpret_cast<uint32_t*>(lambda));
    hipLaunchKernelGGL(kvq_lambda_pow_kernel, dim3((n + 255) / 256), dim3(256), 0, s, lambda, n, alpha, floor_);
    return hipGetLastError();
}

hipError_t kvq_launch_stream_read(const void* buf, size_t bytes, int n_workgroups, uint32_t* sink, hipStream_t s) {
    hipLaunchKernelGGL(kvq_stream_read_kernel, dim3((unsigned)n_workgroups), dim3(256), 0, s,
                       static_cast<const u32x4*>(buf), bytes / 16, sink);
    return hipGetLastError();
}

hipError_t kvq_launch_fill_u32(uint32_t* dst, uint32_t value, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(kvq_fill_u32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, value, n);
    return hipGetLastError();
}
