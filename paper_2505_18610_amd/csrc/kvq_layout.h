// Device layout of the packed KV cache, shared by the host bookkeeping and the HIP kernels.
//
// A *tile* is 32 consecutive tokens x 128 channels of K (or of V) of one (sequence, KV head).  Its 4096
// elements are spread over the 64 lanes of a wavefront, 64 *slots* per lane, in exactly the arrangement in
// which v_mfma_f32_16x16x32_f16 wants its operands, so the attention kernel streams a tile with 16-byte
// loads and feeds the matrix cores without any cross-lane movement:
//
//   lane = 16*j + n   (j = 0..3, n = 0..15)
//   K: slot s = (sub*4 + grp)*8 + i   <->  token 8*(n/4) + 4*sub + (n%4),  channel 32*grp + 8*j + i
//        (scores = K q^T: A operand row n of sub-tile `sub`, k-range of lane quarter j inside group grp)
//   V: slot s = nt*8 + i              <->  token 8*j + i,                   channel 16*nt + n
//        (out^T = V^T p^T: A operand row n of channel block nt, k-range = the 8 tokens of quarter j; these
//         are exactly the tokens whose scores the same lane quarter holds after the K product)
//
// A lane's 64 slots are packed little-endian, b bits each (raw fp16 for b = 16), into 8*b bytes; that string
// is cut into 16-byte chunks and chunk c of lane l is stored at byte (c*64 + l)*16 of the tile, so every
// 16-byte load of a wavefront is one contiguous kilobyte.  A tile of width b takes 512*b bytes.
//
// A tile of the integer 16-bit tier (16-bit codes with scales and zero points, the INT16 format of Sec. 4.1.2)
// is two 8-bit tiles back to back: first the high bytes of the 64 codes of every lane, laid out exactly like an
// 8-bit tile (4 KiB), then the low bytes (4 KiB).  Bytes are exact fp16 integers, so the matrix cores can take
// the two planes separately, and the Direct and Modified Right Shift to 8 bits are a copy of the first plane.
//
// Per tile 1 KiB of metadata (fp16), quantized widths and the integer 16-bit tier only:
//   [   0, 256) K scales  S[token][grp]            [ 256, 512) K zero points, same order
//   [ 512, 768) V scales  S[grp][8*j + 2*v + hi]  for token 8*j + v + 4*hi   (the pairing of MFMA operand
//   [ 768,1024) V zero points, same order           registers: register v holds slots v and v+4)
//
// A *page* is page_tokens tokens of all (sequence, KV head) units at one width: a code block
// [unit][tile]{K tile, V tile} and, for quantized widths, a metadata block [unit][tile]{1 KiB}.
#ifndef KVQ_LAYOUT_H
#define KVQ_LAYOUT_H

#include <stdint.h>

#define KVQ_D 128
#define KVQ_G 32
#define KVQ_NGRP 4
#define KVQ_TILE_TOKENS 32
#define KVQ_META_TILE_BYTES 1024
#define KVQ_MAX_SPLITS 128
#define KVQ_MAX_GQA 16

#if defined(__HIPCC__)
#define KVQ_HD __host__ __device__ inline
#else
#define KVQ_HD inline
#endif

struct KvqPageDesc {       // one entry of a block's device page table
    uint32_t code_off256;  // code block offset from the arena base, in 256-byte units
    uint32_t meta_off256;  // metadata block offset, in 256-byte units (unused for raw fp16 pages)
    uint32_t bits;         // 16, 8, 4, 2
    uint32_t int16;        // 1: a 16-bit page of the integer tier (two byte planes and metadata); else 0
};

KVQ_HD uint32_t kvq_tile_code_bytes(int bits) { return 512u * (uint32_t)bits; }   // one K or V tile

// K element (token t in tile, channel d) -> lane, slot
KVQ_HD void kvq_k_slot(int t, int d, int* lane, int* slot) {
    int hi = t >> 3, sub = (t >> 2) & 1, lo = t & 3;
    int n = hi * 4 + lo;
    int grp = d >> 5, j = (d >> 3) & 3, i = d & 7;
    *lane = j * 16 + n;
    *slot = (sub * 4 + grp) * 8 + i;
}
// V element (token t in tile, channel d) -> lane, slot
KVQ_HD void kvq_v_slot(int t, int d, int* lane, int* slot) {
    int j = t >> 3, i = t & 7;
    int nt = d >> 4, n = d & 15;
    *lane = j * 16 + n;
    *slot = nt * 8 + i;
}
// byte offset inside a tile of the byte holding bit `bitpos` of lane's packed string
KVQ_HD uint32_t kvq_tile_byte(int lane, uint32_t string_byte) {
    return ((string_byte >> 4) * 64u + (uint32_t)lane) * 16u + (string_byte & 15u);
}
// index (in fp16 elements) of token t's entry for group g inside the V scale / zero-point block of a tile
KVQ_HD int kvq_vmeta_index(int t, int g) {
    int j = t >> 3, i = t & 7;
    return g * 32 + j * 8 + (i & 3) * 2 + (i >> 2);
}

#endif
