// Internal interface between the host bookkeeping (kvq_host.cpp) and the kernel translation units.
#ifndef KVQ_INTERNAL_H
#define KVQ_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>
#include "kvq_layout.h"

struct KvqRequantJob {        // one page to re-quantize
    uint32_t src_code_off256; // source code block
    uint32_t dst_code_off256; // destination code block
    uint32_t meta_off256;     // metadata block (updated in place for 2b -> b, written for fp16 -> b)
    uint32_t n_tiles;         // tiles of the page that hold tokens; the kernels leave the others alone
};

// Up to KVQ_JOBS_BY_ARG jobs ride in the kernel arguments (no table upload in front of the launch);
// longer lists are read from the uploaded table.
#define KVQ_JOBS_BY_ARG 192
struct KvqJobArgs {
    int32_t n;  // 0: read the table
    int32_t pad[3];
    KvqRequantJob jobs[KVQ_JOBS_BY_ARG];
};

struct KvqAttnParams {
    const uint8_t* arena;
    const KvqPageDesc* table;  // this block's page table
    const void* q;             // fp16 [batch, n_q_heads, 128]
    const float* lambda;       // [n_kv_heads][128] reparameterization factors applied to q at load, or null
    void* out;                 // [batch, n_q_heads, 128] fp16 or fp32
    float* part_o;             // [unit][split][16][128] un-normalised partial outputs
    float* part_ml;            // [unit][split][16] pairs (running max in log2 units, sum)
    uint32_t* counters;        // [unit] arrival counters of the fused merge (kept at zero between launches)
    const uint32_t* flags;     // [0] bit 0: some V scale of the cache is >= 256 (set by the quantizing kernels)
    int32_t n_tokens;
    int32_t tiles_per_page;
    uint32_t tpp_magic;        // ceil(2^32 / tiles_per_page) (unused when tiles_per_page == 1)
    int32_t gqa;               // query heads per KV head
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t n_splits;
    int32_t out_fp32;
    int32_t fused_merge;
    int32_t deterministic;     // 1: static chunk-to-wavefront assignment (bit-reproducible summation order)
    int32_t int16_tier;        // 1: 16-bit pages hold integer codes in byte planes (selects the kernel)
    float scale_log2;          // softmax scale * log2(e)
    int32_t split_begin[KVQ_MAX_SPLITS + 1];  // tile index where each split starts
    // a one-token append into the 16-bit tier done by the workgroup that owns the last tile (app_t_old < 0: none)
    int32_t app_t_old;         // tokens before the append; n_tokens already counts the new one
    KvqPageDesc app_desc;      // page of the new token
    const void* app_k;         // fp16 [batch, n_kv_heads, 1, 128]
    const void* app_v;
    const float* app_rope;     // [1][128] cos | sin of the new position, or null
    const float* app_rinv;     // [n_kv_heads][128] reciprocal reparameterization factors, or null
    int32_t app_gspan;         // quantization group / 32 (integer 16-bit tier: the new token is quantized, Eq. 1-2)
};

// kvq_quant.hip
// One append call takes fewer than 2^23 tokens per sequence: the kernels address the rows of a unit's input through a
// buffer descriptor with 32-bit byte offsets (256 bytes per row; offsets up to a few tiles beyond the last row occur).
#define KVQ_MAX_APPEND_TOKENS (1 << 23)
hipError_t kvq_launch_append(int bits, uint8_t* arena, const KvqPageDesc* table, const void* k_in,
                             const void* v_in, int t_old, int n_new, int tiles_per_page, int units,
                             const KvqPageDesc* first_two, int first_page, uint32_t* flags, int group,
                             const float* rinv, int n_kv_heads, const float* rope, bool int16, hipStream_t s);
hipError_t kvq_launch_shrink(int dst_bits, int strategy, uint8_t* arena, const KvqRequantJob* jobs_dev,
                             const KvqRequantJob* jobs_host, int n_jobs, int tiles_per_page, int units,
                             uint32_t* flags, hipStream_t s);
hipError_t kvq_launch_quant16(int dst_bits, uint8_t* arena, const KvqRequantJob* jobs_dev,
                              const KvqRequantJob* jobs_host, int n_jobs, int tiles_per_page, int units,
                              uint32_t* flags, int group, hipStream_t s);
hipError_t kvq_launch_reparam_store(const float* lambda, float* dst, int n, hipStream_t s);
hipError_t kvq_launch_calibrate(const void* k, int batch, int n_kv_heads, int n_tokens, float alpha, float floor_,
                                float* lambda, hipStream_t s);
hipError_t kvq_launch_error(bool l1, const uint8_t* arena, const KvqPageDesc* table, const void* k_ref,
                            const void* v_ref, const float* gk, const float* gv, int n_tokens, int tiles_per_page,
                            int units, double* err, hipStream_t s);
hipError_t kvq_launch_stream_read(const void* buf, size_t bytes, int n_workgroups, uint32_t* sink, hipStream_t s);
hipError_t kvq_launch_fill_u32(uint32_t* dst, uint32_t value, size_t n, hipStream_t s);

// A ragged batch: several caches (each with its own length, widths and tables) served by one attention launch.  The
// parameter blocks sit in device memory; the map tells a workgroup which cache it works for.
#define KVQ_MAX_BATCH_CACHES 64
struct KvqBatchMap {
    int32_t n;
    int32_t wg_begin[KVQ_MAX_BATCH_CACHES + 1];  // first workgroup of every cache; [n] = grid size
};

// Static scratch of kvq_decode_attention_static (kvq_attention.hip): room for the partials of KVQ_STATIC_MAX_WGS
// workgroups (units * splits of one launch) and the arrival counters of KVQ_STATIC_MAX_UNITS units.
#define KVQ_STATIC_MAX_WGS 512
#define KVQ_STATIC_MAX_UNITS 4096
#define KVQ_STATIC_PART_O_BYTES ((size_t)KVQ_STATIC_MAX_WGS * 16 * KVQ_D * sizeof(float))
#define KVQ_STATIC_PART_ML_BYTES ((size_t)KVQ_STATIC_MAX_WGS * 32 * sizeof(float))
#define KVQ_STATIC_COUNTER_BYTES ((size_t)KVQ_STATIC_MAX_UNITS * sizeof(uint32_t))
#define KVQ_STATIC_SCRATCH_BYTES (KVQ_STATIC_PART_O_BYTES + KVQ_STATIC_PART_ML_BYTES + KVQ_STATIC_COUNTER_BYTES)
// Device address of the scratch array on the current device (looked up once per device, no allocation).
hipError_t kvq_static_scratch(unsigned char** ptr);

// kvq_attention.hip
hipError_t kvq_launch_attention(const KvqAttnParams& p, int units, hipStream_t s);
hipError_t kvq_launch_merge(const KvqAttnParams& p, int units, hipStream_t s);
hipError_t kvq_launch_attention_i16_append(const KvqAttnParams& p, int units, hipStream_t s);  // kernel only, no merge
// kvq_attention_batch.hip: the bare kernel launch kvq_launch_attention_batch wraps
hipError_t kvq_launch_attention_batch_kernel(const KvqAttnParams* params_dev, const KvqBatchMap& map, bool int16,
                                             hipStream_t s);
// params_dev: the n parameter blocks in device memory (in stream order); params_host: the same blocks on the host;
// units[i]: (sequence, KV head) units of cache i
hipError_t kvq_launch_attention_batch(const KvqAttnParams* params_dev, const KvqAttnParams* params_host,
                                      const int* units, int n, hipStream_t s);

#endif
