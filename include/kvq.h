/*
 * kvq.h -- C ABI of libkvq: decode attention over a progressively quantized KV cache on AMD MI355X (gfx950).
 *
 * The library implements the online half of PM-KVQ (arXiv 2505.18610): tokens enter a transformer block's
 * KV cache at 16 bits; when the block's byte budget would be exceeded the bit-width of the existing cache
 * is halved, 16 -> 8 -> 4 -> 2, never below the block's final bit-width "Fbit" (Sec. 3.1); single-token
 * grouped-query attention reads the mixed-width cache directly.
 *
 * Conventions for every entry point
 *   - Pointers named *_dev are device (HIP) pointers, *_host are host pointers.  No entry point takes or
 *     returns a framework type.
 *   - The caller owns the arena, the q/k/v/out buffers and the stream.  The library owns the kvq_cache_t
 *     (host tables) and sub-allocates inside the arena; it never allocates or frees device memory.
 *   - Every kernel is enqueued on the given HIP stream (hipStream_t passed as void*, NULL = default stream).
 *     No entry point waits for the stream, except the three that copy results to the host
 *     (kvq_cache_export_segment, kvq_cache_sq_error, kvq_cache_sensitivity).  Small host-to-device uploads (page
 *     tables, job lists, the parameter blocks of a ragged batch) travel through a pinned staging ring of 4 segments of
 *     1 MiB whose reuse is guarded by one HIP event per segment: a call blocks the host only when it has run a whole
 *     ring of uploads ahead of the device, and then only until the oldest segment has been consumed.
 *   - Stream capture: kvq_decode_attention and kvq_decode_attention_static enqueue kernels only and may be captured
 *     into a HIP graph (the cache must not change between capture and replay).  Calls that change a cache or stage
 *     parameter blocks (append, requant, the *_batch calls, set_reparam) use the staging ring and its events and must
 *     not be captured.
 *   - All calls on one cache must be issued from one thread at a time and on one stream (the host tables
 *     are updated at enqueue time, the device tables in stream order).
 *   - Errors are reported as kvq_status_t; argument, state and budget errors are detected on the host before
 *     anything is enqueued and leave the cache unchanged.  Nothing throws or aborts across this boundary.
 *     KVQ_E_OOM of an append is found before anything changes as well (the blocks of the new pages and those that
 *     pages leaving the window are quantized into are taken first).  A HIP failure (KVQ_E_HIP) while a call is
 *     being enqueued can strike after the host tables have been updated; the block is then marked unusable: every
 *     later call on it returns KVQ_E_STATE until kvq_cache_reset empties it (other blocks are unaffected).
 *   - All sequences of one cache have the same length and share one page table per block; sequences of different
 *     lengths live in caches of their own and are served together by the *_batch entry points.
 *   - head_dim is 128, group is 32, 64 or 128 channels (128 is the paper's setting, Sec. 4.1.2),
 *     1 <= n_q_heads / n_kv_heads <= 16.
 */
#ifndef KVQ_H
#define KVQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvq_cache kvq_cache_t;

typedef enum {
    KVQ_OK = 0,
    KVQ_E_INVALID = 1, /* null pointer, bad shape, bits not in {16,8,4,2}, unsupported config            */
    KVQ_E_BUDGET = 2,  /* the append would exceed the block's byte budget (nothing was written), or a    */
                       /* shrink was asked for but the policy has nothing left to lower above Fbit        */
    KVQ_E_OOM = 3,     /* the arena has no free block of the needed size                                  */
    KVQ_E_STATE = 4,   /* the call does not fit the cache state (width change inside a page, max_tokens   */
                       /* exceeded, no such segment, compute call on an accounting-only cache)            */
    KVQ_E_HIP = 5,     /* a HIP runtime call or kernel launch failed                                      */
    KVQ_E_LIMIT = 6    /* kvq_decode_attention_static: the launch needs more than the library's static scratch */
} kvq_status_t;

enum { KVQ_POLICY_PAPER = 0, KVQ_POLICY_OLDEST_FIRST = 1 };
enum { KVQ_WHICH_K = 0, KVQ_WHICH_V = 1 };

typedef struct {
    int32_t n_layers;      /* transformer blocks sharing the arena                                        */
    int32_t batch;         /* sequences (all of equal length)                                             */
    int32_t n_q_heads;     /* query heads; query head h reads KV head h / (n_q_heads / n_kv_heads)        */
    int32_t n_kv_heads;
    int32_t head_dim;      /* must be 128                                                                 */
    int32_t group;         /* quantization group: consecutive channels of one token of one head; 32 | 64 | 128 */
    int32_t max_tokens;    /* maximum context length per sequence                                         */
    int32_t window;        /* most recent tokens kept at 16 bits (Sec. 4.1.2); multiple of page_tokens    */
    int32_t n_sink;        /* first tokens kept at 16 bits (Sec. 4.1.2); multiple of page_tokens          */
    int32_t page_tokens;   /* bookkeeping and allocation granularity in tokens; multiple of 32            */
    int32_t policy;        /* KVQ_POLICY_*                                                                */
    int32_t count_metadata_in_budget; /* 1: scales and zero points count toward the byte budget           */
} kvq_config_t;

typedef struct {
    int32_t token_begin;   /* first token of the run                                                      */
    int32_t token_end;     /* one past its last token                                                     */
    int32_t bits;          /* 16, 8, 4 or 2                                                               */
} kvq_segment_info_t;

/* Arena size (bytes) that holds the library's device tables plus `payload_bytes` of cache pages.
 * payload_bytes is rounded up to whole allocation blocks.  Returns 0 on an invalid config. */
uint64_t kvq_arena_bytes(const kvq_config_t* cfg, uint64_t payload_bytes);

/* Bytes one cached token of one KV head occupies at `bits`, K and V together (codes, plus one fp16
 * scale/zero pair per group for K and for V when count_metadata != 0; 16-bit tokens carry such pairs only when
 * int16_tier != 0, see KVQ_OPT_TIER16).  This is the Mem(.) of Sec. 3.2 as the library accounts it.  Returns 0 for
 * bits outside {16,8,4,2}. */
uint64_t kvq_bytes_per_token_head(int32_t bits, int32_t head_dim, int32_t group, int32_t count_metadata,
                                  int32_t int16_tier);

/* Create a cache over a caller-owned device arena (Sec. 3.1: per-block Fbit and byte budget).
 *   block_budget_bytes_host[n_layers], block_fbit_host[n_layers] (each 16, 8, 4 or 2): host arrays, copied.
 *   arena_dev: device memory of arena_bytes bytes, 256-byte aligned; must outlive the cache.  The library
 *   enqueues nothing here; device tables are initialised lazily in stream order.
 *   arena_dev == NULL creates an accounting-only cache: append/requant update the host tables exactly as
 *   they would, launch nothing, and kvq_decode_attention / export return KVQ_E_STATE (capacity planning).
 * Returns KVQ_E_INVALID for an unsupported config, KVQ_E_OOM if the arena cannot hold the device tables. */
kvq_status_t kvq_cache_create(const kvq_config_t* cfg, const uint64_t* block_budget_bytes_host,
                              const uint8_t* block_fbit_host, void* arena_dev, uint64_t arena_bytes,
                              kvq_cache_t** out);

/* Frees the host tables and the pinned staging memory (freeing it makes the HIP runtime wait for the device, so work
 * already enqueued that still reads it completes first); the arena is the caller's. */
void kvq_cache_destroy(kvq_cache_t* cache);

/* Quantize-on-append (Sec. 2.2 Eq. 1-2; Sec. 3.1).
 *   k_dev, v_dev: fp16 [batch, n_kv_heads, n_new, head_dim], contiguous; keys already carry RoPE.
 *   n_new < 2^23 tokens per call (KVQ_E_INVALID beyond; append longer inputs in pieces).
 *   entry_bits: 0 = the policy's entry width (16 while a window is configured or under OLDEST_FIRST, else
 *   the block's current width); 16/8/4/2 = store at exactly that width (state construction).  A width that
 *   differs from the partially filled last page's width is KVQ_E_STATE.
 *   Quantized widths use asymmetric min-max per group: Z = min, S = (max - Z)/(2^b - 1) in fp32 rounded to
 *   fp16, code = rne((x - Z)/S) with the stored S, clamped; S == 0 gives code 0.
 *   Under KVQ_POLICY_PAPER with a window, pages leaving the window are quantized to the block's current
 *   width inside this call.  KVQ_E_BUDGET (cache unchanged) if bytes after the append exceed the budget. */
kvq_status_t kvq_quantize_append(kvq_cache_t* cache, int32_t layer, const void* k_dev, const void* v_dev,
                                 int32_t n_new, int32_t entry_bits, void* hip_stream);

/* kvq_quantize_append for keys that do not carry RoPE yet: the rotation of Sec. 3.3, Eq. 9 (channel i paired with
 * i + 64) is applied to every new key inside the append kernel, before the reparameterization and Eq. 1-2:
 *   K~_i = K_i cos_i - K_{i+64} sin_i,  K~_{i+64} = K_i sin_i + K_{i+64} cos_i    (i = 0..63),
 * each product and the sum a separate fp32 operation, the result rounded to fp16 - exactly what the plain call stores
 * when it is handed keys rotated that way.  cos_sin_dev: device, fp32 [n_new][128]: row r holds cos(m theta_i), i = 0..63,
 * then sin(m theta_i), for the position m of the r-th new token (the caller chooses positions, base and any positional
 * interpolation, Eq. 10).  NULL makes the call identical to kvq_quantize_append.  V is not rotated. */
kvq_status_t kvq_quantize_append_rope(kvq_cache_t* cache, int32_t layer, const void* k_dev, const void* v_dev,
                                      int32_t n_new, int32_t entry_bits, const float* cos_sin_dev, void* hip_stream);

/* Progressive bit-width shrinking (Sec. 3.1 Eq. 3, appendix theorem):
 *   X_b = ((2^2b - 2^b + 1)(X_2b + 2^(b-1))) >> 3b,  S_b = fp16((2^b + 1) S_2b),  Z_b = Z_2b;
 *   pages still holding raw fp16 values are quantized directly to 8 bits (Eq. 1-2), which by the theorem
 *   is what an integer 16-bit tier followed by Eq. 3 would give; with KVQ_TIER16_INT16 the 16-bit pages are that
 *   integer tier and 16 -> 8 is Eq. 3 at b = 8 (multiplier 65281, offset 128, shift 24, in unsigned 32-bit).
 *   segment >= 0: lower every page of that run (kvq_cache_describe order) one step; KVQ_E_STATE if it is
 *   already at 2 bits or does not exist, or if the run ends in the partly filled last page while the policy appends
 *   at 16 bits (OLDEST_FIRST, or a window): that page could take no further token.  Tiles of a partly filled page
 *   that hold no token yet are left untouched.
 *   segment == -1, KVQ_POLICY_PAPER: halve the block's current width: every page at that width outside the
 *   sink and the window is lowered one step.  KVQ_E_BUDGET if the block is already at Fbit.
 *   segment == -1, KVQ_POLICY_OLDEST_FIRST: while bytes_used + reserve_tokens 16-bit tokens exceed the
 *   budget, lower the oldest complete page outside sink/window whose width is above Fbit by one step;
 *   KVQ_E_BUDGET when none is left (steps already taken stay).
 *   *n_pages_done (may be NULL) receives the number of page re-quantizations enqueued. */
kvq_status_t kvq_progressive_requant(kvq_cache_t* cache, int32_t layer, int32_t segment,
                                     int32_t reserve_tokens, void* hip_stream, int32_t* n_pages_done);

/* Single-token GQA decode attention over the block's whole cache (no mask; append the current token first):
 *   out[b, h, :] = softmax_t( q[b, h, :] . K_hat[b, h/g, t, :] * softmax_scale ) V_hat[b, h/g, t, :]
 *   with X_hat = code * S + Z (or the raw fp16 value).  fp16 operands, fp32 accumulation (16-bit codes enter the
 *   matrix cores as their high and low bytes, both exact).
 *   q_dev: fp16 [batch, n_q_heads, head_dim]; out_dev: [batch, n_q_heads, head_dim], fp32 if out_is_fp32
 *   else fp16; softmax_scale 0 means 1/sqrt(head_dim).  KVQ_E_STATE if the block is empty. */
kvq_status_t kvq_decode_attention(kvq_cache_t* cache, int32_t layer, const void* q_dev, void* out_dev,
                                  int32_t out_is_fp32, float softmax_scale, void* hip_stream);

/* kvq_decode_attention for callers that cannot allocate device memory or hand over a workspace at call time -- code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result (to
 * floating-point summation order), same kernels; the split partials and arrival counters of the launch live in a
 * static array of the library's device image (4,276,224 bytes per GPU, held until the process ends) instead of the
 * arena.  The call allocates nothing and frees nothing on host-visible HIP interfaces: it looks the array's device
 * address up once per device (first call on that device), clears the counters with a small fill kernel and launches.
 * Limits: batch * n_kv_heads * splits <= 512 workgroups and batch * n_kv_heads <= 4096, else KVQ_E_LIMIT and nothing is
 * enqueued (the automatic split count never exceeds one workgroup per compute unit; KVQ_OPT_SPLITS can).
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different streams, or
 * different caches on different streams) race; issue them on one stream. */
kvq_status_t kvq_decode_attention_static(kvq_cache_t* cache, int32_t layer, const void* q_dev, void* out_dev,
                                         int32_t out_is_fp32, float softmax_scale, void* hip_stream);

/* One decode step of a block in one launch: kvq_quantize_append_rope of one token (n_new = 1, entry_bits = 0; k_dev,
 * v_dev: fp16 [batch, n_kv_heads, 1, 128]; cos_sin_dev: fp32 [1][128] or NULL for keys that already carry RoPE)
 * followed by kvq_decode_attention over the block including that token.  When the token enters the 16-bit tier
 * (a window is configured, the policy is OLDEST_FIRST, or the block is still at 16 bits) it is written by the attention
 * kernel itself - by the workgroup that owns the last tile, which reads it back only after its stores have
 * completed; with KVQ_TIER16_INT16 that workgroup quantizes it (Eq. 1-2, 2^16 - 1 levels) - so the small append launch
 * and its gap disappear; otherwise the two kernels are launched one after the other.  Bookkeeping, budget check, page allocation and window evictions are those of kvq_quantize_append; the
 * cache contents afterwards are bit-identical to the two separate calls, the outputs equal up to summation order.
 * Errors of the append part leave the cache unchanged and nothing is computed. */
kvq_status_t kvq_append_decode_attention(kvq_cache_t* cache, int32_t layer, const void* k_dev, const void* v_dev,
                                         const float* cos_sin_dev, const void* q_dev, void* out_dev,
                                         int32_t out_is_fp32, float softmax_scale, void* hip_stream);

/* Ragged batches: sequences of different lengths decode together when every sequence (or group of equally long
 * sequences) has a cache of its own -- its own length, widths, budget and shrink history, as the method keeps them per
 * sequence (Sec. 3.1) -- and one launch serves block `layer` of all of them.
 *   caches[n_caches]: host array of distinct caches (1..64) that all use the same kind of 16-bit tier; they may differ
 *   in batch, head counts, page size, length and state.  q_dev[i], out_dev[i], k_dev[i], v_dev[i], cos_sin_dev[i]: host
 *   arrays of device pointers with the shapes the single-cache calls take for caches[i] (cos_sin_dev itself or any of
 *   its entries may be NULL).
 * kvq_decode_attention_batch: kvq_decode_attention of every cache in one launch.
 * kvq_append_decode_attention_batch: kvq_append_decode_attention of every cache -- one new token each, then attention
 *   -- in one attention launch (plus the small append and eviction launches of those caches whose token does not enter
 *   the raw fp16 tier).  The bookkeeping of all appends is checked before the first one is carried out: on
 *   KVQ_E_BUDGET / KVQ_E_STATE no cache has changed.  (An arena that runs out of pages, KVQ_E_OOM, is only found while
 *   carrying them out; caches before the failing one then hold their new token.)
 * The device's workgroups are shared among the caches in proportion to the time their tiles take.  Results per cache
 * are those of the single-cache calls up to floating-point summation order.  The parameter blocks of the launch are
 * read from the pinned staging memory of caches[0]: calls that involve that cache must be issued on one stream. */
kvq_status_t kvq_decode_attention_batch(kvq_cache_t* const* caches, int32_t n_caches, int32_t layer,
                                        const void* const* q_dev, void* const* out_dev, int32_t out_is_fp32,
                                        float softmax_scale, void* hip_stream);
kvq_status_t kvq_append_decode_attention_batch(kvq_cache_t* const* caches, int32_t n_caches, int32_t layer,
                                               const void* const* k_dev, const void* const* v_dev,
                                               const float* const* cos_sin_dev, const void* const* q_dev,
                                               void* const* out_dev, int32_t out_is_fp32, float softmax_scale,
                                               void* hip_stream);

/* Bookkeeping read-out (host only): maximal runs of pages with equal width, oldest first.
 *   segs_host[cap] receives min(cap, *n) entries; n, bytes_used, n_tokens, current_bits may each be NULL.
 *   bytes_used = sum over tokens of batch * n_kv_heads * kvq_bytes_per_token_head(bits of that token). */
kvq_status_t kvq_cache_describe(const kvq_cache_t* cache, int32_t layer, kvq_segment_info_t* segs_host,
                                int32_t cap, int32_t* n, uint64_t* bytes_used, int32_t* n_tokens,
                                int32_t* current_bits);

/* Copies one run of K (which = KVQ_WHICH_K) or V to the host in the canonical format, synchronising the
 * stream.  n = token_end - token_begin, D = head_dim, G = group:
 *   16-bit run: codes_host receives fp16 [batch, n_kv_heads, n, D]; scales/zeros are not written.  With
 *               KVQ_TIER16_INT16 it is a b-bit run with b = 16: two bytes per code, low byte first, and metadata.
 *   b-bit run : codes_host uint8 [batch, n_kv_heads, n, D*b/8], element i of a row at bit (i*b)%8 of byte
 *               (i*b)/8, low bits first; scales_host and zeros_host fp16 [batch, n_kv_heads, n, D/G]. */
kvq_status_t kvq_cache_export_segment(kvq_cache_t* cache, int32_t layer, int32_t segment, int32_t which,
                                      void* codes_host, void* scales_host, void* zeros_host,
                                      void* hip_stream);

/* Tuning options (the results do not depend on them beyond floating-point summation order).
 *   KVQ_OPT_SPLITS: number of token-range splits kvq_decode_attention uses per (sequence, KV head),
 *                   1..128; 0 restores the automatic choice.
 *   KVQ_OPT_FUSED_MERGE: 1 = the last workgroup of a (sequence, KV head) merges the split partials inside
 *                   the attention kernel; 0 = a second small kernel does.
 *   KVQ_OPT_DETERMINISTIC: 1 = tiles are dealt to wavefronts in a fixed order, so repeated calls on the same
 *                   cache give bit-identical outputs; 0 (default) = wavefronts claim tiles dynamically, which
 *                   is faster and changes only the floating-point summation order from call to call.
 *   KVQ_OPT_TILE_COST_{2,4,8,16}BIT: relative time one 32-token tile of that width costs the attention kernel
 *                   (1..1000000); the token range of a (sequence, KV head) is cut into splits of equal cost.
 *   KVQ_OPT_SHIFT_STRATEGY: how later 2b -> b steps of kvq_progressive_requant treat codes, S and Z, for the
 *                   comparison of Sec. 4.3.1 (the step from raw fp16 values is Eq. 1-2 under every strategy):
 *                   KVQ_SHIFT_EQUIVALENT (default, Eq. 3): X_b = ((2^2b - 2^b + 1)(X_2b + 2^(b-1))) >> 3b,
 *                       S_b = (2^b + 1) S_2b, Z kept;
 *                   KVQ_SHIFT_DIRECT:   X_b = X_2b >> b, S_b = (2^b + 1) S_2b, Z kept;
 *                   KVQ_SHIFT_MODIFIED: X_b = X_2b >> b, S_b = 2^b S_2b, Z_b = Z_2b + (S_b - S_2b) / 2.
 *                   S_b and Z_b are formed in fp32 and rounded to nearest-even into fp16.
 *   KVQ_OPT_TIER16: what a 16-bit token is.  Only while every block is empty (else KVQ_E_STATE).
 *                   KVQ_TIER16_FP16 (default): the raw fp16 values, no metadata.
 *                   KVQ_TIER16_INT16: the INT16 format of Sec. 4.1.2, the X_2b of the appendix theorem at b = 8:
 *                       Eq. 1-2 with 2^16 - 1 levels, fp16 S and Z per group (the clamp to 65535 matters: S rounded
 *                       down puts the group maximum up to ~32 codes higher, more for subnormal S), 16-bit codes
 *                       exported as two bytes, low byte first.  Such tokens carry metadata in the byte accounting,
 *                       pages leaving the window go 16 -> 8 -> ... by successive shift steps instead of a direct
 *                       quantization, and the shift strategy applies to the 16 -> 8 step as well. */
enum { KVQ_OPT_SPLITS = 0, KVQ_OPT_FUSED_MERGE = 1, KVQ_OPT_DETERMINISTIC = 2, KVQ_OPT_TILE_COST_2BIT = 3,
       KVQ_OPT_TILE_COST_4BIT = 4, KVQ_OPT_TILE_COST_8BIT = 5, KVQ_OPT_TILE_COST_16BIT = 6,
       KVQ_OPT_SHIFT_STRATEGY = 7, KVQ_OPT_TIER16 = 8 };
enum { KVQ_SHIFT_EQUIVALENT = 0, KVQ_SHIFT_DIRECT = 1, KVQ_SHIFT_MODIFIED = 2 };
enum { KVQ_TIER16_FP16 = 0, KVQ_TIER16_INT16 = 1 };
kvq_status_t kvq_cache_set_option(kvq_cache_t* cache, int32_t option, int32_t value);

/* Channel-wise reparameterization of one block (Sec. 3.3, Eq. 7): P = (Q Lambda) Q((K Lambda^-1)^T).  After this call
 * kvq_quantize_append stores the block's keys as K Lambda^-1 at every width (fp32 product of the fp16 key with the
 * fp32 reciprocal 1 / lambda of its channel, rounded to nearest-even into fp16, before Eq. 1-2), and
 * kvq_decode_attention multiplies the queries by lambda when it loads them (fp32 product, rounded to fp16).  V is
 * untouched.  lambda_dev: device, fp32 [n_kv_heads][128], finite and > 0 (not checked); it is copied, together with
 * its reciprocals, into the arena by a kernel on the stream, so the caller's array may be released afterwards.
 * lambda_dev == NULL switches the reparameterization off.  KVQ_E_STATE unless the block is empty. */
kvq_status_t kvq_cache_set_reparam(kvq_cache_t* cache, int32_t layer, const float* lambda_dev, void* hip_stream);

/* Calibration of the factors (Sec. 3.3, Eq. 8): lambda[h][i] = (max_m |K[., h, m, i]|)^alpha over the sequences and
 * token positions of the calibration keys (magnitudes; maxima below 1e-5 count as 1e-5), pow in fp64 rounded to
 * fp32.  k_calib_dev: device, fp16 [batch, n_kv_heads, n_tokens, 128], keys as they would be appended (rotated; for
 * the paper's calibration with positional interpolation, Eq. 10, rotated at positions s * m).  lambda_dev: device,
 * fp32 [n_kv_heads][128], written.  0 <= alpha <= 4.  Needs no cache; enqueues three small kernels on the stream. */
kvq_status_t kvq_calibrate_lambda(const void* k_calib_dev, int32_t batch, int32_t n_kv_heads, int32_t n_tokens,
                                  float alpha, float* lambda_dev, void* hip_stream);

/* Reconstruction error of a block's cache against the fp16 tensors it was built from (the model-free measure used
 * to compare the bit-width shrinking strategies of Sec. 4.3.1): sq_err_host[0] = sum over all cached K elements of
 * (K_hat - K)^2 with K_hat = code * S + Z (raw value in the 16-bit tier), sq_err_host[1] the same for V.
 * k_ref_dev, v_ref_dev: device, fp16 [batch, n_kv_heads, n_tokens, 128] with n_tokens the block's current length.
 * sq_err_host: host, 2 doubles.  Squares are added in fp32 inside a 32-token tile and in fp64 across tiles.
 * Enqueues on the stream, then waits for it (like kvq_cache_export_segment).  KVQ_E_STATE on an empty block or an
 * accounting-only cache. */
kvq_status_t kvq_cache_sq_error(kvq_cache_t* cache, int32_t layer, const void* k_ref_dev, const void* v_ref_dev,
                                double* sq_err_host, void* hip_stream);

/* The two terms of the sensitivity of Sec. 3.2, Eq. 5, for a block as it is cached now:
 * s_host[0] = || G_K * (K - K_hat) ||_1, s_host[1] = || G_V * (V - V_hat) ||_1 (* element-wise; K_hat = code * S + Z, raw
 * value in the 16-bit tier); s_{i,b} of Eq. 5 is their sum for block i held at width b.  k_ref_dev, v_ref_dev as in
 * kvq_cache_sq_error; gk_dev, gv_dev: device, fp32 [batch, n_kv_heads, n_tokens, 128], the gradients of the loss with
 * respect to K and V, or NULL for all-ones (no model at hand: plain L1 reconstruction error).  For a block with
 * reparameterization the stored keys are K Lambda^-1: pass references in that space.  fp32 inside a tile, fp64 across
 * tiles.  Enqueues on the stream, then waits for it. */
kvq_status_t kvq_cache_sensitivity(kvq_cache_t* cache, int32_t layer, const void* k_ref_dev, const void* v_ref_dev,
                                   const float* gk_dev, const float* gv_dev, double* s_host, void* hip_stream);

/* Block-wise memory allocation, the integer program of Sec. 3.2, Eq. 6, solved exactly on the host (multiple-choice
 * knapsack by lists of non-dominated states): choose one width per block, choice_out[i] in [0, n_choices), minimising
 * sum_i s[i][choice_i] subject to sum_i mem[i][choice_i] <= budget.  s: host, [n_blocks][n_choices], finite, >= 0 (the
 * sensitivities s_{i,b}); mem: host, [n_blocks][n_choices] bytes (e.g. tokens * batch * n_kv_heads *
 * kvq_bytes_per_token_head(b)).  Among equally cheap solutions the one using less memory is returned.  total_s_out,
 * total_mem_out: optional.  The chosen widths and mem[i][choice_i] are the block_fbit / block_budget_bytes vectors of
 * kvq_cache_create.  KVQ_E_BUDGET if no choice fits; KVQ_E_OOM beyond 4 M states; needs no GPU.
 * 1 <= n_blocks <= 4096, 1 <= n_choices <= 16. */
kvq_status_t kvq_allocate_bits(int32_t n_blocks, int32_t n_choices, const double* s, const uint64_t* mem,
                               uint64_t budget, int32_t* choice_out, double* total_s_out, uint64_t* total_mem_out);

/* Measurement aid, not part of the method: enqueues one plain streaming-read kernel (16-byte loads, no
 * arithmetic) over buf_dev[0, bytes) with n_workgroups workgroups of 256 threads.  Timed by the caller, it gives
 * the device's practical HBM read ceiling, next to which the attention kernel's bandwidth is reported.
 * buf_dev: 16-byte aligned device memory the caller owns; nothing is written to it. */
kvq_status_t kvq_stream_read_probe(kvq_cache_t* cache, const void* buf_dev, uint64_t bytes, int32_t n_workgroups,
                                   void* hip_stream);

/* Empties block `layer` (-1: every block) so that the cache can take a new sequence: its pages go back to the arena
 * (reused only by work enqueued later, so on the cache's stream nothing in flight is disturbed), its token count to
 * zero; budget, Fbit, options and the block's reparameterization factors stay (kvq_cache_set_reparam may be called
 * again, the block being empty).  Host bookkeeping only; nothing is enqueued.  Once every block is empty, the
 * device-side flags of the cache (the mark that a V scale >= 256 was seen, which selects the slower overflow-proof
 * attention path) are cleared by the next call that enqueues work, in stream order. */
kvq_status_t kvq_cache_reset(kvq_cache_t* cache, int32_t layer);

/* Free bytes left in the arena's page area (host bookkeeping). */
uint64_t kvq_cache_arena_free_bytes(const kvq_cache_t* cache);

const char* kvq_status_string(kvq_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_H */
