// Decode attention over one cache -- one kernel for a raw fp16 16-bit tier (the default), one for an integer 16-bit
// tier (a cache has one kind, so neither carries the other's path) -- the split-merge kernel and the launchers.  The
// device code is in kvq_attention_body.h; the ragged-batch kernels that share it are compiled on their own, so that
// they do not change the inlining and register allocation of these.
#include "kvq_attention_body.h"

#include <mutex>

namespace {

// Scratch of kvq_decode_attention_static: split partials, (max, sum) pairs and arrival counters in the device image
// of this library instead of the caller's arena, for callers that cannot allocate.  Every GPU the library runs on
// holds its own copy until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[KVQ_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, looked up once

// grid = (splits, units); 512 threads = 8 wavefronts, one workgroup per compute unit.
__global__ __launch_bounds__(KVQ_ATTN_THREADS) void kvq_attention_kernel(const KvqAttnParams P) {
    __shared__ AttnShared sh;
    if (__builtin_amdgcn_readfirstlane(P.flags[0] & 1u)) attention_body<true, false, false, false>(P, sh);
    else attention_body<false, false, false, false>(P, sh);
}

// The same with a one-token append into the raw fp16 tier in front (kvq_append_decode_attention).
__global__ __launch_bounds__(KVQ_ATTN_THREADS) void kvq_attention_append_kernel(const KvqAttnParams P) {
    __shared__ AttnShared sh;
    if (__builtin_amdgcn_readfirstlane(P.flags[0] & 1u)) attention_body<true, false, false, true>(P, sh);
    else attention_body<false, false, false, true>(P, sh);
}

// The same for a cache whose 16-bit tier holds integer codes in byte planes (KVQ_TIER16_INT16).
__global__ __launch_bounds__(KVQ_ATTN_THREADS) void kvq_attention_i16_kernel(const KvqAttnParams P) {
    __shared__ AttnShared sh;
    if (__builtin_amdgcn_readfirstlane(P.flags[0] & 1u)) attention_body<true, true>(P, sh);
    else attention_body<false, true>(P, sh);
}

// Same thread count as the attention kernel, so both merge variants add in the same order.
__global__ __launch_bounds__(KVQ_ATTN_THREADS) void kvq_merge_kernel(const KvqAttnParams P) {
    __shared__ float lds[KVQ_MERGE_LDS_FLOATS];
    merge_splits<false>(P, blockIdx.x, threadIdx.x, lds);
}

}  // namespace

#ifdef KVQ_PHASE_STAMPS
// Measurement build only: copies the stamps of the last launch of the single-cache kernels to the host.
extern "C" int kvq_phase_stamps_read(unsigned long long* host) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(kvq_phase_stamps), sizeof(unsigned long long) * KVQ_STAMP_WGS * KVQ_STAMP_SLOTS);
}
#endif

hipError_t kvq_static_scratch(unsigned char** ptr) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t kvq_launch_merge(const KvqAttnParams& p, int units, hipStream_t s) {
    hipLaunchKernelGGL(kvq_merge_kernel, dim3(units), dim3(KVQ_ATTN_THREADS), 0, s, p);
    return hipGetLastError();
}

hipError_t kvq_launch_attention(const KvqAttnParams& p, int units, hipStream_t s) {
    if (p.int16_tier && p.app_t_old >= 0) { hipError_t e0 = kvq_launch_attention_i16_append(p, units, s); if (e0 != hipSuccess) return e0; }
    else if (p.int16_tier) hipLaunchKernelGGL(kvq_attention_i16_kernel, dim3(p.n_splits, units), dim3(KVQ_ATTN_THREADS), 0, s, p);
    else if (p.app_t_old >= 0) hipLaunchKernelGGL(kvq_attention_append_kernel, dim3(p.n_splits, units), dim3(KVQ_ATTN_THREADS), 0, s, p);
    else hipLaunchKernelGGL(kvq_attention_kernel, dim3(p.n_splits, units), dim3(KVQ_ATTN_THREADS), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.n_splits > 1 && !p.fused_merge) e = kvq_launch_merge(p, units, s);
    return e;
}

hipError_t kvq_launch_attention_batch(const KvqAttnParams* params_dev, const KvqAttnParams* params_host,
                                      const int* units, int n, hipStream_t s) {
    if (n < 1 || n > KVQ_MAX_BATCH_CACHES) return hipErrorInvalidValue;
    KvqBatchMap map;
    map.n = n;
    int wgs = 0;
    for (int i = 0; i < n; ++i) {
        map.wg_begin[i] = wgs;
        wgs += params_host[i].n_splits * units[i];
    }
    for (int i = n; i <= KVQ_MAX_BATCH_CACHES; ++i) map.wg_begin[i] = wgs;
    hipError_t e = kvq_launch_attention_batch_kernel(params_dev, map, params_host[0].int16_tier != 0, s);
    for (int i = 0; i < n && e == hipSuccess; ++i)
        if (params_host[i].n_splits > 1 && !params_host[i].fused_merge) e = kvq_launch_merge(params_host[i], units[i], s);
    return e;
}
