// Decode attention over a ragged batch: grid.x = sum over the caches of splits * units.  A workgroup looks its cache
// up in the map, takes that cache's parameter block from device memory (read-only for the whole launch) and runs the
// same body as the single-cache kernels.
#include "kvq_attention_body.h"

namespace {

template <bool I16>
__device__ __forceinline__ void batch_body(const KvqAttnParams* __restrict__ params, const KvqBatchMap& map, AttnShared& sh) {
    const int wg = blockIdx.x;
    int ci = 0;
    for (int i = 1; i < map.n; ++i) ci = (wg >= map.wg_begin[i]) ? i : ci;
    const KvqAttnParams& P = params[ci];
    const int local = wg - map.wg_begin[ci];
    const int unit = local / P.n_splits, split = local - unit * P.n_splits;  // splits of a unit are neighbours
    if (__builtin_amdgcn_readfirstlane(P.flags[0] & 1u)) attention_body<true, I16, true>(P, sh, split, unit);
    else attention_body<false, I16, true>(P, sh, split, unit);
}
__global__ __launch_bounds__(KVQ_ATTN_THREADS) void kvq_attention_batch_kernel(const KvqAttnParams* __restrict__ params,
                                                                               const KvqBatchMap map) {
    __shared__ AttnShared sh;
    batch_body<false>(params, map, sh);
}
__global__ __launch_bounds__(KVQ_ATTN_THREADS) void kvq_attention_batch_i16_kernel(const KvqAttnParams* __restrict__ params,
                                                                                   const KvqBatchMap map) {
    __shared__ AttnShared sh;
    batch_body<true>(params, map, sh);
}

}  // namespace

hipError_t kvq_launch_attention_batch_kernel(const KvqAttnParams* params_dev, const KvqBatchMap& map, bool int16,
                                             hipStream_t s) {
    const int wgs = map.wg_begin[map.n];
    if (int16) hipLaunchKernelGGL(kvq_attention_batch_i16_kernel, dim3(wgs), dim3(KVQ_ATTN_THREADS), 0, s, params_dev, map);
    else hipLaunchKernelGGL(kvq_attention_batch_kernel, dim3(wgs), dim3(KVQ_ATTN_THREADS), 0, s, params_dev, map);
    return hipGetLastError();
}
