// Decode attention over a cache with an integer 16-bit tier, with the one-token append of kvq_append_decode_attention in
// front: the workgroup that owns the last tile quantizes the new token (Eq. 1-2 with 2^16 - 1 levels) into the tile's
// byte planes before it attends.  A translation unit of its own, like the ragged-batch kernels: what shares a unit
// with the main kernels changes their inlining and register allocation.
#define KVQ_WITH_I16_APPEND
#include "kvq_attention_body.h"

namespace {

__global__ __launch_bounds__(KVQ_ATTN_THREADS) void kvq_attention_i16_append_kernel(const KvqAttnParams P) {
    __shared__ AttnShared sh;
    if (__builtin_amdgcn_readfirstlane(P.flags[0] & 1u)) attention_body<true, true, false, true>(P, sh);
    else attention_body<false, true, false, true>(P, sh);
}

}  // namespace

hipError_t kvq_launch_attention_i16_append(const KvqAttnParams& p, int units, hipStream_t s) {
    hipLaunchKernelGGL(kvq_attention_i16_append_kernel, dim3(p.n_splits, units), dim3(KVQ_ATTN_THREADS), 0, s, p);
    return hipGetLastError();
}
