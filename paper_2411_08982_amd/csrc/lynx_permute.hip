// lynx_permute: token assignment for the grouped expert FFN (paper Sec. 4: the remapper hands every expert its tokens) as a
// stand-alone call: one workgroup builds the per-expert token bit sets in LDS with atomic ORs
// (order-free) and derives offsets, the stable permutation and the invoked-expert list from them.
#include "lynx_permute_core.h"

namespace lynx {

constexpr int kPermThreads = 1024;

__global__ __launch_bounds__(kPermThreads) void permute_kernel(const int32_t *__restrict__ idx, int T, int N, int k,
                                                               int32_t *__restrict__ expert_offsets,
                                                               int32_t *__restrict__ perm,
                                                               int32_t *__restrict__ active_experts,
                                                               int32_t *__restrict__ num_active)
{
    __shared__ PermuteShared sh;
    const int tid = threadIdx.x;
    const int W = (T + 31) / 32;
    const int P = T * k;
    for (int i = tid; i < N * W; i += kPermThreads) sh.member[i] = 0u;
    for (int p = tid; p < P; p += kPermThreads) perm[p] = -1;
    __syncthreads();
    for (int p = tid; p < P; p += kPermThreads) {
        const int e = idx[p];
        const int t = p / k;
        if (e >= 0 && e < N) atomicOr(&sh.member[e * W + (t >> 5)], 1u << (t & 31));
    }
    __syncthreads();
    permute_from_bitsets<kPermThreads>(sh, idx, T, N, k, expert_offsets, perm, active_experts, num_active);
}

}  // namespace lynx

extern "C" int lynx_permute(const int32_t *idx, int T, int N, int k, int32_t *expert_offsets, int32_t *perm,
                            int32_t *active_experts, int32_t *num_active, void *stream)
{
    using namespace lynx;
    if (T < 0 || N <= 0 || k <= 0) return fail(LYNX_ERR_INVALID_ARG, "lynx_permute: negative or zero size");
    if (N > LYNX_MAX_N || k > LYNX_MAX_K || T > LYNX_MAX_T || k > N)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_permute: need k<=N<=%d, k<=%d, T<=%d", LYNX_MAX_N, LYNX_MAX_K, LYNX_MAX_T);
    if (!expert_offsets || !active_experts || !num_active || (T > 0 && (!idx || !perm)))
        return fail(LYNX_ERR_INVALID_ARG, "lynx_permute: null pointer");
    hipLaunchKernelGGL(permute_kernel, dim3(1), dim3(kPermThreads), 0, (hipStream_t)stream, idx, T, N, k,
                       expert_offsets, perm, active_experts, num_active);
    return check_launch("lynx_permute");
}
