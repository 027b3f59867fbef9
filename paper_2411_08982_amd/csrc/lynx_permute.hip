// lynx_permute: token assignment for the grouped expert FFN (paper Sec. 4, "assigns tokens").
//
// A token holds k distinct experts, so an expert sees a token at most once: the membership of the
// batch in each expert is a T-bit set.  The workgroup builds those bit sets in LDS with atomic ORs
// (order-free), pair counts are popcounts, and the stable position of pair (t, slot) inside its
// expert is the popcount of the bits below t.  No sort, no ordered atomics, same result every run.
#include "lynx_common.h"

namespace lynx {

constexpr int kPermThreads = 1024;
constexpr int kWords = LYNX_MAX_T / 32;

__global__ __launch_bounds__(kPermThreads) void permute_kernel(const int32_t *__restrict__ idx, int T, int N, int k,
                                                               int32_t *__restrict__ expert_offsets,
                                                               int32_t *__restrict__ perm,
                                                               int32_t *__restrict__ active_experts,
                                                               int32_t *__restrict__ num_active)
{
    __shared__ unsigned member[LYNX_MAX_N * kWords];   // member[e][w] bit b: token 32*w+b uses expert e
    __shared__ int count[LYNX_MAX_N];
    __shared__ int offs[LYNX_MAX_N + 1];
    __shared__ int arank[LYNX_MAX_N + 1];

    const int tid = threadIdx.x;
    const int W = (T + 31) / 32;
    const int P = T * k;
    for (int i = tid; i < N * W; i += kPermThreads) member[i] = 0u;
    for (int p = tid; p < P; p += kPermThreads) perm[p] = -1;
    __syncthreads();
    for (int p = tid; p < P; p += kPermThreads) {
        const int e = idx[p];
        const int t = p / k;
        if (e >= 0 && e < N) atomicOr(&member[e * W + (t >> 5)], 1u << (t & 31));
    }
    __syncthreads();
    if (tid < N) {
        int c = 0;
        for (int w = 0; w < W; ++w) c += __popc(member[tid * W + w]);
        count[tid] = c;
    }
    __syncthreads();
    // exclusive prefixes over experts: pair offsets and rank among the invoked experts
    if (tid < kWave) {
        int carry_o = 0, carry_a = 0;
        for (int base = 0; base < N; base += kWave) {
            const int e = base + tid;
            const int c = (e < N) ? count[e] : 0;
            const int a = c > 0 ? 1 : 0;
            int so = c, sa = a;
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const int uo = __shfl_up(so, d, kWave), ua = __shfl_up(sa, d, kWave);
                if (tid >= d) {
                    so += uo;
                    sa += ua;
                }
            }
            if (e < N) {
                offs[e] = carry_o + so - c;
                arank[e] = carry_a + sa - a;
            }
            carry_o += __shfl(so, kWave - 1, kWave);
            carry_a += __shfl(sa, kWave - 1, kWave);
        }
        if (tid == 0) {
            offs[N] = carry_o;
            arank[N] = carry_a;
        }
    }
    __syncthreads();
    for (int p = tid; p < P; p += kPermThreads) {
        const int e = idx[p];
        if (e < 0 || e >= N) continue;
        const int t = p / k;
        int pos = offs[e];
        const int wt = t >> 5;
        for (int w = 0; w < wt; ++w) pos += __popc(member[e * W + w]);
        pos += __popc(member[e * W + wt] & ((1u << (t & 31)) - 1u));
        perm[pos] = p;   // pos < offs[N] <= P by construction
    }
    for (int e = tid; e <= N; e += kPermThreads) expert_offsets[e] = offs[e];
    const int na = arank[N];
    for (int e = tid; e < N; e += kPermThreads) {
        if (count[e] > 0) active_experts[arank[e]] = e;
        if (e >= na) active_experts[e] = -1;
    }
    if (tid == 0) num_active[0] = na;
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
