// Token assignment from per-expert token bit sets (paper Sec. 4: the remapper hands every expert its tokens), shared by the
// stand-alone lynx_permute kernel and by the last workgroup of the fused remap kernel.
//
// A token holds k distinct experts, so an expert sees a token at most once: the membership of the batch
// in each expert is a T-bit set.  Pair counts are popcounts, and the stable position of pair (t, slot)
// inside its expert is the popcount of the bits below t.  No sort, no ordered atomics.
#pragma once

#include "lynx_plan.h"

namespace lynx {

template <int MAXW>   // capacity in 32-token words per expert
struct PermuteSharedT {
    unsigned member[LYNX_MAX_N * MAXW];   // member[e*W + w] bit b: token 32*w+b uses expert e
    uint16_t before[LYNX_MAX_N * MAXW];   // before[e*W + w] = tokens of expert e in the words below w
    int count[LYNX_MAX_N];
    int offs[LYNX_MAX_N + 1];
    int arank[LYNX_MAX_N + 1];
    int blk0[LYNX_MAX_N];                 // first block of the expert in the FFN's work plan
};
typedef PermuteSharedT<LYNX_MAX_T / 32> PermuteShared;

// Every thread of the workgroup calls this with sh.member filled (and visible: barrier before).
// perm must have been pre-filled with -1 where invalid indices can occur.  With ps.units_gu > 0 it also writes the
// work plan of the expert FFN into the workspace ws (lynx_plan.h).
template <int THREADS, typename Shared>
__device__ __forceinline__ void permute_from_bitsets(Shared &sh, const int32_t *__restrict__ idx, int T, int N,
                                                     int k, int32_t *__restrict__ expert_offsets,
                                                     int32_t *__restrict__ perm, int32_t *__restrict__ active_experts,
                                                     int32_t *__restrict__ num_active, const PlanShape &ps = PlanShape{0, 0, 0, 0, 0},
                                                     int32_t *__restrict__ ws = nullptr)
{
    const int tid = threadIdx.x;
    const int W = (T + 31) / 32;
    const int P = T * k;
    if (tid < N) {
        int c = 0;
        for (int w = 0; w < W; ++w) {
            sh.before[tid * W + w] = (uint16_t)c;
            c += __popc(sh.member[tid * W + w]);
        }
        sh.count[tid] = c;
    }
    __syncthreads();
    // exclusive prefixes over experts: pair offsets and rank among the invoked experts, both in one scan (the pair
    // count of the whole batch is at most LYNX_MAX_T * LYNX_MAX_K < 2^16: it leaves the upper half to the ranks)
    static_assert(LYNX_MAX_T * LYNX_MAX_K < 65536 && LYNX_MAX_N < 32768, "packed prefix sums");
    if (tid < kWave) {
        int carry_o = 0, carry_a = 0;
        for (int base = 0; base < N; base += kWave) {
            const int e = base + tid;
            const int c = (e < N) ? sh.count[e] : 0;
            const int a = c > 0 ? 1 : 0;
            const int s = wave_prefix_sum_i32(c | (a << 16));
            if (e < N) {
                sh.offs[e] = carry_o + (s & 0xffff) - c;
                sh.arank[e] = carry_a + (s >> 16) - a;
            }
            const int total = __builtin_amdgcn_readlane(s, kWave - 1);
            carry_o += total & 0xffff;
            carry_a += total >> 16;
        }
        if (tid == 0) {
            sh.offs[N] = carry_o;
            sh.arank[N] = carry_a;
        }
    }
    __syncthreads();
    build_plan<THREADS>(ps, N, sh.count, sh.offs, sh.blk0, ws);
    __syncthreads();
    // (the indices are read with device-coherent loads: in the fused kernel another workgroup of this launch
    // wrote them; such loads go to memory, so several are requested before the first is used)
    constexpr int kBatch = 8;
    for (int p0 = tid; p0 < P; p0 += THREADS * kBatch) {
        int ev[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int p = p0 + u * THREADS;
            ev[u] = p < P ? load_coherent(idx + p) : -1;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int p = p0 + u * THREADS, e = ev[u];
            if (e < 0 || e >= N) continue;
            const int t = p / k;
            const int wt = t >> 5;
            const int pos = sh.offs[e] + sh.before[e * W + wt] + __popc(sh.member[e * W + wt] & ((1u << (t & 31)) - 1u));
            perm[pos] = p;   // pos < offs[N] <= P by construction
            plan_file_pair(ps, sh.blk0, e, sh.count[e], pos - sh.offs[e], p, ws);
        }
    }
    for (int e = tid; e <= N; e += THREADS) expert_offsets[e] = sh.offs[e];
    const int na = sh.arank[N];
    for (int e = tid; e < N; e += THREADS) {
        if (sh.count[e] > 0) active_experts[sh.arank[e]] = e;
        if (e >= na) active_experts[e] = -1;
    }
    if (tid == 0) num_active[0] = na;
}

}  // namespace lynx
