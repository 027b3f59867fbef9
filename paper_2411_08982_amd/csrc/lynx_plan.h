// The device-built work plan of the grouped expert FFN.
//
// The number of experts a batch invokes after the remap, and how many tokens each of them got, are device-side
// values (paper Sec. 4: the remapper compacts the active list and hands every expert its tokens; Sec. 5.9 names the
// dispatch parameters for a variable number of activated experts as the open tuning point).  The host sizes the FFN
// grid for the most work the batch could cause; which workgroup does what is decided on the device from three small
// tables in the workspace that the token assignment writes as its last step:
//   hdr     [0] = B, the number of (expert, token block) pairs of the batch, [1] = units per down-projection work
//           item, [2] = invoked experts;
//   blk     [q] = {expert id | tokens << 16, offset of the expert's pairs in the permutation, token block, 0} for
//           block q < B, the invoked experts by ascending id, an expert's blocks in a row;
//   pairs   [q][i], 16 bits each: the (token, slot) pair id of the i-th token of block q, for the blocks of experts
//           with at most kDirectMaxTokens tokens (entries past the expert's tokens are not written).
// An expert with at most kDirectMaxTokens tokens is one token block; a larger one is cut into blocks of tok_block tokens
// (one pass of the staged path each), which go to workgroups of their own.  The work items of a projection are
// numbered block-major, unit-minor: item = block * units + unit, so a workgroup knows from its index alone which
// records to read, and one round trip to memory tells it its expert, its tokens and where their rows are: nothing
// it needs for its first weight and token loads depends on a second load.
#pragma once

#include "lynx_common.h"

namespace lynx {

constexpr int kDirectMaxTokens = 16;         // experts with more tokens take the staged path
constexpr int kTokBlock = 64;                // tokens per pass of the staged path (batches of up to 64 tokens)
constexpr int kTokBlockBig = 128;            // the same in the kernels launched for larger batches

// What the host knows of the FFN launch when the plan is built.
struct PlanShape {
    int units_gu;    // gate/up work items per (expert, token block): 64-row units of the F rows; 0 = build no plan
    int units_dn;    // down-projection row units per (expert, token block)
    int tok_block;   // tokens per block of an expert on the staged path
    int dn_cap;      // down items the grid is sized for: the device takes the fewest units per item that fit it
    int dn_m_max;    // most units per down item
};

constexpr int kPlanB = 0, kPlanM = 1, kPlanNa = 2;   // words of the header

__host__ __device__ __forceinline__ int plan_token_blocks(int te, int tok_block)
{
    return te <= kDirectMaxTokens ? 1 : (te + tok_block - 1) / tok_block;
}

// Most (expert, token block) pairs a batch of T tokens with k picks each can have.
inline int plan_max_blocks(int T, int N, int k, int tok_block)
{
    const long P = (long)T * k;
    const long experts = P < N ? P : N;
    if (T <= kDirectMaxTokens) return (int)experts;
    return (int)(experts + P / tok_block);   // an expert with te tokens has at most 1 + te / tok_block blocks
}

// Units per down item the device will choose for B blocks (same rule on the host, for the grid size).
__host__ __device__ __forceinline__ int plan_down_units_per_item(const PlanShape &ps, int B)
{
    int m = 1;
    while (m < ps.dn_m_max && (long)((ps.units_dn + m - 1) / m) * B > ps.dn_cap) m *= 2;
    return m;
}

// Down items the grid must hold for a batch with at most max_blocks blocks.
inline int plan_down_grid(const PlanShape &ps, int max_blocks)
{
    long worst = 0;
    for (int m = 1; m <= ps.dn_m_max; m *= 2) {
        // m is chosen when m/2 did not fit the cap and m does (or m is the largest): the most blocks with that choice
        const long per = (ps.units_dn + m - 1) / m;
        long b = m == ps.dn_m_max ? max_blocks : ps.dn_cap / per;
        if (b > max_blocks) b = max_blocks;
        if (per * b > worst) worst = per * b;
    }
    return (int)worst;
}

// Builds the header and the block records.  Every thread of the workgroup calls it (one wave does the work); count[e] /
// offs[e] (pairs of expert e and where they start in the permutation) are in LDS and complete (barrier before).
// blk0[e] (LDS) receives the first block of expert e, for the caller to file the pair ids under (barrier after).
// ws = the routing part of the workspace.
template <int THREADS>
__device__ __forceinline__ void build_plan(const PlanShape &ps, int N, const int *count, const int *offs, int *blk0,
                                           int32_t *__restrict__ ws)
{
    if (ps.units_gu <= 0) return;
    const int tid = threadIdx.x;
    if (tid >= kWave) return;
    // exclusive prefixes over the experts in one packed scan: rank among the invoked experts (low half) and token
    // blocks before (high half; at most kPlanMaxBlocks < 2^15)
    int carry_r = 0, carry_b = 0;
    for (int base = 0; base < N; base += kWave) {
        const int e = base + tid;
        const int c = e < N ? count[e] : 0;
        const int a = c > 0 ? 1 : 0;
        const int nb = c > 0 ? plan_token_blocks(c, ps.tok_block) : 0;
        const int s = wave_prefix_sum_i32(a | (nb << 16));
        if (e < N) blk0[e] = carry_b + (s >> 16) - nb;
        if (a) {
            const int q0 = carry_b + (s >> 16) - nb;
            for (int j = 0; j < nb && q0 + j < kPlanMaxBlocks; ++j)
                *reinterpret_cast<int4 *>(ws + kWsPlanBlk + 4 * (q0 + j)) = make_int4(e | (c << 16), offs[e], j, 0);
        }
        const int total = __builtin_amdgcn_readlane(s, kWave - 1);
        carry_r += total & 0xffff;
        carry_b += total >> 16;
    }
    if (tid == 0) {
        ws[kWsPlanHdr + kPlanB] = min(carry_b, kPlanMaxBlocks);
        ws[kWsPlanHdr + kPlanM] = plan_down_units_per_item(ps, carry_b);
        ws[kWsPlanHdr + kPlanNa] = carry_r;
    }
}

// Files pair id p, the i-th of expert e's te pairs, under the expert's block (experts on the direct path only).
__device__ __forceinline__ void plan_file_pair(const PlanShape &ps, const int *blk0, int e, int te, int i, int p,
                                               int32_t *__restrict__ ws)
{
    if (ps.units_gu <= 0 || te > kDirectMaxTokens) return;
    reinterpret_cast<uint16_t *>(ws + kWsPlanPairs)[blk0[e] * kDirectMaxTokens + i] = (uint16_t)p;
}

}  // namespace lynx
