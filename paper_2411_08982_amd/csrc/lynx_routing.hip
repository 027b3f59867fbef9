// Routing side of the Lynx decode step: router logits, softmax and top-k (paper Sec. 2.1),
// AffinityBinning (Sec. 3.2.1), batch-wide expert scoring and active-set selection (Sec. 3.3.1),
// remapping with gate renormalisation (Secs. 3.4, 4) and, in the fused whole-layer path, the token
// assignment (Sec. 4).
//
// These steps are latency-bound (microseconds).  On a chip with one L2 per XCD every dependent launch
// costs a few microseconds of its own (first loads miss, last stores are written back), so the layout
// minimises dependent launches and dependent memory round trips inside them:
//   logits_kernel         (token tile x expert group)  fp32 dot products: the router row is prefetched
//                         into registers while the 4 tokens are staged in LDS; lanes split H; transposing
//                         butterfly reduction.  Always its own launch (it needs the whole chip).  Above
//                         128 tokens logits_mfma_kernel does the same on the fp32 matrix cores.
//   T <= 16:  routing_small_kernel  ONE workgroup does everything else with all state in LDS: top-k,
//                         bins + histogram, scores + score order, nominations, fill, remap, gates, counts
//                         and (fused path) the token assignment.  Two launches for the whole routing side.
//   T  > 16:  token_kernel -> nominate_kernel -> remap_kernel, one wave per token over many workgroups, one
//                         launch per batch-level dependency (finished histogram; finished active set).
//                         Scores/order and the fill are recomputed by every workgroup in its prologue
//                         instead of costing a launch; the last workgroup of remap_kernel (atomic ticket,
//                         device-coherent stores and loads instead of a fence: nobody waits, nothing can
//                         hang) assigns the tokens.
//   lynx_affinity_bin_biased: token_kernel -> biased_remap_kernel (the score-biased selection variant).
// Nomination: with the experts laid out across the lanes in score order, "the best-scoring expert that
// qualifies" is a ballot followed by find-first-set.  All decisions are integer (bins from one fp32
// subtract and one fp32 multiply, scores as base-T integers, ties to the lower expert index), so results
// do not depend on the order in which waves or workgroups run.
#include "lynx_permute_core.h"

namespace lynx {

constexpr int kRouteTT = 4;        // tokens per logits workgroup
constexpr int kRouteHC = 4096;     // hidden columns staged in LDS per pass
constexpr int kTokThreads = 256;   // multi-workgroup token kernels: 4 waves = 4 tokens per workgroup (one per SIMD)
constexpr int kTokWaves = kTokThreads / kWave;
constexpr int kRemapWideMinT = 256;   // batches from which remap_kernel runs with 1024 threads per workgroup
constexpr int kSmallThreads = 1024;   // single-workgroup path: 16 waves = 16 tokens
constexpr int kSmallWaves = kSmallThreads / kWave;
constexpr int kLogitsMfmaMinT = 128;   // larger batches compute the logits on the fp32 matrix cores (measured crossover)

struct ZeroList {
    int32_t *ptr[8];
    int count[8];
    int n;
};

__device__ __forceinline__ void zero_slices(const ZeroList &z, int wg, int nwg, int tid, int nthreads)
{
    for (int a = 0; a < z.n; ++a)
        for (int i = wg * nthreads + tid; i < z.count[a]; i += nwg * nthreads) z.ptr[a][i] = 0;
}

__global__ __launch_bounds__(256) void zero_kernel(ZeroList z)
{
    zero_slices(z, blockIdx.x, gridDim.x, threadIdx.x, blockDim.x);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// logits[t,e] = sum_h x[t,h] * Wr[e,h] + bias[e].  Grid (ceil(T/4), ceil(N/4)); wave w owns expert
// 4*blockIdx.y + w for the workgroup's 4 tokens.  Also clears the scratch of the kernels that follow.
__global__ __launch_bounds__(256) void logits_kernel(const uint16_t *__restrict__ x, const float *__restrict__ Wr,
                                                     const float *__restrict__ bias, int T, int H, int N,
                                                     float *__restrict__ logits, ZeroList z)
{
    __shared__ __attribute__((aligned(16))) uint16_t xs[kRouteTT * kRouteHC];
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    zero_slices(z, blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y, tid, 256);
    const int t0 = blockIdx.x * kRouteTT;
    const int ntok = min(kRouteTT, T - t0);
    const int e = blockIdx.y * 4 + wave;
    const int ec = min(e, N - 1);   // surplus waves redo the last expert and drop the result
    float acc[kRouteTT];
#pragma unroll
    for (int tt = 0; tt < kRouteTT; ++tt) acc[tt] = 0.f;

    constexpr int kIter = kRouteHC / (kWave * 8);   // 8 column groups of 512 per pass
    for (int h0 = 0; h0 < H; h0 += kRouteHC) {
        const int hc = min(kRouteHC, H - h0);
        const int ppr = hc / 8;   // 16-byte pieces per token row
        // the router row of this pass goes to registers first, so that it is in flight while x is staged
        const float *w = Wr + (size_t)ec * H + h0;
        float4 w0[kIter], w1[kIter];
#pragma unroll
        for (int i = 0; i < kIter; ++i) {
            const int h = lane * 8 + i * kWave * 8;
            const int hcl = min(h, hc - 8);   // past the end: re-read the last piece, weight it with zero below
            w0[i] = *reinterpret_cast<const float4 *>(w + hcl);
            w1[i] = *reinterpret_cast<const float4 *>(w + hcl + 4);
            if (h >= hc) {
                w0[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                w1[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
        if (h0 > 0) __syncthreads();
        for (int q = tid; q < kRouteTT * ppr; q += 256) {
            const int tt = q / ppr, pc = q % ppr;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (tt < ntok) v = *reinterpret_cast<const uint4 *>(x + (size_t)(t0 + tt) * H + h0 + pc * 8);
            *reinterpret_cast<uint4 *>(xs + tt * kRouteHC + pc * 8) = v;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kIter; ++i) {
            const int h = min(lane * 8 + i * kWave * 8, hc - 8);
#pragma unroll
            for (int tt = 0; tt < kRouteTT; ++tt) {
                const uint4 xv = *reinterpret_cast<const uint4 *>(xs + tt * kRouteHC + h);
                float a = acc[tt];
                a = fmaf(bf16_lo(xv.x), w0[i].x, a);
                a = fmaf(bf16_hi(xv.x), w0[i].y, a);
                a = fmaf(bf16_lo(xv.y), w0[i].z, a);
                a = fmaf(bf16_hi(xv.y), w0[i].w, a);
                a = fmaf(bf16_lo(xv.z), w1[i].x, a);
                a = fmaf(bf16_hi(xv.z), w1[i].y, a);
                a = fmaf(bf16_lo(xv.w), w1[i].z, a);
                a = fmaf(bf16_hi(xv.w), w1[i].w, a);
                acc[tt] = a;
            }
        }
    }
    // transposing butterfly: after two exchange steps each quarter of the wave owns one token's sum
    const bool hi32 = (lane & 32) != 0;
    float a0 = hi32 ? acc[2] : acc[0], a1 = hi32 ? acc[3] : acc[1];
    const float s0 = hi32 ? acc[0] : acc[2], s1 = hi32 ? acc[1] : acc[3];
    a0 += __shfl_xor(s0, 32, kWave);
    a1 += __shfl_xor(s1, 32, kWave);
    const bool hi16 = (lane & 16) != 0;
    float keep = hi16 ? a1 : a0;
    const float send = hi16 ? a0 : a1;
    keep += __shfl_xor(send, 16, kWave);
#pragma unroll
    for (int m = 8; m > 0; m >>= 1) keep += __shfl_xor(keep, m, kWave);
    const int tok = (hi32 ? 2 : 0) + (hi16 ? 1 : 0);
    if ((lane & 15) == 0 && tok < ntok && e < N) {
        float zv = keep;
        if (bias) zv += bias[e];
        logits[(size_t)(t0 + tok) * N + e] = zv;
    }
}

// The same for larger batches on the fp32 matrix cores: one workgroup per 16 tokens x 16 experts, its four
// waves split H and are summed in a fixed order through LDS.  v_mfma_f32_16x16x4_f32 takes fp32 operands
// (x is exact in fp32) and accumulates in fp32.  A = x (lane l: token l%16, k group l/16), B = Wr (lane l:
// expert l%16, k group l/16), D: lane l holds expert l%16 for tokens 4*(l/16) .. +3.  A k-step is 32 columns:
// a lane loads the 8 consecutive columns of its k group (16 bytes of x, 32 bytes of Wr) and the j-th of its
// 8 values goes into the j-th of 8 MFMAs (any assignment of columns to MFMAs is right as long as A and B
// agree).  Against the 4 x 4 output tiles of logits_kernel this reads 4 times less through L2; its lanes read 16
// rows at once, which costs latency, so it only pays for large batches (about 10 us at any size; logits_kernel:
// 6 us at 32 tokens, 26 us at 512).
typedef float logits_f32x4 __attribute__((ext_vector_type(4)));
constexpr int kLogitsRing = 4;    // k-steps in flight per wave
constexpr int kLogitsWaves = 4;   // waves of a workgroup, splitting H

struct LogitsStep {
    uint4 xv;
    float4 w0, w1;
};

__device__ __forceinline__ LogitsStep logits_load(const uint16_t *__restrict__ xrow, const float *__restrict__ wrow, int step)
{
    asm volatile("" : "+v"(step));   // keeps the prefetch ring: see the weight ring of the expert kernels
    LogitsStep r;
    r.xv = *reinterpret_cast<const uint4 *>(xrow + step * 32);
    r.w0 = *reinterpret_cast<const float4 *>(wrow + step * 32);
    r.w1 = *reinterpret_cast<const float4 *>(wrow + step * 32 + 4);
    return r;
}

__global__ __launch_bounds__(kLogitsWaves * kWave) void logits_mfma_kernel(const uint16_t *__restrict__ x, const float *__restrict__ Wr,
                                                          const float *__restrict__ bias, int T, int H, int N,
                                                          float *__restrict__ logits, ZeroList z)
{
    __shared__ logits_f32x4 part[kLogitsWaves - 1][kWave];
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    zero_slices(z, blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y, tid, kLogitsWaves * kWave);
    const int t0 = blockIdx.x * 16, e0 = blockIdx.y * 16;
    const int KT = H / 32;                                   // k-steps; wave w takes [kb, kb + n)
    const int per = (KT + kLogitsWaves - 1) / kLogitsWaves;
    const int kb = min(wave * per, KT), n = min(KT, kb + per) - kb;
    const int kbc = n > 0 ? kb : 0, last = max(n, 1) - 1;
    // rows past the end re-read the last row; their results are not stored
    const uint16_t *xrow = x + (size_t)min(t0 + (lane & 15), T - 1) * H + kbc * 32 + (lane >> 4) * 8;
    const float *wrow = Wr + (size_t)min(e0 + (lane & 15), N - 1) * H + kbc * 32 + (lane >> 4) * 8;
    logits_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    LogitsStep ring[kLogitsRing];
#pragma unroll
    for (int j = 0; j < kLogitsRing; ++j) ring[j] = logits_load(xrow, wrow, min(j, last));
    for (int s0 = 0; s0 < n; s0 += kLogitsRing) {
#pragma unroll
        for (int u = 0; u < kLogitsRing; ++u) {
            const int s = s0 + u;
            const bool live = s < n;
            const LogitsStep c = ring[u];
            const float a[8] = {bf16_lo(c.xv.x), bf16_hi(c.xv.x), bf16_lo(c.xv.y), bf16_hi(c.xv.y),
                                bf16_lo(c.xv.z), bf16_hi(c.xv.z), bf16_lo(c.xv.w), bf16_hi(c.xv.w)};
            const float b[8] = {c.w0.x, c.w0.y, c.w0.z, c.w0.w, c.w1.x, c.w1.y, c.w1.z, c.w1.w};
#pragma unroll
            for (int j = 0; j < 8; ++j)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(live ? a[j] : 0.f, b[j], acc, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            ring[u] = logits_load(xrow, wrow, min(s + kLogitsRing, last));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (wave > 0) part[wave - 1][lane] = acc;
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int w = 0; w < kLogitsWaves - 1; ++w) acc += part[w][lane];   // fixed order
    const int e = e0 + (lane & 15);
    if (e >= N) return;
    const float bv = bias ? bias[e] : 0.f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int t = t0 + 4 * (lane >> 4) + v;
        if (t < T) logits[(size_t)t * N + e] = acc[v] + bv;
    }
}

// One wave holds one token's logits: lane l, slot i <-> expert l + 64*i.
// NS = slots per lane = ceil(N / 64): the kernels are instantiated for 1, 2 and 4 so that a router with
// few experts does not pay for empty slots.
template <int NS>
struct TokenLogits {
    float v[NS];
    unsigned have;   // bit i: slot i is a real expert
};

template <int NS>
__device__ __forceinline__ TokenLogits<NS> load_token(const float *__restrict__ z, int N)
{
    TokenLogits<NS> t;
    t.have = 0;
    const int lane = lane_id();
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int e = lane + kWave * i;
        t.v[i] = (e < N) ? z[e] : -INFINITY;
        t.have |= (e < N) ? (1u << i) : 0u;
    }
    return t;
}

template <int NS>
__device__ __forceinline__ float token_max(const TokenLogits<NS> &t)
{
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < NS; ++i) m = fmaxf(m, t.v[i]);
    return wave_max(m);
}

// Group-limited routers (the paper's Sec. 1 names expert grouping and gives no rule; the reading: groups of
// N / n_group consecutive experts, group score = its largest logit, a token may only use the experts of its topk_group
// best groups, equal group scores to the lower group).  Returns the token's logits with the other experts taken out:
// value -inf (logits are finite, so -inf marks "not allowed" wherever a value travels between lanes) and no
// candidate bit.  Wave-uniform control flow; every lane of the wave must call it.
template <int NS>
__device__ __forceinline__ TokenLogits<NS> limit_groups(const TokenLogits<NS> &raw, int N, const RouterKind &rk)
{
    if (rk.n_group <= 1 || rk.topk_group >= rk.n_group) return raw;
    const int lane = lane_id();
    const int gs = N / rk.n_group;
    int grp[NS], key[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int e = lane + kWave * i;
        grp[i] = ((raw.have >> i) & 1u) ? e / gs : -1;
        key[i] = order_key(raw.v[i]);
    }
    const int none = order_key(-INFINITY);
    float gscore[1] = {-INFINITY};   // lane g: score of group g
    for (int g = 0; g < rk.n_group; ++g) {
        int m = none;
#pragma unroll
        for (int i = 0; i < NS; ++i) m = (grp[i] == g) ? max(m, key[i]) : m;
        const int best = wave_max_i32(m);
        if (lane == g) gscore[0] = key_value(best);
    }
    unsigned long long chosen = 0ull;   // bit g: group g is one of the token's groups
    wave_topk(gscore, lane < rk.n_group ? 1u : 0u, rk.topk_group, [&](int, int g, float) {
        if (g != INT_MAX) chosen |= 1ull << g;
    });
    TokenLogits<NS> t;
    t.have = 0;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const bool ok = grp[i] >= 0 && ((chosen >> grp[i]) & 1ull);
        t.v[i] = ok ? raw.v[i] : -INFINITY;
        t.have |= ok ? (1u << i) : 0u;
    }
    return t;
}

// Gates of a selection held one per lane (lane j < k: expert mye, logit myz): softmax over the selected
// logits (paper Sec. 4: the weights are renormalised over the new selection), or, for a sigmoid-gated router
// (gate_fn = 1; Sec. 3.2.1 names such routers), the selected sigmoid scores over their sum.  Returns this lane's
// gate; num = sum of the numerators.
constexpr int kGateSoftmax = 0, kGateSigmoid = 1;
__device__ __forceinline__ float selection_gate(int k, int mye, float myz, int gate_fn, float &num, float &zref)
{
    zref = wave_max(myz);
    float mynum = 0.f;
    if (lane_id() < k && mye >= 0) mynum = gate_fn == kGateSigmoid ? 1.0f / (1.0f + expf(-myz)) : expf(myz - zref);
    num = wave_sum(mynum);
    return mynum / num;
}

// ---- per-token steps (one wave per token), shared by the single-workgroup and the multi-workgroup paths ----

// The "top-k weight sum" of a selection (paper Sec. 4): with num = sum over the selected experts of exp(z - zref) it is
// num over the same sum taken over all N experts; for a sigmoid-gated router the sum of the selected scores itself.
template <int NS>
__device__ __forceinline__ void selection_mass(const TokenLogits<NS> &raw, int t, int gate_fn, float num, float zref,
                                               float *__restrict__ out)
{
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < NS; ++i)
        if ((raw.have >> i) & 1u) part += expf(raw.v[i] - zref);
    const float den = wave_sum(part);
    if (lane_id() == 0) out[t] = gate_fn == kGateSigmoid ? num : num / den;
}

// Softmax + top-k (Sec. 2.1): lane j < k returns the j-th pick in mye; writes idx / gate / psum (softmax: the
// selected probability mass; sigmoid-gated: the sum of the selected scores).
// tl = the experts the token may use, raw = all of them (the same unless the router is group-limited): the softmax
// denominator runs over all.
template <int NS>
__device__ __forceinline__ int token_topk(const TokenLogits<NS> &tl, const TokenLogits<NS> &raw, int t, int k, int gate_fn,
                                          int32_t *__restrict__ topk_idx, float *__restrict__ topk_gate,
                                          float *__restrict__ topk_psum)
{
    const int lane = lane_id();
    int mye = -1;
    float myz = -INFINITY;
    wave_topk(tl.v, tl.have, k, [&](int j, int e, float z) {
        put_lane(mye, j, (e == INT_MAX) ? -1 : e);
        put_lane(myz, j, z);
    });
    float num, zref;
    const float g = selection_gate(k, mye, myz, gate_fn, num, zref);
    if (lane < k) {
        topk_idx[(size_t)t * k + lane] = mye;
        topk_gate[(size_t)t * k + lane] = g;
    }
    selection_mass(raw, t, gate_fn, num, zref, topk_psum);
    return mye;
}

// Bins of every expert for this token into the (LDS) histogram, and the token's pairs per expert.
template <int NS>
__device__ __forceinline__ void token_bins(const TokenLogits<NS> &tl, int k, int mye, float alpha, int beta, int *hist,
                                           int *cntb)
{
    const int lane = lane_id();
    const float zmax = token_max(tl);
#pragma unroll
    for (int i = 0; i < NS; ++i)
        if ((tl.have >> i) & 1u) {
            const int q = bin_of(zmax, tl.v[i], alpha, beta);
            if (q >= 0 && q < beta) atomicAdd(&hist[(lane + kWave * i) * beta + q], 1);
        }
    if (lane < k && mye >= 0) atomicAdd(&cntb[mye], 1);
}

// Value of expert e (wave-uniform or per-lane) out of a token's logits held across the lanes.
template <int NS>
__device__ __forceinline__ float logit_of(const TokenLogits<NS> &tl, int e)
{
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const float c = __shfl(tl.v[i], e & (kWave - 1), kWave);
        r = ((e >> 6) == i) ? c : r;
    }
    return r;
}

// Nominations of one token (Sec. 3.3.1 under the stated reading).  order[r] = expert with the r-th best
// score, inU[e] = the batch invokes e, sel = the token's own picks in rank order; sets inA[e] = 1.
// The logits stay in registers: the experts are brought into score order with lane permutations.
template <int NS>
__device__ __forceinline__ void token_nominate(const TokenLogits<NS> &tl, int N, int k, float alpha, int beta,
                                               const int *order, const int *inU, const int32_t *sel, int *inA)
{
    const int lane = lane_id();
    const float zmax = token_max(tl);
    int er[NS], qr[NS];
    unsigned avail = 0;   // bit i: the expert at score rank lane+64*i is invoked by the batch and not used yet
#pragma unroll
    for (int i = 0; i < NS; ++i) {
        const int r = lane + kWave * i;
        er[i] = (r < N) ? order[r] : 0;
        // every lane takes part in the lane exchange, also those past the last rank: a lane that sits out cannot
        // be read by the others, and the expert at this lane's rank may live in any lane
        const float zr = logit_of(tl, er[i]);
        qr[i] = (r < N && zr != -INFINITY) ? bin_of(zmax, zr, alpha, beta) : INT_MAX;   // -inf: not one of the token's groups
        if (r < N && inU[er[i]]) avail |= 1u << i;
    }
    // bins of the token's own picks, one per lane
    int myq = beta;
    {
        const int es = (lane < k) ? sel[lane] : -1;
        const bool ok = es >= 0 && es < N;
        const float zs = logit_of(tl, ok ? es : 0);
        if (ok) myq = bin_of(zmax, zs, alpha, beta);
    }
    for (int s = 0; s < k; ++s) {
        const int qs = __builtin_amdgcn_readlane(myq, s);
        if (qs >= beta) break;   // out of range (or no valid pick): this and all later picks constrain nothing
        bool found = false;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            if (found) continue;
            const bool ok = ((avail >> i) & 1u) && qr[i] <= qs;
            const unsigned long long b = __ballot(ok);
            if (b != 0ull) {
                found = true;
                if (lane == __ffsll((long long)b) - 1) {
                    avail &= ~(1u << i);
                    inA[er[i]] = 1;
                }
            }
        }
    }
}

// Fill of the active set up to k from the invoked experts in score order (one wave; inA / inU in LDS).
// Returns the number of invoked experts |U|.
__device__ __forceinline__ int wave_fill_active(int N, int k, const int *order, const int *inU, int *inA, bool do_fill)
{
    const int lane = lane_id();
    int nA = 0, nU = 0;
    for (int base = 0; base < N; base += kWave) {
        const int e = base + lane;
        nA += __popcll(__ballot(e < N && inA[e] != 0));
        nU += __popcll(__ballot(e < N && inU[e] != 0));
    }
    int need = do_fill ? k - nA : 0;
    for (int base = 0; base < N && need > 0; base += kWave) {
        const int r = base + lane;
        const int e = (r < N) ? order[r] : 0;
        const bool c = r < N && inU[e] && !inA[e];
        const unsigned long long b = __ballot(c);
        if (c && __popcll(b & ((1ull << lane) - 1ull)) < need) inA[e] = 1;
        need -= __popcll(b);
    }
    return nU;
}

// Selection of one token inside the active set (or its unchanged selection when bypassed) and its gates
// (Secs. 3.4, 4).  Lane j < k returns the j-th expert; writes new_idx / new_gate.
// new_psum (may be null): what token_topk writes as topk_psum, for the new selection: its share of the softmax over all
// N experts (raw), or the sum of its sigmoid scores.  Same arithmetic as there, so an unchanged selection gives the
// same bits.
template <int NS>
__device__ __forceinline__ int token_remap(const TokenLogits<NS> &tl, const TokenLogits<NS> &raw, int t, int N, int k, bool bypass,
                                           int gate_fn, const int *inA, const int32_t *sel, int32_t *__restrict__ new_idx,
                                           float *__restrict__ new_gate, float *__restrict__ new_psum)
{
    const int lane = lane_id();
    int mye = -1;
    float myz = -INFINITY;
    if (bypass) {
        const int es = (lane < k) ? sel[lane] : -1;
        const bool ok = es >= 0 && es < N;
        const float zs = logit_of(tl, ok ? es : 0);
        if (ok) {
            mye = es;
            myz = zs;
        }
    } else {
        unsigned cand = 0;
#pragma unroll
        for (int i = 0; i < NS; ++i)
            if (((tl.have >> i) & 1u) && inA[lane + kWave * i]) cand |= 1u << i;
        wave_topk(tl.v, cand, k, [&](int j, int e, float zz) {
            put_lane(mye, j, (e == INT_MAX) ? -1 : e);
            put_lane(myz, j, zz);
        });
        // A group-limited token can find fewer than k members of the active set among its experts (without groups
        // the active set holds at least k for everybody).  Then all of them were taken, and the slots left keep the
        // token's own picks that are not in the active set, in rank order.
        int slot = __popcll(__ballot(lane < k && mye >= 0));
        if (slot < k) {
            const int es = (lane < k) ? sel[lane] : -1;
            const bool ok = es >= 0 && es < N;
            const float zs = logit_of(tl, ok ? es : 0);
            unsigned long long rest = __ballot(ok && !inA[ok ? es : 0]);
            while (rest != 0ull && slot < k) {
                const int src = __ffsll((long long)rest) - 1;
                rest &= rest - 1ull;
                const int e = __shfl(es, src, kWave);
                const float zz = __shfl(zs, src, kWave);
                if (lane == slot) {
                    mye = e;
                    myz = zz;
                }
                ++slot;
            }
        }
    }
    float num, zref;
    const float g = selection_gate(k, mye, myz, gate_fn, num, zref);
    if (lane < k) {
        store_coherent(&new_idx[(size_t)t * k + lane], mye);   // read by the workgroup that assigns the tokens
        new_gate[(size_t)t * k + lane] = g;
    }
    if (new_psum) selection_mass(raw, t, gate_fn, num, zref, new_psum);
    return mye;
}

// Scores as base-T integers (most significant digit = bin 0) from a histogram, and the score order:
// order[r] = expert with the r-th best score, equal scores to the lower index.  Threads tid < N take part;
// the caller puts barriers around it.
__device__ __forceinline__ void score_of(int tid, int N, int T, int beta, const int *hist, unsigned long long *score)
{
    if (tid < N) {
        unsigned long long s = 0;
        for (int j = 0; j < beta; ++j) s = s * (unsigned long long)T + (unsigned long long)hist[tid * beta + j];
        score[tid] = s;
    }
}
// The rank of an expert is the number of experts that come before it: N comparisons per thread.  A turn of that loop
// on 64-bit scores with the index as tie-break costs 64 cycles (measured: 6.8 us at N = 256, 3.6 us at N = 128): the
// 64-bit compares run at a quarter of the rate.  Whenever score * N + (N - 1 - index) fits 32 bits (always for
// beta <= 2, T <= 1024) that one key orders the experts the same way, and a turn is one 32-bit compare.  Every
// thread of the workgroup must call this (it holds a barrier); key is LDS scratch of N words.
__device__ __forceinline__ void rank_of(int tid, int N, int T, int beta, const unsigned long long *score, unsigned *key,
                                        int *order)
{
    // a score is at most T^beta (all T tokens in bin 0), so the largest key is T^beta * N + N - 1
    unsigned long long lim = (unsigned long long)N;
    for (int j = 0; j < beta && lim < (1ull << 32); ++j) lim *= (unsigned long long)T;
    if (lim + (unsigned long long)N <= (1ull << 32)) {
        if (tid < N) key[tid] = (unsigned)score[tid] * (unsigned)N + (unsigned)(N - 1 - tid);
        __syncthreads();
        if (tid < N) {
            const unsigned s = key[tid];
            int r = 0;
            for (int e = 0; e < N; ++e) r += key[e] > s ? 1 : 0;
            order[r] = tid;
        }
        return;
    }
    if (tid < N) {
        const unsigned long long s = score[tid];
        int r = 0;
        for (int e = 0; e < N; ++e) {
            const unsigned long long o = score[e];
            r += (o > s || (o == s && e < tid)) ? 1 : 0;
        }
        order[r] = tid;
    }
}

// True on every thread of the workgroup that takes the ticket last.  Nobody waits for anybody.  What the
// last workgroup reads of the others' results must have been written with atomics or store_coherent and must
// be read with load_coherent: there is no device-wide fence here (see lynx_common.h).
__device__ __forceinline__ bool last_workgroup(int32_t *ticket, int *flag_lds)
{
    wait_memory_complete();
    __syncthreads();
    if (threadIdx.x == 0) *flag_lds = (atomicAdd(ticket, 1) == (int)gridDim.x - 1) ? 1 : 0;
    __syncthreads();
    return *flag_lds != 0;
}

// ---- small batches (T <= kSmallT): everything after the logits in ONE workgroup, all state in LDS -----------

constexpr int kSmallT = 16;   // one token per wave; beyond that one CU's ALUs are the bottleneck (measured)

struct SmallShared {
    PermuteSharedT<1> perm;
    int hist[LYNX_MAX_N * LYNX_MAX_BETA];
    unsigned long long score[LYNX_MAX_N];
    int cntb[LYNX_MAX_N], cnta[LYNX_MAX_N], order[LYNX_MAX_N], inU[LYNX_MAX_N], inA[LYNX_MAX_N];
    unsigned key[LYNX_MAX_N];
    int32_t sel[kSmallT * LYNX_MAX_K];      // the tokens' own picks
    int32_t newsel[kSmallT * LYNX_MAX_K];   // the remapped picks
    int n_before, n_after;
};
static_assert(kSmallT <= kSmallWaves && kSmallT <= 32, "one wave per token, one 32-token word per expert");

// One workgroup, wave t owns token t and keeps its logits in registers from the first step to the last.
template <int NS, bool DO_TOPK, bool DO_PERMUTE>
__global__ __launch_bounds__(kSmallThreads) void routing_small_kernel(
    const float *__restrict__ logits, int T, int N, int k, float alpha, int beta, int bypass, RouterKind rk,
    int32_t *__restrict__ topk_idx, float *__restrict__ topk_gate, float *__restrict__ topk_psum,
    int32_t *__restrict__ new_idx, float *__restrict__ new_gate, float *__restrict__ new_psum,
    int32_t *__restrict__ cnt_before, int32_t *__restrict__ cnt_after, int32_t *__restrict__ bin_hist,
    int32_t *__restrict__ num_active, int32_t *__restrict__ expert_offsets, int32_t *__restrict__ perm,
    int32_t *__restrict__ active_experts, int32_t *__restrict__ num_active_perm, PlanShape ps, int32_t *__restrict__ ws)
{
    __shared__ SmallShared sh;
    const int tid = threadIdx.x, lane = lane_id(), t = wave_id();
    const bool has_token = t < T;
    // the token's logits (and, if given, its picks) are requested first; everything below overlaps the loads
    const TokenLogits<NS> raw = load_token<NS>(logits + (size_t)(has_token ? t : 0) * N, N);
    int given = -1;
    if (!DO_TOPK && has_token && lane < k) given = topk_idx[(size_t)t * k + lane];
    for (int i = tid; i < N * beta; i += kSmallThreads) sh.hist[i] = 0;
    for (int i = tid; i < N; i += kSmallThreads) {
        sh.cntb[i] = 0;
        sh.cnta[i] = 0;
        sh.inA[i] = 0;
        if (DO_PERMUTE) sh.perm.member[i] = 0u;
    }
    if (DO_PERMUTE)
        for (int p = tid; p < T * k; p += kSmallThreads) perm[p] = -1;
    if (tid == 0) sh.n_after = 0;
    const TokenLogits<NS> tl = limit_groups(raw, N, rk);
    __syncthreads();
    // top-k (or the given picks), bins, histogram
    if (has_token) {
        int mye = -1;
        if (DO_TOPK) {
            mye = token_topk(tl, raw, t, k, rk.gate_fn, topk_idx, topk_gate, topk_psum);
        } else if (lane < k) {
            mye = (given < 0 || given >= N) ? -1 : given;
        }
        if (lane < k) sh.sel[t * k + lane] = mye;
        token_bins(tl, k, mye, alpha, beta, sh.hist, sh.cntb);
    }
    __syncthreads();
    score_of(tid, N, T, beta, sh.hist, sh.score);
    if (tid < N) sh.inU[tid] = sh.cntb[tid] > 0;
    __syncthreads();
    rank_of(tid, N, T, beta, sh.score, sh.key, sh.order);
    __syncthreads();
    if (!bypass) {
        if (has_token) token_nominate(tl, N, k, alpha, beta, sh.order, sh.inU, sh.sel + t * k, sh.inA);
        __syncthreads();
    }
    if (t == 0) {
        const int nU = wave_fill_active(N, k, sh.order, sh.inU, sh.inA, !bypass);
        if (lane == 0) sh.n_before = nU;
    }
    __syncthreads();
    if (has_token) {
        const int mye = token_remap(tl, raw, t, N, k, bypass != 0, rk.gate_fn, sh.inA, sh.sel + t * k, new_idx, new_gate,
                                    new_psum);
        if (lane < k) {
            sh.newsel[t * k + lane] = mye;
            if (mye >= 0) {
                atomicAdd(&sh.cnta[mye], 1);
                if (DO_PERMUTE) atomicOr(&sh.perm.member[mye], 1u << t);
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < N * beta; i += kSmallThreads) bin_hist[i] = sh.hist[i];
    for (int i = tid; i < N; i += kSmallThreads) {
        cnt_before[i] = sh.cntb[i];
        cnt_after[i] = sh.cnta[i];
        if (sh.cnta[i] > 0) atomicAdd(&sh.n_after, 1);
    }
    __syncthreads();
    if (tid == 0) {
        num_active[0] = sh.n_before;
        num_active[1] = sh.n_after;
    }
    if constexpr (DO_PERMUTE)
        permute_from_bitsets<kSmallThreads>(sh.perm, sh.newsel, T, N, k, expert_offsets, perm, active_experts,
                                            num_active_perm, ps, ws);
}

// ---- large batches: one wave per token over many workgroups, one launch per batch-level dependency ----------

// Softmax + top-k (DO_TOPK) and/or bins + histogram + pairs per expert (DO_BINS, accumulated with atomics
// into the zeroed outputs).
template <int NS, bool DO_TOPK, bool DO_BINS>
__global__ __launch_bounds__(kTokThreads) void token_kernel(const float *__restrict__ logits, int T, int N, int k,
                                                            float alpha, int beta, RouterKind rk,
                                                            int32_t *__restrict__ topk_idx,
                                                            float *__restrict__ topk_gate,
                                                            float *__restrict__ topk_psum,
                                                            int32_t *__restrict__ bin_hist,
                                                            int32_t *__restrict__ cnt_before)
{
    __shared__ int hist[DO_BINS ? LYNX_MAX_N * LYNX_MAX_BETA : 1];
    __shared__ int cntb[DO_BINS ? LYNX_MAX_N : 1];
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    if (DO_BINS) {
        for (int i = tid; i < N * beta; i += kTokThreads) hist[i] = 0;
        for (int i = tid; i < N; i += kTokThreads) cntb[i] = 0;
        __syncthreads();
    }
    const int t = blockIdx.x * kTokWaves + wave;
    if (t < T) {
        const TokenLogits<NS> raw = load_token<NS>(logits + (size_t)t * N, N);
        const TokenLogits<NS> tl = limit_groups(raw, N, rk);
        int mye = -1;
        if (DO_TOPK) {
            mye = token_topk(tl, raw, t, k, rk.gate_fn, topk_idx, topk_gate, topk_psum);
        } else if (lane < k) {
            mye = topk_idx[(size_t)t * k + lane];
            if (mye < 0 || mye >= N) mye = -1;
        }
        if (DO_BINS) token_bins(tl, k, mye, alpha, beta, hist, cntb);
    }
    if (!DO_BINS) return;
    __syncthreads();
    for (int i = tid; i < N * beta; i += kTokThreads)
        if (hist[i]) atomicAdd(&bin_hist[i], hist[i]);
    for (int i = tid; i < N; i += kTokThreads)
        if (cntb[i]) atomicAdd(&cnt_before[i], cntb[i]);
}

// Every workgroup first turns the finished histogram into scores and the score order (cheap, and it saves a
// launch), then nominates for its tokens.  Workgroup 0 also publishes the order for the remap kernel.
template <int NS>
__global__ __launch_bounds__(kTokThreads) void nominate_kernel(const float *__restrict__ logits,
                                                               const int32_t *__restrict__ topk_idx,
                                                               const int32_t *__restrict__ bin_hist,
                                                               const int32_t *__restrict__ cnt_before, int T, int N,
                                                               int k, float alpha, int beta, RouterKind rk,
                                                               int32_t *__restrict__ ws)
{
    __shared__ unsigned long long score[LYNX_MAX_N];
    __shared__ int order[LYNX_MAX_N], inU[LYNX_MAX_N], inA[LYNX_MAX_N];
    __shared__ unsigned key[LYNX_MAX_N];
    __shared__ int32_t sel[kTokWaves * LYNX_MAX_K];
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    const int t = blockIdx.x * kTokWaves + wave;
    // the token's logits and picks are requested first; the score prologue overlaps the loads
    const TokenLogits<NS> raw = load_token<NS>(logits + (size_t)(t < T ? t : 0) * N, N);
    if (lane < k) sel[wave * k + lane] = (t < T) ? topk_idx[(size_t)t * k + lane] : -1;
    score_of(tid, N, T, beta, bin_hist, score);
    if (tid < N) {
        inU[tid] = cnt_before[tid] > 0;
        inA[tid] = 0;
    }
    const TokenLogits<NS> tl = limit_groups(raw, N, rk);
    __syncthreads();
    rank_of(tid, N, T, beta, score, key, order);
    __syncthreads();
    if (blockIdx.x == 0 && tid < N) ws[kWsOrder + tid] = order[tid];
    if (t < T) token_nominate(tl, N, k, alpha, beta, order, inU, sel + wave * k, inA);
    __syncthreads();
    if (tid < N && inA[tid]) ws[kWsActive + tid] = 1;
}

template <bool DO_PERMUTE>
struct RemapShared {
    int inA[LYNX_MAX_N], inU[LYNX_MAX_N], order[LYNX_MAX_N], cnta[LYNX_MAX_N];
    int flag, n_after;
};
template <>
struct RemapShared<true> {
    PermuteShared perm;
    int inA[LYNX_MAX_N], inU[LYNX_MAX_N], order[LYNX_MAX_N], cnta[LYNX_MAX_N];
    int flag, n_after;
};

// Every workgroup first completes the active set (fill up to k) from the finished nominations, then selects
// inside it for its tokens.  The last workgroup to finish counts the invoked experts and, with DO_PERMUTE,
// assigns the tokens (offsets, permutation, invoked-expert list) from the token bit sets.
template <int NS, bool DO_PERMUTE, int TT = kTokThreads>
__global__ __launch_bounds__(TT) void remap_kernel(const float *__restrict__ logits,
                                                            const int32_t *__restrict__ topk_idx,
                                                            const int32_t *__restrict__ cnt_before, int T, int N, int k,
                                                            int bypass, RouterKind rk, int32_t *__restrict__ ws,
                                                            int32_t *__restrict__ new_idx, float *__restrict__ new_gate,
                                                            float *__restrict__ new_psum,
                                                            int32_t *__restrict__ cnt_after,
                                                            int32_t *__restrict__ num_active,
                                                            int32_t *__restrict__ expert_offsets,
                                                            int32_t *__restrict__ perm,
                                                            int32_t *__restrict__ active_experts,
                                                            int32_t *__restrict__ num_active_perm, PlanShape ps)
{
    __shared__ RemapShared<DO_PERMUTE> sh;
    __shared__ int32_t sel[(TT / kWave) * LYNX_MAX_K];
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    const int W = (T + 31) / 32;
    const int t = blockIdx.x * (TT / kWave) + wave;
    // the token's logits and picks are requested first; the prologue overlaps the loads
    const TokenLogits<NS> raw = load_token<NS>(logits + (size_t)(t < T ? t : 0) * N, N);
    if (lane < k) sel[wave * k + lane] = (t < T) ? topk_idx[(size_t)t * k + lane] : -1;
    if (tid < N) {
        sh.inA[tid] = bypass ? 0 : ws[kWsActive + tid];
        sh.inU[tid] = cnt_before[tid] > 0;
        sh.order[tid] = bypass ? tid : ws[kWsOrder + tid];
        sh.cnta[tid] = 0;
    }
    if (tid == 0) sh.n_after = 0;
    const TokenLogits<NS> tl = limit_groups(raw, N, rk);
    if (DO_PERMUTE) {   // pairs whose expert is invalid stay unassigned
        const int p0 = blockIdx.x * (TT / kWave) * k, p1 = min(T * k, p0 + (TT / kWave) * k);
        for (int p = p0 + tid; p < p1; p += TT) store_coherent(&perm[p], -1);   // overwritten by the last workgroup
    }
    __syncthreads();
    if (wave == 0) {
        const int nU = wave_fill_active(N, k, sh.order, sh.inU, sh.inA, !bypass);
        if (blockIdx.x == 0 && lane == 0) num_active[0] = nU;
    }
    __syncthreads();
    if (t < T) {
        const int mye = token_remap(tl, raw, t, N, k, bypass != 0, rk.gate_fn, sh.inA, sel + wave * k, new_idx, new_gate,
                                    new_psum);
        if (lane < k && mye >= 0) {
            atomicAdd(&sh.cnta[mye], 1);
            if (DO_PERMUTE) atomicOr(reinterpret_cast<unsigned *>(ws + kWsMember) + mye * W + (t >> 5), 1u << (t & 31));
        }
    }
    __syncthreads();
    if (tid < N && sh.cnta[tid]) atomicAdd(&cnt_after[tid], sh.cnta[tid]);
    if (!last_workgroup(ws + kWsTickets + 2, &sh.flag)) return;
    if (tid < N && load_coherent(&cnt_after[tid]) > 0) atomicAdd(&sh.n_after, 1);
    if constexpr (DO_PERMUTE) {
        const unsigned *member = reinterpret_cast<const unsigned *>(ws + kWsMember);
        constexpr int kBatch = 8;   // device-coherent loads go to memory: request several before using the first
        for (int i0 = tid; i0 < N * W; i0 += TT * kBatch) {
            unsigned mv[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int i = i0 + u * TT;
                mv[u] = i < N * W ? load_coherent(&member[i]) : 0u;
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int i = i0 + u * TT;
                if (i < N * W) sh.perm.member[i] = mv[u];
            }
        }
    }
    __syncthreads();
    if (tid == 0) num_active[1] = sh.n_after;
    if constexpr (DO_PERMUTE)
        permute_from_bitsets<TT>(sh.perm, new_idx, T, N, k, expert_offsets, perm, active_experts,
                                          num_active_perm, ps, ws);
}

// ---- score-biased selection (the variant of Sec. 3.3.1 that adds the batch score to the logits) ------------------

// Every workgroup first turns the finished histogram into the bias gamma * score / T^beta (one fp64 division
// rounded to fp32, one fp32 multiply), then every wave selects for its token: the top-ranked expert stays, the
// other k-1 slots go to the invoked experts of largest logit + bias; gates from the original logits.  The last
// workgroup to finish counts the invoked experts before and after.
template <int NS>
__global__ __launch_bounds__(kTokThreads) void biased_remap_kernel(const float *__restrict__ logits,
                                                                   const int32_t *__restrict__ topk_idx,
                                                                   const int32_t *__restrict__ cnt_before,
                                                                   const int32_t *__restrict__ bin_hist, int T, int N,
                                                                   int k, int beta, float gamma, double tpow, int bypass,
                                                                   int32_t *__restrict__ ws, int32_t *__restrict__ new_idx,
                                                                   float *__restrict__ new_gate,
                                                                   float *__restrict__ new_psum,
                                                                   int32_t *__restrict__ cnt_after,
                                                                   int32_t *__restrict__ num_active)
{
    __shared__ float bias[LYNX_MAX_N];
    __shared__ int inU[LYNX_MAX_N];
    __shared__ int cnta[LYNX_MAX_N];
    __shared__ int counts[2];
    __shared__ int flag;
    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
    const int t = blockIdx.x * kTokWaves + wave;
    const TokenLogits<NS> tl = load_token<NS>(logits + (size_t)(t < T ? t : 0) * N, N);
    if (tid < N) {
        unsigned long long sc = 0;
        for (int j = 0; j < beta; ++j) sc = sc * (unsigned long long)T + (unsigned long long)bin_hist[tid * beta + j];
        const float se = __double2float_rn(__ddiv_rn((double)sc, tpow));
        bias[tid] = __fmul_rn(gamma, se);
        inU[tid] = cnt_before[tid] > 0;
        cnta[tid] = 0;
    }
    if (tid < 2) counts[tid] = 0;
    __syncthreads();
    if (t < T) {
        int mye = -1;
        float myz = -INFINITY;
        const int es = (lane < k) ? topk_idx[(size_t)t * k + lane] : -1;   // the token's own picks, rank order
        const bool ok = es >= 0 && es < N;
        const float zs = logit_of(tl, ok ? es : 0);
        if (bypass) {
            if (ok) {
                mye = es;
                myz = zs;
            }
        } else {
            const int top = __shfl(ok ? es : -1, 0, kWave);
            if (lane == 0 && ok) {
                mye = es;
                myz = zs;
            }
            float zb[NS];
            unsigned cand = 0;
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                const int e = lane + kWave * i;
                const bool have = (tl.have >> i) & 1u;
                zb[i] = have ? __fadd_rn(tl.v[i], bias[e]) : -INFINITY;
                if (have && inU[e] && e != top) cand |= 1u << i;
            }
            wave_topk(zb, cand, k - 1, [&](int j, int e, float) { put_lane(mye, j + 1, (e == INT_MAX) ? -1 : e); });
            const float zo = logit_of(tl, mye >= 0 ? mye : 0);   // gates come from the original logits
            if (lane > 0 && mye >= 0) myz = zo;
        }
        float num, zref;
        const float g = selection_gate(k, mye, myz, kGateSoftmax, num, zref);
        if (lane < k) {
            new_idx[(size_t)t * k + lane] = mye;
            new_gate[(size_t)t * k + lane] = g;
            if (mye >= 0) atomicAdd(&cnta[mye], 1);
        }
        if (new_psum) selection_mass(tl, t, kGateSoftmax, num, zref, new_psum);
    }
    __syncthreads();
    if (tid < N && cnta[tid]) atomicAdd(&cnt_after[tid], cnta[tid]);
    if (!last_workgroup(ws + kWsTickets + 3, &flag)) return;
    if (tid < N) {
        if (inU[tid]) atomicAdd(&counts[0], 1);
        if (load_coherent(&cnt_after[tid]) > 0) atomicAdd(&counts[1], 1);
    }
    __syncthreads();
    if (tid < 2) num_active[tid] = counts[tid];
}

static int check_routing_sizes(const char *who, int T, int N, int k)
{
    if (T < 0 || N <= 0 || k <= 0) return fail(LYNX_ERR_INVALID_ARG, "%s: negative or zero size (T=%d N=%d k=%d)", who, T, N, k);
    if (k > N || N > LYNX_MAX_N || k > LYNX_MAX_K || T > LYNX_MAX_T)
        return fail(LYNX_ERR_UNSUPPORTED, "%s: need k<=N<=%d, k<=%d, T<=%d (T=%d N=%d k=%d)", who, LYNX_MAX_N, LYNX_MAX_K,
                    LYNX_MAX_T, T, N, k);
    return LYNX_OK;
}

static int check_bin_params(const char *who, int T, float alpha, int beta)
{
    if (beta < 1 || !(alpha >= 0.0f) || alpha > 3.0e38f)
        return fail(LYNX_ERR_INVALID_ARG, "%s: alpha must be finite and >= 0, beta >= 1 (alpha=%g beta=%d)", who,
                    (double)alpha, beta);
    if (beta > LYNX_MAX_BETA) return fail(LYNX_ERR_UNSUPPORTED, "%s: beta <= %d", who, LYNX_MAX_BETA);
    double lim = 1.0;
    for (int j = 0; j < beta; ++j) lim *= (double)(T > 1 ? T : 1);
    if (lim >= 4611686018427387904.0)
        return fail(LYNX_ERR_UNSUPPORTED, "%s: T^beta must stay below 2^62 (T=%d beta=%d)", who, T, beta);
    return LYNX_OK;
}

int check_router_kind(const char *who, int N, int k, const RouterKind &rk)
{
    if (rk.gate_fn != kGateSoftmax && rk.gate_fn != kGateSigmoid)
        return fail(LYNX_ERR_INVALID_ARG, "%s: gate_fn must be 0 (softmax) or 1 (sigmoid), got %d", who, rk.gate_fn);
    if (rk.n_group < 1 || rk.topk_group < 1 || rk.topk_group > rk.n_group || (N % rk.n_group) != 0)
        return fail(LYNX_ERR_INVALID_ARG, "%s: need 1 <= topk_group <= n_group and n_group dividing N (N=%d n_group=%d topk_group=%d)",
                    who, N, rk.n_group, rk.topk_group);
    if ((long long)rk.topk_group * (N / rk.n_group) < k)
        return fail(LYNX_ERR_INVALID_ARG, "%s: topk_group groups of %d experts hold fewer than k=%d", who, N / rk.n_group, k);
    if (rk.n_group > kWave) return fail(LYNX_ERR_UNSUPPORTED, "%s: n_group <= %d (n_group=%d)", who, kWave, rk.n_group);
    return LYNX_OK;
}

static void add_zero(ZeroList &z, int32_t *p, int count)
{
    z.ptr[z.n] = p;
    z.count[z.n] = count;
    ++z.n;
}

static void launch_logits(const uint16_t *x, const float *Wr, const float *bias, int T, int H, int N, float *logits,
                          const ZeroList &z, hipStream_t st)
{
    if (T > kLogitsMfmaMinT)
        hipLaunchKernelGGL(logits_mfma_kernel, dim3((T + 15) / 16, (N + 15) / 16), dim3(kLogitsWaves * kWave), 0, st, x, Wr, bias, T, H, N,
                           logits, z);
    else
        hipLaunchKernelGGL(logits_kernel, dim3((T + kRouteTT - 1) / kRouteTT, (N + 3) / 4), dim3(256), 0, st, x, Wr, bias,
                           T, H, N, logits, z);
}

// Everything after the logits.  DO_TOPK: compute the top-k (else topk_idx is an input); DO_PERMUTE: also
// assign the tokens.  clear_first: the multi-workgroup path accumulates into zeroed arrays; true = clear them
// with a launch of their own, false = the caller already had them cleared (by the logits kernel).
template <int NS, bool DO_TOPK, bool DO_PERMUTE>
static int launch_after_logits_ns(const char *who, const float *logits, int T, int N, int k, float alpha, int beta,
                               int enable, RouterKind rk, int32_t *topk_idx, float *topk_gate, float *topk_psum, int32_t *new_idx,
                               float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist,
                               int32_t *num_active, int32_t *expert_offsets, int32_t *perm, int32_t *active_experts,
                               int32_t *num_active_perm, int32_t *ws, bool clear_first, hipStream_t st, const PlanShape &ps)
{
    const int bypass = (!enable || T <= 1) ? 1 : 0;
    if (T <= kSmallT) {
        hipLaunchKernelGGL((routing_small_kernel<NS, DO_TOPK, DO_PERMUTE>), dim3(1), dim3(kSmallThreads), 0, st, logits, T, N, k,
                           alpha, beta, bypass, rk, topk_idx, topk_gate, topk_psum, new_idx, new_gate, new_psum, cnt_before,
                           cnt_after, bin_hist, num_active, expert_offsets, perm, active_experts, num_active_perm, ps, ws);
        return check_launch(who);
    }
    int rc;
    if (clear_first) {
        ZeroList z;
        z.n = 0;
        add_zero(z, ws + kWsTickets, 16);
        add_zero(z, ws + kWsActive, N);
        if (DO_PERMUTE) add_zero(z, ws + kWsMember, N * ((T + 31) / 32));
        add_zero(z, bin_hist, N * beta);
        add_zero(z, cnt_before, N);
        add_zero(z, cnt_after, N);
        hipLaunchKernelGGL(zero_kernel, dim3(8), dim3(256), 0, st, z);
        rc = check_launch(who);
        if (rc != LYNX_OK) return rc;
    }
    const dim3 tgrid((T + kTokWaves - 1) / kTokWaves), tblock(kTokThreads);
    hipLaunchKernelGGL((token_kernel<NS, DO_TOPK, true>), tgrid, tblock, 0, st, logits, T, N, k, alpha, beta, rk, topk_idx,
                       topk_gate, topk_psum, bin_hist, cnt_before);
    rc = check_launch(who);
    if (rc != LYNX_OK) return rc;
    if (!bypass) {
        hipLaunchKernelGGL((nominate_kernel<NS>), tgrid, tblock, 0, st, logits, topk_idx, bin_hist, cnt_before, T, N, k, alpha,
                           beta, rk, ws);
        rc = check_launch(who);
        if (rc != LYNX_OK) return rc;
    }
    // Large batches: sixteen tokens per workgroup, so that the last workgroup, which assigns the tokens of the whole
    // batch, has four times the threads for it (512 tokens: 16.2 -> 13.2 us, 256 tokens: 11.4 -> 10.5 us; equal below).
    if (T >= kRemapWideMinT) {
        constexpr int kWide = 1024;
        hipLaunchKernelGGL((remap_kernel<NS, DO_PERMUTE, kWide>), dim3((T + kWide / kWave - 1) / (kWide / kWave)), dim3(kWide), 0,
                           st, logits, topk_idx, cnt_before, T, N, k, bypass, rk, ws, new_idx, new_gate, new_psum, cnt_after,
                           num_active, expert_offsets, perm, active_experts, num_active_perm, ps);
        return check_launch(who);
    }
    hipLaunchKernelGGL((remap_kernel<NS, DO_PERMUTE>), tgrid, tblock, 0, st, logits, topk_idx, cnt_before, T, N, k, bypass, rk, ws,
                       new_idx, new_gate, new_psum, cnt_after, num_active, expert_offsets, perm, active_experts,
                       num_active_perm, ps);
    return check_launch(who);
}

template <bool DO_TOPK, bool DO_PERMUTE>
static int launch_after_logits(const char *who, const float *logits, int T, int N, int k, float alpha, int beta,
                               int enable, RouterKind rk, int32_t *topk_idx, float *topk_gate, float *topk_psum, int32_t *new_idx,
                               float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist,
                               int32_t *num_active, int32_t *expert_offsets, int32_t *perm, int32_t *active_experts,
                               int32_t *num_active_perm, int32_t *ws, bool clear_first, hipStream_t st,
                               const PlanShape &ps = PlanShape{0, 0, 0, 0, 0})
{
#define LYNX_ROUTING_ARGS                                                                                             \
    who, logits, T, N, k, alpha, beta, enable, rk, topk_idx, topk_gate, topk_psum, new_idx, new_gate, new_psum, cnt_before, \
        cnt_after, bin_hist, num_active, expert_offsets, perm, active_experts, num_active_perm, ws, clear_first, st, ps
    if (N <= kWave) return launch_after_logits_ns<1, DO_TOPK, DO_PERMUTE>(LYNX_ROUTING_ARGS);
    if (N <= 2 * kWave) return launch_after_logits_ns<2, DO_TOPK, DO_PERMUTE>(LYNX_ROUTING_ARGS);
    return launch_after_logits_ns<4, DO_TOPK, DO_PERMUTE>(LYNX_ROUTING_ARGS);
#undef LYNX_ROUTING_ARGS
}

// The whole routing side of lynx_moe_layer: two launches for T <= kSmallT, four otherwise.  T >= 1, arguments checked.
int routing_fused(const uint16_t *x, const float *Wr, const float *bias, int T, int H, int N, int k, float alpha,
                  int beta, int enable, RouterKind rk, float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum,
                  int32_t *new_idx, float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist,
                  int32_t *num_active, int32_t *expert_offsets, int32_t *perm, int32_t *active_experts,
                  int32_t *num_active_perm, void *workspace, hipStream_t st, const PlanShape &ps)
{
    int32_t *ws = reinterpret_cast<int32_t *>(workspace);
    ZeroList z;
    z.n = 0;
    add_zero(z, ws + kWsDone, kWsDoneWords + 16);   // the FFN's completion counters and flags
    if (T > kSmallT) {   // the logits kernel clears what the multi-workgroup kernels accumulate into
        add_zero(z, ws + kWsTickets, 16);
        add_zero(z, ws + kWsActive, N);
        add_zero(z, ws + kWsMember, N * ((T + 31) / 32));
        add_zero(z, bin_hist, N * beta);
        add_zero(z, cnt_before, N);
        add_zero(z, cnt_after, N);
    }
    launch_logits(x, Wr, bias, T, H, N, logits, z, st);
    int rc = check_launch("lynx_moe_layer(logits)");
    if (rc != LYNX_OK) return rc;
    return launch_after_logits<true, true>("lynx_moe_layer(routing)", logits, T, N, k, alpha, beta, enable, rk, topk_idx,
                                           topk_gate, topk_psum, new_idx, new_gate, new_psum, cnt_before, cnt_after, bin_hist,
                                           num_active, expert_offsets, perm, active_experts, num_active_perm, ws, false, st, ps);
}

}  // namespace lynx

extern "C" int lynx_affinity_bin_biased(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha,
                                        int beta, float gamma, int enable, int32_t *new_idx, float *new_gate,
                                        float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist,
                                        int32_t *num_active, void *workspace, void *stream)
{
    using namespace lynx;
    int rc = check_routing_sizes("lynx_affinity_bin_biased", T, N, k);
    if (rc != LYNX_OK) return rc;
    rc = check_bin_params("lynx_affinity_bin_biased", T, alpha, beta);
    if (rc != LYNX_OK) return rc;
    if (!(gamma >= 0.0f) || gamma > 3.0e38f)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin_biased: gamma must be finite and >= 0 (gamma=%g)", (double)gamma);
    if (!cnt_before || !cnt_after || !bin_hist || !num_active || !workspace)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin_biased: null output or workspace pointer");
    if (T > 0 && (!logits || !topk_idx || !new_idx || !new_gate))
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin_biased: null pointer");
    hipStream_t st = (hipStream_t)stream;
    int32_t *ws = reinterpret_cast<int32_t *>(workspace);
    ZeroList z;
    z.n = 0;
    add_zero(z, ws + kWsTickets, 16);
    add_zero(z, bin_hist, N * beta);
    add_zero(z, cnt_before, N);
    add_zero(z, cnt_after, N);
    add_zero(z, num_active, 2);
    hipLaunchKernelGGL(zero_kernel, dim3(4), dim3(256), 0, st, z);
    rc = check_launch("lynx_affinity_bin_biased(clear)");
    if (rc != LYNX_OK || T == 0) return rc;
    double tpow = 1.0;   // T^beta by repeated multiplication (below 2^62: checked above)
    for (int j = 0; j < beta; ++j) tpow *= (double)(T > 1 ? T : 1);
    const int bypass = (!enable || T <= 1) ? 1 : 0;
    const dim3 tgrid((T + kTokWaves - 1) / kTokWaves), tblock(kTokThreads);
#define LYNX_BIASED(NS)                                                                                                 \
    do {                                                                                                                \
        hipLaunchKernelGGL((token_kernel<NS, false, true>), tgrid, tblock, 0, st, logits, T, N, k, alpha, beta,         \
                           RouterKind{kGateSoftmax, 1, 1}, const_cast<int32_t *>(topk_idx), nullptr, nullptr, bin_hist, \
                           cnt_before);                                                                                 \
        rc = check_launch("lynx_affinity_bin_biased(bins)");                                                            \
        if (rc != LYNX_OK) return rc;                                                                                   \
        hipLaunchKernelGGL((biased_remap_kernel<NS>), tgrid, tblock, 0, st, logits, topk_idx, cnt_before, bin_hist, T,  \
                           N, k, beta, gamma, tpow, bypass, ws, new_idx, new_gate, new_psum, cnt_after, num_active);    \
    } while (0)
    if (N <= kWave)
        LYNX_BIASED(1);
    else if (N <= 2 * kWave)
        LYNX_BIASED(2);
    else
        LYNX_BIASED(4);
#undef LYNX_BIASED
    return check_launch("lynx_affinity_bin_biased(select)");
}

static int route_impl(const uint16_t *x_bf16, const float *Wr, const float *bias, int T, int H, int N, int k,
                      lynx::RouterKind rk, float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum, void *stream)
{
    using namespace lynx;
    int rc = check_routing_sizes("lynx_route", T, N, k);
    if (rc != LYNX_OK) return rc;
    rc = check_router_kind("lynx_route", N, k, rk);
    if (rc != LYNX_OK) return rc;
    if (H <= 0) return fail(LYNX_ERR_INVALID_ARG, "lynx_route: H must be positive");
    if ((H % 32) != 0) return fail(LYNX_ERR_UNSUPPORTED, "lynx_route: H must be a multiple of 32 (H=%d)", H);
    if (T == 0) return LYNX_OK;
    if (!x_bf16 || !Wr || !logits || !topk_idx || !topk_gate || !topk_psum)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_route: null pointer");
    hipStream_t st = (hipStream_t)stream;
    ZeroList z;
    z.n = 0;
    launch_logits(x_bf16, Wr, bias, T, H, N, logits, z, st);
    rc = check_launch("lynx_route(logits)");
    if (rc != LYNX_OK) return rc;
    const dim3 tgrid((T + kTokWaves - 1) / kTokWaves), tblock(kTokThreads);
    if (N <= kWave)
        hipLaunchKernelGGL((token_kernel<1, true, false>), tgrid, tblock, 0, st, logits, T, N, k, 0.f, 1, rk, topk_idx,
                           topk_gate, topk_psum, nullptr, nullptr);
    else if (N <= 2 * kWave)
        hipLaunchKernelGGL((token_kernel<2, true, false>), tgrid, tblock, 0, st, logits, T, N, k, 0.f, 1, rk, topk_idx,
                           topk_gate, topk_psum, nullptr, nullptr);
    else
        hipLaunchKernelGGL((token_kernel<4, true, false>), tgrid, tblock, 0, st, logits, T, N, k, 0.f, 1, rk, topk_idx,
                           topk_gate, topk_psum, nullptr, nullptr);
    return check_launch("lynx_route(top-k)");
}

extern "C" int lynx_route(const uint16_t *x_bf16, const float *Wr, const float *bias, int T, int H, int N, int k,
                          float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum, void *stream)
{
    return route_impl(x_bf16, Wr, bias, T, H, N, k, lynx::RouterKind{lynx::kGateSoftmax, 1, 1}, logits, topk_idx, topk_gate,
                      topk_psum, stream);
}

extern "C" int lynx_route_sigmoid(const uint16_t *x_bf16, const float *Wr, const float *bias, int T, int H, int N, int k,
                                  float *logits, int32_t *topk_idx, float *topk_gate, float *topk_ssum, void *stream)
{
    return route_impl(x_bf16, Wr, bias, T, H, N, k, lynx::RouterKind{lynx::kGateSigmoid, 1, 1}, logits, topk_idx, topk_gate,
                      topk_ssum, stream);
}

extern "C" int lynx_route_grouped(const uint16_t *x_bf16, const float *Wr, const float *bias, int T, int H, int N, int k,
                                  int n_group, int topk_group, int gate_fn, float *logits, int32_t *topk_idx,
                                  float *topk_gate, float *topk_third, void *stream)
{
    return route_impl(x_bf16, Wr, bias, T, H, N, k, lynx::RouterKind{gate_fn, n_group, topk_group}, logits, topk_idx,
                      topk_gate, topk_third, stream);
}

static int affinity_bin_impl(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha, int beta,
                             int enable, int gate_fn, int32_t *new_idx, float *new_gate, float *new_psum, int32_t *cnt_before,
                             int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active, void *workspace, void *stream)
{
    using namespace lynx;
    int rc = check_routing_sizes("lynx_affinity_bin", T, N, k);
    if (rc != LYNX_OK) return rc;
    rc = check_bin_params("lynx_affinity_bin", T, alpha, beta);
    if (rc != LYNX_OK) return rc;
    if (!cnt_before || !cnt_after || !bin_hist || !num_active || !workspace)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin: null output or workspace pointer");
    if (T > 0 && (!logits || !topk_idx || !new_idx || !new_gate))
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin: null pointer");
    hipStream_t st = (hipStream_t)stream;
    int32_t *ws = reinterpret_cast<int32_t *>(workspace);
    if (T == 0) {
        ZeroList z;
        z.n = 0;
        add_zero(z, bin_hist, N * beta);
        add_zero(z, cnt_before, N);
        add_zero(z, cnt_after, N);
        add_zero(z, num_active, 2);
        hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(256), 0, st, z);
        return check_launch("lynx_affinity_bin(clear)");
    }
    return launch_after_logits<false, false>("lynx_affinity_bin", logits, T, N, k, alpha, beta, enable,
                                             RouterKind{gate_fn, 1, 1},
                                             const_cast<int32_t *>(topk_idx), nullptr, nullptr, new_idx, new_gate, new_psum,
                                             cnt_before, cnt_after, bin_hist, num_active, nullptr, nullptr, nullptr,
                                             nullptr, ws, true, st);
}

extern "C" int lynx_affinity_bin(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha,
                                 int beta, int enable, int32_t *new_idx, float *new_gate, float *new_psum,
                                 int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                                 void *workspace, void *stream)
{
    return affinity_bin_impl(logits, topk_idx, T, N, k, alpha, beta, enable, lynx::kGateSoftmax, new_idx, new_gate,
                             new_psum, cnt_before, cnt_after, bin_hist, num_active, workspace, stream);
}

extern "C" int lynx_affinity_bin_sigmoid(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha,
                                         int beta, int enable, int32_t *new_idx, float *new_gate, float *new_ssum,
                                         int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                                         void *workspace, void *stream)
{
    return affinity_bin_impl(logits, topk_idx, T, N, k, alpha, beta, enable, lynx::kGateSigmoid, new_idx, new_gate,
                             new_ssum, cnt_before, cnt_after, bin_hist, num_active, workspace, stream);
}

extern "C" int lynx_affinity_bin_grouped(const float *logits, int T, int N, int k, int n_group, int topk_group, int gate_fn,
                                         float alpha, int beta, int enable, int32_t *topk_idx, float *topk_gate,
                                         float *topk_third, int32_t *new_idx, float *new_gate, float *new_third,
                                         int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                                         void *workspace, void *stream)
{
    using namespace lynx;
    const RouterKind rk = {gate_fn, n_group, topk_group};
    int rc = check_routing_sizes("lynx_affinity_bin_grouped", T, N, k);
    if (rc != LYNX_OK) return rc;
    rc = check_router_kind("lynx_affinity_bin_grouped", N, k, rk);
    if (rc != LYNX_OK) return rc;
    rc = check_bin_params("lynx_affinity_bin_grouped", T, alpha, beta);
    if (rc != LYNX_OK) return rc;
    if (!cnt_before || !cnt_after || !bin_hist || !num_active || !workspace)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin_grouped: null output or workspace pointer");
    if (T > 0 && (!logits || !topk_idx || !topk_gate || !topk_third || !new_idx || !new_gate))
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin_grouped: null pointer");
    hipStream_t st = (hipStream_t)stream;
    if (T == 0) {
        ZeroList z;
        z.n = 0;
        add_zero(z, bin_hist, N * beta);
        add_zero(z, cnt_before, N);
        add_zero(z, cnt_after, N);
        add_zero(z, num_active, 2);
        hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(256), 0, st, z);
        return check_launch("lynx_affinity_bin_grouped(clear)");
    }
    return launch_after_logits<true, false>("lynx_affinity_bin_grouped", logits, T, N, k, alpha, beta, enable, rk, topk_idx,
                                            topk_gate, topk_third, new_idx, new_gate, new_third, cnt_before, cnt_after, bin_hist,
                                            num_active, nullptr, nullptr, nullptr, nullptr,
                                            reinterpret_cast<int32_t *>(workspace), true, st);
}
