// lynx_affinity_bin: AffinityBinning, batch-wide expert scoring, active-set selection, remapping and
// gate renormalisation (paper Secs. 3.2.1, 3.3.1, 3.4, 4) for one decode batch.
//
// All decisions are integer: bin magnitudes come from one fp32 subtract and one fp32 multiply, scores
// are base-T integers built from the bin histogram, and every tie goes to the lower expert index, so
// the result does not depend on the order in which waves run.
//
// One workgroup owns the batch (the batch-level steps need all tokens).  A wave owns a token at a
// time: its 64 lanes hold the token's N <= 256 logits, four per lane.
//   1. bins + histogram + pairs per expert      (wave per token, LDS integer atomics)
//   2. scores, and the experts ordered by score  (thread per expert)
//   3. nominations: with the experts laid out in score order across the lanes, "the best-scoring
//      expert that qualifies" is a ballot followed by find-first-set
//   4. fill to k, then per token the top-k by original logit inside the active set, and the gates.
#include "lynx_common.h"

namespace lynx {

constexpr int kBinThreads = 1024;
constexpr int kBinWaves = kBinThreads / kWave;

__global__ __launch_bounds__(kBinThreads) void affinity_bin_kernel(
    const float *__restrict__ logits, const int32_t *__restrict__ topk_idx, int T, int N, int k, float alpha, int beta,
    int enable, int32_t *__restrict__ new_idx, float *__restrict__ new_gate, int32_t *__restrict__ cnt_before,
    int32_t *__restrict__ cnt_after, int32_t *__restrict__ bin_hist, int32_t *__restrict__ num_active)
{
    __shared__ int hist[LYNX_MAX_N * LYNX_MAX_BETA];
    __shared__ int cntb[LYNX_MAX_N];
    __shared__ int cnta[LYNX_MAX_N];
    __shared__ unsigned long long score[LYNX_MAX_N];
    __shared__ int order[LYNX_MAX_N];   // order[r] = expert with the r-th best score
    __shared__ int inA[LYNX_MAX_N];
    __shared__ int n_before, n_after;

    const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();

    for (int i = tid; i < N * beta; i += kBinThreads) hist[i] = 0;
    for (int i = tid; i < N; i += kBinThreads) {
        cntb[i] = 0;
        cnta[i] = 0;
        inA[i] = 0;
    }
    if (tid == 0) {
        n_before = 0;
        n_after = 0;
    }
    __syncthreads();

    // 1. bins, histogram, pairs per expert
    for (int t = wave; t < T; t += kBinWaves) {
        const float *z = logits + (size_t)t * N;
        float v[kSlots];
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < kSlots; ++i) {
            const int e = lane + kWave * i;
            v[i] = (e < N) ? z[e] : -INFINITY;
            m = fmaxf(m, v[i]);
        }
        const float zmax = wave_max(m);
#pragma unroll
        for (int i = 0; i < kSlots; ++i) {
            const int e = lane + kWave * i;
            if (e < N) {
                const int q = bin_of(zmax, v[i], alpha, beta);
                if (q >= 0 && q < beta) atomicAdd(&hist[e * beta + q], 1);
            }
        }
        if (lane < k) {
            const int e = topk_idx[(size_t)t * k + lane];
            if (e >= 0 && e < N) atomicAdd(&cntb[e], 1);
        }
    }
    __syncthreads();

    // 2. scores as base-T integers (most significant digit = bin 0) and the score order
    if (tid < N) {
        unsigned long long s = 0;
        for (int j = 0; j < beta; ++j) s = s * (unsigned long long)T + (unsigned long long)hist[tid * beta + j];
        score[tid] = s;
        if (cntb[tid] > 0) atomicAdd(&n_before, 1);
    }
    __syncthreads();
    if (tid < N) {
        const unsigned long long s = score[tid];
        int r = 0;
        for (int e = 0; e < N; ++e) {
            const unsigned long long o = score[e];
            r += (o > s || (o == s && e < tid)) ? 1 : 0;
        }
        order[r] = tid;
    }
    __syncthreads();

    const bool bypass = (!enable) || T <= 1;
    if (!bypass) {
        // 3. nominations
        for (int t = wave; t < T; t += kBinWaves) {
            const float *z = logits + (size_t)t * N;
            float m = -INFINITY;
#pragma unroll
            for (int i = 0; i < kSlots; ++i) {
                const int e = lane + kWave * i;
                if (e < N) m = fmaxf(m, z[e]);
            }
            const float zmax = wave_max(m);
            int er[kSlots], qr[kSlots];
            unsigned avail = 0;   // bit i: the expert at score rank lane+64*i is invoked by the batch and not used yet
#pragma unroll
            for (int i = 0; i < kSlots; ++i) {
                const int r = lane + kWave * i;
                er[i] = (r < N) ? order[r] : 0;
                qr[i] = (r < N) ? bin_of(zmax, z[er[i]], alpha, beta) : INT_MAX;
                if (r < N && cntb[er[i]] > 0) avail |= 1u << i;
            }
            for (int s = 0; s < k; ++s) {
                const int es = topk_idx[(size_t)t * k + s];
                if (es < 0 || es >= N) break;
                const int qs = bin_of(zmax, z[es], alpha, beta);
                if (qs >= beta) break;
                bool found = false;
#pragma unroll
                for (int i = 0; i < kSlots; ++i) {
                    if (found) continue;
                    const bool ok = ((avail >> i) & 1u) && qr[i] <= qs;
                    const unsigned long long b = __ballot(ok);
                    if (b != 0ull) {
                        found = true;
                        const int first = __ffsll((long long)b) - 1;
                        if (lane == first) {
                            avail &= ~(1u << i);
                            inA[er[i]] = 1;
                        }
                    }
                }
            }
        }
        __syncthreads();
        // 4a. fill to k from the invoked experts in score order
        if (tid == 0) {
            int nA = 0;
            for (int e = 0; e < N; ++e) nA += inA[e];
            for (int r = 0; r < N && nA < k; ++r) {
                const int e = order[r];
                if (cntb[e] > 0 && !inA[e]) {
                    inA[e] = 1;
                    ++nA;
                }
            }
        }
        __syncthreads();
    }

    // 4b. selection inside the active set (or the unchanged selection) and gates
    for (int t = wave; t < T; t += kBinWaves) {
        const float *z = logits + (size_t)t * N;
        int mye = -1;
        float myz = -INFINITY;
        if (bypass) {
            if (lane < k) {
                mye = topk_idx[(size_t)t * k + lane];
                if (mye < 0 || mye >= N) mye = -1;
                if (mye >= 0) myz = z[mye];
            }
        } else {
            float v[kSlots];
            unsigned cand = 0;
#pragma unroll
            for (int i = 0; i < kSlots; ++i) {
                const int e = lane + kWave * i;
                v[i] = (e < N) ? z[e] : -INFINITY;
                if (e < N && inA[e]) cand |= 1u << i;
            }
            wave_topk(v, cand, k, [&](int j, int e, float zz) {
                if (lane == j) {
                    mye = (e == INT_MAX) ? -1 : e;
                    myz = zz;
                }
            });
        }
        // gates: softmax over the selected logits; the largest selected logit is the reference
        const float zref = wave_max(myz);
        const float mynum = (lane < k && mye >= 0) ? expf(myz - zref) : 0.f;
        const float num = wave_sum(mynum);
        if (lane < k) {
            new_idx[(size_t)t * k + lane] = mye;
            new_gate[(size_t)t * k + lane] = mynum / num;
            if (mye >= 0) atomicAdd(&cnta[mye], 1);
        }
    }
    __syncthreads();
    if (tid < N && cnta[tid] > 0) atomicAdd(&n_after, 1);
    __syncthreads();
    for (int i = tid; i < N * beta; i += kBinThreads) bin_hist[i] = hist[i];
    for (int i = tid; i < N; i += kBinThreads) {
        cnt_before[i] = cntb[i];
        cnt_after[i] = cnta[i];
    }
    if (tid == 0) {
        num_active[0] = n_before;
        num_active[1] = n_after;
    }
}

}  // namespace lynx

extern "C" int lynx_affinity_bin(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha,
                                 int beta, int enable, int32_t *new_idx, float *new_gate, int32_t *cnt_before,
                                 int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active, void *workspace,
                                 void *stream)
{
    using namespace lynx;
    (void)workspace;
    if (T < 0 || N <= 0 || k <= 0 || beta < 1 || !(alpha >= 0.0f) || alpha > 3.0e38f)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin: bad size, alpha or beta (T=%d N=%d k=%d alpha=%g beta=%d)", T,
                    N, k, (double)alpha, beta);
    if (k > N || N > LYNX_MAX_N || k > LYNX_MAX_K || T > LYNX_MAX_T || beta > LYNX_MAX_BETA)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_affinity_bin: need k<=N<=%d, k<=%d, T<=%d, beta<=%d", LYNX_MAX_N,
                    LYNX_MAX_K, LYNX_MAX_T, LYNX_MAX_BETA);
    {
        double lim = 1.0;
        for (int j = 0; j < beta; ++j) lim *= (double)(T > 1 ? T : 1);
        if (lim >= 4611686018427387904.0)
            return fail(LYNX_ERR_UNSUPPORTED, "lynx_affinity_bin: T^beta must stay below 2^62 (T=%d beta=%d)", T, beta);
    }
    if (!cnt_before || !cnt_after || !bin_hist || !num_active)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin: null output pointer");
    if (T > 0 && (!logits || !topk_idx || !new_idx || !new_gate))
        return fail(LYNX_ERR_INVALID_ARG, "lynx_affinity_bin: null pointer");
    hipLaunchKernelGGL(affinity_bin_kernel, dim3(1), dim3(kBinThreads), 0, (hipStream_t)stream, logits, topk_idx, T, N,
                       k, alpha, beta, enable, new_idx, new_gate, cnt_before, cnt_after, bin_hist, num_active);
    return check_launch("lynx_affinity_bin");
}
