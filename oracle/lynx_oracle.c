/*
 * lynx_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, obviously-correct CPU statement of what one batched MoE-layer decode step of
 * Lynx (arXiv 2411.08982) computes: router logits, softmax and top-k (Sec. 2.1), AffinityBinning
 * (Sec. 3.2.1), batch-wide expert scoring (Sec. 3.3.1), expert remapping (Sec. 3.4), token
 * assignment / compaction / renormalisation (Sec. 4), and the grouped SwiGLU expert FFN with the
 * gate-weighted combine that the remapper dispatches.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.  It shares
 * no code with the HIP path.  Floating point is fp64 except where a floating-point value decides
 * an integer (top-k comparisons and the bin index): those are taken in fp32, the precision of the
 * router logits, with exactly one rounded subtract and one rounded multiply.
 *
 * Where the paper gives prose only (it prints no formula for the pruning rule and no values for
 * alpha and beta) the reading implemented here is written out step by step at each function.
 *
 * Pins (tests/test_oracle_*.py): library fp64 matmul / softmax / stable argsort for the plain
 * steps; hand-worked 4x4 example; invariants the paper states (k distinct experts per token,
 * remap onto already-active experts, top-1 of a confident token kept, invoked count never rises);
 * closed-form special cases; exhaustive subset search on tiny batches.  The widenings at the end of
 * the file (score-biased selection; FP8 E4M3 and MXFP4 expert weights) have pins of their own: exact
 * rational arithmetic and exhaustive search for the bias, the published element tables, an
 * independent library cast (FP8), brute-force rounding on exact rationals, block exponents and error
 * bounds (MXFP4), and a numpy fp64 contraction of the dequantised weights for the quantised FFNs; the
 * gates of sigmoid-gated routers: closed forms, a library logistic function, and what tells them from softmax;
 * group-limited routers: hand-worked cases, a numpy statement of the mask, and the reduction of the grouped
 * remap to the ungrouped one on logits whose forbidden entries are pushed far down.
 * Parity unpinned against the paper: the values of alpha and beta, the bias scale gamma, the
 * weight formats, the gate formula of sigmoid-gated routers and the rule for expert groups (the paper prints
 * none of them).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_ERR_INVALID_ARG (-1)
#define ORC_ERR_UNSUPPORTED (-2)

#define ORC_MAX_BETA 6

static double bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* k largest entries of z among the allowed experts, in descending order; equal values go to the
 * lower expert index.  allowed == NULL means every expert.  Returns how many were found. */
static int topk_select(const float *z, const uint8_t *allowed, int N, int k, int32_t *out)
{
    uint8_t *taken = (uint8_t *)calloc((size_t)N, 1);
    int found = 0;
    for (int j = 0; j < k; ++j) {
        int best = -1;
        for (int e = 0; e < N; ++e) {
            if (taken[e] || (allowed && !allowed[e])) continue;
            if (best < 0 || z[e] > z[best]) best = e; /* strict: ties keep the lower index */
        }
        if (best < 0) break;
        taken[best] = 1;
        out[found++] = best;
    }
    free(taken);
    return found;
}

/* Gates of a selection: softmax over the k selected logits only (Sec. 4: the weights are renormalised over the new selection). */
static void gates_of_selection(const float *z, const int32_t *sel, int k, double *gate)
{
    double zmax = (double)z[sel[0]];
    for (int j = 1; j < k; ++j)
        if ((double)z[sel[j]] > zmax) zmax = (double)z[sel[j]];
    double den = 0.0;
    for (int j = 0; j < k; ++j) den += exp((double)z[sel[j]] - zmax);
    for (int j = 0; j < k; ++j) gate[j] = exp((double)z[sel[j]] - zmax) / den;
}

/* Softmax + top-k of one token's logits (Sec. 2.1): selection, renormalised gates, selected mass. */
static void select_and_weigh(const float *z, int N, int k, int32_t *sel, double *gate, double *psum)
{
    topk_select(z, NULL, N, k, sel);
    double zmax = (double)z[sel[0]], den = 0.0, num = 0.0;
    for (int e = 0; e < N; ++e) den += exp((double)z[e] - zmax);
    for (int j = 0; j < k; ++j) num += exp((double)z[sel[j]] - zmax);
    *psum = num / den;
    gates_of_selection(z, sel, k, gate);
}

/* Softmax + top-k from given fp32 logits [T,N] (the second half of orc_route on its own). */
int orc_topk(const float *logits, int T, int N, int k, int32_t *topk_idx, double *topk_gate, double *topk_psum)
{
    if (T < 0 || N <= 0 || k <= 0) return ORC_ERR_INVALID_ARG;
    if (k > N) return ORC_ERR_UNSUPPORTED;
    for (int t = 0; t < T; ++t)
        select_and_weigh(logits + (size_t)t * N, N, k, topk_idx + (size_t)t * k, topk_gate + (size_t)t * k,
                         topk_psum + t);
    return ORC_OK;
}

/* The "top-k weight sum" of any selection idx [T,k] (Sec. 4 lists these sums among the kernels' outputs): the share of
 * the softmax over all N experts that the selected experts hold, psum[t] = sum_j p[t, idx[t,j]].  For the router's own
 * top-k it is orc_topk's psum; for a remapped selection it says how much probability mass the remap kept.  Entries
 * outside [0,N) are skipped. */
int orc_selection_mass(const float *logits, const int32_t *idx, int T, int N, int k, double *psum)
{
    if (T < 0 || N <= 0 || k <= 0) return ORC_ERR_INVALID_ARG;
    for (int t = 0; t < T; ++t) {
        const float *z = logits + (size_t)t * N;
        double zmax = (double)z[0], den = 0.0, num = 0.0;
        for (int e = 1; e < N; ++e)
            if ((double)z[e] > zmax) zmax = (double)z[e];
        for (int e = 0; e < N; ++e) den += exp((double)z[e] - zmax);
        for (int j = 0; j < k; ++j) {
            const int32_t e = idx[(size_t)t * k + j];
            if (e >= 0 && e < N) num += exp((double)z[e] - zmax);
        }
        psum[t] = num / den;
    }
    return ORC_OK;
}

/*
 * Sigmoid-gated routers (Sec. 3.2.1 closes with the case of routers that do not use softmax: the bins are then
 * taken from differences of the scores before the sigmoid, i.e. of the logits, exactly as above; so binning, scoring,
 * nominations and the remap are orc_affinity_bin unchanged).  What differs is the weight of a selected expert.  The
 * paper prints no formula for it; the reading here is the usual one for such routers: score s = 1 / (1 + exp(-z)),
 * the k experts of largest score per token, and gates = the selected scores divided by their sum.  The sigmoid is
 * strictly increasing, so the selection is taken on the fp32 logits themselves (descending, ties to the lower index):
 * in floating point distinct logits can share a score, and both sides of a parity test must break such ties alike.
 *
 * orc_sigmoid_gates: gates [T,k] (fp64) and the sum of the selected scores ssum [T] for a given selection idx [T,k].
 * orc_topk_sigmoid: selection by logit, then the same.
 */
static double sigmoid64(double z) { return z >= 0.0 ? 1.0 / (1.0 + exp(-z)) : exp(z) / (1.0 + exp(z)); }

int orc_sigmoid_gates(const float *logits, const int32_t *idx, int T, int N, int k, double *gate, double *ssum)
{
    if (T < 0 || N <= 0 || k <= 0) return ORC_ERR_INVALID_ARG;
    if (k > N) return ORC_ERR_UNSUPPORTED;
    for (int t = 0; t < T; ++t) {
        double sum = 0.0;
        for (int j = 0; j < k; ++j) {
            const int32_t e = idx[(size_t)t * k + j];
            if (e < 0 || e >= N) return ORC_ERR_INVALID_ARG;
            sum += sigmoid64((double)logits[(size_t)t * N + e]);
        }
        for (int j = 0; j < k; ++j)
            gate[(size_t)t * k + j] = sigmoid64((double)logits[(size_t)t * N + idx[(size_t)t * k + j]]) / sum;
        if (ssum) ssum[t] = sum;
    }
    return ORC_OK;
}

int orc_topk_sigmoid(const float *logits, int T, int N, int k, int32_t *topk_idx, double *topk_gate, double *topk_ssum)
{
    if (T < 0 || N <= 0 || k <= 0) return ORC_ERR_INVALID_ARG;
    if (k > N) return ORC_ERR_UNSUPPORTED;
    for (int t = 0; t < T; ++t) topk_select(logits + (size_t)t * N, NULL, N, k, topk_idx + (size_t)t * k);
    return orc_sigmoid_gates(logits, topk_idx, T, N, k, topk_gate, topk_ssum);
}

/*
 * Router (Sec. 2.1): z[t,e] = sum_h x[t,h] * Wr[e,h] + bias[e], accumulated in fp64 and rounded
 * once to fp32; p = softmax(z); the k experts of largest z per token (descending, ties to the
 * lower index); psum = sum of the selected softmax probabilities; gates = the selected
 * probabilities renormalised to sum 1.
 */
int orc_route(const uint16_t *x_bf16, const float *Wr, const float *bias, int T, int H, int N, int k,
              float *logits, int32_t *topk_idx, double *topk_gate, double *topk_psum)
{
    if (T < 0 || H <= 0 || N <= 0 || k <= 0) return ORC_ERR_INVALID_ARG;
    if (k > N) return ORC_ERR_UNSUPPORTED;
    for (int t = 0; t < T; ++t) {
        float *z = logits + (size_t)t * N;
        for (int e = 0; e < N; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                acc += bf16_to_f64(x_bf16[(size_t)t * H + h]) * (double)Wr[(size_t)e * H + h];
            if (bias) acc += (double)bias[e];
            z[e] = (float)acc;
        }
        select_and_weigh(z, N, k, topk_idx + (size_t)t * k, topk_gate + (size_t)t * k, topk_psum + t);
    }
    return ORC_OK;
}

/*
 * AffinityBinning + adaptive expert scorer + expert remapper (Secs. 3.2.1, 3.3.1, 3.4, 4).
 *
 * Bins (Sec. 3.2.1).  The affinity of expert e for token t is log(p_e / p_top1) = z_e - z_max.
 * With d = z_max - z_e >= 0 taken as one fp32 subtract, the bin magnitude is
 *     q[t,e] = min(floor(alpha * d), beta)          (one fp32 multiply, then floor)
 * so the paper's bin value is -q; bin 0 holds the top-1; bin width is 1/alpha; q = beta means
 * "deeper than the beta allowed bins" and carries no weight.
 *
 * Score (Sec. 3.3.1).  Every (token, expert) pair with q < beta votes B^(-q) for the expert, where
 * the base B is the batch size T.  With Hst[e][j] = #{t : q[t,e] = j} the score is
 * sum_j Hst[e][j] * T^(-j); it is held exactly as the integer S[e] = sum_j Hst[e][j] * T^(beta-1-j).
 *
 * Active set.  U = experts some token selected.  Token by token, slot by slot in rank order, the
 * token nominates the highest-scoring expert of U that sits in a bin at least as good as the
 * slot's own pick and that the token has not nominated yet (equal scores: lower index).  A slot
 * whose own pick is out of range (q = beta) ends the token's nominations.  A = all nominations;
 * if fewer than k experts were nominated, A is filled from U by descending score.
 *
 * Remap (Sec. 3.4, Sec. 4).  Each token takes its top-k among A by the original logits; gates are
 * the softmax over the k selected original logits.
 *
 * enable = 0 (batch not memory-bound, Sec. 3.1.1 / 3.5) or T = 1 leaves the selection as it is.
 *
 * q_out [T,N], score_out [N], active_out [N] (0/1) are optional diagnostics (may be NULL).
 *
 * allow [T,N] (0/1) or NULL restricts, per token, the experts the token may be sent to (group-limited routers, see
 * orc_group_allowed below); NULL = every expert, which is the method as the paper states it.  With a mask, a
 * (token, expert) pair that is not allowed has no bin (it does not vote), is never nominated by that token and is
 * never selected for it; the token's own picks must be allowed.  A token whose allowed experts hold fewer than k
 * members of the active set keeps, for the slots that stay empty, its own picks in rank order (those not chosen yet).
 */
static int affinity_bin_core(const float *logits, const int32_t *topk_idx, const uint8_t *allow, int T, int N, int k,
                             float alpha, int beta, int enable, int32_t *new_idx, double *new_gate, int32_t *cnt_before,
                             int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active, int32_t *q_out,
                             uint64_t *score_out, int32_t *active_out)
{
    if (T < 0 || N <= 0 || k <= 0 || beta < 1 || !(alpha >= 0.0f) || isinf(alpha)) return ORC_ERR_INVALID_ARG;
    if (k > N || beta > ORC_MAX_BETA) return ORC_ERR_UNSUPPORTED;
    {
        double lim = 1.0;
        for (int j = 0; j < beta; ++j) lim *= (double)(T > 1 ? T : 1);
        if (lim >= 4611686018427387904.0) return ORC_ERR_UNSUPPORTED; /* T^beta must stay below 2^62 */
    }
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            int32_t e = topk_idx[(size_t)t * k + j];
            if (e < 0 || e >= N) return ORC_ERR_INVALID_ARG;
            if (allow && !allow[(size_t)t * N + e]) return ORC_ERR_INVALID_ARG;
            for (int i = 0; i < j; ++i)
                if (topk_idx[(size_t)t * k + i] == e) return ORC_ERR_INVALID_ARG;
        }

    int32_t *q = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1) * N);
    uint8_t *mask = (uint8_t *)calloc((size_t)N, 1);
    uint64_t *score = (uint64_t *)calloc((size_t)N, sizeof(uint64_t));
    uint8_t *inU = (uint8_t *)calloc((size_t)N, 1);
    uint8_t *inA = (uint8_t *)calloc((size_t)N, 1);
    uint8_t *used = (uint8_t *)calloc((size_t)N, 1);

    /* bins */
    for (int t = 0; t < T; ++t) {
        const float *z = logits + (size_t)t * N;
        float zmax = z[0];
        for (int e = 1; e < N; ++e)
            if (z[e] > zmax) zmax = z[e];
        for (int e = 0; e < N; ++e) {
            volatile float d = zmax - z[e];
            volatile float scaled = alpha * d;
            float qf = floorf(scaled);
            q[(size_t)t * N + e] = (qf >= (float)beta) ? beta : (int32_t)qf;
        }
    }
    /* histogram of bins per expert, votes of the original selection */
    memset(bin_hist, 0, sizeof(int32_t) * (size_t)N * beta);
    memset(cnt_before, 0, sizeof(int32_t) * (size_t)N);
    memset(cnt_after, 0, sizeof(int32_t) * (size_t)N);
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < N; ++e) {
            int32_t b = q[(size_t)t * N + e];
            if (allow && !allow[(size_t)t * N + e]) continue;
            if (b < beta) bin_hist[(size_t)e * beta + b] += 1;
        }
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) cnt_before[topk_idx[(size_t)t * k + j]] += 1;
    int nU = 0;
    for (int e = 0; e < N; ++e) {
        inU[e] = cnt_before[e] > 0;
        nU += inU[e];
    }
    /* score as a base-T integer with beta digits, most significant digit = bin 0 */
    for (int e = 0; e < N; ++e) {
        uint64_t s = 0;
        for (int j = 0; j < beta; ++j) s = s * (uint64_t)T + (uint64_t)bin_hist[(size_t)e * beta + j];
        score[e] = s;
    }

    if (!enable || T <= 1) {
        for (int t = 0; t < T; ++t) {
            for (int j = 0; j < k; ++j) new_idx[(size_t)t * k + j] = topk_idx[(size_t)t * k + j];
            gates_of_selection(logits + (size_t)t * N, new_idx + (size_t)t * k, k, new_gate + (size_t)t * k);
        }
        for (int e = 0; e < N; ++e) {
            cnt_after[e] = cnt_before[e];
            inA[e] = inU[e];
        }
        num_active[0] = nU;
        num_active[1] = nU;
    } else {
        /* nominations */
        for (int t = 0; t < T; ++t) {
            const int32_t *qt = q + (size_t)t * N;
            memset(used, 0, (size_t)N);
            for (int i = 0; i < k; ++i) {
                int32_t qi = qt[topk_idx[(size_t)t * k + i]];
                if (qi >= beta) break;
                int best = -1;
                for (int e = 0; e < N; ++e) {
                    if (!inU[e] || used[e] || qt[e] > qi) continue;
                    if (allow && !allow[(size_t)t * N + e]) continue;
                    if (best < 0 || score[e] > score[best]) best = e;
                }
                /* With the picks in rank order (descending logit, as top-k gives them) this is never empty: the
                 * slot's own pick and the picks before it all qualify, and fewer than that are used.  Picks handed
                 * over in another order can leave a slot without a candidate: it nominates nothing. */
                if (best < 0) continue;
                used[best] = 1;
                inA[best] = 1;
            }
        }
        /* fill to k */
        int nA = 0;
        for (int e = 0; e < N; ++e) nA += inA[e];
        while (nA < k) {
            int best = -1;
            for (int e = 0; e < N; ++e) {
                if (!inU[e] || inA[e]) continue;
                if (best < 0 || score[e] > score[best]) best = e;
            }
            if (best < 0) break; /* cannot happen for T >= 1: |U| >= k */
            inA[best] = 1;
            ++nA;
        }
        /* remap */
        for (int t = 0; t < T; ++t) {
            const float *z = logits + (size_t)t * N;
            int32_t *sel = new_idx + (size_t)t * k;
            for (int e = 0; e < N; ++e) mask[e] = inA[e] && (!allow || allow[(size_t)t * N + e]);
            int found = topk_select(z, mask, N, k, sel);
            for (int j = 0; j < k && found < k; ++j) { /* only with an allow mask: see the header */
                const int32_t own = topk_idx[(size_t)t * k + j];
                int chosen = 0;
                for (int i = 0; i < found; ++i) chosen |= sel[i] == own;
                if (!chosen) sel[found++] = own;
            }
            gates_of_selection(z, sel, k, new_gate + (size_t)t * k);
            for (int j = 0; j < k; ++j) cnt_after[sel[j]] += 1;
        }
        int nAfter = 0;
        for (int e = 0; e < N; ++e) nAfter += cnt_after[e] > 0;
        num_active[0] = nU;
        num_active[1] = nAfter;
    }

    if (q_out) memcpy(q_out, q, sizeof(int32_t) * (size_t)T * N);
    if (score_out) memcpy(score_out, score, sizeof(uint64_t) * (size_t)N);
    if (active_out)
        for (int e = 0; e < N; ++e) active_out[e] = inA[e];
    free(q);
    free(score);
    free(inU);
    free(inA);
    free(used);
    free(mask);
    return ORC_OK;
}

int orc_affinity_bin(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha, int beta,
                     int enable, int32_t *new_idx, double *new_gate, int32_t *cnt_before, int32_t *cnt_after,
                     int32_t *bin_hist, int32_t *num_active, int32_t *q_out, uint64_t *score_out,
                     int32_t *active_out)
{
    return affinity_bin_core(logits, topk_idx, NULL, T, N, k, alpha, beta, enable, new_idx, new_gate, cnt_before,
                             cnt_after, bin_hist, num_active, q_out, score_out, active_out);
}

/*
 * Group-limited routers.  Sec. 1 lists expert grouping among the architectures the method has to cover and says no
 * more about it.  The reading here: the N experts form n_group groups of N / n_group consecutive experts; a token
 * may only be sent to experts of its topk_group best groups, the score of a group being the largest logit in it
 * (softmax and sigmoid are increasing, so this is also the largest probability or score), equal group scores to the
 * lower group; the router's selection is the top-k among those experts; and the remap keeps every token inside its
 * own groups, so whatever the limit buys (a bound on the devices a token's activations travel to) survives it.
 * Everything else is orc_affinity_bin with that mask (see there for what the mask does).
 *
 * orc_group_allowed: allow [T,N] (0/1).
 * orc_topk_grouped: the group-limited selection, its gates (gate_fn 0: softmax over the selected logits, 1: the
 *   selected sigmoid scores over their sum) and the third output (0: the selected share of the softmax over ALL
 *   N experts, 1: the sum of the selected scores).
 * orc_affinity_bin_grouped: the remap under the mask; topk_idx is the selection of orc_topk_grouped.  Gates as in
 *   orc_affinity_bin (softmax); for sigmoid gates apply orc_sigmoid_gates to new_idx.
 */
int orc_group_allowed(const float *logits, int T, int N, int n_group, int topk_group, uint8_t *allow)
{
    if (T < 0 || N <= 0 || n_group <= 0 || topk_group <= 0 || topk_group > n_group || (N % n_group) != 0)
        return ORC_ERR_INVALID_ARG;
    const int gs = N / n_group;
    float *gscore = (float *)malloc(sizeof(float) * (size_t)n_group);
    int32_t *best = (int32_t *)malloc(sizeof(int32_t) * (size_t)topk_group);
    for (int t = 0; t < T; ++t) {
        const float *z = logits + (size_t)t * N;
        for (int g = 0; g < n_group; ++g) {
            gscore[g] = z[(size_t)g * gs];
            for (int i = 1; i < gs; ++i)
                if (z[(size_t)g * gs + i] > gscore[g]) gscore[g] = z[(size_t)g * gs + i];
        }
        const int found = topk_select(gscore, NULL, n_group, topk_group, best);
        memset(allow + (size_t)t * N, 0, (size_t)N);
        for (int j = 0; j < found; ++j) memset(allow + (size_t)t * N + (size_t)best[j] * gs, 1, (size_t)gs);
    }
    free(gscore);
    free(best);
    return ORC_OK;
}

int orc_topk_grouped(const float *logits, int T, int N, int k, int n_group, int topk_group, int gate_fn,
                     int32_t *topk_idx, double *topk_gate, double *topk_third)
{
    if (T < 0 || N <= 0 || k <= 0 || (gate_fn != 0 && gate_fn != 1)) return ORC_ERR_INVALID_ARG;
    if (k > N) return ORC_ERR_UNSUPPORTED;
    if (n_group <= 0 || topk_group <= 0 || topk_group > n_group || (N % n_group) != 0 ||
        (long)topk_group * (N / n_group) < k)
        return ORC_ERR_INVALID_ARG;
    uint8_t *allow = (uint8_t *)malloc((size_t)(T > 0 ? T : 1) * N);
    int rc = orc_group_allowed(logits, T, N, n_group, topk_group, allow);
    for (int t = 0; t < T && rc == ORC_OK; ++t) {
        const float *z = logits + (size_t)t * N;
        int32_t *sel = topk_idx + (size_t)t * k;
        topk_select(z, allow + (size_t)t * N, N, k, sel);
        if (gate_fn == 0) {
            double zmax = (double)z[0], den = 0.0, num = 0.0;
            for (int e = 1; e < N; ++e)
                if ((double)z[e] > zmax) zmax = (double)z[e];
            for (int e = 0; e < N; ++e) den += exp((double)z[e] - zmax);
            for (int j = 0; j < k; ++j) num += exp((double)z[sel[j]] - zmax);
            topk_third[t] = num / den;
            gates_of_selection(z, sel, k, topk_gate + (size_t)t * k);
        }
    }
    if (rc == ORC_OK && gate_fn == 1) rc = orc_sigmoid_gates(logits, topk_idx, T, N, k, topk_gate, topk_third);
    free(allow);
    return rc;
}

int orc_affinity_bin_grouped(const float *logits, const int32_t *topk_idx, int T, int N, int k, int n_group,
                             int topk_group, float alpha, int beta, int enable, int32_t *new_idx, double *new_gate,
                             int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                             int32_t *active_out)
{
    if (T < 0 || N <= 0) return ORC_ERR_INVALID_ARG;
    uint8_t *allow = (uint8_t *)malloc((size_t)(T > 0 ? T : 1) * N);
    int rc = orc_group_allowed(logits, T, N, n_group, topk_group, allow);
    if (rc == ORC_OK)
        rc = affinity_bin_core(logits, topk_idx, allow, T, N, k, alpha, beta, enable, new_idx, new_gate, cnt_before,
                               cnt_after, bin_hist, num_active, NULL, NULL, active_out);
    free(allow);
    return rc;
}

/*
 * Score-biased selection, the literal reading of the passage of Sec. 3.3.1 that describes the scorer as adding
 * to an expert's router logit a weighted score that grows with how often the batch's other tokens prefer that
 * expert, as a variant of orc_affinity_bin:
 * bins, histogram and base-T scores exactly as there; then, instead of nominations and an active set,
 *   s_e    = score_e / T^beta                 in [0, 1] (fp64 division, rounded once to fp32),
 *   z'[t,e] = z[t,e] + gamma * s_e            (one fp32 multiply, one fp32 add),
 * and every token keeps its top-ranked expert (Sec. 3.3.1: high-confidence tokens are always mapped to their
 * top-ranked expert) and takes for its other k-1 slots the experts of largest z' among those the batch already
 * invokes (Sec. 1: redirected to experts the batch is already activating), equal z' to the lower index.
 * Gates: softmax over the selected ORIGINAL logits.  gamma = 0 reproduces the unchanged selection.
 * bias_out [N] (optional) receives gamma * s_e.
 */
int orc_affinity_bin_biased(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha, int beta,
                            float gamma, int enable, int32_t *new_idx, double *new_gate, int32_t *cnt_before,
                            int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active, float *bias_out)
{
    if (T < 0 || N <= 0 || k <= 0 || beta < 1 || !(alpha >= 0.0f) || isinf(alpha) || !(gamma >= 0.0f) || isinf(gamma))
        return ORC_ERR_INVALID_ARG;
    if (k > N || beta > ORC_MAX_BETA) return ORC_ERR_UNSUPPORTED;
    double tpow = 1.0; /* T^beta, by repeated multiplication */
    for (int j = 0; j < beta; ++j) tpow *= (double)(T > 1 ? T : 1);
    if (tpow >= 4611686018427387904.0) return ORC_ERR_UNSUPPORTED;
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            int32_t e = topk_idx[(size_t)t * k + j];
            if (e < 0 || e >= N) return ORC_ERR_INVALID_ARG;
            for (int i = 0; i < j; ++i)
                if (topk_idx[(size_t)t * k + i] == e) return ORC_ERR_INVALID_ARG;
        }
    uint8_t *allowed = (uint8_t *)calloc((size_t)N, 1);
    float *bias = (float *)calloc((size_t)N, sizeof(float));
    float *zb = (float *)malloc(sizeof(float) * (size_t)N);

    memset(bin_hist, 0, sizeof(int32_t) * (size_t)N * beta);
    memset(cnt_before, 0, sizeof(int32_t) * (size_t)N);
    memset(cnt_after, 0, sizeof(int32_t) * (size_t)N);
    for (int t = 0; t < T; ++t) {
        const float *z = logits + (size_t)t * N;
        float zmax = z[0];
        for (int e = 1; e < N; ++e)
            if (z[e] > zmax) zmax = z[e];
        for (int e = 0; e < N; ++e) {
            volatile float d = zmax - z[e];
            volatile float scaled = alpha * d;
            float qf = floorf(scaled);
            if (qf < (float)beta) bin_hist[(size_t)e * beta + (int32_t)qf] += 1;
        }
        for (int j = 0; j < k; ++j) cnt_before[topk_idx[(size_t)t * k + j]] += 1;
    }
    int nU = 0;
    for (int e = 0; e < N; ++e) nU += cnt_before[e] > 0;
    for (int e = 0; e < N; ++e) {
        uint64_t sc = 0;
        for (int j = 0; j < beta; ++j) sc = sc * (uint64_t)T + (uint64_t)bin_hist[(size_t)e * beta + j];
        volatile float se = (float)((double)sc / tpow);
        volatile float b = gamma * se;
        bias[e] = b;
    }
    const int bypass = !enable || T <= 1;
    for (int t = 0; t < T; ++t) {
        const float *z = logits + (size_t)t * N;
        int32_t *sel = new_idx + (size_t)t * k;
        if (bypass) {
            for (int j = 0; j < k; ++j) sel[j] = topk_idx[(size_t)t * k + j];
        } else {
            const int32_t top = topk_idx[(size_t)t * k];
            sel[0] = top;
            for (int e = 0; e < N; ++e) {
                allowed[e] = cnt_before[e] > 0 && e != top;
                volatile float v = z[e] + bias[e];
                zb[e] = v;
            }
            if (k > 1) topk_select(zb, allowed, N, k - 1, sel + 1);
        }
        gates_of_selection(z, sel, k, new_gate + (size_t)t * k);
        for (int j = 0; j < k; ++j) cnt_after[sel[j]] += 1;
    }
    int nAfter = 0;
    for (int e = 0; e < N; ++e) nAfter += cnt_after[e] > 0;
    num_active[0] = nU;
    num_active[1] = nAfter;
    if (bias_out) memcpy(bias_out, bias, sizeof(float) * (size_t)N);
    free(allowed);
    free(bias);
    free(zb);
    return ORC_OK;
}

/*
 * Token assignment (Sec. 4): per-expert pair counts, exclusive offsets by expert id, and the list
 * of (token, slot) pairs t*k+slot grouped by expert, ascending in t then slot inside an expert.
 * active_experts holds the invoked expert ids ascending; entries past num_active are -1.
 */
int orc_permute(const int32_t *idx, int T, int N, int k, int32_t *expert_offsets, int32_t *perm,
                int32_t *active_experts, int32_t *num_active)
{
    if (T < 0 || N <= 0 || k <= 0) return ORC_ERR_INVALID_ARG;
    for (int i = 0; i < T * k; ++i)
        if (idx[i] < 0 || idx[i] >= N) return ORC_ERR_INVALID_ARG;
    int32_t *count = (int32_t *)calloc((size_t)N, sizeof(int32_t));
    for (int i = 0; i < T * k; ++i) count[idx[i]] += 1;
    expert_offsets[0] = 0;
    for (int e = 0; e < N; ++e) expert_offsets[e + 1] = expert_offsets[e] + count[e];
    int na = 0;
    for (int e = 0; e < N; ++e) {
        active_experts[e] = -1;
        if (count[e] > 0) active_experts[na++] = e;
    }
    num_active[0] = na;
    memset(count, 0, sizeof(int32_t) * (size_t)N);
    for (int i = 0; i < T * k; ++i) { /* i = t*k+slot ascending: stable */
        int e = idx[i];
        perm[expert_offsets[e] + count[e]] = i;
        count[e] += 1;
    }
    free(count);
    return ORC_OK;
}

/* One SwiGLU FFN applied to a list of tokens: out[i,:] = Wd * (silu(Wg x) .* (Wu x)).
 * Wg, Wu are [F,H], Wd is [H,F], all bf16 row-major; xs is [T,H] fp64; out is [ntok,H] fp64. */
static void swiglu_ffn(const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd, int H, int F,
                       const double *xs, const int32_t *tok, int ntok, double *out)
{
    double *hbuf = (double *)malloc(sizeof(double) * (size_t)ntok * F);
#pragma omp parallel
    {
        double *row = (double *)malloc(sizeof(double) * (size_t)(H > F ? H : F) * 2);
        double *rowg = row, *rowu = row + (H > F ? H : F);
#pragma omp for schedule(static)
        for (int f = 0; f < F; ++f) {
            for (int h = 0; h < H; ++h) {
                rowg[h] = bf16_to_f64(Wg[(size_t)f * H + h]);
                rowu[h] = bf16_to_f64(Wu[(size_t)f * H + h]);
            }
            for (int i = 0; i < ntok; ++i) {
                const double *x = xs + (size_t)tok[i] * H;
                double a = 0.0, b = 0.0;
                for (int h = 0; h < H; ++h) {
                    a += rowg[h] * x[h];
                    b += rowu[h] * x[h];
                }
                hbuf[(size_t)i * F + f] = (a / (1.0 + exp(-a))) * b;
            }
        }
#pragma omp for schedule(static)
        for (int r = 0; r < H; ++r) {
            for (int f = 0; f < F; ++f) rowg[f] = bf16_to_f64(Wd[(size_t)r * F + f]);
            for (int i = 0; i < ntok; ++i) {
                const double *hv = hbuf + (size_t)i * F;
                double o = 0.0;
                for (int f = 0; f < F; ++f) o += rowg[f] * hv[f];
                out[(size_t)i * H + r] = o;
            }
        }
        free(row);
    }
    free(hbuf);
}

/*
 * Grouped expert FFN and combine: y[t] = sum_j gate[t,j] * FFN_{idx[t,j]}(x[t]) + sum_s FFN_s(x[t]),
 * shared experts entering with weight 1 (Sec. 3.3.1, last paragraph).  The intermediate vector is
 * never rounded.  Routed weights: Wg, Wu [N,F,H], Wd [N,H,F]; shared: Sg, Su [n_shared,F_shared,H],
 * Sd [n_shared,H,F_shared]; all bf16 row-major.  y is [T,H] fp64.
 */
int orc_moe_ffn(const uint16_t *x_bf16, const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd,
                const uint16_t *Sg, const uint16_t *Su, const uint16_t *Sd, int n_shared, int F_shared,
                const int32_t *idx, const double *gate, int T, int H, int F, int N, int k, double *y)
{
    if (T < 0 || H <= 0 || F <= 0 || N <= 0 || k <= 0 || n_shared < 0) return ORC_ERR_INVALID_ARG;
    if (n_shared > 0 && (F_shared <= 0 || !Sg || !Su || !Sd)) return ORC_ERR_INVALID_ARG;
    for (int i = 0; i < T * k; ++i)
        if (idx[i] < 0 || idx[i] >= N) return ORC_ERR_INVALID_ARG;
    if (T == 0) return ORC_OK;
    double *xs = (double *)malloc(sizeof(double) * (size_t)T * H);
    for (size_t i = 0; i < (size_t)T * H; ++i) xs[i] = bf16_to_f64(x_bf16[i]);
    for (size_t i = 0; i < (size_t)T * H; ++i) y[i] = 0.0;
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    int32_t *slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    double *out = (double *)malloc(sizeof(double) * (size_t)T * H);
    /* per-pair expert outputs o[t,j,:], kept so that the combine sums slots in rank order */
    double *o = (double *)calloc((size_t)T * k * H, sizeof(double));
    for (int e = 0; e < N; ++e) {
        int n = 0;
        for (int t = 0; t < T; ++t)
            for (int j = 0; j < k; ++j)
                if (idx[(size_t)t * k + j] == e) {
                    tok[n] = t;
                    slot[n] = j;
                    ++n;
                }
        if (n == 0) continue;
        swiglu_ffn(Wg + (size_t)e * F * H, Wu + (size_t)e * F * H, Wd + (size_t)e * H * F, H, F, xs, tok, n, out);
        for (int i = 0; i < n; ++i)
            memcpy(o + ((size_t)tok[i] * k + slot[i]) * H, out + (size_t)i * H, sizeof(double) * (size_t)H);
    }
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            double g = gate[(size_t)t * k + j];
            const double *oj = o + ((size_t)t * k + j) * H;
            for (int h = 0; h < H; ++h) y[(size_t)t * H + h] += g * oj[h];
        }
    for (int t = 0; t < T; ++t) tok[t] = t;
    for (int s = 0; s < n_shared; ++s) {
        swiglu_ffn(Sg + (size_t)s * F_shared * H, Su + (size_t)s * F_shared * H, Sd + (size_t)s * H * F_shared, H,
                   F_shared, xs, tok, T, out);
        for (size_t i = 0; i < (size_t)T * H; ++i) y[i] += out[i];
    }
    free(o);
    free(out);
    free(slot);
    free(tok);
    free(xs);
    return ORC_OK;
}

/* ------------------------------------------------------------------------------------------------------------
 * Expert weights in 8-bit floating point, weight-only (activations stay bf16): a widening beyond the paper's
 * bf16 runs (its Sec. 5 shows the method is additive to weight quantisation).  Format: OCP FP8 E4M3 (1 sign,
 * 4 exponent bits with bias 7, 3 mantissa bits, subnormals, no infinities, S.1111.111 = NaN, largest finite
 * value 448), one fp32 scale per weight-matrix row.
 * ------------------------------------------------------------------------------------------------------------ */

/* Value of an E4M3 code. */
double orc_e4m3_decode(uint8_t c)
{
    const int sgn = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0)
        v = ldexp((double)m, -9); /* subnormal: m/8 * 2^-6 */
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sgn ? -v : v;
}

/* Nearest E4M3 code of v, ties to the even code, magnitudes of 448 and above to +-448, NaN to NaN. */
uint8_t orc_e4m3_encode(float v)
{
    const uint8_t sgn = signbit(v) ? 0x80 : 0x00;
    if (isnan(v)) return (uint8_t)(sgn | 0x7f);
    const double a = fabs((double)v);
    if (a >= 448.0) return (uint8_t)(sgn | 0x7e);
    int code;
    if (a < ldexp(1.0, -6)) {
        code = (int)rint(ldexp(a, 9)); /* multiples of 2^-9; 8 is the smallest normal */
    } else {
        int e;
        const double fr = frexp(a, &e); /* a = fr * 2^e, fr in [0.5, 1) */
        const int ex = e - 1;           /* a = (2 fr) * 2^ex, 2 fr in [1, 2) */
        int q = (int)rint((2.0 * fr - 1.0) * 8.0);
        code = ((ex + 7) << 3) + q;     /* q = 8 carries into the exponent */
    }
    if (code > 0x7e) code = 0x7e;
    return (uint8_t)(sgn | code);
}

/*
 * Row-wise quantisation of bf16 weights W [rows, K]: scale = amax / 448 (one fp32 division; 1 for an all-zero
 * row), code = encode(w / scale) (one fp32 division).  The dequantised weight is decode(code) * scale.
 */
int orc_quantize_rows_e4m3(const uint16_t *W_bf16, long rows, int K, uint8_t *codes, float *scales)
{
    if (rows < 0 || K <= 0) return ORC_ERR_INVALID_ARG;
    for (long r = 0; r < rows; ++r) {
        const uint16_t *w = W_bf16 + (size_t)r * K;
        float amax = 0.0f;
        for (int i = 0; i < K; ++i) {
            const float a = fabsf((float)bf16_to_f64(w[i]));
            if (a > amax) amax = a;
        }
        volatile float sc = amax / 448.0f;
        if (amax == 0.0f) sc = 1.0f;
        scales[r] = sc;
        for (int i = 0; i < K; ++i) {
            volatile float q = (float)bf16_to_f64(w[i]) / sc;
            codes[(size_t)r * K + i] = orc_e4m3_encode(q);
        }
    }
    return ORC_OK;
}

/* swiglu_ffn with quantised weights: rows of codes with one scale each. */
static void swiglu_ffn_q8(const uint8_t *Qg, const uint8_t *Qu, const uint8_t *Qd, const float *sg, const float *su,
                          const float *sd, int H, int F, const double *xs, const int32_t *tok, int ntok, double *out)
{
    double *hbuf = (double *)malloc(sizeof(double) * (size_t)ntok * F);
#pragma omp parallel
    {
        double *row = (double *)malloc(sizeof(double) * (size_t)(H > F ? H : F) * 2);
        double *rowg = row, *rowu = row + (H > F ? H : F);
#pragma omp for schedule(static)
        for (int f = 0; f < F; ++f) {
            for (int h = 0; h < H; ++h) {
                rowg[h] = orc_e4m3_decode(Qg[(size_t)f * H + h]);
                rowu[h] = orc_e4m3_decode(Qu[(size_t)f * H + h]);
            }
            for (int i = 0; i < ntok; ++i) {
                const double *x = xs + (size_t)tok[i] * H;
                double a = 0.0, b = 0.0;
                for (int h = 0; h < H; ++h) {
                    a += rowg[h] * x[h];
                    b += rowu[h] * x[h];
                }
                a *= (double)sg[f];
                b *= (double)su[f];
                hbuf[(size_t)i * F + f] = (a / (1.0 + exp(-a))) * b;
            }
        }
#pragma omp for schedule(static)
        for (int r = 0; r < H; ++r) {
            for (int f = 0; f < F; ++f) rowg[f] = orc_e4m3_decode(Qd[(size_t)r * F + f]);
            for (int i = 0; i < ntok; ++i) {
                const double *hv = hbuf + (size_t)i * F;
                double o = 0.0;
                for (int f = 0; f < F; ++f) o += rowg[f] * hv[f];
                out[(size_t)i * H + r] = o * (double)sd[r];
            }
        }
        free(row);
    }
    free(hbuf);
}

/*
 * orc_moe_ffn with E4M3 weights: Qg, Qu [N,F,H], Qd [N,H,F] codes; sg, su [N,F], sd [N,H] scales; shared
 * experts likewise (SQ*, ss*).  Everything else as orc_moe_ffn.
 */
int orc_moe_ffn_q8(const uint16_t *x_bf16, const uint8_t *Qg, const uint8_t *Qu, const uint8_t *Qd, const float *sg,
                   const float *su, const float *sd, const uint8_t *SQg, const uint8_t *SQu, const uint8_t *SQd,
                   const float *ssg, const float *ssu, const float *ssd, int n_shared, int F_shared, const int32_t *idx,
                   const double *gate, int T, int H, int F, int N, int k, double *y)
{
    if (T < 0 || H <= 0 || F <= 0 || N <= 0 || k <= 0 || n_shared < 0) return ORC_ERR_INVALID_ARG;
    if (n_shared > 0 && (F_shared <= 0 || !SQg || !SQu || !SQd || !ssg || !ssu || !ssd)) return ORC_ERR_INVALID_ARG;
    for (int i = 0; i < T * k; ++i)
        if (idx[i] < 0 || idx[i] >= N) return ORC_ERR_INVALID_ARG;
    if (T == 0) return ORC_OK;
    double *xs = (double *)malloc(sizeof(double) * (size_t)T * H);
    for (size_t i = 0; i < (size_t)T * H; ++i) xs[i] = bf16_to_f64(x_bf16[i]);
    for (size_t i = 0; i < (size_t)T * H; ++i) y[i] = 0.0;
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    int32_t *slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)T);
    double *out = (double *)malloc(sizeof(double) * (size_t)T * H);
    double *o = (double *)calloc((size_t)T * k * H, sizeof(double));
    for (int e = 0; e < N; ++e) {
        int n = 0;
        for (int t = 0; t < T; ++t)
            for (int j = 0; j < k; ++j)
                if (idx[(size_t)t * k + j] == e) {
                    tok[n] = t;
                    slot[n] = j;
                    ++n;
                }
        if (n == 0) continue;
        swiglu_ffn_q8(Qg + (size_t)e * F * H, Qu + (size_t)e * F * H, Qd + (size_t)e * H * F, sg + (size_t)e * F,
                      su + (size_t)e * F, sd + (size_t)e * H, H, F, xs, tok, n, out);
        for (int i = 0; i < n; ++i)
            memcpy(o + ((size_t)tok[i] * k + slot[i]) * H, out + (size_t)i * H, sizeof(double) * (size_t)H);
    }
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            double g = gate[(size_t)t * k + j];
            const double *oj = o + ((size_t)t * k + j) * H;
            for (int h = 0; h < H; ++h) y[(size_t)t * H + h] += g * oj[h];
        }
    for (int t = 0; t < T; ++t) tok[t] = t;
    for (int s = 0; s < n_shared; ++s) {
        swiglu_ffn_q8(SQg + (size_t)s * F_shared * H, SQu + (size_t)s * F_shared * H, SQd + (size_t)s * H * F_shared,
                      ssg + (size_t)s * F_shared, ssu + (size_t)s * F_shared, ssd + (size_t)s * H, H, F_shared, xs, tok,
                      T, out);
        for (size_t i = 0; i < (size_t)T * H; ++i) y[i] += out[i];
    }
    free(o);
    free(out);
    free(slot);
    free(tok);
    free(xs);
    return ORC_OK;
}

/* ------------------------------------------------------------------------------------------------------------
 * Expert weights in 4-bit floating point with shared block scales, weight-only: the OCP Microscaling format
 * MXFP4.  Elements are FP4 E2M1 (1 sign, 2 exponent bits with bias 1, 1 mantissa bit: magnitudes 0, 0.5, 1, 1.5,
 * 2, 3, 4, 6; no infinities, no NaN); every block of 32 consecutive elements of a weight-matrix row shares one
 * scale X = 2^(E - 127), stored as the 8-bit exponent E (E8M0; 255 = NaN, not produced here).  The weight a
 * code stands for is decode(code) * X: a power of two times a two-bit significand, hence exactly a bf16 number,
 * so the FFN over MXFP4 weights IS the bf16 FFN (orc_moe_ffn) over the dequantised weights.
 * ------------------------------------------------------------------------------------------------------------ */

static const double kE2M1[8] = {0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0};

/* Value of an E2M1 code (low four bits of c). */
double orc_e2m1_decode(uint8_t c)
{
    const double v = kE2M1[c & 7];
    return (c & 8) ? -v : v;
}

/* Nearest E2M1 code of v: ties to the even code, magnitudes above 6 to +-6 (NaN to +-6 as well: the format has
 * no NaN). */
uint8_t orc_e2m1_encode(float v)
{
    const uint8_t sgn = signbit(v) ? 8 : 0;
    if (isnan(v)) return (uint8_t)(sgn | 7);
    const double a = fabs((double)v);
    if (a >= 6.0) return (uint8_t)(sgn | 7); /* saturation (also keeps the distances below exact for huge a) */
    int best = 0;
    for (int c = 1; c < 8; ++c) {
        const double d = fabs(a - kE2M1[c]), db = fabs(a - kE2M1[best]);
        if (d < db || (d == db && (c & 1) == 0)) best = c;
    }
    return (uint8_t)(sgn | best);
}

/*
 * Block quantisation of bf16 weights W [rows, K], K a multiple of 32, as the MX specification's conversion: per
 * block of 32, E - 127 = floor(log2(max |w|)) - 2 (2 = exponent of the largest E2M1 magnitude, 6 = 1.5 * 2^2),
 * clamped to the E8M0 range; an all-zero block gets X = 1; code = encode(w / X), which saturates the part of the
 * block above 6 X.  codes: one code per byte [rows, K]; scales: E [rows, K/32].
 */
int orc_quantize_mxfp4(const uint16_t *W_bf16, long rows, int K, uint8_t *codes, uint8_t *scales)
{
    if (rows < 0 || K <= 0 || (K % 32) != 0) return ORC_ERR_INVALID_ARG;
    const int nb = K / 32;
    for (long r = 0; r < rows; ++r)
        for (int b = 0; b < nb; ++b) {
            const uint16_t *w = W_bf16 + (size_t)r * K + (size_t)b * 32;
            double amax = 0.0;
            for (int i = 0; i < 32; ++i) {
                const double a = fabs(bf16_to_f64(w[i]));
                if (a > amax) amax = a;
            }
            int E = 127;
            if (amax > 0.0) {
                int ex;
                (void)frexp(amax, &ex); /* amax = fr * 2^ex with fr in [0.5, 1): floor(log2 amax) = ex - 1 */
                E = (ex - 1) - 2 + 127;
                if (E < 0) E = 0;
                if (E > 254) E = 254;
            }
            scales[(size_t)r * nb + b] = (uint8_t)E;
            for (int i = 0; i < 32; ++i)
                codes[(size_t)r * K + (size_t)b * 32 + i] = orc_e2m1_encode((float)ldexp(bf16_to_f64(w[i]), 127 - E));
        }
    return ORC_OK;
}

/* The bf16 weights that codes and scales stand for (exact; fails if a product is not a bf16 number). */
int orc_dequantize_mxfp4(const uint8_t *codes, const uint8_t *scales, long rows, int K, uint16_t *W_bf16)
{
    if (rows < 0 || K <= 0 || (K % 32) != 0) return ORC_ERR_INVALID_ARG;
    const int nb = K / 32;
    for (long r = 0; r < rows; ++r)
        for (int i = 0; i < K; ++i) {
            const int E = scales[(size_t)r * nb + i / 32];
            if (E == 255) return ORC_ERR_INVALID_ARG;
            const double v = ldexp(orc_e2m1_decode(codes[(size_t)r * K + i]), E - 127);
            const float f = (float)v;
            uint32_t u;
            memcpy(&u, &f, 4);
            if ((double)f != v || (u & 0xffffu) != 0 || isinf(f)) return ORC_ERR_INVALID_ARG;
            W_bf16[(size_t)r * K + i] = (uint16_t)(u >> 16);
        }
    return ORC_OK;
}
