/*
 * lynx.h -- C ABI of the MI355X (gfx950) implementation of the batched MoE-layer decode step of
 * Lynx (arXiv 2411.08982): router logits, softmax and top-k (Sec. 2.1); AffinityBinning, batch-wide
 * expert scoring and remapping (Secs. 3.2.1, 3.3.1, 3.4); token assignment and weight
 * renormalisation (Sec. 4); grouped SwiGLU expert FFN over the experts still invoked, and the
 * gate-weighted combine (the expert computation that the remapper dispatches, Sec. 3.4).
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer owned by the caller unless it says "host".  The library
 *    allocates nothing and keeps no state between calls (one exception, stated there: lynx_moe_layer_static
 *    remembers, per GPU, where its built-in scratch array lives).
 *  - Every call only enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the null
 *    stream).  No call synchronises with the host or reads device results on the host, so a sequence
 *    of calls can be captured into a hipGraph.
 *  - All matrices are dense row-major unless a packed layout is named.  bf16 values travel as
 *    uint16_t bit patterns.  T = decode tokens in the batch, H = hidden size, F = expert FFN width,
 *    N = routed experts, k = experts per token.
 *  - Return value: LYNX_OK, or a negative error; lynx_last_error() gives a host string for the last
 *    error of the calling thread.  On error nothing has been enqueued.
 *  - Inputs are assumed finite.  Indices outside [0,N) in caller-provided index arrays never cause an
 *    out-of-bounds access: such pairs are skipped.
 *  - Limits: T <= LYNX_MAX_T, N <= LYNX_MAX_N, k <= LYNX_MAX_K, beta <= LYNX_MAX_BETA,
 *    H % 32 == 0, F % 32 == 0, F_shared % 32 == 0 (multiples of 64 for the FP8-weight calls, of 128 for MXFP4).
 *  - Beyond the paper's bf16 method the header also declares a variant of the expert scorer
 *    (lynx_affinity_bin_biased), FP8 and MXFP4 expert weights (lynx_*_fp8, lynx_*_fp4), sigmoid-gated and
 *    group-limited routers; each says so.  Measurement aids and test knobs are in lynx_bench.h.
 */
#ifndef LYNX_H
#define LYNX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LYNX_OK 0
#define LYNX_ERR_INVALID_ARG (-1) /* null pointer, negative size, alpha < 0 or not finite, beta < 1 */
#define LYNX_ERR_UNSUPPORTED (-2) /* a documented limit is exceeded (k > N, beta > 6, T^beta >= 2^62, ...) */
#define LYNX_ERR_HIP (-3)         /* a HIP runtime call failed */

#define LYNX_MAX_T 1024
#define LYNX_MAX_N 256
#define LYNX_MAX_K 16
#define LYNX_MAX_BETA 6
#define LYNX_STATIC_SCRATCH_BYTES (64u << 20) /* the built-in scratch array of lynx_moe_layer_static, per GPU */

/* Host string describing the last error on this thread ("" if none). */
const char *lynx_last_error(void);

/* Bytes of device workspace that lynx_affinity_bin, lynx_moe_ffn and lynx_moe_layer need for these
 * sizes (one buffer serves all; contents need not be preserved between calls; calls that share a
 * workspace must not overlap in time).  lynx_affinity_bin alone uses only the first 64 KiB.  N does not
 * enter the size: the per-expert tables are reserved for LYNX_MAX_N experts inside those 64 KiB. */
size_t lynx_workspace_bytes(int T, int H, int F, int N, int k, int n_shared, int F_shared);

/*
 * Router (Sec. 2.1): z[t,e] = sum_h x[t,h] * Wr[e,h] + bias[e] in fp32; p = softmax(z); the k
 * experts of largest z per token, descending, equal logits to the lower expert index.
 *   x_bf16 [T,H] bf16, Wr [N,H] fp32, bias [N] fp32 or NULL.
 *   logits [T,N] fp32 out; topk_idx [T,k] int32 out; topk_gate [T,k] fp32 out = selected
 *   probabilities renormalised to sum 1; topk_psum [T] fp32 out = sum of the selected probabilities.
 * Accuracy of the logits: fp32 multiply-adds over H terms in a fixed order, so a logit differs from the exactly
 * rounded sum by a few ulp of sum_h |x[t,h] * Wr[e,h]|, not of the logit itself.  For hidden states and router rows of
 * ordinary scale (terms that do not cancel by orders of magnitude) that is below 1e-5 * max(1, |z|), the bound the
 * parity tests check; a router whose terms are a thousand times larger than their sum loses the corresponding digits.
 */
int lynx_route(const uint16_t *x_bf16, const float *Wr, const float *bias, int T, int H, int N, int k,
               float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum, void *stream);

/*
 * AffinityBinning, batch-wide scoring, active-set selection, remapping (Secs. 3.2.1, 3.3.1, 3.4, 4).
 *   Bin magnitude q[t,e] = min(floor(alpha * (max_e' z[t,e'] - z[t,e])), beta), one fp32 subtract
 *   and one fp32 multiply (the paper's bin value is -q; bin width 1/alpha; beta allowed bins).
 *   bin_hist[e][j] = #{t : q[t,e] = j}, j < beta.  Score of expert e = sum_j bin_hist[e][j] * T^(-j)
 *   (batch size as the base, bin value as the exponent), compared exactly as a base-T integer.
 *   Each token, slot by slot in rank order, nominates the best-scoring expert among those the batch
 *   already invokes that lies in a bin at least as good as the slot's own pick (and that the token
 *   has not nominated yet; equal scores to the lower index); a slot whose own pick is out of range
 *   (q = beta) ends the token's nominations.  The active set is the union of the nominations, filled
 *   by descending score up to k experts if smaller.  Every token then takes its top-k by original
 *   logit within the active set; gates are the softmax over the k selected original logits.
 *   enable = 0 (batch not memory-bound, Sec. 3.1.1) or T = 1 keeps topk_idx as it is.
 *
 *   logits [T,N] fp32, topk_idx [T,k] int32 (k distinct experts per row, descending logit; a row in another
 *   order is accepted, and a slot that then finds no expert to nominate nominates nothing).
 *   new_idx [T,k] int32 out, new_gate [T,k] fp32 out, new_psum [T] fp32 out or NULL = the share of the softmax over
 *   all N experts that the NEW selection holds (Sec. 4 names the top-k weight sums among the kernels' outputs; beside
 *   lynx_route's topk_psum it says how much probability mass the remap gave up for the token: new_psum <= topk_psum,
 *   equal where the selection did not change), cnt_before [N], cnt_after [N] int32 out (pairs per expert before /
 *   after), bin_hist [N,beta] int32 out, num_active [2] int32 out (experts invoked before, after).
 *   workspace: lynx_workspace_bytes() bytes (the first 64 KiB are used).
 */
int lynx_affinity_bin(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha, int beta,
                      int enable, int32_t *new_idx, float *new_gate, float *new_psum, int32_t *cnt_before,
                      int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active, void *workspace, void *stream);

/*
 * Score-biased selection: the variant of the adaptive expert scorer that takes literally what Sec. 3.3.1 says
 * of it, namely that a weighted batch-level score is added to an expert's router logit.  Bins, histogram and base-T scores exactly as in
 * lynx_affinity_bin; then bias[e] = gamma * score[e] / T^beta (score / T^beta in [0,1]: one fp64 division
 * rounded to fp32, one fp32 multiply), and every token keeps its top-ranked expert (Sec. 3.3.1) and fills
 * its other k-1 slots with the experts of largest logit + bias (one fp32 addition) among those the batch
 * already invokes (Sec. 1), equal values to the lower index.  Gates: softmax over the selected ORIGINAL
 * logits.  gamma >= 0, finite; gamma = 0 or enable = 0 or T <= 1 leaves the selection unchanged.  Other
 * arguments, outputs and the workspace as in lynx_affinity_bin; composes with lynx_permute and lynx_moe_ffn.
 */
int lynx_affinity_bin_biased(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha, int beta,
                             float gamma, int enable, int32_t *new_idx, float *new_gate, float *new_psum,
                             int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                             void *workspace, void *stream);

/*
 * Token assignment (Sec. 4): expert_offsets [N+1] int32 out = exclusive prefix of pairs per expert;
 * perm [T*k] int32 out = pair ids t*k+slot grouped by expert ascending, ascending inside an expert;
 * active_experts [N] int32 out = invoked expert ids ascending, -1 past num_active; num_active [1] out.
 * idx [T,k] int32 must hold k distinct experts per row.
 */
int lynx_permute(const int32_t *idx, int T, int N, int k, int32_t *expert_offsets, int32_t *perm,
                 int32_t *active_experts, int32_t *num_active, void *stream);

/*
 * One-time re-layout of expert weights into the streaming layout lynx_moe_ffn reads (same byte
 * count as the row-major weights).  Input: Wg, Wu [E,F,H], Wd [E,H,F] bf16 row-major.  Output:
 *   Wgu_packed [E][F/16][H/32][2][64][8] bf16: tile (rt,kt), matrix m (0 = gate, 1 = up), entry
 *     (lane l, i) = W_m[rt*16 + l%16][kt*32 + (l/16)*8 + i];
 *   Wd_packed  [E][H/16][F/32][64][8] bf16: entry (lane l, i) = Wd[rt*16 + l%16][kt*32 + (l/16)*8 + i].
 * Each 16-row tile is then one contiguous run, read with 1 KiB wave-wide loads.
 */
int lynx_pack_weights(const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd, int E, int H, int F,
                      uint16_t *Wgu_packed, uint16_t *Wd_packed, void *stream);

/*
 * Grouped SwiGLU expert FFN over the invoked experts and gate-weighted combine:
 *   y[t] = sum_j gate[t,j] * Wd[e] (silu(Wg[e] x_t) .* (Wu[e] x_t)),  e = idx[t,j],
 *          + sum_s Sd[s] (silu(Sg[s] x_t) .* (Su[s] x_t))            (shared experts, weight 1,
 *                                                                      Sec. 3.3.1 last paragraph)
 * bf16 operands, fp32 accumulation; the intermediate vector is rounded to bf16 between the two
 * projections.  Each invoked expert's weights are read once per call (an expert with more tokens than one pass of
 * the kernel holds, 64 or 128, once per pass); experts with no pair are not touched.  Weights in the packed layout of
 * lynx_pack_weights (Sgu/Sd: packed with E = n_shared, F = F_shared; NULL when n_shared = 0).  expert_offsets / perm as
 * written by lynx_permute for the same idx: the invoked experts are those with a non-empty range in expert_offsets
 * (active_experts / num_active are accepted for symmetry with lynx_permute and not read).  y [T,H] fp32 out, overwritten.
 *
 * status: one int32, DEVICE, out, or NULL.  When both projections run as one launch, a down-projection workgroup waits
 * for the gate/up workgroups of its expert, which always precede it in dispatch order; the wait is bounded so that no
 * wave can hang.  If a wait ever runs out, the call does not pass garbage on: every element of y is NaN and *status is
 * 1; otherwise *status is 0.  (The return value cannot say it: the call has returned before the kernels run.)
 */
int lynx_moe_ffn(const uint16_t *x_bf16, const uint16_t *Wgu_packed, const uint16_t *Wd_packed,
                 const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared, int F_shared,
                 const int32_t *idx, const float *gate, const int32_t *expert_offsets, const int32_t *perm,
                 const int32_t *active_experts, const int32_t *num_active, int T, int H, int F, int N, int k,
                 float *y, int32_t *status, void *workspace, void *stream);

/*
 * The whole decode step of one MoE layer: the work of lynx_route, lynx_affinity_bin, lynx_permute and
 * lynx_moe_ffn chained on `stream` with the argument meanings above and identical results (the routing
 * side is issued as two launches up to 16 tokens and four beyond).  All intermediate arrays are outputs; new_psum and
 * status may be NULL.  Every argument check of the four calls is made before anything is enqueued.  stage_events: HOST
 * array of four hipEvent_t (entries may be NULL) or NULL: [0] is recorded on `stream` before the weight-streaming
 * launch(es), [1] and [2] after them, [3] after the combine (for measurement; see lynx_bench.h).
 */
int lynx_moe_layer(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                   const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared,
                   int F_shared, int T, int H, int F, int N, int k, float alpha, int beta, int enable, float *logits,
                   int32_t *topk_idx, float *topk_gate, float *topk_psum, int32_t *new_idx, float *new_gate,
                   float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                   int32_t *expert_offsets, int32_t *perm, int32_t *active_experts, int32_t *num_active_perm, float *y,
                   int32_t *status, void *workspace, void *stream, void *const *stage_events);

/*
 * lynx_moe_layer for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without workspace and
 * stage_events), same kernels and bit-identical results; the scratch memory is a device array built into the library
 * (LYNX_STATIC_SCRATCH_BYTES = 64 MiB; every GPU the library runs on holds its copy until the process ends).  The call
 * allocates and frees nothing.  Sizes whose lynx_workspace_bytes() exceeds the array are refused with
 * LYNX_ERR_UNSUPPORTED before anything is enqueued (all benchmark shapes up to T = 512 fit).  The first call on a device
 * looks up that device's copy of the array (the device must be current, as for any launch on `stream`; make that first
 * call outside a stream capture).  Every call on a GPU uses that GPU's one array, which keeps the last call's contents
 * (what must start at zero is cleared by the first kernel of each call): calls that overlap in time on one GPU race,
 * on any streams; calls on one stream, or ordered by events, are fine.
 */
int lynx_moe_layer_static(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                          const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared,
                          int F_shared, int T, int H, int F, int N, int k, float alpha, int beta, int enable, float *logits,
                          int32_t *topk_idx, float *topk_gate, float *topk_psum, int32_t *new_idx, float *new_gate,
                          float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                          int32_t *expert_offsets, int32_t *perm, int32_t *active_experts, int32_t *num_active_perm, float *y,
                          int32_t *status, void *stream);

/*
 * Expert weights in 8-bit floating point, weight-only (a widening beyond the paper's bf16 runs; its Sec. 5 shows
 * the method is additive to weight quantisation): halves the bytes the decode step is bound by.  Format: OCP FP8
 * E4M3 (largest value 448), one fp32 scale per weight-matrix row: scale = amax(row) / 448 (1 for an all-zero
 * row), code = nearest E4M3 value of w / scale (ties to even; both divisions correctly rounded fp32).
 * lynx_quantize_weights_fp8 quantises row-major bf16 weights (as for lynx_pack_weights; H and F multiples of
 * 64) straight into the streaming layout:
 *   Wgu_q [E][F/16][H/64][2][64][16] bytes, Wd_q [E][H/16][F/64][64][16] bytes (a 1 KiB tile = 16 rows x 64
 *   columns: lane l = row l%16, columns (l/16)*16 .. +15), scales_gu [E][2][F] (gate rows, then up rows),
 *   scales_d [E][H].  All DEVICE.
 */
int lynx_quantize_weights_fp8(const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd, int E, int H, int F,
                              uint8_t *Wgu_q, uint8_t *Wd_q, float *scales_gu, float *scales_d, void *stream);

/*
 * lynx_moe_ffn with FP8 weights (and the stage events of lynx_moe_layer): the codes are converted to bf16 in registers (exact), multiplied on the
 * matrix cores as in the bf16 path, and the accumulated sums are multiplied by the row scales; activations and
 * the intermediate vector stay bf16.  Shared experts quantised likewise (NULL when n_shared = 0).
 * stage_events may be NULL.  H, F, F_shared multiples of 64.
 */
int lynx_moe_ffn_fp8(const uint16_t *x_bf16, const uint8_t *Wgu_q, const uint8_t *Wd_q, const float *scales_gu,
                     const float *scales_d, const uint8_t *Sgu_q, const uint8_t *Sd_q, const float *shared_scales_gu,
                     const float *shared_scales_d, int n_shared, int F_shared, const int32_t *idx, const float *gate,
                     const int32_t *expert_offsets, const int32_t *perm, const int32_t *active_experts,
                     const int32_t *num_active, int T, int H, int F, int N, int k, float *y, int32_t *status,
                     void *workspace, void *stream, void *const *stage_events);

/* lynx_moe_layer with FP8 expert weights (routing unchanged). */
int lynx_moe_layer_fp8(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint8_t *Wgu_q,
                       const uint8_t *Wd_q, const float *scales_gu, const float *scales_d, const uint8_t *Sgu_q,
                       const uint8_t *Sd_q, const float *shared_scales_gu, const float *shared_scales_d, int n_shared,
                       int F_shared, int T, int H, int F, int N, int k, float alpha, int beta, int enable, float *logits,
                       int32_t *topk_idx, float *topk_gate, float *topk_psum, int32_t *new_idx, float *new_gate,
                       float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                       int32_t *expert_offsets, int32_t *perm, int32_t *active_experts, int32_t *num_active_perm,
                       float *y, int32_t *status, void *workspace, void *stream, void *const *stage_events);

/*
 * Expert weights in 4-bit floating point with shared block scales, weight-only (the same widening, a quarter of the
 * bf16 bytes plus 1/32 for the scales): the OCP Microscaling format MXFP4.  Elements are FP4 E2M1 (magnitudes 0,
 * 0.5, 1, 1.5, 2, 3, 4, 6); each block of 32 consecutive columns of a weight-matrix row shares the scale
 * 2^(E - 127), E an 8-bit exponent.  Conversion as in the MX specification: E - 127 = floor(log2(amax(block))) - 2,
 * clamped to [0, 254] (E = 127 for an all-zero block); code = nearest E2M1 value of w / 2^(E - 127), ties to the even
 * code, magnitudes above 6 to 6.  A code times its scale is exactly a bf16 number, so the FFN is the bf16 FFN over
 * the dequantised weights.  (Blocks whose largest magnitude is below 2^-124 are outside the tested range.)
 * lynx_quantize_weights_fp4 quantises row-major bf16 weights (as for lynx_pack_weights; H and F multiples of 128)
 * straight into the streaming layout:
 *   Wgu_q [E][F/16][H/128][2][64][16] bytes, Wd_q [E][H/16][F/128][64][16] bytes (a 1 KiB tile = 16 rows x 128
 *   columns: lane l = row l%16, columns (l/16)*32 .. +31, byte j = columns 2j (low nibble) and 2j+1);
 *   scales_gu [E][F/16][ceil(H/128 / 4)][64][2] dwords (lane, then gate|up; byte i of a dword = k-tile 4j+i),
 *   scales_d [E][H/32][ceil(F/128 / 4)][64][2] dwords (lane, then the first|second row tile of the row pair).
 * lynx_fp4_scale_words(E, rows, K, gate_up) gives the dword count of such a scale array (rows = F, K = H, gate_up
 * = 1 for scales_gu; rows = H, K = F, gate_up = 0 for scales_d).  All DEVICE.
 */
size_t lynx_fp4_scale_words(int E, int rows, int K, int gate_up);
int lynx_quantize_weights_fp4(const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd, int E, int H, int F,
                              uint8_t *Wgu_q, uint8_t *Wd_q, uint32_t *scales_gu, uint32_t *scales_d, void *stream);

/*
 * lynx_moe_ffn with MXFP4 weights (and the stage events of lynx_moe_layer): the codes are converted to bf16, times their block scale, in registers
 * (exact) and multiplied on the same bf16 MFMA path.  Shared experts: Sgu_q, Sd_q and their scale arrays in the
 * same layouts with E = n_shared, F = F_shared (NULL if n_shared == 0).  H, F, F_shared multiples of 128.
 */
int lynx_moe_ffn_fp4(const uint16_t *x_bf16, const uint8_t *Wgu_q, const uint8_t *Wd_q, const uint32_t *scales_gu,
                     const uint32_t *scales_d, const uint8_t *Sgu_q, const uint8_t *Sd_q,
                     const uint32_t *shared_scales_gu, const uint32_t *shared_scales_d, int n_shared, int F_shared,
                     const int32_t *idx, const float *gate, const int32_t *expert_offsets, const int32_t *perm,
                     const int32_t *active_experts, const int32_t *num_active, int T, int H, int F, int N, int k,
                     float *y, int32_t *status, void *workspace, void *stream, void *const *stage_events);

/* lynx_moe_layer with MXFP4 expert weights (routing unchanged). */
int lynx_moe_layer_fp4(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint8_t *Wgu_q,
                       const uint8_t *Wd_q, const uint32_t *scales_gu, const uint32_t *scales_d, const uint8_t *Sgu_q,
                       const uint8_t *Sd_q, const uint32_t *shared_scales_gu, const uint32_t *shared_scales_d,
                       int n_shared, int F_shared, int T, int H, int F, int N, int k, float alpha, int beta, int enable,
                       float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum, int32_t *new_idx,
                       float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist,
                       int32_t *num_active, int32_t *expert_offsets, int32_t *perm, int32_t *active_experts,
                       int32_t *num_active_perm, float *y, int32_t *status, void *workspace, void *stream,
                       void *const *stage_events);

/*
 * Sigmoid-gated routers.  Sec. 3.2.1 closes with routers that do not use softmax: their bins are taken from
 * differences of the scores before the sigmoid, that is of the logits, which is what lynx_affinity_bin computes
 * already; bins, histogram, scores, nominations and the remapped selection are therefore identical.  What
 * differs is the weight of a selected expert, for which the paper prints no formula.  The reading here is the usual
 * one for such routers: score = 1 / (1 + exp(-logit)) in fp32, the k experts of largest logit (the sigmoid is
 * increasing; equal logits to the lower index, decided on the fp32 logits), gate = score / sum of the k selected
 * scores.  The three calls below are lynx_route, lynx_affinity_bin and lynx_moe_layer (bf16 expert weights) with
 * these gates: same arguments, same layouts, same errors.  topk_ssum / new_ssum [T] fp32 out = the sum of the selected
 * scores, of the router's own and of the remapped selection (where the softmax calls give the selected probability
 * mass).  They compose with lynx_permute,
 * lynx_moe_ffn and the quantised FFN calls, which take any gates.
 */
int lynx_route_sigmoid(const uint16_t *x_bf16, const float *Wr, const float *bias, int T, int H, int N, int k,
                       float *logits, int32_t *topk_idx, float *topk_gate, float *topk_ssum, void *stream);
int lynx_affinity_bin_sigmoid(const float *logits, const int32_t *topk_idx, int T, int N, int k, float alpha, int beta,
                              int enable, int32_t *new_idx, float *new_gate, float *new_ssum, int32_t *cnt_before,
                              int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active, void *workspace, void *stream);
int lynx_moe_layer_sigmoid(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                           const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared,
                           int F_shared, int T, int H, int F, int N, int k, float alpha, int beta, int enable,
                           float *logits, int32_t *topk_idx, float *topk_gate, float *topk_ssum, int32_t *new_idx,
                           float *new_gate, float *new_ssum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist,
                           int32_t *num_active, int32_t *expert_offsets, int32_t *perm, int32_t *active_experts,
                           int32_t *num_active_perm, float *y, int32_t *status, void *workspace, void *stream,
                           void *const *stage_events);

/*
 * Group-limited routers.  Sec. 1 lists expert grouping among the architectures the method has to cover and gives no
 * rule for it.  The reading here: the N experts form n_group groups of N / n_group consecutive experts; the score of a
 * group for a token is the largest logit in it; the token may only be sent to experts of its topk_group best groups
 * (equal group scores to the lower group); the router's selection is the top-k among those; and the remap keeps the
 * token inside the same groups: a forbidden (token, expert) pair has no bin and casts no vote, is never nominated and
 * never selected.  A token whose groups hold fewer than k members of the active set takes them all and keeps, for the
 * slots left, its own picks that are not in the active set, in rank order (so new_idx always holds k distinct experts
 * the batch already invoked).  Batch scores, score order, active-set fill, gates, counts and permutation are as in
 * the calls above.  gate_fn: 0 = softmax gates, topk_third [T] = selected share of the softmax over ALL N experts;
 * 1 = sigmoid gates (see above), topk_third = sum of the selected scores; new_third [T] (or NULL) = the same of the
 * remapped selection.
 *
 * n_group >= 1 must divide N, 1 <= topk_group <= n_group, topk_group * N / n_group >= k, gate_fn in {0, 1}, else
 * LYNX_ERR_INVALID_ARG; n_group <= 64, else LYNX_ERR_UNSUPPORTED.  n_group = 1 (or topk_group = n_group) is the
 * router without groups.
 *
 * lynx_route_grouped: lynx_route with the group limit.
 * lynx_affinity_bin_grouped: top-k and remap from given logits in one call (the remap needs the group-limited
 *   selection, so it is computed here, not handed in): topk_idx / topk_gate [T,k] and topk_third [T] are OUTPUTS,
 *   the rest as lynx_affinity_bin.
 * lynx_moe_layer_grouped: lynx_moe_layer (bf16 expert weights) with the group limit.
 */
int lynx_route_grouped(const uint16_t *x_bf16, const float *Wr, const float *bias, int T, int H, int N, int k, int n_group,
                       int topk_group, int gate_fn, float *logits, int32_t *topk_idx, float *topk_gate, float *topk_third,
                       void *stream);
int lynx_affinity_bin_grouped(const float *logits, int T, int N, int k, int n_group, int topk_group, int gate_fn, float alpha,
                              int beta, int enable, int32_t *topk_idx, float *topk_gate, float *topk_third,
                              int32_t *new_idx, float *new_gate, float *new_third, int32_t *cnt_before,
                              int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active, void *workspace, void *stream);
int lynx_moe_layer_grouped(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                           const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared,
                           int F_shared, int T, int H, int F, int N, int k, int n_group, int topk_group, int gate_fn,
                           float alpha, int beta, int enable, float *logits, int32_t *topk_idx, float *topk_gate,
                           float *topk_third, int32_t *new_idx, float *new_gate, float *new_third, int32_t *cnt_before,
                           int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active, int32_t *expert_offsets,
                           int32_t *perm, int32_t *active_experts, int32_t *num_active_perm, float *y, int32_t *status,
                           void *workspace, void *stream, void *const *stage_events);

#ifdef __cplusplus
}
#endif
#endif /* LYNX_H */
