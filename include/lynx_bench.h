/*
 * lynx_bench.h -- measurement aids and test knobs of liblynx.  None of them is a step of the method (lynx.h has
 * those); the benchmark and the tests use them.  Same conventions as lynx.h: C ABI, DEVICE pointers unless a
 * parameter says "host", kernels only enqueued on `stream`, LYNX_OK or a negative error code.
 */
#ifndef LYNX_BENCH_H
#define LYNX_BENCH_H

#include "lynx.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * How many launches of the weight-streaming kernel lynx_moe_ffn issues for this batch size and expert width:
 * 1 (gate/up and down workgroups in one grid) or 2 (one grid each).  For measurement: per-launch figures of
 * a profile are whole-FFN figures divided by this.
 */
int lynx_moe_ffn_launches(int T, int F);

/*
 * lynx_moe_ffn with stage timing (roofline of the weight-streaming kernel): the same work, and additionally
 * records the caller's events on `stream`.  stage_events: HOST array of four hipEvent_t (entries may be NULL):
 * [0] is recorded before the weight-streaming launch(es), [1] and [2] after them (gate/up and down are one kernel,
 * launched once or twice: the two events are adjacent), [3] after the combine.  stage_events == NULL is exactly
 * lynx_moe_ffn.
 */
int lynx_moe_ffn_timed(const uint16_t *x_bf16, const uint16_t *Wgu_packed, const uint16_t *Wd_packed,
                       const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared, int F_shared,
                       const int32_t *idx, const float *gate, const int32_t *expert_offsets, const int32_t *perm,
                       const int32_t *active_experts, const int32_t *num_active, int T, int H, int F, int N, int k,
                       float *y, int32_t *status, void *workspace, void *stream, void *const *stage_events);

/*
 * The residual update that chains MoE layers into a stack (the benchmark times a stack of layers as a whole, each
 * layer's input depending on the layer before): x_next[i] = bf16(float(x[i]) + y[i]) for i < n, one fp32 addition
 * rounded to nearest even.  x_bf16 [n] and x_next_bf16 [n] bf16, y [n] fp32; n even; x_next may be x itself.
 * n == 0 is a no-op.
 */
int lynx_residual_add(const uint16_t *x_bf16, const float *y, size_t n, uint16_t *x_next_bf16, void *stream);

/*
 * Enqueues a plain read-only streaming kernel over buf[0, bytes) (16-byte aligned, bytes a multiple of 16; nothing
 * is modified).  Timed by the caller over a buffer much larger than the caches it gives the read bandwidth the chip
 * delivers in practice, which the benchmark prints beside the rate of the expert-weight stream.  non_temporal != 0:
 * the loads carry the same non-temporal hint as the weight stream.  sink: one uint32_t (kept only so that the loads
 * have a use; practically never written).  bytes == 0 is a no-op.
 */
int lynx_read_probe(const void *buf, size_t bytes, int non_temporal, uint32_t *sink, void *stream);

/*
 * Process-wide knobs, read by the calls that follow (host state; not for use while another thread is inside the
 * library).  value <= 0 (or < 0 where 0 is meaningful) restores the default.
 *   LYNX_DEBUG_SPIN_LIMIT       polls of a completion counter before a down-projection workgroup gives up a wait
 *                               (default 131072; 0 = give up at once).  value < 0 restores the default.
 *   LYNX_DEBUG_TARGET_BIAS      added to the count such a workgroup waits for (default 0).  With a spin limit of 0 and a
 *                               bias the counters never reach, every wait gives up at once and every kernel still
 *                               runs to its end: how the test of lynx_moe_ffn's status output forces the condition.
 *   LYNX_DEBUG_DOWN_ITEM_CAP    down-projection work items the device-side plan aims at (default 768)
 *   LYNX_DEBUG_DOWN_ITEM_UNITS  most row units per down-projection work item (a power of two; default 1)
 *   LYNX_DEBUG_DOWN_K_WAVES     K slices that the four waves of a down-projection workgroup form (1, 2, or 4 for batches
 *                               of at most 16 tokens; default 0 = the library's rule)
 */
#define LYNX_DEBUG_SPIN_LIMIT 1
#define LYNX_DEBUG_TARGET_BIAS 2
#define LYNX_DEBUG_DOWN_ITEM_CAP 3
#define LYNX_DEBUG_DOWN_ITEM_UNITS 4
#define LYNX_DEBUG_DOWN_K_WAVES 5
int lynx_debug_set(int what, int value);

#ifdef __cplusplus
}
#endif
#endif /* LYNX_BENCH_H */
