// Error reporting and the chained whole-layer entry point of liblynx.
#include <stdarg.h>
#include <stdio.h>

#include <mutex>

#include "lynx_plan.h"

namespace lynx {

static thread_local char g_last_error[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof g_last_error, fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char *what)
{
    const hipError_t err = hipGetLastError();
    if (err == hipSuccess) return LYNX_OK;
    return fail(LYNX_ERR_HIP, "%s: %s", what, hipGetErrorString(err));
}

}  // namespace lynx

extern "C" const char *lynx_last_error(void) { return lynx::g_last_error; }

namespace lynx {
int routing_fused(const uint16_t *x, const float *Wr, const float *bias, int T, int H, int N, int k, float alpha,
                  int beta, int enable, RouterKind rk, float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum,
                  int32_t *new_idx, float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist,
                  int32_t *num_active, int32_t *expert_offsets, int32_t *perm, int32_t *active_experts,
                  int32_t *num_active_perm, void *workspace, hipStream_t st, const PlanShape &ps);
int check_router_kind(const char *who, int N, int k, const RouterKind &rk);
PlanShape ffn_plan_shape(int T, int H, int F, int N, int k, int n_shared, int format);
int moe_ffn_validate(const void *x_bf16, const void *Wgu_packed, const void *Wd_packed, const void *Sgu_packed,
                     const void *Sd_packed, int n_shared, int F_shared, const void *idx, const void *gate, const void *perm,
                     const void *offsets, int T, int H, int F, int N, int k, const void *y, const void *workspace,
                     const FfnScales *q8);
int moe_ffn_impl(const uint16_t *x_bf16, const uint16_t *Wgu_packed, const uint16_t *Wd_packed, const uint16_t *Sgu_packed,
                 const uint16_t *Sd_packed, int n_shared, int F_shared, const int32_t *idx, const float *gate,
                 const int32_t *expert_offsets, const int32_t *perm, int T, int H, int F, int N, int k, float *y,
                 int32_t *status, void *workspace, void *stream, void *const *stage_events, bool plan_ready,
                 const FfnScales *q8);
}

// The fused path issues the routing side in two launches up to 16 tokens (logits; everything else in one
// workgroup) and in four beyond (logits; top-k + bins; nominations; remap + token assignment) instead of the
// launches of the separate calls; results are identical.
namespace lynx {
static int moe_layer_impl(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                          const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared,
                          int F_shared, int T, int H, int F, int N, int k, float alpha, int beta, int enable, float *logits,
                          int32_t *topk_idx, float *topk_gate, float *topk_psum, int32_t *new_idx, float *new_gate,
                          float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                          int32_t *expert_offsets, int32_t *perm, int32_t *active_experts, int32_t *num_active_perm,
                          float *y, int32_t *status, void *workspace, void *stream, void *const *stage_events,
                          const FfnScales *q8, RouterKind rk = {0, 1, 1})
{
    int rc;
    bool fused = false;
    const int gate_fn = rk.gate_fn;
    if (rk.n_group > 1 && (T <= 0 || !workspace)) {
        // group-limited router: route + remap in one call, which also reports a missing workspace
        rc = lynx_route_grouped(x_bf16, Wr, bias, T, H, N, k, rk.n_group, rk.topk_group, gate_fn, logits, topk_idx, topk_gate,
                                topk_psum, stream);
        if (rc != LYNX_OK) return rc;
        rc = lynx_affinity_bin_grouped(logits, T, N, k, rk.n_group, rk.topk_group, gate_fn, alpha, beta, enable, topk_idx,
                                       topk_gate, topk_psum, new_idx, new_gate, new_psum, cnt_before, cnt_after, bin_hist,
                                       num_active, workspace, stream);
        if (rc != LYNX_OK) return rc;
        rc = lynx_permute(new_idx, T, N, k, expert_offsets, perm, active_experts, num_active_perm, stream);
        if (rc != LYNX_OK) return rc;
    } else if (T <= 0 || !workspace) {
        // no tokens (or a missing workspace, which the separate calls report): take the separate calls
        rc = (gate_fn ? lynx_route_sigmoid : lynx_route)(x_bf16, Wr, bias, T, H, N, k, logits, topk_idx, topk_gate, topk_psum,
                                                         stream);
        if (rc != LYNX_OK) return rc;
        rc = (gate_fn ? lynx_affinity_bin_sigmoid : lynx_affinity_bin)(logits, topk_idx, T, N, k, alpha, beta, enable, new_idx,
                                                                       new_gate, new_psum, cnt_before, cnt_after, bin_hist,
                                                                       num_active, workspace, stream);
        if (rc != LYNX_OK) return rc;
        rc = lynx_permute(new_idx, T, N, k, expert_offsets, perm, active_experts, num_active_perm, stream);
        if (rc != LYNX_OK) return rc;
    } else {
        // same argument checks as the separate calls, before anything is enqueued
        if (H <= 0 || N <= 0 || k <= 0) return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_layer: negative or zero size");
        rc = check_router_kind("lynx_moe_layer", N, k, rk);
        if (rc != LYNX_OK) return rc;
        if (k > N || N > LYNX_MAX_N || k > LYNX_MAX_K || T > LYNX_MAX_T || (H % 32) != 0 || beta > LYNX_MAX_BETA)
            return fail(LYNX_ERR_UNSUPPORTED, "lynx_moe_layer: need k<=N<=%d, k<=%d, T<=%d, beta<=%d, H%%32==0", LYNX_MAX_N,
                        LYNX_MAX_K, LYNX_MAX_T, LYNX_MAX_BETA);
        if (beta < 1 || !(alpha >= 0.0f) || alpha > 3.0e38f)
            return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_layer: alpha must be finite and >= 0, beta >= 1");
        double lim = 1.0;
        for (int j = 0; j < beta; ++j) lim *= (double)T;
        if (lim >= 4611686018427387904.0) return fail(LYNX_ERR_UNSUPPORTED, "lynx_moe_layer: T^beta must stay below 2^62");
        if (!x_bf16 || !Wr || !logits || !topk_idx || !topk_gate || !topk_psum || !new_idx || !new_gate || !cnt_before ||
            !cnt_after || !bin_hist || !num_active || !expert_offsets || !perm || !active_experts || !num_active_perm)
            return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_layer: null pointer");
        // the FFN's own checks, made here so that an error leaves nothing enqueued
        rc = moe_ffn_validate(x_bf16, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, new_idx, new_gate, perm,
                              expert_offsets, T, H, F, N, k, y, workspace, q8);
        if (rc != LYNX_OK) return rc;
        rc = routing_fused(x_bf16, Wr, bias, T, H, N, k, alpha, beta, enable, rk, logits, topk_idx, topk_gate, topk_psum,
                           new_idx, new_gate, new_psum, cnt_before, cnt_after, bin_hist, num_active, expert_offsets, perm,
                           active_experts, num_active_perm, workspace, (hipStream_t)stream,
                           ffn_plan_shape(T, H, F, N, k, n_shared, q8 ? q8->format : 0));
        if (rc != LYNX_OK) return rc;
        fused = true;   // its kernels have also cleared the FFN's completion counters and written the work plan
    }
    return moe_ffn_impl(x_bf16, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, new_idx, new_gate,
                        expert_offsets, perm, T, H, F, N, k, y, status, workspace, stream, stage_events, fused, q8);
}
}  // namespace lynx

extern "C" int lynx_moe_layer(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                              const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed,
                              int n_shared, int F_shared, int T, int H, int F, int N, int k, float alpha, int beta,
                              int enable, float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum,
                              int32_t *new_idx, float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after,
                              int32_t *bin_hist, int32_t *num_active, int32_t *expert_offsets, int32_t *perm,
                              int32_t *active_experts, int32_t *num_active_perm, float *y, int32_t *status, void *workspace,
                              void *stream, void *const *stage_events)
{
    return lynx::moe_layer_impl(x_bf16, Wr, bias, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, T, H, F,
                                N, k, alpha, beta, enable, logits, topk_idx, topk_gate, topk_psum, new_idx, new_gate, new_psum,
                                cnt_before, cnt_after, bin_hist, num_active, expert_offsets, perm, active_experts,
                                num_active_perm, y, status, workspace, stream, stage_events, nullptr);
}

// ---- the whole layer for callers that cannot allocate ---------------------------------------------------------
// The workspace of lynx_moe_layer (routing tickets and bit sets, completion counters, the intermediate vectors h
// and the per-pair outputs o) lives in a device array of the library instead of a caller's buffer.  The array's
// name is a host-side stand-in for the symbol, not a device address: the address on each GPU comes from
// hipGetSymbolAddress, asked once per device with that device current, and only that pointer is handed to kernels.
namespace lynx {
constexpr size_t kStaticScratchBytes = (size_t)LYNX_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
}  // namespace lynx
static __device__ __align__(256) unsigned char scratch[lynx::kStaticScratchBytes];

namespace lynx {
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];   // per device: where that GPU holds its copy of `scratch`

// The current device's copy of the scratch array (resolved on the first call on that device), or null with the error set.
static void *static_scratch()
{
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        fail(LYNX_ERR_HIP, "lynx_moe_layer_static: hipGetDevice: %s (device %d)", hipGetErrorString(err), dev);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !ptr) {
            fail(LYNX_ERR_HIP, "lynx_moe_layer_static: hipGetSymbolAddress: %s", hipGetErrorString(err));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace lynx

extern "C" int lynx_moe_layer_static(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                                     const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed,
                                     int n_shared, int F_shared, int T, int H, int F, int N, int k, float alpha, int beta,
                                     int enable, float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum,
                                     int32_t *new_idx, float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after,
                                     int32_t *bin_hist, int32_t *num_active, int32_t *expert_offsets, int32_t *perm,
                                     int32_t *active_experts, int32_t *num_active_perm, float *y, int32_t *status, void *stream)
{
    using namespace lynx;
    if (T < 0 || H <= 0 || F <= 0 || N <= 0 || k <= 0 || n_shared < 0 || (n_shared > 0 && F_shared <= 0))
        return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_layer_static: negative or zero size");
    if (T > LYNX_MAX_T || N > LYNX_MAX_N || k > LYNX_MAX_K || k > N)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_moe_layer_static: need k<=N<=%d, k<=%d, T<=%d", LYNX_MAX_N, LYNX_MAX_K, LYNX_MAX_T);
    const size_t need = lynx_workspace_bytes(T, H, F, N, k, n_shared, F_shared);
    if (need > kStaticScratchBytes)
        return fail(LYNX_ERR_UNSUPPORTED,
                    "lynx_moe_layer_static: these sizes need %zu bytes of scratch, the built-in array holds %zu "
                    "(use lynx_moe_layer with a workspace of your own)", need, kStaticScratchBytes);
    void *ws = static_scratch();
    if (!ws) return LYNX_ERR_HIP;
    return moe_layer_impl(x_bf16, Wr, bias, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, T, H, F, N, k,
                          alpha, beta, enable, logits, topk_idx, topk_gate, topk_psum, new_idx, new_gate, new_psum, cnt_before,
                          cnt_after, bin_hist, num_active, expert_offsets, perm, active_experts, num_active_perm, y, status, ws,
                          stream, nullptr, nullptr);
}

extern "C" int lynx_moe_layer_sigmoid(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                                      const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed,
                                      int n_shared, int F_shared, int T, int H, int F, int N, int k, float alpha, int beta,
                                      int enable, float *logits, int32_t *topk_idx, float *topk_gate, float *topk_ssum,
                                      int32_t *new_idx, float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after,
                                      int32_t *bin_hist, int32_t *num_active, int32_t *expert_offsets, int32_t *perm,
                                      int32_t *active_experts, int32_t *num_active_perm, float *y, int32_t *status, void *workspace,
                                      void *stream, void *const *stage_events)
{
    return lynx::moe_layer_impl(x_bf16, Wr, bias, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, T, H, F,
                                N, k, alpha, beta, enable, logits, topk_idx, topk_gate, topk_ssum, new_idx, new_gate, new_psum,
                                cnt_before, cnt_after, bin_hist, num_active, expert_offsets, perm, active_experts,
                                num_active_perm, y, status, workspace, stream, stage_events, nullptr, lynx::RouterKind{1, 1, 1});
}

extern "C" int lynx_moe_layer_grouped(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                                      const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed,
                                      int n_shared, int F_shared, int T, int H, int F, int N, int k, int n_group,
                                      int topk_group, int gate_fn, float alpha, int beta, int enable, float *logits,
                                      int32_t *topk_idx, float *topk_gate, float *topk_third, int32_t *new_idx,
                                      float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist,
                                      int32_t *num_active, int32_t *expert_offsets, int32_t *perm, int32_t *active_experts,
                                      int32_t *num_active_perm, float *y, int32_t *status, void *workspace, void *stream,
                                      void *const *stage_events)
{
    return lynx::moe_layer_impl(x_bf16, Wr, bias, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, T, H, F,
                                N, k, alpha, beta, enable, logits, topk_idx, topk_gate, topk_third, new_idx, new_gate, new_psum,
                                cnt_before, cnt_after, bin_hist, num_active, expert_offsets, perm, active_experts,
                                num_active_perm, y, status, workspace, stream, stage_events, nullptr,
                                lynx::RouterKind{gate_fn, n_group, topk_group});
}

extern "C" int lynx_moe_layer_fp8(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint8_t *Wgu_q,
                                  const uint8_t *Wd_q, const float *scales_gu, const float *scales_d, const uint8_t *Sgu_q,
                                  const uint8_t *Sd_q, const float *shared_scales_gu, const float *shared_scales_d,
                                  int n_shared, int F_shared, int T, int H, int F, int N, int k, float alpha, int beta,
                                  int enable, float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum,
                                  int32_t *new_idx, float *new_gate, float *new_psum, int32_t *cnt_before, int32_t *cnt_after,
                                  int32_t *bin_hist, int32_t *num_active, int32_t *expert_offsets, int32_t *perm,
                                  int32_t *active_experts, int32_t *num_active_perm, float *y, int32_t *status, void *workspace,
                                  void *stream, void *const *stage_events)
{
    const lynx::FfnScales q = {scales_gu, scales_d, shared_scales_gu, shared_scales_d, 1};
    return lynx::moe_layer_impl(x_bf16, Wr, bias, reinterpret_cast<const uint16_t *>(Wgu_q),
                                reinterpret_cast<const uint16_t *>(Wd_q), reinterpret_cast<const uint16_t *>(Sgu_q),
                                reinterpret_cast<const uint16_t *>(Sd_q), n_shared, F_shared, T, H, F, N, k, alpha, beta,
                                enable, logits, topk_idx, topk_gate, topk_psum, new_idx, new_gate, new_psum, cnt_before, cnt_after,
                                bin_hist, num_active, expert_offsets, perm, active_experts, num_active_perm, y, status, workspace,
                                stream, stage_events, &q);
}

extern "C" int lynx_moe_layer_fp4(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint8_t *Wgu_q,
                                  const uint8_t *Wd_q, const uint32_t *scales_gu, const uint32_t *scales_d,
                                  const uint8_t *Sgu_q, const uint8_t *Sd_q, const uint32_t *shared_scales_gu,
                                  const uint32_t *shared_scales_d, int n_shared, int F_shared, int T, int H, int F, int N,
                                  int k, float alpha, int beta, int enable, float *logits, int32_t *topk_idx,
                                  float *topk_gate, float *topk_psum, int32_t *new_idx, float *new_gate, float *new_psum,
                                  int32_t *cnt_before, int32_t *cnt_after, int32_t *bin_hist, int32_t *num_active,
                                  int32_t *expert_offsets, int32_t *perm, int32_t *active_experts,
                                  int32_t *num_active_perm, float *y, int32_t *status, void *workspace, void *stream,
                                  void *const *stage_events)
{
    const lynx::FfnScales q = {reinterpret_cast<const float *>(scales_gu), reinterpret_cast<const float *>(scales_d),
                               reinterpret_cast<const float *>(shared_scales_gu),
                               reinterpret_cast<const float *>(shared_scales_d), 2};
    return lynx::moe_layer_impl(x_bf16, Wr, bias, reinterpret_cast<const uint16_t *>(Wgu_q),
                                reinterpret_cast<const uint16_t *>(Wd_q), reinterpret_cast<const uint16_t *>(Sgu_q),
                                reinterpret_cast<const uint16_t *>(Sd_q), n_shared, F_shared, T, H, F, N, k, alpha, beta,
                                enable, logits, topk_idx, topk_gate, topk_psum, new_idx, new_gate, new_psum, cnt_before, cnt_after,
                                bin_hist, num_active, expert_offsets, perm, active_experts, num_active_perm, y, status, workspace,
                                stream, stage_events, &q);
}
