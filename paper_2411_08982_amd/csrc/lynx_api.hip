// Error reporting and the chained whole-layer entry point of liblynx.
#include <stdarg.h>
#include <stdio.h>

#include "lynx_common.h"

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

extern "C" int lynx_moe_layer(const uint16_t *x_bf16, const float *Wr, const float *bias, const uint16_t *Wgu_packed,
                              const uint16_t *Wd_packed, const uint16_t *Sgu_packed, const uint16_t *Sd_packed,
                              int n_shared, int F_shared, int T, int H, int F, int N, int k, float alpha, int beta,
                              int enable, float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum,
                              int32_t *new_idx, float *new_gate, int32_t *cnt_before, int32_t *cnt_after,
                              int32_t *bin_hist, int32_t *num_active, int32_t *expert_offsets, int32_t *perm,
                              int32_t *active_experts, int32_t *num_active_perm, float *y, void *workspace,
                              void *stream)
{
    int rc = lynx_route(x_bf16, Wr, bias, T, H, N, k, logits, topk_idx, topk_gate, topk_psum, stream);
    if (rc != LYNX_OK) return rc;
    rc = lynx_affinity_bin(logits, topk_idx, T, N, k, alpha, beta, enable, new_idx, new_gate, cnt_before, cnt_after,
                           bin_hist, num_active, workspace, stream);
    if (rc != LYNX_OK) return rc;
    rc = lynx_permute(new_idx, T, N, k, expert_offsets, perm, active_experts, num_active_perm, stream);
    if (rc != LYNX_OK) return rc;
    return lynx_moe_ffn(x_bf16, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, new_idx, new_gate,
                        expert_offsets, perm, active_experts, num_active_perm, T, H, F, N, k, y, workspace, stream);
}
