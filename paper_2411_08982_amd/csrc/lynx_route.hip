// lynx_route: router logits, softmax, top-k (paper Sec. 2.1) for a decode batch.
//
// One workgroup per token.  The four waves share the token's experts: for each expert a wave streams
// the fp32 router row with 16-byte loads, multiplies by the (bf16-exact) hidden state in fp32 and
// reduces over lanes with a fixed butterfly, so a logit does not depend on scheduling.  Wave 0 then
// holds the N logits of the token (N <= 256: four per lane) and does softmax and top-k with shuffles.
#include "lynx_common.h"

namespace lynx {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__global__ __launch_bounds__(256) void route_kernel(const uint16_t *__restrict__ x, const float *__restrict__ Wr,
                                                    const float *__restrict__ bias, int T, int H, int N, int k,
                                                    float *__restrict__ logits, int32_t *__restrict__ topk_idx,
                                                    float *__restrict__ topk_gate, float *__restrict__ topk_psum)
{
    __shared__ float zs[LYNX_MAX_N];
    const int t = blockIdx.x;
    const int lane = lane_id(), wave = wave_id();
    const uint16_t *xt = x + (size_t)t * H;

    for (int e = wave; e < N; e += 4) {
        const float *w = Wr + (size_t)e * H;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        for (int h = lane * 8; h < H; h += kWave * 8) {
            const uint4 xv = *reinterpret_cast<const uint4 *>(xt + h);
            const float4 w0 = *reinterpret_cast<const float4 *>(w + h);
            const float4 w1 = *reinterpret_cast<const float4 *>(w + h + 4);
            a0 = fmaf(bf16_lo(xv.x), w0.x, a0);
            a1 = fmaf(bf16_hi(xv.x), w0.y, a1);
            a2 = fmaf(bf16_lo(xv.y), w0.z, a2);
            a3 = fmaf(bf16_hi(xv.y), w0.w, a3);
            a0 = fmaf(bf16_lo(xv.z), w1.x, a0);
            a1 = fmaf(bf16_hi(xv.z), w1.y, a1);
            a2 = fmaf(bf16_lo(xv.w), w1.z, a2);
            a3 = fmaf(bf16_hi(xv.w), w1.w, a3);
        }
        float z = wave_sum((a0 + a1) + (a2 + a3));
        if (bias) z += bias[e];
        if (lane == 0) {
            zs[e] = z;
            logits[(size_t)t * N + e] = z;
        }
    }
    __syncthreads();
    if (wave != 0) return;

    float v[kSlots];
    unsigned cand = 0;
#pragma unroll
    for (int i = 0; i < kSlots; ++i) {
        const int e = lane + kWave * i;
        v[i] = (e < N) ? zs[e] : -INFINITY;
        cand |= (e < N) ? (1u << i) : 0u;
    }
    // lane j keeps the j-th winner
    int mye = -1;
    float myz = -INFINITY;
    wave_topk(v, cand, k, [&](int j, int e, float z) {
        if (lane == j) {
            mye = (e == INT_MAX) ? -1 : e;
            myz = z;
        }
    });
    const float zmax = __shfl(myz, 0, kWave);
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < kSlots; ++i)
        if (lane + kWave * i < N) part += expf(v[i] - zmax);
    const float den = wave_sum(part);
    const float mynum = (lane < k) ? expf(myz - zmax) : 0.f;
    const float num = wave_sum(mynum);
    if (lane < k) {
        topk_idx[(size_t)t * k + lane] = mye;
        topk_gate[(size_t)t * k + lane] = mynum / num;
    }
    if (lane == 0) topk_psum[t] = num / den;
}

}  // namespace lynx

extern "C" int lynx_route(const uint16_t *x_bf16, const float *Wr, const float *bias, int T, int H, int N, int k,
                          float *logits, int32_t *topk_idx, float *topk_gate, float *topk_psum, void *stream)
{
    using namespace lynx;
    if (T < 0 || H <= 0 || N <= 0 || k <= 0) return fail(LYNX_ERR_INVALID_ARG, "lynx_route: negative or zero size");
    if (k > N || N > LYNX_MAX_N || k > LYNX_MAX_K || T > LYNX_MAX_T || (H % 32) != 0)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_route: need k<=N<=%d, k<=%d, T<=%d, H%%32==0 (T=%d H=%d N=%d k=%d)",
                    LYNX_MAX_N, LYNX_MAX_K, LYNX_MAX_T, T, H, N, k);
    if (T == 0) return LYNX_OK;
    if (!x_bf16 || !Wr || !logits || !topk_idx || !topk_gate || !topk_psum)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_route: null pointer");
    hipLaunchKernelGGL(route_kernel, dim3(T), dim3(256), 0, (hipStream_t)stream, x_bf16, Wr, bias, T, H, N, k, logits,
                       topk_idx, topk_gate, topk_psum);
    return check_launch("lynx_route");
}
