// Measurement aids, not steps of the method.
//
// (1) The residual update that chains MoE layers into a stack, x_next = bf16(x + y), so that a stack of
// layers can be timed as a whole with a true dependency from each layer to the next.
//
// (2) A plain read-only streaming kernel.  Its rate over a buffer
// much larger than the caches is the read bandwidth this chip actually delivers, the practical ceiling that
// the expert-weight stream of the FFN kernels is compared with (the published HBM peak is not reachable by
// any access pattern).
#include <hip/hip_runtime.h>

#include "../../include/lynx_bench.h"
#include "lynx_common.h"

namespace lynx {

typedef unsigned probe_u32x4 __attribute__((ext_vector_type(4)));
constexpr int kProbeUnroll = 8;            // 16-byte loads in flight per thread
constexpr int kProbeBlocks = 256;          // one workgroup per CU: measured to be the fastest plain read on this chip

// Grid-stride over 16-byte pieces: consecutive lanes read consecutive pieces, so every wave-wide load is one
// contiguous KiB, the same access shape as the weight stream.  The XOR of everything read is stored only if
// it equals a value it practically never has: the loads cannot be optimised away and nothing is written.
template <bool NT>
__global__ __launch_bounds__(256) void read_probe_kernel(const probe_u32x4 *__restrict__ p, size_t n16, uint32_t *sink)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    unsigned acc = 0;
    for (; i + (kProbeUnroll - 1) * stride < n16; i += kProbeUnroll * stride) {
        probe_u32x4 r[kProbeUnroll];
#pragma unroll
        for (int j = 0; j < kProbeUnroll; ++j) r[j] = NT ? __builtin_nontemporal_load(p + i + j * stride) : p[i + j * stride];
#pragma unroll
        for (int j = 0; j < kProbeUnroll; ++j) acc ^= r[j].x ^ r[j].y ^ r[j].z ^ r[j].w;
    }
    for (; i < n16; i += stride) {
        const probe_u32x4 r = p[i];
        acc ^= r.x ^ r.y ^ r.z ^ r.w;
    }
    if (acc == 0x9e3779b9u && sink) *sink = acc;
}

__device__ __forceinline__ uint32_t bf16_rne_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// x_next[i] = bf16(float(x[i]) + y[i]), round to nearest even; two elements per thread.
__global__ __launch_bounds__(256) void residual_kernel(const uint32_t *__restrict__ x2, const float2 *__restrict__ y2,
                                                       size_t pairs, uint32_t *__restrict__ out2)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= pairs) return;
    const uint32_t xv = x2[i];
    const float2 yv = y2[i];
    const float lo = __fadd_rn(__uint_as_float(xv << 16), yv.x);
    const float hi = __fadd_rn(__uint_as_float(xv & 0xffff0000u), yv.y);
    out2[i] = bf16_rne_bits(lo) | (bf16_rne_bits(hi) << 16);
}

}  // namespace lynx

extern "C" int lynx_residual_add(const uint16_t *x_bf16, const float *y, size_t n, uint16_t *x_next_bf16, void *stream)
{
    using namespace lynx;
    if (n == 0) return LYNX_OK;
    if (!x_bf16 || !y || !x_next_bf16) return fail(LYNX_ERR_INVALID_ARG, "lynx_residual_add: null pointer");
    if ((n & 1) != 0 || (reinterpret_cast<uintptr_t>(x_bf16) & 3) != 0 || (reinterpret_cast<uintptr_t>(y) & 7) != 0 ||
        (reinterpret_cast<uintptr_t>(x_next_bf16) & 3) != 0)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_residual_add: n must be even and the arrays 4- / 8-byte aligned");
    const size_t pairs = n / 2, blocks = (pairs + 255) / 256;
    if (blocks > 0x7fffffffull) return fail(LYNX_ERR_UNSUPPORTED, "lynx_residual_add: too large for one call");
    hipLaunchKernelGGL(residual_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       reinterpret_cast<const uint32_t *>(x_bf16), reinterpret_cast<const float2 *>(y), pairs,
                       reinterpret_cast<uint32_t *>(x_next_bf16));
    return check_launch("lynx_residual_add");
}

extern "C" int lynx_read_probe(const void *buf, size_t bytes, int non_temporal, uint32_t *sink, void *stream)
{
    using namespace lynx;
    if (bytes == 0) return LYNX_OK;
    if (!buf || !sink) return fail(LYNX_ERR_INVALID_ARG, "lynx_read_probe: null pointer");
    if ((reinterpret_cast<uintptr_t>(buf) & 15) != 0 || (bytes & 15) != 0)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_read_probe: buffer and size must be multiples of 16 bytes");
    const probe_u32x4 *p = reinterpret_cast<const probe_u32x4 *>(buf);
    if (non_temporal)
        hipLaunchKernelGGL(read_probe_kernel<true>, dim3(kProbeBlocks), dim3(256), 0, (hipStream_t)stream, p, bytes / 16, sink);
    else
        hipLaunchKernelGGL(read_probe_kernel<false>, dim3(kProbeBlocks), dim3(256), 0, (hipStream_t)stream, p, bytes / 16, sink);
    return check_launch("lynx_read_probe");
}
