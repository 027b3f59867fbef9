// Internal helpers shared by the HIP translation units of liblynx (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lynx.h"

namespace lynx {

// Records a host-side error string for lynx_last_error() and returns `code`.
int fail(int code, const char *fmt, ...);
// LYNX_OK if the last kernel launch was accepted, else records the HIP error.
int check_launch(const char *what);

constexpr int kWave = 64;
constexpr int kSlots = LYNX_MAX_N / kWave;  // expert slots per lane when a wave holds one token's N logits

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x >> 6); }

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int m = kWave / 2; m > 0; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
    return v;
}

// Butterfly sum: every lane ends with the same value, summed in a fixed order.
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int m = kWave / 2; m > 0; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// Bin magnitude of one (token, expert) pair: min(floor(alpha * (zmax - z)), beta), with exactly one
// rounded fp32 subtract and one rounded fp32 multiply (paper Sec. 3.2.1; bin value = -q).
__device__ __forceinline__ int bin_of(float zmax, float z, float alpha, int beta)
{
    float d = __fsub_rn(zmax, z);
    float qf = floorf(__fmul_rn(alpha, d));
    return (qf >= (float)beta) ? beta : (int)qf;
}

// The wave holds one token's logits: lane l, slot i <-> expert l + 64*i.  Picks the k largest among
// the candidate slots (bit i of `cand`), descending, equal values to the lower expert index, and calls
// emit(j, expert, value) on every lane with the j-th winner (expert = INT_MAX when none is left).
template <typename Emit>
__device__ __forceinline__ void wave_topk(const float (&v)[kSlots], unsigned cand, int k, Emit &&emit)
{
    const int lane = lane_id();
    for (int j = 0; j < k; ++j) {
        float bv = -INFINITY;
        int be = INT_MAX;
#pragma unroll
        for (int i = 0; i < kSlots; ++i)
            if (((cand >> i) & 1u) && (be == INT_MAX || v[i] > bv)) {
                bv = v[i];
                be = lane + kWave * i;
            }
#pragma unroll
        for (int m = kWave / 2; m > 0; m >>= 1) {
            float ov = __shfl_xor(bv, m, kWave);
            int oe = __shfl_xor(be, m, kWave);
            bool take = (oe != INT_MAX) && (be == INT_MAX || ov > bv || (ov == bv && oe < be));
            bv = take ? ov : bv;
            be = take ? oe : be;
        }
        if (be != INT_MAX && (be & (kWave - 1)) == lane) cand &= ~(1u << (be >> 6));
        emit(j, be, bv);
    }
}

}  // namespace lynx
