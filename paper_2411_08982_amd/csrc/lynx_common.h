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
constexpr int kSlots = LYNX_MAX_N / kWave;  // most expert slots per lane when a wave holds one token's N logits

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x >> 6); }

// Wave-wide reductions on the DPP data path (row shifts inside each row of 16 lanes, then the two row
// broadcasts): no LDS crossbar round trips.  After the sequence lane 63 holds the result; it is read back
// as a wave-uniform value.  Lanes that a step does not write keep their own value (max) or add zero (sum).
#define LYNX_DPP_STEP_MAX(ctrl, rmask)                                                                          \
    v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), ctrl, rmask, 0xf, false)))
#define LYNX_DPP_STEP_SUM(ctrl, rmask) \
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, rmask, 0xf, false))

__device__ __forceinline__ float wave_max(float v)
{
    LYNX_DPP_STEP_MAX(0x111, 0xf);   // row_shr:1
    LYNX_DPP_STEP_MAX(0x112, 0xf);   // row_shr:2
    LYNX_DPP_STEP_MAX(0x114, 0xf);   // row_shr:4
    LYNX_DPP_STEP_MAX(0x118, 0xf);   // row_shr:8   -> lane 15 of every row holds the row's maximum
    LYNX_DPP_STEP_MAX(0x142, 0xa);   // row_bcast:15 into rows 1 and 3
    LYNX_DPP_STEP_MAX(0x143, 0xc);   // row_bcast:31 into rows 2 and 3 -> lane 63 holds the wave's maximum
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Fixed summation order (a prefix tree inside rows, then rows 0+1, 2+3, then halves): every lane gets the
// same value, and it does not depend on scheduling.
__device__ __forceinline__ float wave_sum(float v)
{
    LYNX_DPP_STEP_SUM(0x111, 0xf);
    LYNX_DPP_STEP_SUM(0x112, 0xf);
    LYNX_DPP_STEP_SUM(0x114, 0xf);
    LYNX_DPP_STEP_SUM(0x118, 0xf);
    LYNX_DPP_STEP_SUM(0x142, 0xa);
    LYNX_DPP_STEP_SUM(0x143, 0xc);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// The same on integers.  With the identity of the maximum as the value of the lanes a step does not write, a step
// is one instruction (a float step is four: the float maximum has to quieten NaNs first).
#define LYNX_DPP_STEP_IMAX(ctrl, rmask) v = max(v, __builtin_amdgcn_update_dpp(INT_MIN, v, ctrl, rmask, 0xf, false))
__device__ __forceinline__ int wave_max_i32(int v)
{
    LYNX_DPP_STEP_IMAX(0x111, 0xf);
    LYNX_DPP_STEP_IMAX(0x112, 0xf);
    LYNX_DPP_STEP_IMAX(0x114, 0xf);
    LYNX_DPP_STEP_IMAX(0x118, 0xf);
    LYNX_DPP_STEP_IMAX(0x142, 0xa);
    LYNX_DPP_STEP_IMAX(0x143, 0xc);
    return __builtin_amdgcn_readlane(v, 63);
}

// Inclusive prefix sums over the lanes of the wave, same data path: the four row shifts leave every lane with the
// sum of its row up to itself, the two broadcasts add the totals of the rows before.  Every lane gets its prefix.
__device__ __forceinline__ int wave_prefix_sum_i32(int v)
{
#define LYNX_DPP_STEP_IADD(ctrl, rmask) v += __builtin_amdgcn_update_dpp(0, v, ctrl, rmask, 0xf, false)
    LYNX_DPP_STEP_IADD(0x111, 0xf);
    LYNX_DPP_STEP_IADD(0x112, 0xf);
    LYNX_DPP_STEP_IADD(0x114, 0xf);
    LYNX_DPP_STEP_IADD(0x118, 0xf);
    LYNX_DPP_STEP_IADD(0x142, 0xa);
    LYNX_DPP_STEP_IADD(0x143, 0xc);
#undef LYNX_DPP_STEP_IADD
    return v;
}

// Floats as integers that compare the same way (finite values and infinities; -0 is first made +0, so that the two
// stay equal), and back.
__device__ __forceinline__ int order_key(float f)
{
    const int b = __float_as_int(f + 0.0f);
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float key_value(int key) { return __int_as_float(key ^ ((key >> 31) & 0x7fffffff)); }

// Bin magnitude of one (token, expert) pair: min(floor(alpha * (zmax - z)), beta), with exactly one
// rounded fp32 subtract and one rounded fp32 multiply (paper Sec. 3.2.1; bin value = -q).
__device__ __forceinline__ int bin_of(float zmax, float z, float alpha, int beta)
{
    float d = __fsub_rn(zmax, z);
    float qf = floorf(__fmul_rn(alpha, d));
    return (qf >= (float)beta) ? beta : (int)qf;
}

// Writes a value into one lane of a per-lane variable, as a select (no branch).
__device__ __forceinline__ void put_lane(int &var, int lane, int value) { var = (lane_id() == lane) ? value : var; }
__device__ __forceinline__ void put_lane(float &var, int lane, float value) { var = (lane_id() == lane) ? value : var; }

// The wave holds one token's logits: lane l, slot i <-> expert l + 64*i.  Picks the k largest among
// the candidate slots (bit i of `cand`), descending, equal values to the lower expert index, and calls
// emit(j, expert, value) on every lane with the j-th winner, both wave-uniform (expert = INT_MAX when none is left).
// Per pick: one DPP max reduction, then the lowest-indexed holder of that maximum by ballot + find-first
// (slot 0 holds the lower experts, so the first slot with a match wins).  Values are finite: the key of -inf marks
// the entries that are no candidates or already taken.  A pick is a chain of dependent instructions that a lone
// wave issues at one per 8-12 cycles (measured), so the loop body is kept short: 34 instructions for two slots.
template <int NS, typename Emit>
__device__ __forceinline__ void wave_topk(const float (&v)[NS], unsigned cand, int k, Emit &&emit)
{
    const int lane = lane_id();
    // the k wave-wide maxima are taken on order-preserving integer keys: see wave_max_i32
    const int none = order_key(-INFINITY);
    int key[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) key[i] = ((cand >> i) & 1u) ? order_key(v[i]) : none;
    for (int j = 0; j < k; ++j) {
        int m = key[0];
#pragma unroll
        for (int i = 1; i < NS; ++i) m = max(m, key[i]);
        const int best = wave_max_i32(m);
        int e = INT_MAX;
#pragma unroll
        for (int i = NS - 1; i >= 0; --i) {   // descending: the last slot to report is the lowest
            const unsigned long long b = __ballot(key[i] == best);
            if (b != 0ull) e = __ffsll((long long)b) - 1 + kWave * i;
        }
        if (best == none) e = INT_MAX;
#pragma unroll
        for (int i = 0; i < NS; ++i) key[i] = (e == lane + kWave * i) ? none : key[i];
        emit(j, e, key_value(best));
    }
}

// ---- data handed from one workgroup to another inside a launch ---------------------------------------------
// Every XCD has its own L2, and a device-wide fence (write back / invalidate that L2) costs microseconds per
// workgroup.  Instead, the few words that another workgroup of the same launch will read are written with
// device-coherent stores or atomics (they go through to the point where all XCDs meet) and read with
// device-coherent loads; the writer waits for its stores to complete before it takes its ticket.
__device__ __forceinline__ void store_coherent(int32_t *p, int32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int32_t load_coherent(const int32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned load_coherent(const unsigned *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_coherent(uint2 *p, uint2 v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), ((unsigned long long)v.y << 32) | v.x, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
// All memory operations this wave has issued are complete (vmcnt, expcnt, lgkmcnt = 0).
__device__ __forceinline__ void wait_memory_complete() { __builtin_amdgcn_s_waitcnt(0); }

// Scales of quantised expert weights (all DEVICE), for the routed and the shared experts.  format 1 = FP8 E4M3: fp32
// row scales, gate/up [N][2][F] and down [N][H].  format 2 = MXFP4: the block-scale exponents in the streaming layout
// (dwords, passed through these pointers).  A null pointer to this struct means bf16 weights.
// What kind of router the layer has.  gate_fn: 0 = softmax over the selected logits, 1 = selected sigmoid scores over
// their sum.  n_group > 1: group-limited, a token may only use the experts of its topk_group best groups.
struct RouterKind {
    int gate_fn, n_group, topk_group;
};

struct FfnScales {
    const float *gu, *d, *shared_gu, *shared_d;
    int format;
};

// ---- workspace layout (one caller-provided buffer serves every call) -----------------------------------
// [ routing scratch | h: bf16 intermediate vectors | o: fp32 per-pair outputs ]
// Routing scratch (int32 words): tickets of the "last workgroup finishes the batch-level step" pattern,
// the experts in score order, the active-set flags and the per-expert token bit sets of the permutation.
constexpr int kWsTickets = 0;                              // 16 words
constexpr int kWsOrder = 16;                               // LYNX_MAX_N words
constexpr int kWsActive = kWsOrder + LYNX_MAX_N;           // LYNX_MAX_N words
constexpr int kWsMember = kWsActive + LYNX_MAX_N;          // LYNX_MAX_N * LYNX_MAX_T/32 words
constexpr int kWsDone = kWsMember + LYNX_MAX_N * (LYNX_MAX_T / 32);   // FFN: gate/up completion counters
constexpr int kWsDoneWords = 1024;                         // LYNX_MAX_N routed + (shared expert, token block) pairs
constexpr int kWsFlags = kWsDone + kWsDoneWords;           // FFN: bit 0 = a bounded wait ran out
constexpr int kWsPlanHdr = kWsFlags + 16;                  // FFN work plan (lynx_plan.h): header, 16 words
constexpr int kPlanMaxBlocks = 512;                        // most (expert, token block) pairs: LYNX_MAX_N + LYNX_MAX_T * LYNX_MAX_K / 128, rounded up
constexpr int kWsPlanBlk = kWsPlanHdr + 16;                // one record of four words per (expert, token block) pair
constexpr int kWsPlanPairs = kWsPlanBlk + 4 * kPlanMaxBlocks;   // 16 pair ids of 16 bits per block: 8 words each
constexpr int kWsRoutingWords = kWsPlanPairs + 8 * kPlanMaxBlocks;
constexpr size_t kWsRoutingBytes = 98304;
static_assert((size_t)kWsRoutingWords * 4 <= kWsRoutingBytes, "routing scratch does not fit its reservation");

inline int h_stride(int F) { return (F + 63) / 64 * 64; }   // elements between rows of the h scratch

struct Workspace {
    size_t h_elems, o_elems, h_off, o_off, routing_off, total;
};

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// o holds one fp32 row per (token, slot) pair and per (shared expert, K split, token).
inline Workspace workspace_layout(int T, int H, int F, int k, int n_shared, int F_shared, int shared_splits)
{
    Workspace w;
    // rows of the intermediate vectors start on 128-byte lines (a cache line never holds parts of two experts' rows)
    w.h_elems = (size_t)T * k * h_stride(F) + (size_t)n_shared * T * h_stride(F_shared);
    w.o_elems = ((size_t)T * k + (size_t)n_shared * shared_splits * T) * H;
    w.routing_off = 0;
    w.h_off = kWsRoutingBytes;
    w.o_off = w.h_off + align256(w.h_elems * 2);
    w.total = w.o_off + align256(w.o_elems * 4);
    return w;
}

// Number of K slices a shared expert's down projection is cut into, so that a shared expert that is
// several times wider than a routed one still spreads over the chip (each slice owns its output rows).
inline int shared_down_splits(int F, int n_shared, int F_shared)
{
    if (n_shared <= 0 || F_shared <= F) return 1;
    int s = (F_shared + F - 1) / F;
    return s > 8 ? 8 : s;
}

}  // namespace lynx
