// lynx_moe_ffn: grouped SwiGLU expert FFN over the invoked experts + gate-weighted combine, and the
// one-time weight re-layout it streams from.
//
// Decode is bound by streaming expert weights from HBM (paper Sec. 2.1: latency grows with the number
// of experts the batch activates), so the kernels are organised around the weight stream:
//   * weights are pre-packed so that a wave reads a 16-row x 32-column bf16 tile as one contiguous
//     1 KiB load (16 bytes per lane) that IS the A operand of v_mfma_f32_16x16x32_bf16;
//   * a wave owns 16 output rows and walks (a slice of) the contraction dimension with a ring of
//     prefetched tiles in registers, so each weight byte is fetched from HBM once per call;
//   * the tokens of the expert are the B operand.  Experts with few tokens (<= 16, the usual decode
//     case) read the token columns straight from global memory in MFMA layout ("direct" path: no
//     LDS, no barrier in the loop); experts with many tokens stage the token tile through LDS, shared
//     by four row tiles ("staged" path);
//   * the grid is fixed (most experts the batch can invoke + shared experts, times row tiles); a
//     workgroup whose rank is past the device-side num_active leaves at once, so nothing is read back
//     to the host;
//   * gate/up (with the SiLU-multiply epilogue) and down are ONE kernel whose grid holds the workgroups of
//     both; it is launched once (down workgroups wait for their expert's gate/up workgroups through
//     completion counters) or once per projection, whichever measured faster for the shape;
//   * weights are bf16, FP8 E4M3 with one scale per row, or MXFP4 with one scale per block of 32 columns (both
//     converted to bf16 in registers).
// Launches: the expert kernel (once or twice) and a small combine.

#include <atomic>

#include "../../include/lynx_bench.h"
#include "lynx_plan.h"

namespace lynx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kFfnThreads = 256;
constexpr int kFfnWaves = kFfnThreads / kWave;
constexpr int kPF = 8;                       // staged path: weight tiles in flight per wave and matrix
#ifndef LYNX_PFD
#define LYNX_PFD 8
#endif
constexpr int kPFD = LYNX_PFD;               // direct path: the same (most; see DirectDepth for the depth per format)
constexpr int kStageBytes = 2 * 18432;       // two LDS buffers for the staged token tile
constexpr int kStageBytesBig = 2 * 128 * (4 * 64 + 16);   // the same in the large-batch kernels (128 tokens x 4 k-steps)

// Optional per-workgroup timeline of the expert kernel (-DLYNX_TIMELINE; measurement builds only): for every workgroup
// four stamps of the chip-wide 100 MHz clock (start, item known, wait over, work done) and what it was (projection,
// workgroup index, XCC id), read back with lynx_debug_timeline.  The product build defines none of it.
#ifdef LYNX_TIMELINE
constexpr int kTimelineSlots = 1 << 15;
__device__ unsigned long long g_timeline[kTimelineSlots][6];
#define LYNX_TS_BEGIN(kind, b)                                                                                         \
    const int ts_slot_ = (int)blockIdx.x < kTimelineSlots ? (int)blockIdx.x : kTimelineSlots - 1;                      \
    if (threadIdx.x == 0) {                                                                                            \
        unsigned xcc_, hwid_;                                                                                          \
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc_));                                          \
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hwid_));                                          \
        g_timeline[ts_slot_][0] = wall_clock64();                                                                      \
        g_timeline[ts_slot_][4] = ((unsigned long long)(kind) << 32) | (unsigned)(b);                                  \
        g_timeline[ts_slot_][5] = (xcc_ & 0xf) | ((unsigned long long)hwid_ << 8);                                     \
        g_timeline[ts_slot_][1] = g_timeline[ts_slot_][2] = g_timeline[ts_slot_][3] = 0;                               \
    }
#define LYNX_TS(i)                                                                                                     \
    if (threadIdx.x == 0) g_timeline[ts_slot_][i] = wall_clock64()
#else
#define LYNX_TS_BEGIN(kind, b)
#define LYNX_TS(i)
#endif

struct GemmParams {
    const uint16_t *W_routed;   // packed routed weights (gate/up interleaved, or down)
    const uint16_t *W_shared;   // packed shared-expert weights or NULL
    const float *sc_routed;     // FP8 weights: row scales, gate/up [N][2][F] or down [N][H]; MXFP4: the scale dwords; else unused
    const float *sc_shared;     // the same for the shared experts
    const uint16_t *B;          // gate/up: x [T,H]; down: h scratch
    void *out;                  // gate/up: h scratch (bf16); down: o scratch (fp32)
    const int32_t *perm;        // pair ids grouped by expert (the token assignment)
    const int32_t *plan;        // the routing part of the workspace: the work plan (lynx_plan.h)
    int T, N, k, n_shared;
    int R, K;                   // routed: output rows, contraction length
    int ldb_r, ldo_r, ldb_s, ldo_s;   // elements between B rows / output rows, routed and shared
    int Rs, Ks;                 // shared
    int tiles_r, tiles_s;       // row units per (routed expert, token block) / per shared work item
    int tiles_s_stride;         // tiles_s rounded up so that the token blocks of one shared row tile share an XCD
    int shared_tblocks;         // token blocks that a shared expert's tokens are divided into (1 = not divided)
    int tok_block;              // tokens per block: one pass of the staged path
    int routed_blocks, shared_blocks;   // grid = shared blocks first (the longest workgroups), then routed
    int shared_splits;          // K slices per shared expert (down projection only; each slice has its own output rows)
    int dn_m_max;               // most row units per down item that the plan may choose (1: always one)
    long long shared_h_base;    // element offset of the shared experts' h rows in the h scratch
};

// What a workgroup works on, resolved from blockIdx and the device-side routing tables.
struct WorkItem {
    const uint4 *W;      // packed weights of the expert
    const uint16_t *B;   // B-operand rows
    void *out;
    const float *sc;     // FP8 weights: this expert's row scales ([2][R] for gate/up, [R] for down); MXFP4: its scale dwords
    int R, K, tile, Te, off, shared_s, e;
    int te_all;          // all tokens of the expert (Te bounds this item's token block)
    int ldb, ldo;        // elements between B rows / output rows
    int tok0;            // first token of this work item's token block
    int kbeg, ksteps;    // slice of the contraction dimension this work item covers, in weight tiles (32 or 64 columns)
    int out_base;        // shared experts: first output row of this work item
    int pair;            // direct path, routed experts: the pair id of this lane's token column (lane % 16), -1 = none
    bool valid;
};

// Weight formats WF: 0 = bf16 (a 1 KiB tile is 16 rows x 32 columns), 1 = FP8 E4M3 (16 rows x 64 columns, converted to
// bf16 in registers; one fp32 scale per row applied to the accumulated sums), 2 = MXFP4 (16 rows x 128 columns:
// lane l holds row l%16, columns 32*(l/16) .. +31, which is exactly one scale block; converted to bf16 times the
// block's power-of-two scale in registers).  MXFP4 scale exponents: one dword per lane and four consecutive
// k-tiles (byte i = tile 4j+i), stored [row group][k-tile/4][lane][2], the 2 being gate|up, or the two row tiles of
// a down-projection row pair: a lane fetches both of its streams' scales with one 8-byte load.
template <int WF>
struct TileCols {
    static constexpr int value = 32 << WF;
};

// Dwords of MXFP4 scale exponents behind the weights of one expert's projection: row groups (gate/up: R/16 row
// tiles, both matrices; down: R/32 row pairs) x groups of four k-tiles x 64 lanes x 2.
__host__ __device__ __forceinline__ size_t mx_kt4(int K) { return (size_t)((K / 128 + 3) / 4); }
template <bool DUAL>
__host__ __device__ __forceinline__ size_t mx_scale_dwords(int R, int K)
{
    return (size_t)(DUAL ? R / 16 : R / 32) * mx_kt4(K) * 128;
}

// Which work item workgroup b of a projection is: one round trip to memory.  The shared experts' items come first
// (static: they see every token); the routed items follow in the plan's order, item = block * per + unit with
// per = the row units (gate/up) or groups of m row units (down) of one (expert, token block) pair.  The block's
// record, the header and the lane's pair id are requested together; their addresses follow from b alone.
// w.tile = the first row unit of the item, units = how many it covers.
template <bool DUAL, int WF>
__device__ __forceinline__ WorkItem resolve_item(const GemmParams &p, int b, int &units)
{
    constexpr int KC = TileCols<WF>::value;
    WorkItem w;
    w.sc = nullptr;
    w.valid = false;
    w.off = 0;
    w.Te = 0;
    w.te_all = 0;
    w.e = -1;
    w.shared_s = -1;
    w.tok0 = 0;
    w.pair = -1;
    w.B = p.B;
    w.out = p.out;
    units = 1;
    const uint16_t *Wbase;
    if (b >= p.shared_blocks) {
        const int idx = b - p.shared_blocks;
        const int32_t *__restrict__ plan = p.plan;
        // (down items of more than one row unit: their number per block is a device-side value, and the block
        // follows from it: a second round trip, only with that tuning knob set)
        const int m = (DUAL || p.dn_m_max <= 1) ? 1 : max(plan[kWsPlanHdr + kPlanM], 1);
        const int per = (p.tiles_r + m - 1) / m;
        const int q = min(idx / per, kPlanMaxBlocks - 1);
        const int B = plan[kWsPlanHdr + kPlanB];
        const int4 rec = *reinterpret_cast<const int4 *>(plan + kWsPlanBlk + 4 * q);
        const unsigned pv = reinterpret_cast<const uint16_t *>(plan + kWsPlanPairs)[q * kDirectMaxTokens + (lane_id() & 15)];
        if (B <= 0 || idx >= per * B) return w;   // (uniform: the whole workgroup leaves)
        // (the same for every lane: kept in scalar registers, and everything derived from them too)
        const int r0 = __builtin_amdgcn_readfirstlane(rec.x);
        const int e = r0 & 0xffff, te = (int)((unsigned)r0 >> 16);
        const int off = __builtin_amdgcn_readfirstlane(rec.y), tb = __builtin_amdgcn_readfirstlane(rec.z);
        if (e < 0 || e >= p.N || te <= 0 || off < 0 || off + te > p.T * p.k) return w;
        w.e = e;
        w.off = off;
        w.te_all = te;
        if (te > kDirectMaxTokens) {   // one pass of the staged path: tokens [tok0, Te) of the expert
            w.tok0 = tb * p.tok_block;
            w.Te = min(te, w.tok0 + p.tok_block);
            if (w.tok0 >= te) return w;
        } else {
            w.Te = te;
            w.pair = (int)pv;   // (checked where it is used)
        }
        w.tile = (idx % per) * m;
        units = min(m, p.tiles_r - w.tile);
        w.R = p.R;
        w.K = p.K;
        w.ldb = p.ldb_r;
        w.ldo = p.ldo_r;
        w.kbeg = 0;
        w.ksteps = w.K / KC;
        w.out_base = 0;
        Wbase = p.W_routed + (size_t)e * (((size_t)w.R * w.K * (DUAL ? 2 : 1)) >> WF);
        if (WF == 1) w.sc = p.sc_routed + (size_t)e * w.R * (DUAL ? 2 : 1);
        if (WF == 2) w.sc = p.sc_routed + (size_t)e * mx_scale_dwords<DUAL>(w.R, w.K);
    } else {
        // b = ((shared expert, K slice) * token blocks + token block) * stride + row tile.  Workgroups go to the
        // XCDs round-robin and the stride is a multiple of 8, so the token blocks of one row tile read their
        // common weights through one L2.
        w.tile = b % p.tiles_s_stride;
        const int vt = b / p.tiles_s_stride;
        const int v = vt / p.shared_tblocks;   // (shared expert, K slice)
        w.tok0 = (vt % p.shared_tblocks) * p.tok_block;
        w.shared_s = v / p.shared_splits;
        if (w.tile >= p.tiles_s || w.shared_s >= p.n_shared || w.tok0 >= p.T) return w;
        w.Te = p.shared_tblocks > 1 ? min(p.T, w.tok0 + p.tok_block) : p.T;   // tokens [tok0, Te)
        w.te_all = p.T;
        w.R = p.Rs;
        w.K = p.Ks;
        w.ldb = p.ldb_s;
        w.ldo = p.ldo_s;
        const int per = (w.K / KC + p.shared_splits - 1) / p.shared_splits;
        w.kbeg = (v % p.shared_splits) * per;
        w.ksteps = min(w.K / KC, w.kbeg + per) - w.kbeg;
        if (w.ksteps <= 0) return w;
        w.out_base = p.T * p.k + v * p.T;
        Wbase = p.W_shared + (size_t)w.shared_s * (((size_t)w.R * w.K * (DUAL ? 2 : 1)) >> WF);
        if (WF == 1) w.sc = p.sc_shared + (size_t)w.shared_s * w.R * (DUAL ? 2 : 1);
        if (WF == 2) w.sc = p.sc_shared + (size_t)w.shared_s * mx_scale_dwords<DUAL>(w.R, w.K);
        // shared experts keep their h rows in their own region of the scratch
        const size_t hbase = (size_t)p.shared_h_base + (size_t)w.shared_s * p.T * (DUAL ? w.ldo : w.ldb);
        if (DUAL)
            w.out = reinterpret_cast<uint16_t *>(p.out) + hbase;
        else
            w.B = p.B + hbase;
    }
    w.W = reinterpret_cast<const uint4 *>(Wbase);
    w.valid = true;
    return w;
}

// B row (element offset) and output row of the i-th token of the work item; -1 = none.
template <bool DUAL>
__device__ __forceinline__ void token_rows(const GemmParams &p, const WorkItem &w, int i, int &ro, int &orow)
{
    ro = -1;
    orow = -1;
    if (i >= w.Te) return;
    const int P = p.T * p.k;
    if (w.shared_s < 0) {
        const int pv = p.perm[w.off + i];
        const bool ok = pv >= 0 && pv < P;
        if (DUAL) {   // B row = x[token], out row = sorted position in h
            if (!ok) return;
            ro = (pv / p.k) * w.ldb;
            orow = w.off + i;
        } else {      // B row = h[sorted position] (known without the permutation), out row = pair id in o
            ro = (w.off + i) * w.ldb;
            orow = ok ? pv : -1;
        }
    } else if (DUAL) {   // shared: every token
        ro = i * w.ldb;
        orow = i;
    } else {
        ro = i * w.ldb;
        orow = w.out_base + i;
    }
}

// The same for this lane's token column on the direct path, from the pair id that came with the item: no load.
template <bool DUAL>
__device__ __forceinline__ void token_rows_direct(const GemmParams &p, const WorkItem &w, int &ro, int &orow)
{
    const int i = lane_id() & 15;
    ro = -1;
    orow = -1;
    if (i >= w.Te) return;
    if (w.shared_s < 0) {
        const bool ok = w.pair >= 0 && w.pair < p.T * p.k;
        if (DUAL) {
            if (!ok) return;
            ro = (w.pair / p.k) * w.ldb;
            orow = w.off + i;
        } else {
            ro = (w.off + i) * w.ldb;
            orow = ok ? w.pair : -1;
        }
    } else {
        ro = i * w.ldb;
        orow = DUAL ? i : w.out_base + i;
    }
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float silu_mul(float g, float u) { return (g / (1.0f + __expf(-g))) * u; }
__device__ __forceinline__ uint4 zero4() { return make_uint4(0u, 0u, 0u, 0u); }
__device__ __forceinline__ uint4 sel4(bool keep, uint4 v) { return keep ? v : zero4(); }

template <int NT>
__device__ __forceinline__ void clear_acc(f32x4 (&accg)[NT], f32x4 (&accu)[NT])
{
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        accg[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        accu[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
}

// D fragment of v_mfma_f32_16x16x32: lane holds token column (lane & 15) and output rows
// 4*(lane >> 4) .. +3 of the wave's 16.  gate/up: h = silu(g) * u rounded to bf16; down: fp32.
// FP8 weights: the sums are scaled by the row scales first (sc: gate rows [R] then up rows [R], or the down rows).
template <bool DUAL, int NT, int WF>
__device__ __forceinline__ void epilogue(const f32x4 (&accg_in)[NT], const f32x4 (&accu_in)[NT], void *out, int ld, int row0,
                                         const int (&orow)[NT], const float *sc, int R)
{
    const int r = row0 + 4 * (lane_id() >> 4);
    f32x4 sg = {1.f, 1.f, 1.f, 1.f}, su = {1.f, 1.f, 1.f, 1.f};
    if (WF == 1) {
        const float4 a = *reinterpret_cast<const float4 *>(sc + r);
        sg = f32x4{a.x, a.y, a.z, a.w};
        if (DUAL) {
            const float4 b = *reinterpret_cast<const float4 *>(sc + R + r);
            su = f32x4{b.x, b.y, b.z, b.w};
        }
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        if (orow[nt] < 0) continue;
        const f32x4 accg = WF == 1 ? accg_in[nt] * sg : accg_in[nt];
        const f32x4 accu = (WF == 1 && DUAL) ? accu_in[nt] * su : accu_in[nt];
        if (DUAL) {
            uint2 pk;
            pk.x = (uint32_t)f32_to_bf16_rne(silu_mul(accg[0], accu[0])) |
                   ((uint32_t)f32_to_bf16_rne(silu_mul(accg[1], accu[1])) << 16);
            pk.y = (uint32_t)f32_to_bf16_rne(silu_mul(accg[2], accu[2])) |
                   ((uint32_t)f32_to_bf16_rne(silu_mul(accg[3], accu[3])) << 16);
            // read by the down-projection workgroups of the same launch, possibly on another XCD
            store_coherent(reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(out) + (size_t)orow[nt] * ld + r), pk);
        } else {
            *reinterpret_cast<float4 *>(reinterpret_cast<float *>(out) + (size_t)orow[nt] * ld + r) =
                make_float4(accg[0], accg[1], accg[2], accg[3]);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Weight streaming.  Both kernels keep a ring of kPF prefetched 1 KiB weight tiles per wave and matrix
// in registers.  The loop bodies are branch-free on purpose: loads past the end are clamped to the last
// tile (re-reading it from cache) and their MFMA operand is zeroed, so that the compiler can count the
// outstanding loads and wait for exactly the oldest one instead of draining the queue.
// ---------------------------------------------------------------------------------------------------

// Direct: Wt = first weight tile of this wave (uint4 units); n = k-steps of this wave (>= 1);
// boff[nt] = byte offset of this lane's B piece at the wave's first column (4 x 16 bytes = 32 columns per step).
// The address passes through an empty asm so that the compiler treats every ring load as a distinct,
// unmovable-by-value-numbering load: otherwise it merges the prefetch for the next turn of the ring
// with the loads of that turn and issues them only when they are needed.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ring_load(const uint4 *__restrict__ base, int index)
{
    asm volatile("" : "+v"(index));
    return base[index];
}

// B operand (token rows).  For the down projection these are the intermediate vectors that gate/up workgroups
// of the same launch have written with device-coherent stores.  Plain (cached) loads are right for them: caches
// are invalidated when a kernel starts, a row is first touched after its expert's counter says it is complete,
// and rows start on 128-byte lines, so no cache on the reading side can hold an older copy of a line.  (Device-
// coherent loads instead would send every workgroup's re-reads of the same few rows to memory.)
//
// They are read through a buffer resource over the B array with a byte offset per lane.  A lane whose token column
// is empty (an expert with 3 tokens fills 3 of the 16 columns of a fragment) carries an offset past the resource's
// range: the hardware returns zero for it and fetches nothing.  The load path's time goes with the lanes that are in
// range (measured on a cache-resident region: 16 bytes per lane with 2 of 16 token columns in range cost 0.38 of
// the full load), and with 4-bit weights the token fragments are four times the bytes of the weights they meet.
constexpr unsigned kNoToken = 0x80000000u;   // past any resource (the B arrays stay below 2 GiB, checked on the host)
typedef __amdgpu_buffer_rsrc_t BufferRsrc;
__device__ __forceinline__ BufferRsrc token_rows_resource(const uint16_t *B)
{
    // the array is the same for all lanes of a wave: hand the address over as scalars (a resource that the compiler
    // takes for a per-lane value costs a loop over its distinct values around every load)
    const unsigned long long a = reinterpret_cast<unsigned long long>(B);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a), hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(((unsigned long long)hi << 32) | lo), 0, 0x7fffffff,
                                             0x00020000);
}
__device__ __forceinline__ uint4 ring_load_b(BufferRsrc rs, unsigned off, int index)
{
    asm volatile("" : "+v"(index));
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, off + (unsigned)index * 16u, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Expert weights: a non-temporal load (a weight byte is read once per launch, and a stream that does not allocate in
// the caches on its way runs measurably closer to the HBM rate) through a buffer resource over the wave's run of weight
// tiles.  The ring is refilled without branches, so a wave nearing the end of its run still issues its refills; those
// carry an offset past the resource's range, for which the hardware returns zero and fetches nothing.  (Clamping them
// to the last tile instead re-read that tile once per ring slot: with the short runs of small experts, a down
// projection of 12 k-steps behind a ring of 8, two thirds more loads than the weights need.  A streaming probe with
// the same clamped ring reads 12 KiB runs at 5.9 TB/s and runs of 24 KiB and more at 7.0-7.2 TB/s.)
__device__ __forceinline__ BufferRsrc weights_resource(const uint4 *wave_base)
{
    // the run's first tile is the same for all lanes of a wave: hand the address over as scalars
    const unsigned long long a = reinterpret_cast<unsigned long long>(wave_base);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a), hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(((unsigned long long)hi << 32) | lo), 0, 0x7fffffff,
                                             0x00020000);
}
constexpr int kAuxNonTemporal = 2;
// index: in 16-byte units from this lane's piece of the run's first tile; live = false: nothing is fetched, zero returns
__device__ __forceinline__ uint4 ring_load_weights(BufferRsrc rs, int index, bool live)
{
    unsigned off = live ? ((unsigned)index + (unsigned)lane_id()) * 16u : kNoToken;
    asm volatile("" : "+v"(off));
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, kAuxNonTemporal);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Two weight streams share every B fragment: gate and up tiles (interleaved: second = 64, step = 128) or,
// for the down projection, two consecutive row tiles (second = one row tile further, step = 64).
// 16 E4M3 codes (one lane's piece of a 64-column tile) -> two MFMA operands of 8 bf16 (columns 0-7 and 8-15 of
// the lane's group).  The hardware conversion gives fp32; an E4M3 value has 3 mantissa bits, so the upper half
// of the fp32 IS the bf16, exactly.
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t e4m3x2_to_bf16x2(uint32_t codes, bool upper)
{
    const f32x2 f = upper ? __builtin_amdgcn_cvt_pk_f32_fp8((int)codes, true) : __builtin_amdgcn_cvt_pk_f32_fp8((int)codes, false);
    return __builtin_amdgcn_perm(__float_as_uint(f.y), __float_as_uint(f.x), 0x07060302u);
}
__device__ __forceinline__ void e4m3x16_to_bf16(uint4 c, bf16x8 &lo, bf16x8 &hi)
{
    const uint4 l = make_uint4(e4m3x2_to_bf16x2(c.x, false), e4m3x2_to_bf16x2(c.x, true), e4m3x2_to_bf16x2(c.y, false),
                               e4m3x2_to_bf16x2(c.y, true));
    const uint4 h = make_uint4(e4m3x2_to_bf16x2(c.z, false), e4m3x2_to_bf16x2(c.z, true), e4m3x2_to_bf16x2(c.w, false),
                               e4m3x2_to_bf16x2(c.w, true));
    lo = __builtin_bit_cast(bf16x8, l);
    hi = __builtin_bit_cast(bf16x8, h);
}

// 32 E2M1 codes (one lane's piece of a 128-column MXFP4 tile: one scale block) -> four MFMA operands of 8 bf16
// (columns 8j .. 8j+7 of the block), each value already multiplied by the block scale.  The conversion
// instruction takes one byte (two codes, low nibble first) and the scale as a float; value * 2^k is exact in bf16.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t e2m1x2_to_bf16x2(uint32_t codes, float scale, int byte)
{
    bf16x2 r;
    switch (byte) {   // the byte select is an immediate
    case 0: r = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 0); break;
    case 1: r = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 1); break;
    case 2: r = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 2); break;
    default: r = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, scale, 3); break;
    }
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ bf16x8 e2m1x8_to_bf16(uint32_t codes, float scale)
{
    const uint4 v = make_uint4(e2m1x2_to_bf16x2(codes, scale, 0), e2m1x2_to_bf16x2(codes, scale, 1),
                               e2m1x2_to_bf16x2(codes, scale, 2), e2m1x2_to_bf16x2(codes, scale, 3));
    return __builtin_bit_cast(bf16x8, v);
}
// The scale of k-tile kt from the lane's dword of four exponents: 2^(E - 127) is the float with exponent field E.
__device__ __forceinline__ float mx_scale(uint32_t four, int kt) { return __uint_as_float(((four >> (8 * (kt & 3))) & 0xffu) << 23); }

// One weight tile of one stream -> its MFMA A operands (1, 2 or 4 k-steps of 32 columns).
template <int WF>
__device__ __forceinline__ void decode_tile(uint4 w, float scale, bf16x8 (&a)[1 << WF])
{
    if constexpr (WF == 0) {
        a[0] = __builtin_bit_cast(bf16x8, w);
    } else if constexpr (WF == 1) {
        e4m3x16_to_bf16(w, a[0], a[1]);
    } else {
        a[0] = e2m1x8_to_bf16(w.x, scale);
        a[1] = e2m1x8_to_bf16(w.y, scale);
        a[2] = e2m1x8_to_bf16(w.z, scale);
        a[3] = e2m1x8_to_bf16(w.w, scale);
    }
}

// Tiles in flight per wave and stream on the direct path.  MXFP4 tiles carry four k-steps, so the token
// fragments that travel with a slot are 64 bytes per lane, twice the slot's weights: four slots keep the ring
// inside the register file (measured: 3 and 4 equal, 5 and more spill and are slower; an MXFP4 launch at these
// sizes is short enough that the fixed part of a launch weighs more than the depth of the ring).
template <int WF>
struct DirectDepth {
    static constexpr int value = WF == 2 ? 4 : kPFD;
};

struct WeightRing {
    uint4 w0[kPFD], w1[kPFD];
    uint2 sq[kPFD];      // MXFP4: the scale exponents of both streams (see the layout above)
};

// Where a wave of the direct path streams from: needs the expert, not its tokens.
struct DirectPlan {
    const uint4 *Wb;     // the wave's first weight tile (the same for all lanes)
    const uint2 *Sl;     // MXFP4: this lane's scale dwords of the wave's row group, k-tile group 0
    int step, second;    // uint4 strides: next k-step, second stream
    int kb, n;           // first k-step and k-steps of this wave
    int kt0;             // first k-tile actually read (kb, or 0 for a wave without work)
    int rt;              // first 16-row tile
    bool rows_ok;
};

template <bool DUAL, int KW, int WF>
__device__ __forceinline__ DirectPlan plan_direct(const WorkItem &w)
{
    constexpr int RW = kFfnWaves / KW;
    const int wv = wave_id();
    const int rw = wv / KW, kw = wv % KW;
    const int KT = w.K / TileCols<WF>::value;
    DirectPlan d;
    const int grp = w.tile * RW + rw;                  // row group of this wave
    d.rt = DUAL ? grp : 2 * grp;
    d.rows_ok = d.rt * 16 < w.R;                       // (down: R/16 is even, so the second tile exists too)
    const int per = (w.ksteps + KW - 1) / KW;
    d.kb = w.kbeg + kw * per;
    d.n = min(w.kbeg + w.ksteps, d.kb + per) - d.kb;
    const int rtc = d.rows_ok ? d.rt : 0;              // waves past the last row read tile 0 and store nothing
    const int kbc = d.n > 0 ? d.kb : 0;
    d.kt0 = kbc;
    d.step = DUAL ? 2 * kWave : kWave;
    d.second = DUAL ? kWave : KT * kWave;
    d.Wb = w.W + ((size_t)rtc * KT + kbc) * d.step;
    d.Sl = nullptr;
    if (WF == 2)
        d.Sl = reinterpret_cast<const uint2 *>(w.sc) + (size_t)(d.rows_ok ? grp : 0) * mx_kt4(w.K) * kWave + lane_id();
    return d;
}

__device__ __forceinline__ uint2 ring_load_scales(const uint2 *__restrict__ base, int index)
{
    asm volatile("" : "+v"(index));
    return base[index];
}

template <int WF>
__device__ __forceinline__ void prefetch_weights(const DirectPlan &d, WeightRing &r)
{
    constexpr int D = DirectDepth<WF>::value;
    const int last = max(d.n, 1) - 1;
    const BufferRsrc rw = weights_resource(d.Wb);
#pragma unroll
    for (int j = 0; j < D; ++j) {
        const int s = min(j, last);
        r.w0[j] = ring_load_weights(rw, j * d.step, j <= last);
        r.w1[j] = ring_load_weights(rw, j * d.step + d.second, j <= last);
        if (WF == 2) r.sq[j] = ring_load_scales(d.Sl, ((d.kt0 + s) >> 2) * kWave);
    }
}

// The ring arrives with its first turn of weight tiles already requested (prefetch_weights).
template <int NT, int WF>
__device__ __forceinline__ void stream_direct(const DirectPlan &d, WeightRing &r, BufferRsrc rs, const unsigned (&boff)[NT],
                                              f32x4 (&acc0)[NT], f32x4 (&acc1)[NT])
{
    constexpr int D = DirectDepth<WF>::value;
    constexpr int BP = 1 << WF;              // 16-byte pieces of a token row per lane and weight tile = its k-steps
    constexpr int BS = TileCols<WF>::value / 8;   // uint4 units between the pieces of consecutive tiles
    const BufferRsrc rw = weights_resource(d.Wb);
    const int step = d.step, second = d.second;
    const int n = d.rows_ok ? d.n : 0;     // k-steps whose products count
    const int last = max(d.n, 1) - 1;
    uint4 bb[D][NT][BP];
#pragma unroll
    for (int j = 0; j < D; ++j) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int h = 0; h < BP; ++h) bb[j][nt][h] = ring_load_b(rs, j <= last ? boff[nt] : kNoToken, j * BS + h);
    }
    // One turn of the ring: consume the D slots in order, refilling each right after its last read.
    auto turn = [&](int s0) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int s = s0 + u;
            const bool live = s < n;
            // consume slot u ...
            bf16x8 a0[BP], a1[BP];
            const int kt = d.kt0 + min(s, last);
            decode_tile<WF>(sel4(live, r.w0[u]), WF == 2 ? mx_scale(r.sq[u].x, kt) : 1.0f, a0);
            decode_tile<WF>(sel4(live, r.w1[u]), WF == 2 ? mx_scale(r.sq[u].y, kt) : 1.0f, a1);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int h = 0; h < BP; ++h) {
                    const bf16x8 b = __builtin_bit_cast(bf16x8, bb[u][nt][h]);
                    acc0[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[h], b, acc0[nt], 0, 0, 0);
                    acc1[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[h], b, acc1[nt], 0, 0, 0);
                }
            // ... then refill it (the scheduling fences keep the refill behind the last read of the slot,
            // so that it can land in the same registers and the ring needs no copies)
            __builtin_amdgcn_sched_barrier(0);
            const int sn = s + D;          // refills past the end of the run fetch nothing
            const bool more = sn <= last;
            r.w0[u] = ring_load_weights(rw, sn * step, more);
            r.w1[u] = ring_load_weights(rw, sn * step + second, more);
            if (WF == 2) r.sq[u] = ring_load_scales(d.Sl, ((d.kt0 + min(sn, last)) >> 2) * kWave);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int h = 0; h < BP; ++h) bb[u][nt][h] = ring_load_b(rs, more ? boff[nt] : kNoToken, sn * BS + h);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // The first turn is peeled off the loop.  On entry the ring holds the weight loads of prefetch_weights
    // followed by the token loads above; from the first turn on, the loads of a slot are interleaved
    // (weights, weights, tokens).  The compiler inserts the waits for the oldest load from what may be
    // outstanding on ANY path into a block: with the first turn inside the loop it would have to assume the
    // entry order in every turn, and would wait until a third of the ring is left before the first slot.
    if (n > 0) {
        turn(0);
        for (int s0 = D; s0 < n; s0 += D) turn(s0);
    }
}

// One expert with <= 16*NT tokens: the four waves are RW row groups x KW slices of K; the slices are
// summed through LDS at the end.  A row group is one 16-row tile of gate and up (gate/up) or two
// consecutive 16-row tiles (down), so that every token fragment loaded feeds two MFMAs.
// The two halves of one row unit on the direct path.  direct_stream: the wave's products over its slice of K (the
// ring arrives with its first turn of weight tiles requested).  direct_finish: the K slices are summed through LDS and
// the results stored.  Between the two the ring's registers are free, so the caller requests the next unit's first
// tiles there: they are in flight while this unit's sums are exchanged and written.
// ro / orow: B row (element offset) and output row of this lane's token column, the same for every unit of an item.
template <int NT, int KW, int WF>
__device__ __forceinline__ void direct_stream(const WorkItem &w, const DirectPlan &d, WeightRing &ring, const int (&ro)[NT],
                                              f32x4 (&acc0)[NT], f32x4 (&acc1)[NT])
{
    constexpr int KC = TileCols<WF>::value;
    const int lane = lane_id();
    const int kbc = d.n > 0 ? d.kb : 0;
    unsigned boff[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)   // columns without a token fetch nothing and read as zero; their results are never stored
        boff[nt] = ro[nt] < 0 ? kNoToken : 2u * ((unsigned)ro[nt] + (unsigned)kbc * KC + (unsigned)(lane >> 4) * (KC / 4));
    clear_acc<NT>(acc0, acc1);
    stream_direct<NT, WF>(d, ring, token_rows_resource(w.B), boff, acc0, acc1);
}

template <bool DUAL, int NT, int KW, int WF>
__device__ __forceinline__ void direct_finish(const WorkItem &w, const DirectPlan &d, const int (&orow)[NT], f32x4 (&acc0)[NT],
                                              f32x4 (&acc1)[NT], float *red)
{
    constexpr int NACC = NT * 2;
    const int lane = lane_id(), wv = wave_id();
    const int rw = wv / KW, kw = wv % KW;
    if (KW > 1) {
        f32x4 *r4 = reinterpret_cast<f32x4 *>(red);   // [rw][kw-1][NACC][lane]
        if (kw > 0) {
            f32x4 *dst = r4 + ((size_t)(rw * (KW - 1) + (kw - 1)) * NACC) * kWave + lane;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                dst[(size_t)nt * kWave] = acc0[nt];
                dst[(size_t)(NT + nt) * kWave] = acc1[nt];
            }
        }
        __syncthreads();
        if (kw == 0) {
#pragma unroll
            for (int j = 1; j < KW; ++j) {
                const f32x4 *src = r4 + ((size_t)(rw * (KW - 1) + (j - 1)) * NACC) * kWave + lane;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    acc0[nt] += src[(size_t)nt * kWave];
                    acc1[nt] += src[(size_t)(NT + nt) * kWave];
                }
            }
        }
    }
    if (kw == 0 && d.rows_ok) {
        if (DUAL) {
            epilogue<true, NT, WF>(acc0, acc1, w.out, w.ldo, d.rt * 16, orow, w.sc, w.R);
        } else {
            epilogue<false, NT, WF>(acc0, acc0, w.out, w.ldo, d.rt * 16, orow, w.sc, w.R);
            epilogue<false, NT, WF>(acc1, acc1, w.out, w.ldo, d.rt * 16 + 16, orow, w.sc, w.R);
        }
    }
}

// Staged: the token tile is staged through LDS in chunks of KS k-steps, double buffered and shared by
// the four waves, which own four consecutive 16-row tiles and walk all of K.
// PAIR (down projection, 128-row workgroups): the wave owns two consecutive 16-row tiles and walks them together,
// pair_second uint4 units apart, so that every token fragment read from LDS feeds two MFMAs, as gate and up do (accg =
// first tile, accu = second): half the LDS reads per weight byte and half as many down workgroups (measured 2-4 %
// off the launch for every shape beyond 64 tokens).
template <bool DUAL, int NT, int KS, int WF, bool PAIR = false>
__device__ __forceinline__ void stream_staged(const uint4 *__restrict__ Wt, int KT, int K,
                                              const uint16_t *__restrict__ B, const int *rowoff, char *stage,
                                              const uint2 *__restrict__ Sl, int kt0, bool sc_second, int pair_second,
                                              f32x4 (&accg)[NT], f32x4 (&accu)[NT])   // KT weight tiles from Wt; B columns [0, K)
{   // (MXFP4: Sl = this lane's scale dwords of the wave's row group, kt0 = the first k-tile's index, sc_second = a
    // down-projection wave on the second row tile of its pair)
    constexpr bool TWO = DUAL || PAIR;
    const int second = DUAL ? kWave : pair_second;
    constexpr int TS = 1 << WF;                  // 32-column steps of the staged token tile per weight tile
    constexpr int ROWB = KS * 64 + 16;           // LDS bytes per token row (+16: conflict-free 16-byte reads)
    constexpr int BUFB = NT * 16 * ROWB;
    static_assert(2 * BUFB <= (NT > 4 ? kStageBytesBig : kStageBytes), "token tile does not fit the LDS stage");
    constexpr int PIECES = NT * 16 * KS * 4;     // 16-byte pieces per chunk
    static_assert(PIECES % kFfnThreads == 0, "pieces must divide evenly over the workgroup");
    constexpr int PPT = PIECES / kFfnThreads;
    static_assert((kPF * TS) % KS == 0, "a ring turn must hold whole chunks");
    constexpr int WSTEP = DUAL ? 2 * kWave : kWave;

    const int tid = threadIdx.x, lane = lane_id();
    const int last = KT - 1;
    const int lastc = (KT * TS + KS - 1) / KS - 1;

    // This thread's staging pieces: (token row, 16-byte piece inside the chunk).  The rows' offsets stay in the LDS
    // table and are looked up again for every chunk: registers are what this path is short of.  The pieces are read
    // through a buffer resource over the B array; a piece of a row without a token, or past the row's last column
    // (the last chunk of a ragged K, or a row shorter than one chunk), carries an offset out of range: nothing is
    // fetched for it and it arrives as zero, which is what the stage has to hold there.
    const BufferRsrc rb = token_rows_resource(B);
    const int pc0 = (tid % (KS * 4)) * 8;   // column of every piece of this thread inside a chunk (256 % (KS*4) == 0)
    uint4 xr[PPT];
    // chunk c: request it ... (nothing here reads what was loaded: a read would have to wait for the load, and
    // with it for every weight tile requested before it)
    auto load_x = [&](int c) {
        const int col = c * KS * 32 + pc0;
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int ro = rowoff[(tid + kFfnThreads * i) / (KS * 4)];
            xr[i] = ring_load_b(rb, (ro >= 0 && col < K) ? 2u * (unsigned)(ro + col) : kNoToken, 0);
        }
    };
    // ... and, a chunk of weight tiles later, put it into the stage
    auto store_x = [&](int c) {
        char *buf = stage + (c & 1) * BUFB;
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int q = tid + kFfnThreads * i;
            *reinterpret_cast<uint4 *>(buf + (q / (KS * 4)) * ROWB + (q % (KS * 4)) * 16) = xr[i];
        }
    };

    const BufferRsrc rw = weights_resource(Wt);
    uint4 wg[kPF], wu[kPF];
    uint2 sq[kPF];
#pragma unroll
    for (int j = 0; j < kPF; ++j) {
        const int s = min(j, last);
        wg[j] = ring_load_weights(rw, j * WSTEP, j <= last);
        wu[j] = TWO ? ring_load_weights(rw, j * WSTEP + second, j <= last) : zero4();
        if (WF == 2) sq[j] = ring_load_scales(Sl, ((kt0 + s) >> 2) * kWave);
    }
    load_x(0);
    store_x(0);
    __syncthreads();

    // this lane's B-fragment offset inside a token tile (its column group: 8 columns, or 16 for 64-column tiles)
    const int brow = (lane & 15) * ROWB + (lane >> 4) * (16 << WF);
    for (int s0 = 0; s0 < KT; s0 += kPF) {
#pragma unroll
        for (int u = 0; u < kPF; ++u) {
            const int s = s0 + u;
            const int c = (s * TS) / KS;
            if ((u * TS) % KS == 0) {
                load_x(min(c + 1, lastc));
                __builtin_amdgcn_sched_barrier(0);
            }
            // (tiles past the end of the run were not fetched and arrived as zeros; a wave without rows multiplies
            // tile 0 and stores nothing)
            const char *buf = stage + (c & 1) * BUFB + brow + ((u * TS) % KS) * 64;
            bf16x8 ag[TS], au[TS];
            const int kt = kt0 + min(s, last);
            decode_tile<WF>(wg[u], WF == 2 ? mx_scale(sc_second ? sq[u].y : sq[u].x, kt) : 1.0f, ag);
            if (TWO) decode_tile<WF>(wu[u], WF == 2 ? mx_scale(sq[u].y, kt) : 1.0f, au);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int h = 0; h < TS; ++h) {
                    const bf16x8 b = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(buf + nt * 16 * ROWB + 16 * h));
                    accg[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ag[h], b, accg[nt], 0, 0, 0);
                    if (TWO) accu[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(au[h], b, accu[nt], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
            const int sn = s + kPF;        // refills past the end of the run fetch nothing
            wg[u] = ring_load_weights(rw, sn * WSTEP, sn <= last);
            if (TWO) wu[u] = ring_load_weights(rw, sn * WSTEP + second, sn <= last);
            if (WF == 2) sq[u] = ring_load_scales(Sl, ((kt0 + min(sn, last)) >> 2) * kWave);
            __builtin_amdgcn_sched_barrier(0);
            if ((u * TS + TS - 1) % KS == KS - 1) {
                store_x(c + 1);
                __syncthreads();
            }
        }
    }
}

template <bool DUAL, int NT, int KS, int WF, bool PAIR = false>
__device__ __forceinline__ void expert_staged(const WorkItem &w, const int *rowoff, const int *outrow, char *stage)
{
    constexpr int WSTEP = DUAL ? 2 * kWave : kWave;
    constexpr int KC = TileCols<WF>::value;
    const int KT = w.K / KC;
    // w.tile counts 64-row units; a wave of a PAIR pass owns two row tiles of the 128 rows that start there
    const int rt = w.tile * kFfnWaves + (PAIR ? 2 : 1) * wave_id();
    const bool wave_active = rt * 16 < w.R;   // (down: R/16 is even, so the second tile of a pair exists too)
    const int rtc = wave_active ? rt : 0;   // idle waves read tile 0 (in bounds) and contribute nothing
    f32x4 accg[NT], accu[NT];
    clear_acc<NT>(accg, accu);
    const uint2 *Sl = nullptr;
    if (WF == 2)
        Sl = reinterpret_cast<const uint2 *>(w.sc) + (size_t)(DUAL ? rtc : rtc >> 1) * mx_kt4(w.K) * kWave + lane_id();
    stream_staged<DUAL, NT, KS, WF, PAIR>(w.W + ((size_t)rtc * KT + w.kbeg) * WSTEP, w.ksteps, w.ksteps * KC,
                                          w.B + (size_t)w.kbeg * KC, rowoff, stage, Sl, w.kbeg, !DUAL && !PAIR && (rtc & 1),
                                          KT * kWave, accg, accu);
    if (!wave_active) return;
    int orow[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) orow[nt] = outrow[nt * 16 + (lane_id() & 15)];
    if (PAIR) {
        epilogue<false, NT, WF>(accg, accg, w.out, w.ldo, rt * 16, orow, w.sc, w.R);
        epilogue<false, NT, WF>(accu, accu, w.out, w.ldo, rt * 16 + 16, orow, w.sc, w.R);
    } else {
        epilogue<DUAL, NT, WF>(accg, accu, w.out, w.ldo, rt * 16, orow, w.sc, w.R);
    }
}

// Both projections of every invoked and shared expert in ONE launch.  Grid: all gate/up workgroups, then
// all down workgroups; per projection the shared experts' items first, then the routed items in the order of the
// device-built plan (lynx_plan.h): live items are contiguous from the front of each part, and a workgroup past them
// leaves after one load.  A row unit is 16*RW rows of gate and up, or 32*RW rows of down, RW = 4 / KW.  An expert
// with at most kDirectMaxTokens tokens takes the direct path with the workgroup's four waves as RW row tiles x KW
// slices of K.  A larger expert takes the staged path, in which a workgroup covers 64 rows: of every KW
// consecutive workgroups one does the work, one pass of up to 64 (128) tokens per item, and the others leave.  A down
// item covers m consecutive row units, m chosen on the device from the number of (expert, token block) pairs: few
// invoked experts get short items that fill the chip, many get fewer, longer ones, whose start-up (tables, first
// tiles) weighs less.  The gate/up part of the grid ends with spare workgroups: when the last round of live gate/up
// workgroups is small, each of its workgroups is replaced by four of one row tile (see ffn_kernel).
//
// A down workgroup needs the intermediate vectors h of its expert complete.  Every gate/up workgroup adds its
// row tiles (four, or one) to its expert's counter once its h stores have completed; a down workgroup requests its
// first weight tiles and then waits for the counter to reach the expert's row tiles.  Workgroups are dispatched in
// index order, so when a down workgroup runs, every gate/up workgroup has been dispatched, and those wait for
// nothing: the wait always ends.  It is bounded all the same: on running out the workgroup sets a flag in the
// workspace and goes on, so no wave can hang, and the combine kernel turns the flag into NaNs in y and a non-zero
// status word.  The gain: the down projection's start-up overlaps the tail of gate/up instead of following a launch
// boundary.
struct FfnParams {
    GemmParams gu, dn;
    int gu_blocks;
    int block0;       // index of this launch's first workgroup in the (gate/up, down) order
    int gu_split;     // 1: the last, partial round of gate/up workgroups is cut into single row tiles (see ffn_kernel)
    int wait;         // 0: the down workgroups of this launch follow a finished gate/up launch and do not wait
    int spin_limit;   // polls of a completion counter before a down workgroup gives up
    int target_bias;  // added to the count a down workgroup waits for (0; tests of the give-up path set it)
    int32_t *done;    // [LYNX_MAX_N] routed experts, then [n_shared * token blocks]; zero before the launch
    int32_t *flags;
};

constexpr int kSplitRound = 256;     // CUs: workgroups per round of the dispatcher
constexpr int kSplitMaxRem = 128;    // largest partial round that is cut into single row tiles
constexpr int kSplitMaxTokens = 32;  // largest batch for which it is done
constexpr int kSpinLimit = 1 << 17;   // polls of a counter (about a microsecond each) before giving up

__device__ __forceinline__ int done_slot(const GemmParams &p, const WorkItem &w)
{
    return w.shared_s < 0 ? w.e : LYNX_MAX_N + w.shared_s * p.shared_tblocks + w.tok0 / p.tok_block;
}

// sub >= 0 (gate/up, KW = 4 only): the workgroup takes row tile `sub` of the four that workgroup b stands for.
template <bool DUAL, int KW, bool BIG, int WF>
__device__ __forceinline__ void expert_work(const GemmParams &p, int b, const FfnParams &fp, char *stage, int *rowoff,
                                            int *outrow, int sub = -1)
{
    constexpr int TB = BIG ? kTokBlockBig : kTokBlock;   // tokens per pass
    int units;
    LYNX_TS_BEGIN(DUAL ? (sub >= 0 ? 2 : 1) : 0, b);
    WorkItem w = resolve_item<DUAL, WF>(p, b, units);
    if (!w.valid) return;
    if (sub >= 0) w.tile = w.tile * kFfnWaves + sub;
    int32_t *counter = fp.done + done_slot(p, w);
    const int unit0 = w.tile;
    LYNX_TS(1);
    // Waits for this expert's (this token block's) intermediate vectors (down projection in the same launch as
    // gate/up; gate/up workgroups report row tiles: four each, or one for a workgroup of a single tile).
    auto wait_for_h = [&]() {
        if (DUAL || !fp.wait) return;
        const int items = w.shared_s < 0 ? fp.gu.tiles_r * plan_token_blocks(w.te_all, p.tok_block) : fp.gu.tiles_s;
        const int target = kFfnWaves * items + fp.target_bias;
        if (threadIdx.x == 0) {
            int polls = 0;
            while (load_coherent(counter) < target) {
                if (++polls > fp.spin_limit) {
                    atomicOr(fp.flags, 1);
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
        }
        __syncthreads();
    };
    if (w.te_all <= kDirectMaxTokens) {
        // Direct path.  The weight stream starts before anything else is waited for, and the next unit's first tiles
        // are requested before this unit's results are exchanged and stored.
        DirectPlan plan = plan_direct<DUAL, KW, WF>(w);
        WeightRing ring;
        prefetch_weights<WF>(plan, ring);
        int ro[1], orow[1];
        token_rows_direct<DUAL>(p, w, ro[0], orow[0]);
        wait_for_h();
        LYNX_TS(2);
        for (int un = 0; un < units; ++un) {
            f32x4 acc0[1], acc1[1];
            direct_stream<1, KW, WF>(w, plan, ring, ro, acc0, acc1);
            const DirectPlan done = plan;
            if (un + 1 < units) {
                w.tile = unit0 + un + 1;
                plan = plan_direct<DUAL, KW, WF>(w);
                prefetch_weights<WF>(plan, ring);
            }
            direct_finish<DUAL, 1, KW, WF>(w, done, orow, acc0, acc1, reinterpret_cast<float *>(stage));
            if (KW > 1 && un + 1 < units) __syncthreads();   // the next unit reuses the K-slice sums in LDS
        }
    } else {
        wait_for_h();
        LYNX_TS(2);
        // staged path: units of 64 rows.  A direct workgroup covers 16*RW rows (gate/up) or 32*RW rows (down).
        constexpr int kRowsPerWG = 16 * (kFfnWaves / KW) * (DUAL ? 1 : 2);
        constexpr int kUnits = kRowsPerWG >= 64 ? kRowsPerWG / 64 : 1;      // staged units per row unit
        constexpr int kShare = kRowsPerWG >= 64 ? 1 : 64 / kRowsPerWG;      // workgroups that share one staged unit
        // (a gate/up workgroup that shares its unit with others and leaves the work to one of them still reports
        // below: a down workgroup waits for the row tiles of all gate/up workgroups of its expert)
        // (shared experts see every token, so the host knows that they are staged and gives them one workgroup
        // per unit)
        const bool shared = w.shared_s >= 0;
        const int tid = threadIdx.x;
        for (int un = 0; un < units; ++un) {
            const int tile = unit0 + un;
            // Of the workgroups that share a unit one does the work and the others leave.  Which one rotates with the
            // unit and the expert: the sharing workgroups have consecutive indices, so a fixed choice would put all the
            // staged work of the launch on the XCDs that the first of every four workgroups goes to (measured: two of
            // the eight XCDs ended their gate/up work at 44 us, the others at 31 us).
            if (!shared && (tile % kShare) != ((tile / kShare + w.e) % kShare)) continue;
            const int s0 = shared ? tile : (tile / kShare) * kUnits;
            // a 128-row down workgroup does its two 64-row units in one pass, two row tiles per wave
            constexpr bool kPair = !DUAL && kUnits == 2;
            const bool pair = kPair && !shared;
            const int sn = (shared || pair) ? 1 : kUnits;
            for (int su = 0; su < sn; ++su) {
                w.tile = s0 + su;
                if (w.tile * 64 >= w.R) break;
                for (int i0 = w.tok0; i0 < w.Te; i0 += TB) {
                    const int nb = min(w.Te - i0, TB);
                    __syncthreads();   // the previous pass has read rowoff / outrow and the stage
                    if (tid < TB) {
                        int ro, orow;
                        token_rows<DUAL>(p, w, tid < nb ? i0 + tid : w.Te, ro, orow);
                        rowoff[tid] = ro;
                        outrow[tid] = orow;
                    }
                    __syncthreads();
                    if constexpr (kPair) {
                        if (pair) {
                            if (nb <= 32)
                                expert_staged<DUAL, 2, 8, WF, true>(w, rowoff, outrow, stage);
                            else if (!BIG || nb <= 64)
                                expert_staged<DUAL, 4, 4, WF, true>(w, rowoff, outrow, stage);
                            else
                                expert_staged<DUAL, 8, 4, WF, true>(w, rowoff, outrow, stage);
                            continue;
                        }
                    }
                    if (nb <= 32)
                        expert_staged<DUAL, 2, 8, WF>(w, rowoff, outrow, stage);
                    else if (!BIG || nb <= 64)
                        expert_staged<DUAL, 4, 4, WF>(w, rowoff, outrow, stage);
                    else
                        expert_staged<DUAL, 8, 4, WF>(w, rowoff, outrow, stage);
                }
            }
        }
    }
    LYNX_TS(3);
    if (DUAL && fp.wait) {   // report: this workgroup's part of h is complete in memory
        wait_memory_complete();
        __syncthreads();
        if (threadIdx.x == 0) atomicAdd(counter, KW == 1 ? kFfnWaves : 1);
    }
}

#ifndef LYNX_WGCU
#define LYNX_WGCU 2
#endif
constexpr int kWgPerCuSmall = LYNX_WGCU;   // workgroups per CU of the kernels for batches of at most 64 tokens

template <int KWD, bool BIG, int WF>
__global__ __launch_bounds__(kFfnThreads, (BIG || WF != 0) ? 2 : kWgPerCuSmall) void ffn_kernel(FfnParams fp)
{
    // staged token tile, or the K-slice partial sums
    __shared__ __attribute__((aligned(16))) char stage[BIG ? kStageBytesBig : kStageBytes];
    __shared__ int rowoff[BIG ? kTokBlockBig : kTokBlock];   // staged path: element offset of each token's B row, -1 = none
    __shared__ int outrow[BIG ? kTokBlockBig : kTokBlock];   // staged path: output row of each token, -1 = none
    const int b = blockIdx.x + fp.block0;
    if (b < fp.gu_blocks) {
        // Gate/up workgroups take four row tiles, one per wave, and the dispatcher hands workgroups to the CUs
        // breadth first: L live workgroups put two on L mod 256 CUs and one on the rest, and while the stream is
        // HBM-bound the CUs share it evenly, so the CUs with two take twice as long (measured: Qwen3 shape, 312
        // workgroups: 21-24 us against 40-48 us), at the end on a fraction of the chip's waves.  When that last,
        // partial round is small, each of its workgroups is replaced by four workgroups of one row tile (the
        // four waves split K), which the dispatcher spreads over all CUs: at most one or two tiles more per CU.
        // The count of live workgroups is a device-side value, so the mapping is made here.
        // (bf16 weights only: in the kernels of the quantised formats the second code path costs spilled registers)
        int bb = b, sub = -1;
        if (WF == 0 && fp.gu_split) {
            const int live = fp.gu.shared_blocks + max(fp.gu.plan[kWsPlanHdr + kPlanB], 0) * fp.gu.tiles_r;
            const int full = live / kSplitRound * kSplitRound, rem = live - full;
            if (rem > 0 && rem <= kSplitMaxRem && full >= fp.gu.shared_blocks) {
                // The small workgroups come last in the grid: they fill the tail.  (Putting them first when everything
                // is resident at once was tried, so that the small one is the older workgroup on its CU: with the
                // device-built plan it is equal or slower, Qwen3 shapes 32 tokens 51.7 against 49.3 us, 16 tokens
                // 47.4 against 43.1.)
                if (b >= full) {
                    bb = full + (b - full) / kFfnWaves;
                    sub = (b - full) % kFfnWaves;
                    if (bb >= live) return;
                }
            }
        }
        if (WF != 0 || sub < 0)
            expert_work<true, 1, BIG, WF>(fp.gu, bb, fp, stage, rowoff, outrow);
        else if constexpr (WF == 0)
            expert_work<true, kFfnWaves, BIG, WF>(fp.gu, bb, fp, stage, rowoff, outrow, sub);
    } else {
        expert_work<false, KWD, BIG, WF>(fp.dn, b - fp.gu_blocks, fp, stage, rowoff, outrow);
    }
}

// The plan from a caller's token assignment (lynx_moe_ffn after lynx_permute): the experts with a valid, non-empty
// range in expert_offsets are the invoked ones.  One workgroup; also clears the completion counters and the flags.
__global__ __launch_bounds__(256) void plan_kernel(const int32_t *__restrict__ offsets, const int32_t *__restrict__ perm, int N,
                                                   int P, PlanShape ps, int32_t *__restrict__ ws)
{
    __shared__ int count[LYNX_MAX_N], offs[LYNX_MAX_N], blk0[LYNX_MAX_N];
    const int tid = threadIdx.x;
    for (int i = tid; i < kWsDoneWords + 16; i += 256) ws[kWsDone + i] = 0;
    if (tid < N) {
        const int o0 = offsets[tid], o1 = offsets[tid + 1];
        const bool ok = o0 >= 0 && o1 > o0 && o1 <= P;
        count[tid] = ok ? o1 - o0 : 0;
        offs[tid] = ok ? o0 : 0;
    }
    __syncthreads();
    build_plan<256>(ps, N, count, offs, blk0, ws);
    __syncthreads();
    // the pair ids of the experts on the direct path, 16 threads per expert
    for (int e = tid / kDirectMaxTokens; e < N; e += 256 / kDirectMaxTokens) {
        const int i = tid % kDirectMaxTokens;
        if (i < count[e]) {   // (an id outside [0, P) is filed as 0xffff: no such pair, the row is skipped)
            const int pv = perm[offs[e] + i];
            plan_file_pair(ps, blk0, e, count[e], i, (pv >= 0 && pv < P) ? pv : 0xffff, ws);
        }
    }
}

// y[t] = sum_j gate[t,j] * o[t*k+j] + sum_s o[P + s*T + t].  If a workgroup of the expert kernel gave up a bounded wait
// (flags != 0: some rows of o may then be computed from incomplete intermediate vectors) every element of y becomes NaN
// and *status (if given) 1, else *status 0: a failed hand-over cannot pass for a result.
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ o, const int32_t *__restrict__ idx,
                                                      const float *__restrict__ gate, int T, int H, int N, int k,
                                                      int n_shared, float *__restrict__ y,
                                                      const int32_t *__restrict__ flags, int32_t *__restrict__ status)
{
    const int t = blockIdx.y;
    const int h = (blockIdx.x * 256 + threadIdx.x) * 4;
    const bool failed = *flags != 0;
    if (status && t == 0 && blockIdx.x == 0 && threadIdx.x == 0) *status = failed ? 1 : 0;
    if (h >= H) return;
    if (failed) {
        const float q = __int_as_float(0x7fc00000);
        *reinterpret_cast<float4 *>(y + (size_t)t * H + h) = make_float4(q, q, q, q);
        return;
    }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; ++j) {
        const int e = idx[(size_t)t * k + j];
        if (e < 0 || e >= N) continue;
        const float g = gate[(size_t)t * k + j];
        const float4 v = *reinterpret_cast<const float4 *>(o + ((size_t)t * k + j) * H + h);
        acc.x = fmaf(g, v.x, acc.x);
        acc.y = fmaf(g, v.y, acc.y);
        acc.z = fmaf(g, v.z, acc.z);
        acc.w = fmaf(g, v.w, acc.w);
    }
    for (int s = 0; s < n_shared; ++s) {
        const float4 v = *reinterpret_cast<const float4 *>(o + ((size_t)T * k + (size_t)s * T + t) * H + h);
        acc.x += v.x;
        acc.y += v.y;
        acc.z += v.z;
        acc.w += v.w;
    }
    *reinterpret_cast<float4 *>(y + (size_t)t * H + h) = acc;
}

// Row-major -> streaming layout, one 16-byte piece per thread.
__global__ __launch_bounds__(256) void pack_kernel(const uint16_t *__restrict__ Wa, const uint16_t *__restrict__ Wb,
                                                   int nmat, int E, int R, int K, uint16_t *__restrict__ out)
{
    const int KT = K / 32;
    const size_t pieces = (size_t)E * (R / 16) * KT * nmat * kWave;
    const size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= pieces) return;
    const int l = (int)(q % kWave);
    size_t rest = q / kWave;
    const int m = (int)(rest % nmat);
    rest /= nmat;
    const int kt = (int)(rest % KT);
    rest /= KT;
    const int rt = (int)(rest % (R / 16));
    const int e = (int)(rest / (R / 16));
    const uint16_t *src = (m == 0 ? Wa : Wb) + ((size_t)e * R + rt * 16 + (l & 15)) * K + kt * 32 + (l >> 4) * 8;
    *reinterpret_cast<uint4 *>(out + q * 8) = *reinterpret_cast<const uint4 *>(src);
}

// Nearest E4M3 code of v (ties to the even code, 448 and above to +-448, NaN to NaN), in integer and exact
// floating-point steps so that it does not depend on a conversion mode of the hardware.
__device__ __forceinline__ uint32_t e4m3_encode(float v)
{
    const uint32_t sgn = (__float_as_uint(v) >> 24) & 0x80u;
    if (v != v) return sgn | 0x7fu;
    const float a = fabsf(v);
    if (a >= 448.0f) return sgn | 0x7eu;
    uint32_t code;
    if (a < 0.015625f) {                       // below 2^-6: multiples of 2^-9
        code = (uint32_t)rintf(a * 512.0f);
    } else {
        const uint32_t bits = __float_as_uint(a);
        const int ex = (int)(bits >> 23) - 127;                              // a = m * 2^ex, m in [1, 2)
        const float m = __uint_as_float((bits & 0x007fffffu) | 0x3f800000u);
        const uint32_t q = (uint32_t)rintf((m - 1.0f) * 8.0f);               // exact product; 8 carries into the exponent
        code = ((uint32_t)(ex + 7) << 3) + q;
    }
    return sgn | min(code, 0x7eu);
}

// Row-wise FP8 quantisation straight into the streaming layout: one wave per (expert, matrix, row).  scale =
// amax / 448 (1 for an all-zero row), code = encode(w / scale), both divisions correctly rounded fp32.  A 1 KiB
// tile is 16 rows x 64 columns: lane l = row l%16, column group l/16 (16 consecutive columns = 16 bytes).
__global__ __launch_bounds__(256) void quantize_kernel(const uint16_t *__restrict__ Wa, const uint16_t *__restrict__ Wb,
                                                       int nmat, int E, int R, int K, uint8_t *__restrict__ out,
                                                       float *__restrict__ scales)
{
    const long row_id = (long)blockIdx.x * 4 + wave_id();   // (e, m, r)
    if (row_id >= (long)E * nmat * R) return;
    const int lane = lane_id();
    const int r = (int)(row_id % R);
    const int m = (int)((row_id / R) % nmat);
    const int e = (int)(row_id / ((long)R * nmat));
    const uint16_t *src = (m == 0 ? Wa : Wb) + ((size_t)e * R + r) * K;
    float amax = 0.f;
    for (int c = lane * 8; c < K; c += kWave * 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(src + c);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            amax = fmaxf(amax, fabsf(__uint_as_float(w[i] << 16)));
            amax = fmaxf(amax, fabsf(__uint_as_float(w[i] & 0xffff0000u)));
        }
    }
    amax = wave_max(amax);
    const float sc = amax == 0.f ? 1.0f : __fdiv_rn(amax, 448.0f);
    if (lane == 0) scales[((size_t)e * nmat + m) * R + r] = sc;
    const int KT = K / 64;
    for (int c = lane * 16; c < K; c += kWave * 16) {   // 16 consecutive columns = one lane's piece of a tile
        uint32_t packed[4];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const uint4 v = *reinterpret_cast<const uint4 *>(src + c + half * 8);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = e4m3_encode(__fdiv_rn(__uint_as_float(w[i] << 16), sc));
                const uint32_t hi = e4m3_encode(__fdiv_rn(__uint_as_float(w[i] & 0xffff0000u), sc));
                const uint32_t two = lo | (hi << 8);
                if (i % 2 == 0)
                    packed[half * 2 + i / 2] = two;
                else
                    packed[half * 2 + i / 2] |= two << 16;
            }
        }
        const int kt = c / 64, g = (c % 64) / 16;
        const size_t piece = ((((size_t)e * (R / 16) + r / 16) * KT + kt) * nmat + m) * kWave + g * 16 + (r % 16);
        *reinterpret_cast<uint4 *>(out + piece * 16) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
    }
}

// Nearest E2M1 code of q (already divided by the block scale): ties to the even code, magnitudes above 6 to 6.
// The thresholds are the midpoints of 0, 0.5, 1, 1.5, 2, 3, 4, 6; "<=" where the lower neighbour is the even code.
__device__ __forceinline__ uint32_t e2m1_encode(float q)
{
    const uint32_t sgn = (__float_as_uint(q) >> 31) << 3;
    const float a = fabsf(q);
    const uint32_t code = a <= 0.25f ? 0u : a < 0.75f ? 1u : a <= 1.25f ? 2u : a < 1.75f ? 3u : a <= 2.5f ? 4u : a < 3.5f ? 5u : a <= 5.0f ? 6u : 7u;
    return sgn | code;
}

// MXFP4 quantisation straight into the streaming layout: one wave per (expert, matrix, row), a lane per block of
// 32 columns.  Per block: E - 127 = floor(log2(amax)) - 2, clamped to [0, 254] (E = 127 for an all-zero block);
// code = encode(w * 2^(127 - E)), an exact scaling.  Weights: a 1 KiB tile is 16 rows x 128 columns, lane l = row
// l%16, block l/16, 16 bytes, byte j = columns 2j (low nibble) and 2j+1.  Scale exponents: byte kt%4 of dword
// [row group][kt/4][lane][which], (row group, which) = (row tile, matrix) for gate/up or (row pair, tile of the
// pair) for down.
__global__ __launch_bounds__(256) void quantize_fp4_kernel(const uint16_t *__restrict__ Wa, const uint16_t *__restrict__ Wb,
                                                           int nmat, int E, int R, int K, uint8_t *__restrict__ out,
                                                           uint8_t *__restrict__ scales)
{
    const long row_id = (long)blockIdx.x * 4 + wave_id();   // (e, m, r)
    if (row_id >= (long)E * nmat * R) return;
    const int lane = lane_id();
    const int r = (int)(row_id % R);
    const int m = (int)((row_id / R) % nmat);
    const int e = (int)(row_id / ((long)R * nmat));
    const uint16_t *src = (m == 0 ? Wa : Wb) + ((size_t)e * R + r) * K;
    const int KT = K / 128;
    const size_t KT4 = mx_kt4(K);
    const int groups = nmat == 2 ? R / 16 : R / 32;
    const int grp = nmat == 2 ? r / 16 : r / 32;
    const int which = nmat == 2 ? m : (r / 16) & 1;
    for (int c = lane * 32; c < K; c += kWave * 32) {
        uint32_t w[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint4 v = *reinterpret_cast<const uint4 *>(src + c + q * 8);
            w[4 * q] = v.x;
            w[4 * q + 1] = v.y;
            w[4 * q + 2] = v.z;
            w[4 * q + 3] = v.w;
        }
        float amax = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            amax = fmaxf(amax, fabsf(__uint_as_float(w[i] << 16)));
            amax = fmaxf(amax, fabsf(__uint_as_float(w[i] & 0xffff0000u)));
        }
        int Eb = 127;
        if (amax > 0.f) {
            const uint32_t bits = __float_as_uint(amax);
            const int ef = (int)(bits >> 23);
            const int fl = ef != 0 ? ef - 127 : (31 - __clz((int)(bits & 0x007fffffu))) - 149;   // floor(log2(amax))
            Eb = min(max(fl - 2 + 127, 0), 254);
        }
        uint32_t packed[4];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t lo = e2m1_encode(ldexpf(__uint_as_float(w[i] << 16), 127 - Eb));
            const uint32_t hi = e2m1_encode(ldexpf(__uint_as_float(w[i] & 0xffff0000u), 127 - Eb));
            const uint32_t byte = lo | (hi << 4);
            if (i % 4 == 0)
                packed[i / 4] = byte;
            else
                packed[i / 4] |= byte << (8 * (i % 4));
        }
        const int kt = c / 128, g = (c % 128) / 32;
        const int l = g * 16 + (r % 16);
        const size_t piece = ((((size_t)e * (R / 16) + r / 16) * KT + kt) * nmat + m) * kWave + l;
        *reinterpret_cast<uint4 *>(out + piece * 16) = make_uint4(packed[0], packed[1], packed[2], packed[3]);
        const size_t dword = (((size_t)e * groups + grp) * KT4 + kt / 4) * 128 + (size_t)l * 2 + which;
        scales[dword * 4 + (kt % 4)] = (uint8_t)Eb;
    }
}

// How many of a workgroup's four waves split the contraction dimension (the rest split rows).  Long
// per-wave streams amortise the fill and drain of the prefetch ring, so K is only split when the
// batch cannot invoke enough experts to give every CU several waves otherwise.
static int pick_k_waves(int K, bool dual, int T, int max_experts, int bits_per_weight)
{
    // Gate/up: a wave streams a whole row tile of both matrices (2 * K * 32 bytes, contiguous); measured best
    // at every expert count.  It also makes a workgroup exactly one 64-row unit of the staged path.
    if (dual) return 1;
    // Down, more than 16 tokens: some expert may take the staged path, whose unit is 64 rows; two row groups
    // of 32 rows per workgroup cover exactly one (workgroups that only exist to be told they have nothing to
    // do are expensive).
    // Beyond 64 tokens (passes of up to 128 tokens): 128-row workgroups, whose staged passes give every wave two row
    // tiles that share each token fragment read from LDS (measured 2-4 % faster on every shape).
    // (not with quantised weights and at most 8 experts: 256 down workgroups of a Mixtral-shaped layer then carry too
    // few bytes each: FP8 419 against 386 us, MXFP4 360 against 323 us per layer at 128 tokens)
    if (T > kTokBlock && !(bits_per_weight < 16 && max_experts <= 8)) return 1;
    if (T > kDirectMaxTokens) return 2;
    // Down, direct path only.  Measured: splitting K four ways pays when the batch can invoke so few experts
    // that whole row groups would leave the chip with too few, too long workgroups (Mixtral-like shapes); with
    // more experts two ways (64-row workgroups: 4-5 % faster than 128-row ones for DeepSeek-V2-Lite and
    // Qwen1.5-MoE shapes), unless the streams would get too short.
    const long group_bytes = (long)16 * K * 2 * bits_per_weight / 8;      // weight bytes behind one row group
    int kw = max_experts <= 8 ? 4 : 2;
    while (kw > 1 && group_bytes / kw < 32 * 1024) kw >>= 1;              // keep at least 32 KiB per wave
    return kw;
}

// Knobs that tuning runs and the test of the give-up path set through lynx_debug_set (lynx_bench.h); the defaults are
// what the library ships with.
struct Tunables {
    std::atomic<int> spin_limit{kSpinLimit};
    std::atomic<int> target_bias{0};
    std::atomic<int> dn_cap{768};      // down items the grid aims at (two per CU are resident: 512)
    std::atomic<int> dn_m_max{1};      // most row units per down item
    std::atomic<int> dn_kw{0};         // 0 = the rule of pick_k_waves, else the K slices of a down workgroup's waves
};
static Tunables g_tune;

// Everything the host decides from the sizes alone.
struct FfnShape {
    int kwd;            // K slices of a down workgroup's waves
    bool big, single;   // 128-token staged passes; one launch for both projections
    int tok_block;
    int max_blocks;     // most (expert, token block) pairs of a batch
    PlanShape plan;
};

static bool single_launch(int T, int F) { return T >= 1 && (F + 63) / 64 <= 64; }   // (any batch size: see below)

static FfnShape ffn_shape(int T, int H, int F, int N, int k, int n_shared, int format)
{
    FfnShape s;
    const int max_experts = (int)min((long)N, (long)T * k) + n_shared;
    s.kwd = pick_k_waves(F, false, T, max_experts, 16 >> format);
    const int forced = g_tune.dn_kw.load();
    if (forced == 1 || forced == 2 || (forced == 4 && T <= kDirectMaxTokens)) s.kwd = forced;
    s.big = T > kTokBlock;
    s.single = single_launch(T, F);
    s.tok_block = s.big ? kTokBlockBig : kTokBlock;
    s.max_blocks = plan_max_blocks(T, N, k, s.tok_block);
    const int rows_dn = 16 * (kFfnWaves / s.kwd) * 2;
    s.plan.units_gu = (F + 16 * kFfnWaves - 1) / (16 * kFfnWaves);
    s.plan.units_dn = (H + rows_dn - 1) / rows_dn;
    s.plan.tok_block = s.tok_block;
    // Longer down items only where the staged unit and the direct workgroup are the same 64 rows (two K slices).
    s.plan.dn_m_max = s.kwd <= 2 ? max(1, g_tune.dn_m_max.load()) : 1;
    s.plan.dn_cap = max(1, g_tune.dn_cap.load());
    return s;
}

PlanShape ffn_plan_shape(int T, int H, int F, int N, int k, int n_shared, int format)
{
    return ffn_shape(T, H, F, N, k, n_shared, format).plan;
}

static void set_tiles(GemmParams &p, int units_r, int rows_per_wg, int routed_items)
{
    p.tiles_r = units_r;
    // shared experts process all T tokens: staged (units of 64 rows, one per workgroup) when T is past the direct limit
    const int rows_shared = p.T > kDirectMaxTokens ? 64 : rows_per_wg;
    p.tiles_s = p.n_shared ? (p.Rs + rows_shared - 1) / rows_shared : 0;
    // ... and then a workgroup with all T tokens would make one pass per 64 tokens over the same weights and be by
    // far the longest of the launch: the passes go to workgroups of their own instead.
    p.tok_block = p.T > kTokBlock ? kTokBlockBig : kTokBlock;
    p.shared_tblocks = p.T > kDirectMaxTokens ? (p.T + p.tok_block - 1) / p.tok_block : 1;
    p.tiles_s_stride = p.shared_tblocks > 1 ? (p.tiles_s + 7) / 8 * 8 : p.tiles_s;
    p.shared_blocks = p.n_shared * p.shared_splits * p.shared_tblocks * p.tiles_s_stride;
    p.routed_blocks = routed_items;
}

static unsigned grid_blocks(const GemmParams &p) { return (unsigned)(p.shared_blocks + p.routed_blocks); }

// Workgroups per CU.  The dispatcher fills a CU up to its occupancy limit before it moves on, so a grid
// that is small compared with the chip (few invoked experts) would leave CUs idle while others hold three
// workgroups.  A dynamic-LDS pad makes exactly kWgPerCu workgroups fit a CU, which spreads such grids.
constexpr int kLdsPerCu = 160 * 1024;

template <int KWD, bool BIG, int WF>
static int launch_padded(const FfnParams &fp, unsigned blocks, hipStream_t st)
{
    constexpr int kWgPerCu = (BIG || WF != 0) ? 2 : kWgPerCuSmall;
    constexpr int kLdsTargetPerWg = kWgPerCu == 2 ? 56 * 1024 : kLdsPerCu / kWgPerCu / 1024 * 1024;   // (at most 64 KiB per workgroup)
    static_assert(kLdsTargetPerWg * (kWgPerCu + 1) > kLdsPerCu && kLdsTargetPerWg * kWgPerCu <= kLdsPerCu, "LDS pad");
    // what the kernel declares itself: the stage and the two token tables
    constexpr int kStatic = (BIG ? kStageBytesBig : kStageBytes) + 2 * 4 * (BIG ? kTokBlockBig : kTokBlock) ;
    constexpr int pad = kLdsTargetPerWg > kStatic ? kLdsTargetPerWg - kStatic : 0;
    static_assert((kStatic + pad) * kWgPerCu <= kLdsPerCu, "the workgroups must fit a CU");
    hipLaunchKernelGGL((ffn_kernel<KWD, BIG, WF>), dim3(blocks), dim3(kFfnThreads), pad, st, fp);
    return LYNX_OK;
}

// One launch for both projections, or one each (the same kernel over its gate/up and its down workgroups)?
// Measured over the benchmark configurations: with experts of moderate size the single launch is 3-12 % faster beyond
// 16 tokens (the down projection fills the tail of gate/up and there is one start-up less) and 0-5 % faster up to 16
// (DeepSeek-V2-Lite shapes, 16 tokens: 87.6 -> 84.7 us per layer, remap off 150.0 -> 146.5; Qwen1.5-MoE shapes, 8
// tokens: 81.7 -> 81.7, remap off 92.3 -> 87.5); with huge experts (hundreds of gate/up workgroups each, whose
// completion reports then cost more than the overlap gains) it is equal or slower at every batch size.

// Gate/up and down over all invoked and shared experts.  Batches of more than 64 tokens take the
// kernels whose staged path makes passes of up to 128 tokens.
template <int WF>
static int launch_ffn(FfnParams fp, const FfnShape &sh, hipStream_t st)
{
    const GemmParams &d = fp.dn;
    set_tiles(fp.gu, sh.plan.units_gu, 16 * kFfnWaves, sh.plan.units_gu * sh.max_blocks);   // gate/up: four row tiles per workgroup
    set_tiles(fp.dn, sh.plan.units_dn, 16 * (kFfnWaves / sh.kwd) * 2, plan_down_grid(sh.plan, sh.max_blocks));
    fp.gu.dn_m_max = fp.dn.dn_m_max = sh.plan.dn_m_max;
    // the split of the last round needs up to three more workgroups per workgroup it replaces
    // (not for batches of more than 32 tokens: more and more experts are then on the staged path, whose unit is the
    // whole workgroup of four row tiles, and three of the four small workgroups only find out that they leave;
    // measured equal or 3 us slower at 64 tokens, 3-8 us slower at 128 and 256)
    fp.gu_split = (WF == 0 && d.T <= kSplitMaxTokens && fp.gu.shared_blocks < kSplitRound) ? 1 : 0;
    fp.gu_blocks = (int)grid_blocks(fp.gu) + (fp.gu_split ? kSplitMaxRem * (kFfnWaves - 1) : 0);
    const unsigned dn_blocks = grid_blocks(fp.dn);
    int rc = LYNX_OK;
    for (int part = 0; part < (sh.single ? 1 : 2) && rc == LYNX_OK; ++part) {
        fp.wait = sh.single ? 1 : 0;
        fp.block0 = part == 0 ? 0 : fp.gu_blocks;
        const unsigned blocks = sh.single ? (unsigned)fp.gu_blocks + dn_blocks : part == 0 ? (unsigned)fp.gu_blocks : dn_blocks;
        if (sh.big && sh.kwd == 1)
            rc = launch_padded<1, true, WF>(fp, blocks, st);
        else if (sh.big)
            rc = launch_padded<2, true, WF>(fp, blocks, st);
        else if (sh.kwd == 4)
            rc = launch_padded<4, false, WF>(fp, blocks, st);
        else if (sh.kwd == 2)
            rc = launch_padded<2, false, WF>(fp, blocks, st);
        else
            rc = launch_padded<1, false, WF>(fp, blocks, st);
        if (rc == LYNX_OK) rc = check_launch("lynx_moe_ffn(gate/up, down)");
    }
    return rc;
}

}  // namespace lynx

extern "C" size_t lynx_workspace_bytes(int T, int H, int F, int N, int k, int n_shared, int F_shared)
{
    // (N does not enter: the tables per expert are reserved for LYNX_MAX_N experts, inside the first 64 KiB)
    if (T < 0 || H < 0 || F < 0 || N < 0 || k < 0 || n_shared < 0 || F_shared < 0) return 0;
    if (n_shared == 0) F_shared = 0;
    return lynx::workspace_layout(T, H, F, k, n_shared, F_shared, lynx::shared_down_splits(F, n_shared, F_shared)).total;
}

extern "C" int lynx_moe_ffn_launches(int T, int F) { return lynx::single_launch(T, F) ? 1 : 2; }

extern "C" int lynx_debug_set(int what, int value)
{
    using namespace lynx;
    switch (what) {
    case LYNX_DEBUG_SPIN_LIMIT: g_tune.spin_limit.store(value < 0 ? kSpinLimit : value); return LYNX_OK;
    case LYNX_DEBUG_TARGET_BIAS: g_tune.target_bias.store(value); return LYNX_OK;
    case LYNX_DEBUG_DOWN_ITEM_CAP: g_tune.dn_cap.store(value <= 0 ? 768 : value); return LYNX_OK;
    case LYNX_DEBUG_DOWN_ITEM_UNITS: g_tune.dn_m_max.store(value <= 0 ? 1 : value); return LYNX_OK;
    case LYNX_DEBUG_DOWN_K_WAVES: g_tune.dn_kw.store(value <= 0 ? 0 : value); return LYNX_OK;
    default: return fail(LYNX_ERR_INVALID_ARG, "lynx_debug_set: unknown knob %d", what);
    }
}

#ifdef LYNX_TIMELINE
// Measurement builds only: copies the timeline of the last expert-kernel launch to a HOST array of n x 6 uint64.
extern "C" int lynx_debug_timeline(unsigned long long *host_out, int n)
{
    if (n > lynx::kTimelineSlots) n = lynx::kTimelineSlots;
    return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(lynx::g_timeline), (size_t)n * 6 * sizeof(unsigned long long)) == hipSuccess
               ? LYNX_OK
               : LYNX_ERR_HIP;
}
#endif

extern "C" int lynx_pack_weights(const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd, int E, int H, int F,
                                 uint16_t *Wgu_packed, uint16_t *Wd_packed, void *stream)
{
    using namespace lynx;
    if (E < 0 || H <= 0 || F <= 0) return fail(LYNX_ERR_INVALID_ARG, "lynx_pack_weights: bad size");
    if ((H % 32) != 0 || (F % 32) != 0)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_pack_weights: H and F must be multiples of 32 (H=%d F=%d)", H, F);
    if (E == 0) return LYNX_OK;
    if (!Wg || !Wu || !Wd || !Wgu_packed || !Wd_packed) return fail(LYNX_ERR_INVALID_ARG, "lynx_pack_weights: null pointer");
    const size_t pieces_gu = (size_t)E * F * H * 2 / 8, pieces_d = (size_t)E * F * H / 8;
    if ((pieces_gu + 255) / 256 > 0x7fffffffull) return fail(LYNX_ERR_UNSUPPORTED, "lynx_pack_weights: too large for one call");
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((pieces_gu + 255) / 256)), dim3(256), 0, (hipStream_t)stream, Wg, Wu,
                       2, E, F, H, Wgu_packed);
    int rc = check_launch("lynx_pack_weights(gate/up)");
    if (rc != LYNX_OK) return rc;
    hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((pieces_d + 255) / 256)), dim3(256), 0, (hipStream_t)stream, Wd, Wd,
                       1, E, H, F, Wd_packed);
    return check_launch("lynx_pack_weights(down)");
}

namespace lynx {

// Every check of the FFN call that needs no device: sizes, limits, pointers.  lynx_moe_layer runs it before its
// routing kernels are enqueued, so that an error leaves nothing behind.
int moe_ffn_validate(const void *x_bf16, const void *Wgu_packed, const void *Wd_packed, const void *Sgu_packed,
                     const void *Sd_packed, int n_shared, int F_shared, const void *idx, const void *gate, const void *perm,
                     const void *offsets, int T, int H, int F, int N, int k, const void *y, const void *workspace,
                     const FfnScales *q8)
{
    if (T < 0 || H <= 0 || F <= 0 || N <= 0 || k <= 0 || n_shared < 0)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_ffn: bad size");
    if (n_shared > 0 && (F_shared <= 0 || !Sgu_packed || !Sd_packed))
        return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_ffn: shared experts need F_shared > 0 and their weights");
    const int mult = q8 ? 32 << q8->format : 32;   // columns of a weight tile
    if ((H % mult) != 0 || (F % mult) != 0 || (n_shared > 0 && (F_shared % mult) != 0) || N > LYNX_MAX_N ||
        k > LYNX_MAX_K || T > LYNX_MAX_T || k > N)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_moe_ffn: need H,F,F_shared multiples of %d, k<=N<=%d, k<=%d, T<=%d", mult,
                    LYNX_MAX_N, LYNX_MAX_K, LYNX_MAX_T);
    if (q8 && (!q8->gu || !q8->d || (n_shared > 0 && (!q8->shared_gu || !q8->shared_d))))
        return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_ffn_fp8: null scale pointer");
    if (T == 0) return LYNX_OK;
    if (!x_bf16 || !Wgu_packed || !Wd_packed || !idx || !gate || !offsets || !perm || !y || !workspace)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_ffn: null pointer");
    if (n_shared == 0) F_shared = 0;
    const int tok_block = T > kTokBlock ? kTokBlockBig : kTokBlock;
    if (LYNX_MAX_N + (long)n_shared * ((T + tok_block - 1) / tok_block) > kWsDoneWords)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_moe_ffn: too many shared experts for this batch size (n_shared=%d T=%d)",
                    n_shared, T);
    const Workspace ws = workspace_layout(T, H, F, k, n_shared, F_shared, shared_down_splits(F, n_shared, F_shared));
    // (token rows are addressed with 32-bit byte offsets below 2 GiB)
    if (ws.h_elems >= 0x3fffffffull || (unsigned long long)T * H >= 0x3fffffffull || ws.o_elems >= 0x7fffffffull * 4)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_moe_ffn: scratch index would overflow 32 bits");
    return LYNX_OK;
}

// plan_ready: the caller has already had the completion counters in the workspace cleared and the work plan written
// on `stream` (the fused layer path does both in its routing kernels); otherwise a small launch does it here from
// expert_offsets.
int moe_ffn_impl(const uint16_t *x_bf16, const uint16_t *Wgu_packed, const uint16_t *Wd_packed, const uint16_t *Sgu_packed,
                 const uint16_t *Sd_packed, int n_shared, int F_shared, const int32_t *idx, const float *gate,
                 const int32_t *expert_offsets, const int32_t *perm, int T, int H, int F, int N, int k, float *y,
                 int32_t *status, void *workspace, void *stream, void *const *stage_events, bool plan_ready,
                 const FfnScales *q8)
{
    auto mark = [&](int i) -> int {
        if (!stage_events || !stage_events[i]) return LYNX_OK;
        const hipError_t err = hipEventRecord((hipEvent_t)stage_events[i], (hipStream_t)stream);
        return err == hipSuccess ? LYNX_OK : fail(LYNX_ERR_HIP, "lynx_moe_ffn_timed: hipEventRecord: %s", hipGetErrorString(err));
    };
    int rc = moe_ffn_validate(x_bf16, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, idx, gate, perm,
                              expert_offsets, T, H, F, N, k, y, workspace, q8);
    if (rc != LYNX_OK || T == 0) return rc;
    if (n_shared == 0) F_shared = 0;
    const int mult = q8 ? 32 << q8->format : 32;
    // K slices of a shared expert's down projection.  The workspace is sized for the most there can be; a slice holds
    // whole weight tiles, ceil(tiles / slices) of them, so fewer slices may already cover all tiles: an empty slice
    // would leave its output rows unwritten, and the combine adds every slice's rows.
    int splits = shared_down_splits(F, n_shared, F_shared);
    const Workspace ws = workspace_layout(T, H, F, k, n_shared, F_shared, splits);
    if (n_shared > 0) {
        const int kt = F_shared / mult;
        for (;;) {
            const int per = (kt + splits - 1) / splits;
            const int need = (kt + per - 1) / per;
            if (need == splits) break;
            splits = need;
        }
    }
    uint16_t *hbuf = reinterpret_cast<uint16_t *>(reinterpret_cast<char *>(workspace) + ws.h_off);
    float *obuf = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + ws.o_off);
    int32_t *rws = reinterpret_cast<int32_t *>(workspace);
    hipStream_t st = (hipStream_t)stream;
    const FfnShape shape = ffn_shape(T, H, F, N, k, n_shared, q8 ? q8->format : 0);
    if (!plan_ready) {
        hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(256), 0, st, expert_offsets, perm, N, T * k, shape.plan, rws);
        rc = check_launch("lynx_moe_ffn(plan)");
        if (rc != LYNX_OK) return rc;
    }

    FfnParams fp;
    fp.done = rws + kWsDone;
    fp.flags = rws + kWsFlags;
    fp.gu_blocks = 0;
    fp.spin_limit = g_tune.spin_limit.load();
    fp.target_bias = g_tune.target_bias.load();
    GemmParams p;
    p.perm = perm;
    p.plan = rws;
    p.T = T;
    p.N = N;
    p.k = k;
    p.n_shared = n_shared;
    p.shared_splits = 1;
    p.shared_h_base = (long long)T * k * h_stride(F);
    // gate/up: rows = F, contraction = H
    p.W_routed = Wgu_packed;
    p.W_shared = Sgu_packed;
    p.B = x_bf16;
    p.out = hbuf;
    p.R = F;
    p.K = H;
    p.Rs = F_shared;
    p.Ks = H;
    p.sc_routed = q8 ? q8->gu : nullptr;
    p.sc_shared = q8 ? q8->shared_gu : nullptr;
    p.ldb_r = p.ldb_s = H;
    p.ldo_r = h_stride(F);
    p.ldo_s = h_stride(F_shared);
    fp.gu = p;
    // down: rows = H, contraction = F
    p.W_routed = Wd_packed;
    p.W_shared = Sd_packed;
    p.B = hbuf;
    p.out = obuf;
    p.R = H;
    p.K = F;
    p.Rs = H;
    p.Ks = F_shared;
    p.sc_routed = q8 ? q8->d : nullptr;
    p.sc_shared = q8 ? q8->shared_d : nullptr;
    p.ldb_r = h_stride(F);
    p.ldb_s = h_stride(F_shared);
    p.ldo_r = p.ldo_s = H;
    p.shared_splits = splits;
    fp.dn = p;
    rc = mark(0);
    if (rc != LYNX_OK) return rc;
    rc = !q8 ? launch_ffn<0>(fp, shape, st) : q8->format == 2 ? launch_ffn<2>(fp, shape, st) : launch_ffn<1>(fp, shape, st);
    if (rc != LYNX_OK) return rc;
    rc = mark(1);
    if (rc != LYNX_OK) return rc;
    rc = mark(2);
    if (rc != LYNX_OK) return rc;

    hipLaunchKernelGGL(combine_kernel, dim3((H / 4 + 255) / 256, T), dim3(256), 0, st, obuf, idx, gate, T, H, N, k,
                       n_shared * splits, y, fp.flags, status);
    rc = check_launch("lynx_moe_ffn(combine)");
    if (rc != LYNX_OK) return rc;
    return mark(3);
}

}  // namespace lynx

extern "C" int lynx_moe_ffn_timed(const uint16_t *x_bf16, const uint16_t *Wgu_packed, const uint16_t *Wd_packed,
                                  const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared, int F_shared,
                                  const int32_t *idx, const float *gate, const int32_t *expert_offsets,
                                  const int32_t *perm, const int32_t *active_experts, const int32_t *num_active, int T,
                                  int H, int F, int N, int k, float *y, int32_t *status, void *workspace, void *stream,
                                  void *const *stage_events)
{
    (void)active_experts;   // the invoked experts are those with a non-empty range in expert_offsets
    (void)num_active;
    return lynx::moe_ffn_impl(x_bf16, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, idx, gate,
                              expert_offsets, perm, T, H, F, N, k, y, status, workspace, stream, stage_events, false,
                              nullptr);
}

extern "C" int lynx_moe_ffn_fp8(const uint16_t *x_bf16, const uint8_t *Wgu_q, const uint8_t *Wd_q, const float *scales_gu,
                                const float *scales_d, const uint8_t *Sgu_q, const uint8_t *Sd_q,
                                const float *shared_scales_gu, const float *shared_scales_d, int n_shared, int F_shared,
                                const int32_t *idx, const float *gate, const int32_t *expert_offsets, const int32_t *perm,
                                const int32_t *active_experts, const int32_t *num_active, int T, int H, int F, int N,
                                int k, float *y, int32_t *status, void *workspace, void *stream, void *const *stage_events)
{
    (void)active_experts;
    (void)num_active;
    const lynx::FfnScales q = {scales_gu, scales_d, shared_scales_gu, shared_scales_d, 1};
    return lynx::moe_ffn_impl(x_bf16, reinterpret_cast<const uint16_t *>(Wgu_q), reinterpret_cast<const uint16_t *>(Wd_q),
                              reinterpret_cast<const uint16_t *>(Sgu_q), reinterpret_cast<const uint16_t *>(Sd_q), n_shared,
                              F_shared, idx, gate, expert_offsets, perm, T, H, F, N, k, y, status, workspace, stream,
                              stage_events, false, &q);
}

extern "C" int lynx_quantize_weights_fp8(const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd, int E, int H, int F,
                                         uint8_t *Wgu_q, uint8_t *Wd_q, float *scales_gu, float *scales_d, void *stream)
{
    using namespace lynx;
    if (E < 0 || H <= 0 || F <= 0) return fail(LYNX_ERR_INVALID_ARG, "lynx_quantize_weights_fp8: bad size");
    if ((H % 64) != 0 || (F % 64) != 0)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_quantize_weights_fp8: H and F must be multiples of 64 (H=%d F=%d)", H, F);
    if (E == 0) return LYNX_OK;
    if (!Wg || !Wu || !Wd || !Wgu_q || !Wd_q || !scales_gu || !scales_d)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_quantize_weights_fp8: null pointer");
    const size_t rows_gu = (size_t)E * 2 * F, rows_d = (size_t)E * H;
    if ((rows_gu + 3) / 4 > 0x7fffffffull || (rows_d + 3) / 4 > 0x7fffffffull)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_quantize_weights_fp8: too large for one call");
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)((rows_gu + 3) / 4)), dim3(256), 0, (hipStream_t)stream, Wg, Wu, 2, E,
                       F, H, Wgu_q, scales_gu);
    int rc = check_launch("lynx_quantize_weights_fp8(gate/up)");
    if (rc != LYNX_OK) return rc;
    hipLaunchKernelGGL(quantize_kernel, dim3((unsigned)((rows_d + 3) / 4)), dim3(256), 0, (hipStream_t)stream, Wd, Wd, 1, E,
                       H, F, Wd_q, scales_d);
    return check_launch("lynx_quantize_weights_fp8(down)");
}

extern "C" size_t lynx_fp4_scale_words(int E, int rows, int K, int gate_up)
{
    if (E < 0 || rows <= 0 || K <= 0) return 0;
    return (size_t)E * (gate_up ? lynx::mx_scale_dwords<true>(rows, K) : lynx::mx_scale_dwords<false>(rows, K));
}

extern "C" int lynx_quantize_weights_fp4(const uint16_t *Wg, const uint16_t *Wu, const uint16_t *Wd, int E, int H, int F,
                                         uint8_t *Wgu_q, uint8_t *Wd_q, uint32_t *scales_gu, uint32_t *scales_d,
                                         void *stream)
{
    using namespace lynx;
    if (E < 0 || H <= 0 || F <= 0) return fail(LYNX_ERR_INVALID_ARG, "lynx_quantize_weights_fp4: bad size");
    if ((H % 128) != 0 || (F % 128) != 0)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_quantize_weights_fp4: H and F must be multiples of 128 (H=%d F=%d)", H, F);
    if (E == 0) return LYNX_OK;
    if (!Wg || !Wu || !Wd || !Wgu_q || !Wd_q || !scales_gu || !scales_d)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_quantize_weights_fp4: null pointer");
    const size_t rows_gu = (size_t)E * 2 * F, rows_d = (size_t)E * H;
    if ((rows_gu + 3) / 4 > 0x7fffffffull || (rows_d + 3) / 4 > 0x7fffffffull)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_quantize_weights_fp4: too large for one call");
    hipLaunchKernelGGL(quantize_fp4_kernel, dim3((unsigned)((rows_gu + 3) / 4)), dim3(256), 0, (hipStream_t)stream, Wg, Wu, 2,
                       E, F, H, Wgu_q, reinterpret_cast<uint8_t *>(scales_gu));
    int rc = check_launch("lynx_quantize_weights_fp4(gate/up)");
    if (rc != LYNX_OK) return rc;
    hipLaunchKernelGGL(quantize_fp4_kernel, dim3((unsigned)((rows_d + 3) / 4)), dim3(256), 0, (hipStream_t)stream, Wd, Wd, 1,
                       E, H, F, Wd_q, reinterpret_cast<uint8_t *>(scales_d));
    return check_launch("lynx_quantize_weights_fp4(down)");
}

extern "C" int lynx_moe_ffn_fp4(const uint16_t *x_bf16, const uint8_t *Wgu_q, const uint8_t *Wd_q, const uint32_t *scales_gu,
                                const uint32_t *scales_d, const uint8_t *Sgu_q, const uint8_t *Sd_q,
                                const uint32_t *shared_scales_gu, const uint32_t *shared_scales_d, int n_shared, int F_shared,
                                const int32_t *idx, const float *gate, const int32_t *expert_offsets, const int32_t *perm,
                                const int32_t *active_experts, const int32_t *num_active, int T, int H, int F, int N,
                                int k, float *y, int32_t *status, void *workspace, void *stream, void *const *stage_events)
{
    (void)active_experts;
    (void)num_active;
    const lynx::FfnScales q = {reinterpret_cast<const float *>(scales_gu), reinterpret_cast<const float *>(scales_d),
                               reinterpret_cast<const float *>(shared_scales_gu),
                               reinterpret_cast<const float *>(shared_scales_d), 2};
    return lynx::moe_ffn_impl(x_bf16, reinterpret_cast<const uint16_t *>(Wgu_q), reinterpret_cast<const uint16_t *>(Wd_q),
                              reinterpret_cast<const uint16_t *>(Sgu_q), reinterpret_cast<const uint16_t *>(Sd_q), n_shared,
                              F_shared, idx, gate, expert_offsets, perm, T, H, F, N, k, y, status, workspace, stream,
                              stage_events, false, &q);
}

extern "C" int lynx_moe_ffn(const uint16_t *x_bf16, const uint16_t *Wgu_packed, const uint16_t *Wd_packed,
                            const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared, int F_shared,
                            const int32_t *idx, const float *gate, const int32_t *expert_offsets, const int32_t *perm,
                            const int32_t *active_experts, const int32_t *num_active, int T, int H, int F, int N, int k,
                            float *y, int32_t *status, void *workspace, void *stream)
{
    return lynx_moe_ffn_timed(x_bf16, Wgu_packed, Wd_packed, Sgu_packed, Sd_packed, n_shared, F_shared, idx, gate,
                              expert_offsets, perm, active_experts, num_active, T, H, F, N, k, y, status, workspace, stream,
                              nullptr);
}
