// lynx_moe_ffn: grouped SwiGLU expert FFN over the invoked experts + gate-weighted combine, and the
// one-time weight re-layout it streams from.
//
// Decode is bound by streaming expert weights from HBM (paper Sec. 2.1: latency grows with the number
// of experts the batch activates), so the kernels are organised around the weight stream:
//   * weights are pre-packed so that a wave reads a 16-row x 32-column bf16 tile as one contiguous
//     1 KiB load (16 bytes per lane) that IS the A operand of v_mfma_f32_16x16x32_bf16;
//   * a wave owns 16 output rows and walks the whole contraction dimension, keeping a ring of
//     prefetched tiles in registers, so each weight byte is fetched from HBM once per call;
//   * the (few) tokens of the expert are the B operand: staged through LDS in K-chunks, double
//     buffered, shared by the four waves of the workgroup;
//   * a workgroup = (invoked expert, 64 output rows).  The grid is fixed (N experts + shared experts);
//     workgroups whose rank is past the device-side num_active leave at once, so nothing is read
//     back to the host.
// Two launches (gate/up with the SiLU-multiply epilogue, then down) and a small combine.
#include "lynx_common.h"

namespace lynx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kFfnThreads = 256;
constexpr int kFfnWaves = kFfnThreads / kWave;
constexpr int kRowsPerWG = 16 * kFfnWaves;   // output rows per workgroup
constexpr int kNTMax = 8;                    // token tiles (of 16) held in accumulators at once
constexpr int kTokBlock = 16 * kNTMax;
constexpr int kPF = 8;                       // weight tiles in flight per wave and matrix
constexpr int kStageBytes = 2 * 18432;       // two LDS buffers for the token tile

struct GemmParams {
    const uint16_t *W_routed;   // packed routed weights (gate/up interleaved, or down)
    const uint16_t *W_shared;   // packed shared-expert weights or NULL
    const uint16_t *B;          // gate/up: x [T,H]; down: h scratch
    void *out;                  // gate/up: h scratch (bf16); down: o scratch (fp32)
    const int32_t *offsets, *perm, *active, *num_active;
    int T, N, k, n_shared;
    int R, K;                   // routed: output rows, contraction length
    int Rs, Ks;                 // shared
    int tiles_r, tiles_s;       // workgroups per routed / shared expert
    int routed_blocks;
    long long shared_h_base;    // element offset of the shared experts' h rows in the h scratch
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float silu_mul(float g, float u) { return (g / (1.0f + __expf(-g))) * u; }

// One pass over the contraction dimension for NT token tiles.  KS = k-steps (of 32 columns) per LDS
// chunk.  Wt points at this wave's row tile (uint4 units), or the wave is idle (rows past R).
template <bool DUAL, int NT, int KS>
__device__ __forceinline__ void stream_rows(const uint4 *__restrict__ Wt, bool wave_active, int KT, int K,
                                            const uint16_t *__restrict__ B, const int *rowoff, char *stage,
                                            f32x4 (&accg)[NT], f32x4 (&accu)[NT])
{
    constexpr int ROWB = KS * 64 + 16;           // LDS bytes per token row (+16: conflict-free 16-byte reads)
    constexpr int BUFB = NT * 16 * ROWB;
    static_assert(2 * BUFB <= kStageBytes, "token tile does not fit the LDS stage");
    constexpr int PIECES = NT * 16 * KS * 4;     // 16-byte pieces per chunk
    constexpr int PPT = (PIECES + kFfnThreads - 1) / kFfnThreads;
    constexpr int U = KS > kPF ? KS : kPF;
    constexpr int WSTEP = DUAL ? 2 * kWave : kWave;   // uint4 per k-step

    const int tid = threadIdx.x, lane = lane_id();
    const int nchunks = (KT + KS - 1) / KS;
    uint4 xr[PPT];

    auto load_x = [&](int c) {
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int q = tid + kFfnThreads * i;
            uint4 val = make_uint4(0u, 0u, 0u, 0u);
            if (q < PIECES) {
                const int row = q / (KS * 4), pc = q % (KS * 4);
                const int col = c * KS * 32 + pc * 8;
                const int ro = rowoff[row];
                if (ro >= 0 && col < K) val = *reinterpret_cast<const uint4 *>(B + (size_t)ro + col);
            }
            xr[i] = val;
        }
    };
    auto store_x = [&](int c) {
        char *buf = stage + (c & 1) * BUFB;
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const int q = tid + kFfnThreads * i;
            if (q < PIECES) {
                const int row = q / (KS * 4), pc = q % (KS * 4);
                *reinterpret_cast<uint4 *>(buf + row * ROWB + pc * 16) = xr[i];
            }
        }
    };

    uint4 wg[kPF], wu[kPF];
#pragma unroll
    for (int j = 0; j < kPF; ++j) {
        wg[j] = make_uint4(0u, 0u, 0u, 0u);
        wu[j] = make_uint4(0u, 0u, 0u, 0u);
        if (wave_active && j < KT) {
            wg[j] = Wt[(size_t)j * WSTEP + lane];
            if (DUAL) wu[j] = Wt[(size_t)j * WSTEP + kWave + lane];
        }
    }
    load_x(0);
    store_x(0);
    __syncthreads();

    const int brow = (lane & 15) * ROWB + (lane >> 4) * 16;   // this lane's B-fragment offset inside a token tile
    for (int s0 = 0; s0 < KT; s0 += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = s0 + u;
            if (s < KT) {
                const int c = s / KS;
                if (u % KS == 0 && c + 1 < nchunks) load_x(c + 1);
                if (wave_active) {
                    const bf16x8 ag = __builtin_bit_cast(bf16x8, wg[u % kPF]);
                    const bf16x8 au = __builtin_bit_cast(bf16x8, wu[u % kPF]);
                    if (s + kPF < KT) {
                        wg[u % kPF] = Wt[(size_t)(s + kPF) * WSTEP + lane];
                        if (DUAL) wu[u % kPF] = Wt[(size_t)(s + kPF) * WSTEP + kWave + lane];
                    }
                    const char *buf = stage + (c & 1) * BUFB + brow + (u % KS) * 64;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const bf16x8 b = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(buf + nt * 16 * ROWB));
                        accg[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ag, b, accg[nt], 0, 0, 0);
                        if (DUAL) accu[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(au, b, accu[nt], 0, 0, 0);
                    }
                }
                if (u % KS == KS - 1 || s == KT - 1) {
                    if (c + 1 < nchunks) store_x(c + 1);
                    __syncthreads();
                }
            }
        }
    }
}

// Handles one block of up to 16*NT tokens of the workgroup's expert: stream, then epilogue.
template <bool DUAL, int NT, int KS>
__device__ __forceinline__ void expert_block(const uint4 *Wt, bool wave_active, int R, int K, const uint16_t *B,
                                             void *out, int row0, const int *rowoff, const int *outrow, char *stage)
{
    f32x4 accg[NT], accu[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        accg[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        accu[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    stream_rows<DUAL, NT, KS>(Wt, wave_active, K / 32, K, B, rowoff, stage, accg, accu);
    if (!wave_active) return;
    // D fragment: lane holds token column (lane & 15), output rows 4*(lane >> 4) .. +3 of the wave's 16
    const int lane = lane_id();
    const int r = row0 + 4 * (lane >> 4);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int orow = outrow[nt * 16 + (lane & 15)];
        if (orow < 0) continue;
        if (DUAL) {
            uint2 pk;
            pk.x = (uint32_t)f32_to_bf16_rne(silu_mul(accg[nt][0], accu[nt][0])) |
                   ((uint32_t)f32_to_bf16_rne(silu_mul(accg[nt][1], accu[nt][1])) << 16);
            pk.y = (uint32_t)f32_to_bf16_rne(silu_mul(accg[nt][2], accu[nt][2])) |
                   ((uint32_t)f32_to_bf16_rne(silu_mul(accg[nt][3], accu[nt][3])) << 16);
            *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(out) + (size_t)orow * R + r) = pk;
        } else {
            *reinterpret_cast<float4 *>(reinterpret_cast<float *>(out) + (size_t)orow * R + r) =
                make_float4(accg[nt][0], accg[nt][1], accg[nt][2], accg[nt][3]);
        }
    }
}

template <bool DUAL>
__global__ __launch_bounds__(kFfnThreads, 2) void expert_gemm_kernel(GemmParams p)
{
    __shared__ __attribute__((aligned(16))) char stage[kStageBytes];
    __shared__ int rowoff[kTokBlock];   // element offset of each token's B row, -1 = padding (zeros)
    __shared__ int outrow[kTokBlock];   // output row of each token, -1 = none

    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int P = p.T * p.k;
    int R, K, tile, Te, off = 0, shared_s = -1;
    const uint16_t *Wexp;
    if (b < p.routed_blocks) {
        const int rank = b / p.tiles_r;
        tile = b % p.tiles_r;
        const int na = min(*p.num_active, p.N);
        if (rank >= na) return;
        const int e = p.active[rank];
        if (e < 0 || e >= p.N) return;
        off = p.offsets[e];
        Te = p.offsets[e + 1] - off;
        if (off < 0 || Te <= 0 || off + Te > P) return;
        R = p.R;
        K = p.K;
        Wexp = p.W_routed + (size_t)e * ((size_t)R * K * (DUAL ? 2 : 1));
    } else {
        const int bs = b - p.routed_blocks;
        shared_s = bs / p.tiles_s;
        tile = bs % p.tiles_s;
        if (shared_s >= p.n_shared || p.T <= 0) return;
        Te = p.T;
        R = p.Rs;
        K = p.Ks;
        Wexp = p.W_shared + (size_t)shared_s * ((size_t)R * K * (DUAL ? 2 : 1));
    }
    const int KT = K / 32;
    const int rt = tile * kFfnWaves + wave_id();   // 16-row tile of this wave
    const bool wave_active = rt * 16 < R;
    const uint4 *Wt = reinterpret_cast<const uint4 *>(Wexp) + (size_t)rt * KT * (DUAL ? 2 * kWave : kWave);
    const int row0 = rt * 16;

    for (int i0 = 0; i0 < Te; i0 += kTokBlock) {
        const int nb = min(Te - i0, kTokBlock);
        __syncthreads();   // previous block's epilogue has read outrow
        if (tid < kTokBlock) {
            int ro = -1, orow = -1;
            const int i = i0 + tid;
            if (tid < nb) {
                if (shared_s < 0) {
                    const int pv = p.perm[off + i];
                    if (pv >= 0 && pv < P) {
                        if (DUAL) {   // B row = x[token], out row = sorted position in h
                            ro = (pv / p.k) * K;
                            orow = off + i;
                        } else {      // B row = h[sorted position], out row = pair id in o
                            ro = (off + i) * K;
                            orow = pv;
                        }
                    }
                } else if (DUAL) {    // shared: every token, h rows after the routed ones
                    ro = i * K;
                    orow = i;
                } else {
                    ro = i * K;
                    orow = P + shared_s * p.T + i;
                }
            }
            rowoff[tid] = ro;
            outrow[tid] = orow;
        }
        __syncthreads();
        // shared experts keep their h rows in their own region of the scratch
        const uint16_t *B = p.B;
        void *out = p.out;
        if (shared_s >= 0) {
            const size_t hbase = (size_t)p.shared_h_base + (size_t)shared_s * p.T * (DUAL ? R : K);
            if (DUAL)
                out = reinterpret_cast<uint16_t *>(p.out) + hbase;
            else
                B = p.B + hbase;
        }
        if (nb <= 16)
            expert_block<DUAL, 1, 16>(Wt, wave_active, R, K, B, out, row0, rowoff, outrow, stage);
        else if (nb <= 32)
            expert_block<DUAL, 2, 8>(Wt, wave_active, R, K, B, out, row0, rowoff, outrow, stage);
        else if (nb <= 64)
            expert_block<DUAL, 4, 4>(Wt, wave_active, R, K, B, out, row0, rowoff, outrow, stage);
        else
            expert_block<DUAL, 8, 2>(Wt, wave_active, R, K, B, out, row0, rowoff, outrow, stage);
    }
}

// y[t] = sum_j gate[t,j] * o[t*k+j] + sum_s o[P + s*T + t]
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ o, const int32_t *__restrict__ idx,
                                                      const float *__restrict__ gate, int T, int H, int N, int k,
                                                      int n_shared, float *__restrict__ y)
{
    const int t = blockIdx.y;
    const int h = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (h >= H) return;
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

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Workspace {
    size_t h_elems, o_elems, h_off, o_off, total;
};

static Workspace workspace_layout(int T, int H, int F, int N, int k, int n_shared, int F_shared)
{
    (void)N;
    Workspace w;
    w.h_elems = (size_t)T * k * F + (size_t)n_shared * T * F_shared;
    w.o_elems = ((size_t)T * k + (size_t)n_shared * T) * H;
    w.h_off = 0;
    w.o_off = align256(w.h_elems * 2);
    w.total = w.o_off + align256(w.o_elems * 4) + 65536;
    return w;
}

}  // namespace lynx

extern "C" size_t lynx_workspace_bytes(int T, int H, int F, int N, int k, int n_shared, int F_shared)
{
    if (T < 0 || H < 0 || F < 0 || N < 0 || k < 0 || n_shared < 0 || F_shared < 0) return 0;
    return lynx::workspace_layout(T, H, F, N, k, n_shared, F_shared).total;
}

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

extern "C" int lynx_moe_ffn(const uint16_t *x_bf16, const uint16_t *Wgu_packed, const uint16_t *Wd_packed,
                            const uint16_t *Sgu_packed, const uint16_t *Sd_packed, int n_shared, int F_shared,
                            const int32_t *idx, const float *gate, const int32_t *expert_offsets, const int32_t *perm,
                            const int32_t *active_experts, const int32_t *num_active, int T, int H, int F, int N, int k,
                            float *y, void *workspace, void *stream)
{
    using namespace lynx;
    if (T < 0 || H <= 0 || F <= 0 || N <= 0 || k <= 0 || n_shared < 0)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_ffn: bad size");
    if (n_shared > 0 && (F_shared <= 0 || !Sgu_packed || !Sd_packed))
        return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_ffn: shared experts need F_shared > 0 and their weights");
    if ((H % 32) != 0 || (F % 32) != 0 || (n_shared > 0 && (F_shared % 32) != 0) || N > LYNX_MAX_N || k > LYNX_MAX_K ||
        T > LYNX_MAX_T || k > N)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_moe_ffn: need H,F,F_shared multiples of 32, k<=N<=%d, k<=%d, T<=%d",
                    LYNX_MAX_N, LYNX_MAX_K, LYNX_MAX_T);
    if (T == 0) return LYNX_OK;
    if (!x_bf16 || !Wgu_packed || !Wd_packed || !idx || !gate || !expert_offsets || !perm || !active_experts ||
        !num_active || !y || !workspace)
        return fail(LYNX_ERR_INVALID_ARG, "lynx_moe_ffn: null pointer");
    if (n_shared == 0) F_shared = 0;
    const Workspace ws = workspace_layout(T, H, F, N, k, n_shared, F_shared);
    if (ws.h_elems >= 0x7fffffffull || ws.o_elems >= 0x7fffffffull * 4)
        return fail(LYNX_ERR_UNSUPPORTED, "lynx_moe_ffn: scratch index would overflow 32 bits");
    uint16_t *hbuf = reinterpret_cast<uint16_t *>(reinterpret_cast<char *>(workspace) + ws.h_off);
    float *obuf = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + ws.o_off);
    hipStream_t st = (hipStream_t)stream;

    GemmParams p;
    p.offsets = expert_offsets;
    p.perm = perm;
    p.active = active_experts;
    p.num_active = num_active;
    p.T = T;
    p.N = N;
    p.k = k;
    p.n_shared = n_shared;
    p.shared_h_base = (long long)T * k * F;

    // gate/up: rows = F, contraction = H
    p.W_routed = Wgu_packed;
    p.W_shared = Sgu_packed;
    p.B = x_bf16;
    p.out = hbuf;
    p.R = F;
    p.K = H;
    p.Rs = F_shared;
    p.Ks = H;
    p.tiles_r = (F + kRowsPerWG - 1) / kRowsPerWG;
    p.tiles_s = n_shared ? (F_shared + kRowsPerWG - 1) / kRowsPerWG : 0;
    p.routed_blocks = N * p.tiles_r;
    hipLaunchKernelGGL(expert_gemm_kernel<true>, dim3(p.routed_blocks + n_shared * p.tiles_s), dim3(kFfnThreads), 0, st, p);
    int rc = check_launch("lynx_moe_ffn(gate/up)");
    if (rc != LYNX_OK) return rc;

    // down: rows = H, contraction = F
    p.W_routed = Wd_packed;
    p.W_shared = Sd_packed;
    p.B = hbuf;
    p.out = obuf;
    p.R = H;
    p.K = F;
    p.Rs = H;
    p.Ks = F_shared;
    p.tiles_r = (H + kRowsPerWG - 1) / kRowsPerWG;
    p.tiles_s = n_shared ? p.tiles_r : 0;
    p.routed_blocks = N * p.tiles_r;
    hipLaunchKernelGGL(expert_gemm_kernel<false>, dim3(p.routed_blocks + n_shared * p.tiles_s), dim3(kFfnThreads), 0, st, p);
    rc = check_launch("lynx_moe_ffn(down)");
    if (rc != LYNX_OK) return rc;

    hipLaunchKernelGGL(combine_kernel, dim3((H / 4 + 255) / 256, T), dim3(256), 0, st, obuf, idx, gate, T, H, N, k,
                       n_shared, y);
    return check_launch("lynx_moe_ffn(combine)");
}
