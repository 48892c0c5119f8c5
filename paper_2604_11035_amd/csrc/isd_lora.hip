// Segment-gated LoRA projection of the lossless variant (App. G "Per-position computation"):
//     h_j = W x_j + 1[j is a MASK position] * B (A x_j)
// as two launches of one bf16 MFMA kernel (v_mfma_f32_16x16x32_bf16, fp32 accumulation):
//   1. shrink:  u_j = A x_j for the token tiles that hold a MASK row, rows of clean tokens zeroed;
//   2. project: h = [x | u] [W | B]^T, i.e. the reduction over d_in continues over the r columns
//      of u with B as the weight; token tiles without a MASK row stop after d_in.
// A clean token's row of u is exactly zero, so its accumulators after the second segment hold the
// bits they held after the first: its output is that of the base layer alone.
//
// Both operands of the contraction are K-contiguous ("NT" product).  A workgroup owns a
// BM x BN tile of the output and walks K in steps of 64.  Per step its wavefronts copy the two
// operand tiles from global memory straight into LDS (global_load_lds_dwordx4: no staging
// registers, no LDS store instructions); one such load moves 8 rows x 128 bytes, i.e. whole cache
// lines (rows of 64 bytes per load measured half the fetch rate, and the fetch rate is what bounds
// this kernel).  Lane i of a load deposits its 16 bytes at entry i of a 1 KB unit, so the layout in
// LDS is chosen through the address each lane fetches: lane (r, s) of unit u fetches row r ^ (u & 1),
// 16-byte chunk s ^ row.  With that XOR pattern an MFMA operand read (16 rows, one chunk per lane
// group) spreads over all banks and runs at the LDS's full rate (measured: 8 clocks per wavefront
// read of 1 KB; the same rows without the XOR take twice as long).
// The stages form a ring: the loads of the next NSTAGE-1 steps are in flight while a step is
// multiplied, one barrier per step, and a wavefront only ever waits for the oldest stage
// (s_waitcnt vmcnt(n) with the younger loads still outstanding).  The weight fragment is the A
// operand and the token fragment the B operand of the MFMA, so a lane ends up with four consecutive
// output features of one token; the tile is rounded to bf16, transposed through LDS and written
// with full 16-byte row segments.
#include "idlm_common.h"

namespace idlm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kBK = 64;          // K elements per pipeline step (128 bytes of a row: one cache line)
constexpr int kGroupM = 4;       // token-tile rows that share a band of weight tiles in the launch order

struct LoraGemmParams {
    const uint16_t* x;     // [T, K0]  tokens (first K segment)
    const uint16_t* w;     // [N, K0]  weights of the first segment
    const uint16_t* x2;    // [T, K1]  second segment of the token operand (u), or unused when K1 = 0
    const uint16_t* w2;    // [N, K1]
    uint16_t* out;         // [T, N]
    const uint8_t* gate;   // [T] or NULL: then the gate of token t is (t % S) > n_draft[t / S]
    const int32_t* n_draft;
    int S;
    int T, N, K0, K1;
    int tiles_m, tiles_n;
    int splits;            // > 1: the K range is cut into this many parts, one workgroup each, which write
    float* partial;        //      fp32 tiles to partial[split][T][N] for the reduction kernel
};

__device__ __forceinline__ bool token_gated(const LoraGemmParams& p, int t)
{
    if (p.gate) return p.gate[t] != 0;
    const int b = t / p.S;
    const int nd = max(0, min(p.n_draft[b], p.S - 1));
    return (t - b * p.S) > nd;
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 v;
    v.x = (__bf16)lo;
    v.y = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// 16 bytes per lane from global memory to LDS entry (base + lane); base is wavefront-uniform.
__device__ __forceinline__ void load_to_lds(const uint16_t* src, u32x4* lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
}

// Waits until at most N of this wavefront's vector-memory operations are outstanding (they retire
// in order), leaving the other counters alone.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// WT x WF wavefronts; a wavefront multiplies FT token fragments by FF weight fragments; NSTAGE
// stages of LDS, each one step (64 columns of K) of both operand tiles.
// SHRINK: the launch that produces u (rows of clean tokens are written as zeros, token tiles
// without a MASK row are not multiplied at all); otherwise the projection, whose second K segment
// is skipped for token tiles without a MASK row.
template <int WT, int WF, int FT, int FF, int NSTAGE, bool SHRINK>
__global__ __launch_bounds__(WT * WF * 64) void isd_gated_lora_gemm_kernel(const LoraGemmParams p)
{
    constexpr int NW = WT * WF;
    constexpr int NTH = NW * 64;
    constexpr int BM = WT * FT * 16;        // tokens per tile
    constexpr int BN = WF * FF * 16;        // output features per tile
    constexpr int BKS = kBK;                // K elements per step
    constexpr int UX = BM / 8;              // 1 KB units (8 rows x 128 bytes) of the token tile per step
    constexpr int UW = BN / 8;
    static_assert(UX % NW == 0 && UW % NW == 0 && NW % 2 == 0, "units must divide among the wavefronts");
    constexpr int LX = UX / NW, LW = UW / NW;
    constexpr int L = LX + LW;              // loads of a wavefront per step
    constexpr int STAGE = (UX + UW) * 64;   // 16-byte entries per stage
    constexpr int OUT_LD = BN + 8;          // padded row of the bf16 output tile in LDS (elements)
    static_assert(NSTAGE >= 2 && (NSTAGE - 1) * L < 64, "loads in flight must fit the counter");

    extern __shared__ u32x4 lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = wave_id();
    const int wt = wv / WF, wf = wv - wt * WF;

    // launch order -> tile: the workgroups that one XCD receives (every 8th) cover a compact
    // rectangle of the tile grid, kGroupM token tiles high, so that its L2 holds few operand tiles
    int tm, tn;
    {
        const int nb = p.tiles_m * p.tiles_n;
        const int bid = blockIdx.x % nb;
        const int xcd = bid & 7, local = bid >> 3;
        const int per = nb >> 3, rem = nb & 7;
        const int Lin = xcd * per + min(xcd, rem) + local;
        const int band = kGroupM * p.tiles_n;
        const int g = Lin / band;
        const int first = g * kGroupM;
        const int rows = min(kGroupM, p.tiles_m - first);
        const int within = Lin - g * band;
        tn = within / rows;
        tm = first + (within - tn * rows);
    }
    const int row0 = tm * BM, n0 = tn * BN;
    const int split = blockIdx.x / (p.tiles_m * p.tiles_n);

    // does this token tile hold a MASK row?  (a projection without an adapter never asks)
    int any = 0;
    if (SHRINK || p.K1 > 0) {
        for (int i = tid; i < BM; i += NTH)
            if (row0 + i < p.T) any |= token_gated(p, row0 + i) ? 1 : 0;
        any = __syncthreads_or(any);
    }

    if (SHRINK && !any) {   // u of a tile of clean tokens: zeros (with splits the reduction writes them)
        if (p.splits == 1)
            for (int c = tid; c < BM * (BN / 8); c += NTH) {
                const int r = c / (BN / 8), c8 = c - r * (BN / 8);
                if (row0 + r < p.T && n0 + c8 * 8 < p.N)
                    *reinterpret_cast<u32x4*>(p.out + (size_t)(row0 + r) * p.N + n0 + c8 * 8) = u32x4{0u, 0u, 0u, 0u};
            }
        return;
    }

    // this workgroup's steps: its share of the first K segment and, for the last split only, the
    // second segment (so that the terms of the first segment are summed in the same order whether
    // or not a second segment exists)
    const int steps0 = p.K0 / BKS;
    const int k_begin = (int)((int64_t)steps0 * split / p.splits);
    const int nk0 = (int)((int64_t)steps0 * (split + 1) / p.splits) - k_begin;
    const int nk = nk0 + ((!SHRINK && any && split == p.splits - 1) ? p.K1 / BKS : 0);

    // this lane's source: unit u = wv + NW*i of a step covers rows 8u .. 8u+7; the lane fetches row
    // (lane / 8) ^ (u & 1) of them (u & 1 = wv & 1 for all its units) and chunk (lane % 8) ^ row
    const int srow = (lane >> 3) ^ (wv & 1);
    const int schunk = (lane & 7) ^ srow;
    const uint16_t* px[LX];
    const uint16_t* pw[LW];
    auto set_segment = [&](const uint16_t* xb, const uint16_t* wb, int ld, int first_step) {
#pragma unroll
        for (int i = 0; i < LX; ++i) {
            const int row = min(row0 + (wv + NW * i) * 8 + srow, p.T - 1);
            px[i] = xb + (size_t)row * ld + first_step * BKS + schunk * 8;
        }
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const int row = min(n0 + (wv + NW * i) * 8 + srow, p.N - 1);
            pw[i] = wb + (size_t)row * ld + first_step * BKS + schunk * 8;
        }
    };
    set_segment(p.x, p.w, p.K0, k_begin);

    auto issue = [&](int ki) {   // the loads of step ki, into stage ki % NSTAGE
        if (ki == nk0) set_segment(p.x2, p.w2, p.K1, 0);
        u32x4* st = lds + (ki % NSTAGE) * STAGE;
#pragma unroll
        for (int i = 0; i < LX; ++i) { load_to_lds(px[i], st + (wv + NW * i) * 64); px[i] += BKS; }
#pragma unroll
        for (int i = 0; i < LW; ++i) { load_to_lds(pw[i], st + (UX + wv + NW * i) * 64); pw[i] += BKS; }
    };

    // operand reads: lane (rr, cc) of a 16-row fragment needs row rr, chunk 4*kk + cc of the step:
    // unit rr / 8 of the fragment's two, entry ((rr % 8) ^ (unit & 1)) * 8 + (chunk ^ (rr % 8))
    const int rr = lane & 15, cc = lane >> 4;
    int frag_off[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
        frag_off[kk] = (rr >> 3) * 64 + (((rr & 7) ^ (rr >> 3)) << 3) + ((kk * 4 + cc) ^ (rr & 7));

    f32x4 acc[FF][FT];
#pragma unroll
    for (int j = 0; j < FF; ++j)
#pragma unroll
        for (int i = 0; i < FT; ++i) acc[j][i] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int s = 0; s < NSTAGE - 1; ++s)
        if (s < nk) issue(s);

    for (int kt = 0; kt < nk; ++kt) {
        // step kt has landed once only the loads of the NSTAGE-2 younger steps are outstanding;
        // near the end fewer steps are in flight and the wait is for everything
        if (kt + NSTAGE - 2 < nk) wait_vmcnt<(NSTAGE - 2) * L>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();   // every wavefront's part of step kt is in LDS; step kt-1 is no longer read
        if (kt + NSTAGE - 1 < nk) issue(kt + NSTAGE - 1);
        const u32x4* sxp = lds + (kt % NSTAGE) * STAGE;
        const u32x4* swp = sxp + UX * 64;
        // The step is multiplied in groups of (32 columns) x (all token fragments) x (FH weight
        // fragments).  The operands of group g+1 are requested from LDS before the multiplications
        // of group g are issued, into a second set of registers, so that the matrix pipeline does not
        // wait for LDS except at the first group after the barrier.
        constexpr int NH = (FF >= 8) ? 2 : 1;   // weight fragments are read in halves when there are many
        constexpr int FH = FF / NH;
        constexpr int NG = 2 * NH;
        bf16x8 fx[2][FT], fw[2][FH];
        auto read_x = [&](int kk, bf16x8 (&f)[FT]) {
#pragma unroll
            for (int i = 0; i < FT; ++i) f[i] = __builtin_bit_cast(bf16x8, sxp[(wt * FT + i) * 128 + frag_off[kk]]);
        };
        auto read_w = [&](int kk, int h, bf16x8 (&f)[FH]) {
#pragma unroll
            for (int j = 0; j < FH; ++j)
                f[j] = __builtin_bit_cast(bf16x8, swp[(wf * FF + h * FH + j) * 128 + frag_off[kk]]);
        };
        read_w(0, 0, fw[0]);
        read_x(0, fx[0]);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int kk = g / NH, h = g % NH;
            if (g + 1 < NG) {
                const int kk1 = (g + 1) / NH, h1 = (g + 1) % NH;
                read_w(kk1, h1, fw[(g + 1) & 1]);
                if (h1 == 0) read_x(kk1, fx[kk1 & 1]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < FT; ++i)
#pragma unroll
                for (int j = 0; j < FH; ++j)
                    acc[h * FH + j][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[g & 1][j], fx[kk & 1][i],
                                                                                 acc[h * FH + j][i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (p.splits > 1) {   // fp32 partial tile, four consecutive features per lane
        float* part = p.partial + (size_t)split * p.T * p.N;
#pragma unroll
        for (int j = 0; j < FF; ++j)
#pragma unroll
            for (int i = 0; i < FT; ++i) {
                const int tok = row0 + (wt * FT + i) * 16 + (lane & 15);
                const int feat = n0 + (wf * FF + j) * 16 + (lane >> 4) * 4;
                if (tok < p.T && feat < p.N) *reinterpret_cast<f32x4*>(part + (size_t)tok * p.N + feat) = acc[j][i];
            }
        return;
    }
    __syncthreads();   // the stages are free: they become the output tile

    // accumulators -> bf16 tile [BM][OUT_LD] in LDS: lane = token (lane % 16) of fragment i,
    // features 4*(lane / 16) .. +3 of fragment j
    uint16_t* ot = reinterpret_cast<uint16_t*>(lds);
#pragma unroll
    for (int j = 0; j < FF; ++j)
#pragma unroll
        for (int i = 0; i < FT; ++i) {
            const int tok = (wt * FT + i) * 16 + rr;
            const int feat = (wf * FF + j) * 16 + cc * 4;
            u32x2 v;
            v.x = pack_bf16(acc[j][i].x, acc[j][i].y);
            v.y = pack_bf16(acc[j][i].z, acc[j][i].w);
            *reinterpret_cast<u32x2*>(ot + tok * OUT_LD + feat) = v;
        }
    __syncthreads();
    for (int c = tid; c < BM * (BN / 8); c += NTH) {
        const int r = c / (BN / 8), c8 = c - r * (BN / 8);
        if (row0 + r < p.T && n0 + c8 * 8 < p.N) {
            u32x4 v = *reinterpret_cast<const u32x4*>(ot + r * OUT_LD + c8 * 8);
            if (SHRINK && !token_gated(p, row0 + r)) v = u32x4{0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4*>(p.out + (size_t)(row0 + r) * p.N + n0 + c8 * 8) = v;
        }
    }
}

// Sums the fp32 partial tiles of the K splits in split order, rounds to bf16, 8 features per thread.
// apply_gate: rows of clean tokens become zeros (u), whatever the partial buffers hold for them.
__global__ __launch_bounds__(256) void isd_lora_splitk_reduce_kernel(const LoraGemmParams p, int apply_gate)
{
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int per_row = p.N / 8;
    if (c >= (int64_t)p.T * per_row) return;
    const int t = (int)(c / per_row), c8 = (int)(c - (int64_t)t * per_row);
    u32x4 v = {0u, 0u, 0u, 0u};
    if (!apply_gate || token_gated(p, t)) {
        const float* src = p.partial + (size_t)t * p.N + c8 * 8;
        f32x4 a = *reinterpret_cast<const f32x4*>(src), b = *reinterpret_cast<const f32x4*>(src + 4);
        for (int z = 1; z < p.splits; ++z) {
            src += (size_t)p.T * p.N;
            a += *reinterpret_cast<const f32x4*>(src);
            b += *reinterpret_cast<const f32x4*>(src + 4);
        }
        v.x = pack_bf16(a.x, a.y); v.y = pack_bf16(a.z, a.w);
        v.z = pack_bf16(b.x, b.y); v.w = pack_bf16(b.z, b.w);
    }
    *reinterpret_cast<u32x4*>(p.out + (size_t)t * p.N + c8 * 8) = v;
}

template <int WT, int WF, int FT, int FF, int NSTAGE>
constexpr size_t gemm_lds_bytes()
{
    constexpr size_t BM = WT * FT * 16, BN = WF * FF * 16;
    constexpr size_t stages = (size_t)NSTAGE * (BM + BN) * 128;
    constexpr size_t tile = BM * (BN + 8) * 2;
    return stages > tile ? stages : tile;
}

template <int WT, int WF, int FT, int FF, int NSTAGE, bool SHRINK>
static int launch_gemm(LoraGemmParams p, hipStream_t st)
{
    constexpr int BM = WT * FT * 16, BN = WF * FF * 16;
    constexpr size_t lds_bytes = gemm_lds_bytes<WT, WF, FT, FF, NSTAGE>();
    static_assert(lds_bytes <= 160 * 1024, "LDS of a compute unit");
    p.tiles_m = (p.T + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    const int64_t blocks = (int64_t)p.tiles_m * p.tiles_n * p.splits;
    if (blocks >= INT32_MAX) return IDLM_ERR_SHAPE;
    auto kern = isd_gated_lora_gemm_kernel<WT, WF, FT, FF, NSTAGE, SHRINK>;
    if (lds_bytes > 64 * 1024 &&   // beyond the default limit
        hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_bytes) != hipSuccess)
        return IDLM_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(WT * WF * 64), lds_bytes, st, p);
    if (p.splits > 1) {
        const int64_t chunks = (int64_t)p.T * (p.N / 8);
        hipLaunchKernelGGL(isd_lora_splitk_reduce_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, st, p,
                           SHRINK ? 1 : 0);
    }
    return IDLM_OK;
}

}  // namespace idlm

using namespace idlm;

static bool lora_shape_ok(int32_t T, int32_t d_in, int32_t d_out, int32_t r)
{
    return T >= 0 && d_in >= kBK && d_in % kBK == 0 && d_out >= 8 && d_out % 8 == 0 && r >= 0 && r % kBK == 0 &&
           r <= 4096 && (int64_t)T * d_in < ((int64_t)1 << 40) && (int64_t)T * d_out < ((int64_t)1 << 40);
}

namespace {

// Launch shapes, a function of the sizes alone (the workspace size follows from them): token tile
// of the projection, K splits of the projection and of the shrink.  256 = compute units of the part.
struct LoraPlan {
    int bm, splits, shrink_splits;
    size_t u_off, part_off, total;
};

constexpr int kUnits = 256;

int pick_splits(int64_t tiles, int steps, int max_splits)
{
    // enough workgroups for every compute unit, at least four steps each
    int z = (int)((kUnits + tiles - 1) / tiles);
    if (z > max_splits) z = max_splits;
    if (z > steps / 4) z = steps / 4;
    return z < 1 ? 1 : z;
}

// Estimated time of the projection for a token tile and a number of reduction parts, in microseconds
// as measured on an MI355X (only the order of the candidates matters).  One workgroup runs per compute
// unit at a time, so the launch takes ceil(workgroups / units) rounds; a 64-wide reduction step costs a
// 64 / 128 / 256-token tile about 0.66 / 1.0 / 1.5 us; partial sums are written and read once more by
// the second kernel.
static double projection_cost(int64_t T, int64_t d_out, int steps, int lora_steps, int bm, int splits)
{
    const int64_t tiles = ((T + bm - 1) / bm) * ((d_out + 255) / 256);
    const int64_t rounds = (tiles * splits + kUnits - 1) / kUnits;
    const double step_us = bm == 64 ? 0.66 : bm == 128 ? 1.0 : 1.5;
    const int per_part = (steps + splits - 1) / splits + lora_steps;      // the adapter's columns go to the last part
    double us = 4.0 + (double)rounds * per_part * step_us;
    if (splits > 1) us += 3.0 + (double)splits * (double)T * (double)d_out * 4.0 / 4.0e6;
    return us;
}

LoraPlan make_lora_plan(int32_t T, int32_t d_in, int32_t d_out, int32_t r, int32_t tile_tokens, int32_t k_splits)
{
    LoraPlan pl{};
    const int steps = d_in / kBK;
    // token tile and reduction parts: what was asked for, else the cheapest of the candidates
    int bm = tile_tokens, best_splits = k_splits;
    if (tile_tokens == 0 || k_splits == 0) {
        double best = 0.0;
        bool have = false;
        for (int cb = 64; cb <= 256; cb *= 2) {
            if (tile_tokens != 0 && cb != tile_tokens) continue;
            if (tile_tokens == 0 && cb > 64 && cb / 2 >= T) continue;          // a tile twice the batch computes padding only
            for (int cs = 1; cs <= (k_splits ? 16 : 8); ++cs) {
                if (k_splits != 0 && cs != k_splits) continue;
                if (k_splits == 0 && cs > 1 && steps / cs < 4) break;          // at least four steps per part
                const double c = projection_cost(T, d_out, steps, r / kBK, cb, cs);
                if (!have || c < best) { best = c; bm = cb; best_splits = cs; have = true; }
            }
        }
        if (!have) { bm = tile_tokens ? tile_tokens : 64; best_splits = k_splits ? k_splits : 1; }
    }
    pl.bm = bm;
    pl.splits = best_splits;
    if (pl.splits > d_in / kBK) pl.splits = d_in / kBK;
    pl.shrink_splits = 1;
    if (r > 0) {
        const int64_t stiles = (int64_t)((T + 63) / 64) * ((r + 127) / 128);
        pl.shrink_splits = k_splits > 0 ? k_splits : pick_splits(stiles, d_in / kBK, 16);
        if (pl.shrink_splits > d_in / kBK) pl.shrink_splits = d_in / kBK;
    }
    size_t off = 0;
    pl.u_off = off;
    off += ((size_t)T * r * 2 + 255) & ~(size_t)255;
    pl.part_off = off;   // one buffer serves the shrink's partial tiles and then the projection's
    size_t part = 0;
    if (pl.shrink_splits > 1) part = (size_t)pl.shrink_splits * T * r * 4;
    if (pl.splits > 1 && (size_t)pl.splits * T * d_out * 4 > part) part = (size_t)pl.splits * T * d_out * 4;
    off += (part + 255) & ~(size_t)255;
    pl.total = off;
    return pl;
}

}  // namespace

extern "C" size_t idlm_gated_lora_linear_workspace(int32_t T, int32_t d_in, int32_t d_out, int32_t r,
                                                   int32_t tile_tokens, int32_t k_splits)
{
    if (!lora_shape_ok(T, d_in, d_out, r) || T == 0) return 0;
    if (tile_tokens != 0 && tile_tokens != 64 && tile_tokens != 128 && tile_tokens != 256) return 0;
    if (k_splits < 0 || k_splits > 16) return 0;
    return make_lora_plan(T, d_in, d_out, r, tile_tokens, k_splits).total;
}

extern "C" int idlm_gated_lora_linear(const uint16_t* x, const uint16_t* W, const uint16_t* A, const uint16_t* Bm,
                                      const uint8_t* gate, const int32_t* n_draft, int32_t S, uint16_t* h,
                                      int32_t T, int32_t d_in, int32_t d_out, int32_t r, int32_t tile_tokens,
                                      int32_t k_splits, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!lora_shape_ok(T, d_in, d_out, r)) return IDLM_ERR_SHAPE;
    if (tile_tokens != 0 && tile_tokens != 64 && tile_tokens != 128 && tile_tokens != 256) return IDLM_ERR_SHAPE;
    if (k_splits < 0 || k_splits > 16) return IDLM_ERR_SHAPE;
    if (r > 0 && !gate && (S < 1 || T % S != 0)) return IDLM_ERR_SHAPE;
    if (T == 0) return IDLM_OK;
    if (!x || !W || !h || (r > 0 && (!A || !Bm || (!gate && !n_draft)))) return IDLM_ERR_NULL;
    if (!aligned(x, 16) || !aligned(W, 16) || !aligned(h, 16) || (r > 0 && (!aligned(A, 16) || !aligned(Bm, 16))))
        return IDLM_ERR_ALIGN;
    const LoraPlan pl = make_lora_plan(T, d_in, d_out, r, tile_tokens, k_splits);
    if (pl.total && (!workspace || workspace_bytes < pl.total)) return IDLM_ERR_WORKSPACE;
    if (pl.total && !aligned(workspace, 256)) return IDLM_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();

    char* ws = static_cast<char*>(workspace);
    uint16_t* u = reinterpret_cast<uint16_t*>(ws + pl.u_off);
    LoraGemmParams p{};
    p.gate = gate; p.n_draft = n_draft; p.S = S > 0 ? S : 1; p.T = T;
    p.partial = reinterpret_cast<float*>(ws + pl.part_off);
    int rc = IDLM_OK;
    if (r > 0) {   // u = gate * (x A^T)
        p.x = x; p.w = A; p.x2 = nullptr; p.w2 = nullptr; p.out = u; p.N = r; p.K0 = d_in; p.K1 = 0;
        p.splits = pl.shrink_splits;
        rc = launch_gemm<1, 4, 4, 2, 3, true>(p, st);
        if (rc != IDLM_OK) return rc;
    } else {
        p.gate = nullptr; p.n_draft = nullptr;
    }
    p.x = x; p.w = W; p.x2 = u; p.w2 = Bm; p.out = h; p.N = d_out; p.K0 = d_in; p.K1 = r;
    p.splits = pl.splits;
    if (pl.bm == 256) rc = launch_gemm<2, 4, 8, 4, 2, false>(p, st);
    else if (pl.bm == 128) rc = launch_gemm<1, 8, 8, 2, 3, false>(p, st);
    else rc = launch_gemm<1, 8, 4, 2, 3, false>(p, st);
    if (rc != IDLM_OK) return rc;
    return launch_status();
}
