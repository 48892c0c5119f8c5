// Device-side definitions shared by the attention kernels: vector types, the kernel parameters, the tile list of a
// KV head and its partition into slices of equal cost, small lane-level helpers.
#pragma once
#include "idlm_common.h"

namespace idlm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

constexpr int kMaxWorkgroups = 1024;      // upper bound of a forced persistent grid
constexpr int kDefaultWorkgroups = 256;   // upper bound of the grid the library chooses itself (one workgroup per compute unit)

struct AttnParams {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    uint16_t* out;
    void* ws_o;     // [2*NW][NB][4][64] partial outputs of a slot (2v: first sequence of wavefront v's slice, 2v+1: its
                    //                   last): D/16 fp16 per entry, normalised per row to a largest magnitude of 1
    f32x4* ws_ml;   // [2*NW][NB][16]    per row: reference exponent, denominator l, largest magnitude of O / l, unused
    int B, S, Hq, Hkv, G, M, RG, max_pages, Mpad;   // RG groups of Mpad = 16*NB rows share a KV head
    int num_pages;
    int partial_layout;   // which values an entry of a partial result holds: 0 = streaming kernel, 1 = shared-tile kernel
    int xcd_bias;   // streaming kernel: 1024 x the share of a slice that wavefronts on even XCDs take over from those on odd
                    // ones (0 = equal slices); only with a multiple of eight virtual heads and an even number of slices
    unsigned long long* wave_trace;   // nullptr, or [wavefronts of the grid][4]: start, end (100 MHz clock), tiles, sequence parts
    int64_t page_stride, head_stride, token_stride;
    float scale_log2;
};

// A rescale of the running reference exponent is skipped while no score exceeds it by more
// than this many powers of two: probabilities then stay below 2^12, harmless in fp32 / bf16
// (bf16 has fp32's exponent range), and after the first tile the rescale almost never runs.
constexpr float kRescaleSlack = 12.0f;

// ---- the tile list and its partition -------------------------------------------------------

// The list is cut into slices of equal COST, not of equal tile count: besides its tiles every
// sequence costs a wavefront about three tiles' worth of time (Q in, rows out; measured 8 us per
// sequence part against 2.6 us per tile on the serving workload), so positions are counted in
// "weights", tiles + kSeqCost per sequence.  A cut that falls into a sequence's extra weight is
// moved to the end of that sequence.
constexpr int kSeqCost = 3;

template <int NWAVES>
struct TilePlanT {              // static LDS of the kernels; NWAVES wavefronts per workgroup
    int incl[64 * NWAVES];      // inclusive prefix sums of the per-thread sequence weights
    int wave_sum[NWAVES];       // weight counted by each of the block's wavefronts
};
typedef TilePlanT<4> TilePlan;

// x of the lane whose number differs in bit 0 (XOR_LANE = 1) or bit 1 (XOR_LANE = 2): a permutation inside each quad
// of lanes, done by the vector ALU's data-parallel-primitive path in one instruction instead of a round trip through LDS.
template <int XOR_LANE>
__device__ __forceinline__ uint32_t quad_xor(uint32_t x)
{
    constexpr int ctrl = XOR_LANE == 1 ? 0xB1 : 0x4E;   // quad_perm [1,0,3,2] / [2,3,0,1]
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, ctrl, 0xF, 0xF, false);
}

// One 32-bit value into / out of an accumulation register.  In this file the matrix instructions keep their results
// in ordinary vector registers, so the accumulation registers are free storage: the finished output rows of up to
// two whole sequences wait there until the wavefront has no K/V left to read.
__device__ __forceinline__ uint32_t acc_park(uint32_t v)
{
    uint32_t a;
    asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a) : "v"(v));
    return a;
}
__device__ __forceinline__ uint32_t acc_fetch(uint32_t a)
{
    uint32_t v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// The value of x, hidden from the optimiser: what is computed from it is computed here and now
// instead of once, ahead of the loops, and then kept in (or spilled from) a register.
__device__ __forceinline__ int opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// 32-token tiles of sequence b (for one KV head).  A context longer than the block table can
// describe is a broken precondition; the table is never walked past its end.
__device__ __forceinline__ int seq_tiles(const AttnParams& p, const int32_t* __restrict__ ctx_lens, int b)
{
    const int c = min(ctx_lens[b], p.max_pages * 16);
    return c > 0 ? (c + 31) >> 5 : 0;
}

// Block-wide inclusive scan of sequence weights (thread t sums sequences [t*per, (t+1)*per)): a
// shuffle scan inside each wavefront, then the wavefront totals through LDS - two barriers in all.
// Returns the total weight of one head's list (its tiles + kSeqCost * B).  Every thread of the
// block must call it.  The sequences are spread over the first 256 threads whatever the block size, so the
// lookups below only read that part of the plan.
template <int NWAVES>
__device__ __forceinline__ int plan_scan(const AttnParams& p, const int32_t* __restrict__ ctx_lens, TilePlanT<NWAVES>& plan)
{
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int per = (p.B + 255) >> 8;
    const int b0 = min(p.B, tid * per), b1 = min(p.B, b0 + per);
    int x = 0;
    for (int b = b0; b < b1; ++b) x += seq_tiles(p, ctx_lens, b) + kSeqCost;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    if (lane == 63) plan.wave_sum[w] = x;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int k = 0; k < NWAVES; ++k) {
        const int sk = plan.wave_sum[k];
        before += (k < w) ? sk : 0;
        total += sk;
    }
    plan.incl[tid] = x + before;
    __syncthreads();
    return __builtin_amdgcn_readfirstlane(total);   // wave-uniform: keep it in a scalar register
}

// Sequence b whose weight range holds weight position y (0 <= y < total weight) and the weight
// before it.  A wavefront-level lookup (after plan_scan): y must be the same in all lanes of the
// calling wavefront, different wavefronts may look up different positions, nobody waits for anybody.
template <int NWAVES>
__device__ __forceinline__ void plan_locate(const AttnParams& p, const int32_t* __restrict__ ctx_lens,
                                            const TilePlanT<NWAVES>& plan, int y, int& b, int& before)
{
    const int lane = threadIdx.x & 63;
    int fb = 0, fpre = 0;
    bool found = false;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int t = lane + 64 * k;
        const int incl = plan.incl[t];
        const int excl = t ? plan.incl[t - 1] : 0;
        if (excl <= y && y < incl) {     // true for exactly one t of the 256
            const int per = (p.B + 255) >> 8;
            int bb = t * per, acc = excl;
            for (;;) {
                const int wgt = seq_tiles(p, ctx_lens, bb) + kSeqCost;
                if (y < acc + wgt) break;
                acc += wgt;
                ++bb;
            }
            fb = bb;
            fpre = acc;
            found = true;
        }
    }
    // the same value in every lane: scalar registers, so that everything derived from it
    // (table pointer, page ids, loop bounds) stays on the scalar unit
    const unsigned long long mask = __ballot(found);
    const int src = __builtin_amdgcn_readfirstlane((int)__ffsll((long long)mask) - 1);
    b = __builtin_amdgcn_readlane(fb, src);
    before = __builtin_amdgcn_readlane(fpre, src);
}

// Where slice j of virtual head vh starts, in 1/1024 of a mean slice: the odd cuts are shifted by p.xcd_bias, so that slices 2i
// grow and slices 2i + 1 shrink, or the other way round for the heads whose bit 2 is set (they start on an odd XCD).
__device__ __forceinline__ int64_t slice_cut_numerator(const AttnParams& p, int vh, int j)
{
    const int shift = (vh & 4) ? -p.xcd_bias : p.xcd_bias;
    return 1024 * (int64_t)j + ((j & 1) ? shift : 0);
}

// First tile (position in the head's tile list) of slice j of the Wg slices of virtual head vh, the sequence b that
// holds it and the tiles before b.  j >= Wg gives the end of the list (b and pre are then not set).
// Wavefront-level like plan_locate.
template <int NWAVES>
__device__ __forceinline__ int slice_first_tile(const AttnParams& p, const int32_t* __restrict__ ctx_lens,
                                                const TilePlanT<NWAVES>& plan, int total_weight, int Wg, int j, int vh,
                                                int& b, int& pre)
{
    const int total_tiles = total_weight - kSeqCost * p.B;
    if (j >= Wg) return total_tiles;
    const int y = (int)((int64_t)total_weight * slice_cut_numerator(p, vh, j) / (1024 * (int64_t)Wg));
    int before;
    plan_locate(p, ctx_lens, plan, y, b, before);
    pre = before - kSeqCost * b;
    int nt = seq_tiles(p, ctx_lens, b);
    const int x = pre + min(y - before, nt);
    // a cut at the end of a sequence belongs to the next sequence that has tiles
    while (x >= pre + nt && x < total_tiles) {
        pre += nt;
        ++b;
        nt = seq_tiles(p, ctx_lens, b);
    }
    return x;
}

// Debug aid (idlm_isd_attention_wave_trace): what a wavefront did and when, on the constant 100 MHz clock that all compute
// units share.  A wavefront that has no tiles writes nothing (the host clears the array).
__device__ __forceinline__ void wave_trace_write(const AttnParams& p, int wavefront, unsigned long long t_start, int tiles, int parts)
{
    if (p.wave_trace != nullptr && (threadIdx.x & 63) == 0) {
        unsigned long long* r = p.wave_trace + 4 * (size_t)wavefront;
        r[0] = t_start;
        r[1] = __builtin_amdgcn_s_memrealtime();
        r[2] = (unsigned long long)tiles;
        r[3] = (unsigned long long)parts;
    }
}

// A lane's share of a V row (and of an output row) is a chunk of D/16 consecutive values, 8 or 16 bytes.
template <int D> struct LaneChunk;
template <> struct LaneChunk<128> { typedef u32x4 type; };
template <> struct LaneChunk<64> { typedef u32x2 type; };

// The kernel for 65 .. 256 query rows per KV head (bf16, D = 128): the four wavefronts of a workgroup, 32 rows each, share
// every K/V tile through LDS; two workgroups per compute unit.  W workgroups of 256 threads; layout as the streaming
// kernel's LAYOUT; NB = 2, p.RG = wavefront-level row groups per KV head (4 or 8), p.Mpad = 32, p.partial_layout = 1.
size_t shared_kernel_lds_bytes();
int launch_shared_kernel(int layout, int W, hipStream_t st, const AttnParams& p, const int32_t* block_table,
                         const int32_t* ctx_lens);

}  // namespace idlm
