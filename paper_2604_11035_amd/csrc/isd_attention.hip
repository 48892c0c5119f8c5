// Paged causal attention of one ISD step's stride of S query rows per sequence
// (strict causal masking, Sec. 3.1; single paged kernel over prefix + stride, Sec. 3.3 (1),
// App. D) for gfx950.
//
// bf16 path.  Per KV head the work is the list of 32-token tiles of every sequence, in sequence
// order.  The launch has one persistent workgroup per compute unit; workgroup w works on head
// w % Hkv and owns slice w / Hkv of W / Hkv equal contiguous slices of that list ("stream-K"),
// which it finds by itself with a block-wide prefix sum over ctx_lens: no host round trip, no
// empty workgroups, equal bytes per compute unit whatever the length mix.  A slice is a run of
// segments (one sequence, a tile range); a segment that covers its whole sequence writes the
// final output, any other leaves an fp32 partial (at most two per workgroup) that a small
// second kernel joins.
//
// Inside a segment the S*G query rows that share the KV head form the N side of every MFMA and
// everything is computed transposed, so that no cross-lane data movement is needed between
// the two contractions:
//     St[token][row] = K[token][:] . Qt[:][row]          v_mfma_f32_16x16x32_bf16, A = K, B = Q
//     Ot[d][row]    += Vt[d][token] . Pt[token][row]     A = V transposed, B = P
// The accumulator layout of St (lane = row, 4 consecutive tokens per register quad) is exactly
// the B-operand layout of the second MFMA once the contraction index is numbered accordingly.
// K rows are read from HBM directly in A-operand layout with 16-byte loads, and V rows are read
// with 16-byte loads of full 256-byte rows and transposed inside each lane (8 tokens x 8 dims of
// 16-bit values held by one lane).  The four wavefronts of a workgroup take the segment's tiles
// round-robin (and, when S*G > 64, split the query rows), keep private online-softmax state
// and are merged once through LDS at the end of the segment.
//
// HBM-bound for S*G below the machine's flop/byte ridge: algorithmic traffic is one read of
// the sequence's K and V rows (2 * Hkv * D * 2 bytes per context token).
#include "idlm_common.h"

namespace idlm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kMaxWorkgroups = 1024;   // upper bound of the persistent grid (sizes the workspace)

struct AttnParams {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    uint16_t* out;
    float* ws_o;    // [2*W][Mpad][128] unnormalised partial outputs (slot 2w: first segment of
    float* ws_ml;   // [2*W][Mpad][2]   workgroup w, 2w+1: its last) and (reference exponent, denominator)
    int B, S, Hq, Hkv, G, M, max_pages, Mpad;
    int64_t page_stride, head_stride, token_stride;
    float scale_log2;
};

// A rescale of the running reference exponent is skipped while no score exceeds it by more
// than this many powers of two: probabilities then stay below 2^12, harmless in fp32 / bf16
// (bf16 has fp32's exponent range), and after the first tile the rescale almost never runs.
constexpr float kRescaleSlack = 12.0f;

struct KVTile {
    bf16x8 k[2][4];   // [16-token block][k-step]: A operand of St
    u32x4 v[8];       // [slot j']: token 16*(j'/4) + 4*g + j'%4, dims 8*n .. 8*n+7
};

// ---- the tile list and its partition -------------------------------------------------------

struct TilePlan {     // static LDS of both kernels
    int incl[256];    // inclusive prefix sums of the per-thread tile counts
    int found_b;      // sequence that holds a looked-up position ...
    int found_pre;    // ... and the number of tiles (one head) before it
};

// 32-token tiles of sequence b (for one KV head).  A context longer than the block table can
// describe is a broken precondition; the table is never walked past its end.
__device__ __forceinline__ int seq_tiles(const AttnParams& p, const int32_t* __restrict__ ctx_lens, int b)
{
    const int c = min(ctx_lens[b], p.max_pages * 16);
    return c > 0 ? (c + 31) >> 5 : 0;
}

// Block-wide inclusive scan of tile counts (thread t sums sequences [t*per, (t+1)*per)).
// Returns the total number of tiles of one head.  Every thread of the block must call it.
__device__ __forceinline__ int plan_scan(const AttnParams& p, const int32_t* __restrict__ ctx_lens, TilePlan& plan)
{
    const int tid = threadIdx.x;
    const int per = (p.B + 255) >> 8;
    const int b0 = tid * per, b1 = min(p.B, b0 + per);
    int local = 0;
    for (int b = b0; b < b1; ++b) local += seq_tiles(p, ctx_lens, b);
    plan.incl[tid] = local;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const int add = (tid >= off) ? plan.incl[tid - off] : 0;
        __syncthreads();
        plan.incl[tid] += add;
        __syncthreads();
    }
    return __builtin_amdgcn_readfirstlane(plan.incl[255]);   // wave-uniform: keep it in a scalar register
}

// Sequence b that holds per-head tile position x (0 <= x < total) and the tiles before it.
// Every thread of the block must call it (after plan_scan).
__device__ __forceinline__ void plan_locate(const AttnParams& p, const int32_t* __restrict__ ctx_lens, TilePlan& plan,
                                            int x, int& b, int& pre)
{
    const int tid = threadIdx.x;
    const int incl = plan.incl[tid];
    const int excl = tid ? plan.incl[tid - 1] : 0;
    if (excl <= x && x < incl) {
        const int per = (p.B + 255) >> 8;
        int bb = tid * per, acc = excl;
        for (;;) {
            const int nt = seq_tiles(p, ctx_lens, bb);
            if (x < acc + nt) break;
            acc += nt;
            ++bb;
        }
        plan.found_b = bb;
        plan.found_pre = acc;
    }
    __syncthreads();
    // the same value in every lane: scalar registers, so that everything derived from it
    // (table pointer, page ids, loop bounds) stays on the scalar unit
    b = __builtin_amdgcn_readfirstlane(plan.found_b);
    pre = __builtin_amdgcn_readfirstlane(plan.found_pre);
    __syncthreads();
}

// The block table and the context lengths are separate __restrict__ kernel arguments: nothing
// the kernel stores can alias them, so their wave-uniform loads stay on the scalar unit and do
// not tie up the vector-memory counter that the K/V prefetch relies on.
template <int NB, int RG>
__global__ __launch_bounds__(256, (NB <= 2 ? 2 : 1)) void isd_attention_bf16_kernel(const AttnParams p,
                                                                 const int32_t* __restrict__ block_table,
                                                                 const int32_t* __restrict__ ctx_lens)
{
    constexpr int TS = 4 / RG;            // wavefronts that split the tiles of one row group
    constexpr int NREG = 32 * NB + 2 * NB;
    extern __shared__ float lds[];
    __shared__ TilePlan plan;

    // ---- this workgroup's head and its slice of that head's tile list ----
    // W >= Hkv: workgroup w works on head w % Hkv and takes slice w / Hkv of Wg = W / Hkv equal
    // slices of the per-head tile list.  Workgroups w, w+1, .. of one slice index run side by side
    // and read the Hkv adjacent 4 KB head blocks of the same pages at about the same time
    // (DRAM row and TLB locality).  W < Hkv: workgroup w takes heads w, w+W, .. whole.
    const int total = plan_scan(p, ctx_lens, plan);
    const int W = gridDim.x, wg = blockIdx.x;
    const int Wg = W >= p.Hkv ? W / p.Hkv : 1;
    const int slice = W >= p.Hkv ? wg / p.Hkv : 0;
    const int head0 = W >= p.Hkv ? wg % p.Hkv : wg;
    const int head_step = W >= p.Hkv ? p.Hkv : W;
    if (slice >= Wg) return;
    const int slice_begin = (int)((int64_t)total * slice / Wg), slice_end = (int)((int64_t)total * (slice + 1) / Wg);
    if (slice_begin >= slice_end) return;
    int b0, pre0;
    plan_locate(p, ctx_lens, plan, slice_begin, b0, pre0);

    const int lane = threadIdx.x & 63;
    const int w = wave_id();
    const int rg = w / TS, ts = w % TS;
    const int n = lane & 15, g = lane >> 4;
    const int rowbase = rg * 16 * NB;
    const int S = p.S, G = p.G, M = p.M;
    const float cs = p.scale_log2;

    int qpos[NB];   // stride position i of this lane's row in each 16-row block
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) qpos[nb] = (rowbase + 16 * nb + n) / G;
    u32x4* qlds = reinterpret_cast<u32x4*>(lds) + (size_t)rg * NB * 4 * 64;

    for (int kvh = head0; kvh < p.Hkv; kvh += head_step) {
    int b = b0;
    int ntiles = seq_tiles(p, ctx_lens, b);
    int seg_a = slice_begin - pre0;
    int pos = slice_begin;
    bool first_segment = true;

    while (pos < slice_end) {
        const int seg_b = min(ntiles, seg_a + (slice_end - pos));   // tiles [seg_a, seg_b) of item (b, kvh)
        const bool complete = seg_a == 0 && seg_b == ntiles;
        const int ctx = min(ctx_lens[b], p.max_pages * 16);
        const int npages = (ctx + 15) >> 4;

        // ---- Q as B operands, parked in LDS: lane (row n, group g) of k-step s holds dims
        //      8*(4s+g) .. +7; slot [(rg*NB + nb)*4 + s][lane] is read back conflict-free ----
        __syncthreads();   // the previous segment's merge buffers share this LDS
        if (ts == 0) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int row = rowbase + 16 * nb + n;
                if (row < M) {
                    const int gq = row - qpos[nb] * G;
                    const uint16_t* qp = p.q + ((size_t)(b * S + qpos[nb]) * p.Hq + kvh * G + gq) * 128;
#pragma unroll
                    for (int s = 0; s < 4; ++s)
                        qlds[(nb * 4 + s) * 64 + lane] = *reinterpret_cast<const u32x4*>(qp + (4 * s + g) * 8);
                } else {
#pragma unroll
                    for (int s = 0; s < 4; ++s) qlds[(nb * 4 + s) * 64 + lane] = u32x4{0u, 0u, 0u, 0u};
                }
            }
        }
        __syncthreads();

        f32x4 oacc[8][NB];
        float mref[NB], lsum[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            mref[nb] = -INFINITY;
            lsum[nb] = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) oacc[e][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

        const int32_t* __restrict__ tab = block_table + (size_t)b * p.max_pages;
        const uint16_t* kh = p.k + kvh * p.head_stride;
        const uint16_t* vh = p.v + kvh * p.head_stride;

        // Page ids of tile kt (two 16-token pages).  The second id is only read when that page
        // belongs to the sequence; otherwise the first page is read again and masked out.
        auto page_ids = [&](int kt, int& pg0, int& pg1) {
            const int pi = kt * 2;
            pg0 = tab[pi];
            pg1 = (pi + 1 < npages) ? tab[pi + 1] : pg0;
        };
        auto load_k = [&](int pg0, int pg1, KVTile& T_) {
            const uint16_t* k0 = kh + (size_t)pg0 * p.page_stride + n * p.token_stride + g * 8;
            const uint16_t* k1 = kh + (size_t)pg1 * p.page_stride + n * p.token_stride + g * 8;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                T_.k[0][s] = *reinterpret_cast<const bf16x8*>(k0 + 32 * s);
                T_.k[1][s] = *reinterpret_cast<const bf16x8*>(k1 + 32 * s);
            }
        };
        auto load_v = [&](int pg0, int pg1, KVTile& T_) {
            const uint16_t* v0 = vh + (size_t)pg0 * p.page_stride + (4 * g) * p.token_stride + n * 8;
            const uint16_t* v1 = vh + (size_t)pg1 * p.page_stride + (4 * g) * p.token_stride + n * 8;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                T_.v[j] = *reinterpret_cast<const u32x4*>(v0 + j * p.token_stride);
                T_.v[4 + j] = *reinterpret_cast<const u32x4*>(v1 + j * p.token_stride);
            }
        };

        // ---- main loop: this wavefront's tiles seg_a+ts, +TS, ...  One register image of a
        //      tile; the next tile's K is requested as soon as St has consumed K, its V as soon
        //      as Ot has consumed V, so loads stay in flight across the softmax and the other
        //      contraction ----
        KVTile T_;
        int npg0 = 0, npg1 = 0;
        if (seg_a + ts < seg_b) {
            page_ids(seg_a + ts, npg0, npg1);
            load_k(npg0, npg1, T_);
            load_v(npg0, npg1, T_);
            if (seg_a + ts + TS < seg_b) page_ids(seg_a + ts + TS, npg0, npg1);
        }
        for (int kt = seg_a + ts; kt < seg_b; kt += TS) {
            const bool has_next = kt + TS < seg_b;
            const int tb = 32 * kt;
            // ---- St = K Qt ----
            f32x4 sacc[NB][2];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                sacc[nb][0] = f32x4{0.f, 0.f, 0.f, 0.f};
                sacc[nb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const bf16x8 qb = __builtin_bit_cast(bf16x8, qlds[(nb * 4 + s) * 64 + lane]);
                    sacc[nb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(T_.k[0][s], qb, sacc[nb][0], 0, 0, 0);
                    sacc[nb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(T_.k[1][s], qb, sacc[nb][1], 0, 0, 0);
                }
            if (has_next) load_k(npg0, npg1, T_);   // K registers are free again: next tile's K goes in flight
            // ---- causal mask and end of context: only tiles that reach the stride's own rows ----
            if (tb + 32 > ctx - S + 1) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int lim = ctx - S + qpos[nb];   // last key this row may see
#pragma unroll
                    for (int tblk = 0; tblk < 2; ++tblk)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (tb + 16 * tblk + 4 * g + j > lim) sacc[nb][tblk][j] = -INFINITY;
                }
                // value rows beyond the context may hold anything (NaN included): zero them
#pragma unroll
                for (int jj = 0; jj < 8; ++jj)
                    if (tb + 16 * (jj >> 2) + 4 * g + (jj & 3) >= ctx) T_.v[jj] = u32x4{0u, 0u, 0u, 0u};
            }
            // ---- running reference exponent: rescale only when a score overshoots it ----
            bool overshoot = false;
            float lmax[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                float mx = fmaxf(fmaxf(sacc[nb][0][0], sacc[nb][0][1]), fmaxf(sacc[nb][0][2], sacc[nb][0][3]));
                mx = fmaxf(mx, fmaxf(fmaxf(sacc[nb][1][0], sacc[nb][1][1]), fmaxf(sacc[nb][1][2], sacc[nb][1][3])));
                lmax[nb] = mx * cs;
                overshoot |= lmax[nb] > mref[nb] + kRescaleSlack;
            }
            if (__any(overshoot)) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    float rm = lmax[nb];
                    rm = fmaxf(rm, __shfl_xor(rm, 16));
                    rm = fmaxf(rm, __shfl_xor(rm, 32));
                    const float mnew = fmaxf(mref[nb], rm);
                    const float alpha = (mnew == -INFINITY) ? 1.f : fast_exp2(mref[nb] - mnew);
                    lsum[nb] *= alpha;
#pragma unroll
                    for (int e = 0; e < 8; ++e) oacc[e][nb] *= alpha;
                    mref[nb] = mnew;
                }
            }
            // ---- Pt = 2^(St*scale - ref), packed straight into B-operand order ----
            bf16x8 pt[NB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const float mr = (mref[nb] == -INFINITY) ? 0.f : mref[nb];
                float sum = 0.f;
#pragma unroll
                for (int tblk = 0; tblk < 2; ++tblk)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float pv = fast_exp2(fmaf(sacc[nb][tblk][j], cs, -mr));
                        sum += pv;
                        pt[nb][4 * tblk + j] = (__bf16)pv;
                    }
                lsum[nb] += sum;
            }
            // ---- Vt: transpose the lane's 8 tokens x 8 dims, then Ot += Vt Pt ----
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                u32x4 vt;
#pragma unroll
                for (int wp = 0; wp < 4; ++wp) {
                    const uint32_t x = T_.v[2 * wp][e >> 1], y = T_.v[2 * wp + 1][e >> 1];
                    vt[wp] = (e & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
                }
                const bf16x8 va = __builtin_bit_cast(bf16x8, vt);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    oacc[e][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pt[nb], oacc[e][nb], 0, 0, 0);
            }
            if (has_next) {
                load_v(npg0, npg1, T_);                  // V registers are free again
                if (kt + 2 * TS < seg_b) page_ids(kt + 2 * TS, npg0, npg1);
            }
        }

        // denominators: add the four lanes (g = 0..3) that share a row
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            lsum[nb] += __shfl_xor(lsum[nb], 16);
            lsum[nb] += __shfl_xor(lsum[nb], 32);
        }

        // ---- merge the TS wavefronts of a row group through LDS (same register layout on both sides) ----
        auto spill = [&](int slot) {
            float* dst = lds + (size_t)slot * NREG * 64 + lane;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int j = 0; j < 4; ++j) dst[((nb * 8 + e) * 4 + j) * 64] = oacc[e][nb][j];
                dst[(32 * NB + 2 * nb) * 64] = mref[nb];
                dst[(32 * NB + 2 * nb + 1) * 64] = lsum[nb];
            }
        };
        auto absorb = [&](int slot) {
            const float* src = lds + (size_t)slot * NREG * 64 + lane;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const float m2 = src[(32 * NB + 2 * nb) * 64];
                const float l2 = src[(32 * NB + 2 * nb + 1) * 64];
                const float mnew = fmaxf(mref[nb], m2);
                const float a1 = (mref[nb] == -INFINITY) ? 0.f : fast_exp2(mref[nb] - mnew);
                const float a2 = (m2 == -INFINITY) ? 0.f : fast_exp2(m2 - mnew);
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        oacc[e][nb][j] = oacc[e][nb][j] * a1 + src[((nb * 8 + e) * 4 + j) * 64] * a2;
                lsum[nb] = lsum[nb] * a1 + l2 * a2;
                mref[nb] = mnew;
            }
        };
        if constexpr (TS > 1) __syncthreads();   // every wavefront is done with Q: its LDS is reused below
        if constexpr (TS == 4) {
            if (ts >= 2) spill(ts - 2);
            __syncthreads();
            if (ts < 2) absorb(ts);
            __syncthreads();
            if (ts == 1) spill(0);
            __syncthreads();
            if (ts == 0) absorb(0);
        } else if constexpr (TS == 2) {
            if (ts == 1) spill(rg);
            __syncthreads();
            if (ts == 0) absorb(rg);
        }

        // ---- write: lane (row n, group g) holds dims 32g + 8j + e of its rows ----
        if (ts == 0) {
            const size_t wslot = (size_t)(2 * wg + (first_segment ? 0 : 1)) * p.Mpad;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int row = rowbase + 16 * nb + n;
                if (row >= M) continue;
                if (complete) {
                    const float inv = 1.f / lsum[nb];
                    const int i = qpos[nb], gq = row - i * G;
                    uint16_t* op = p.out + ((size_t)(b * S + i) * p.Hq + kvh * G + gq) * 128 + 32 * g;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        bf16x8 o;
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[e] = (__bf16)(oacc[e][nb][j] * inv);
                        *reinterpret_cast<bf16x8*>(op + 8 * j) = o;
                    }
                } else {
                    float* op = p.ws_o + (wslot + row) * 128 + 32 * g;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        *reinterpret_cast<f32x4*>(op + 8 * j) = f32x4{oacc[0][nb][j], oacc[1][nb][j], oacc[2][nb][j], oacc[3][nb][j]};
                        *reinterpret_cast<f32x4*>(op + 8 * j + 4) = f32x4{oacc[4][nb][j], oacc[5][nb][j], oacc[6][nb][j], oacc[7][nb][j]};
                    }
                    if (g == 0) {
                        p.ws_ml[(wslot + row) * 2] = mref[nb];
                        p.ws_ml[(wslot + row) * 2 + 1] = lsum[nb];
                    }
                }
            }
        }

        // ---- next segment: the next non-empty sequence ----
        pos += seg_b - seg_a;
        first_segment = false;
        seg_a = 0;
        if (pos < slice_end) {
            do { ++b; ntiles = seq_tiles(p, ctx_lens, b); } while (ntiles == 0);
        }
    }
    }   // heads
}

// Joins the partials of items that span several workgroups.  Block (h, j) looks at the cut
// between slices j-1 and j of head h's tile list (the main kernel's partition); the block of the
// first cut that falls inside an item merges all of that item's partials:
// out = sum_k 2^(m_k - m*) O_k / sum_k 2^(m_k - m*) l_k.
__global__ __launch_bounds__(256) void isd_attention_merge_kernel(const AttnParams p, int Wg,
                                                                  const int32_t* __restrict__ ctx_lens)
{
    __shared__ TilePlan plan;
    const int total = plan_scan(p, ctx_lens, plan);
    const int kvh = blockIdx.x % p.Hkv;
    const int jcut = blockIdx.x / p.Hkv + 1;       // cut = start of slice jcut
    const int cut = (int)((int64_t)total * jcut / Wg);
    if (cut <= 0 || cut >= total) return;
    int b, pre;
    plan_locate(p, ctx_lens, plan, cut, b, pre);
    const int ntiles = seq_tiles(p, ctx_lens, b);
    const int a = cut - pre;
    if (a == 0) return;                            // the cut coincides with the start of an item
    const int item_begin = pre, item_end = pre + ntiles;
    auto slice_start = [&](int j) { return (int)((int64_t)total * j / Wg); };
    if (slice_start(jcut - 1) > item_begin) return;   // an earlier cut is inside the same item
    // slices jcut-1 .. hold this item's partials, written by workgroup j*Hkv + kvh into slot 2w if
    // the item is the first segment of that slice (the slice starts inside the item), 2w+1 if it
    // is its last
    auto slot_of = [&](int j, int jbeg) { return 2 * (j * p.Hkv + kvh) + (jbeg >= item_begin ? 0 : 1); };
    for (int idx = threadIdx.x; idx < p.M * 32; idx += 256) {
        const int row = idx >> 5, d4 = idx & 31;
        float mstar = -INFINITY;
        for (int j = jcut - 1; j < Wg; ++j) {
            const int jbeg = slice_start(j), jend = slice_start(j + 1);
            if (jbeg >= item_end) break;
            if (jbeg == jend) continue;
            mstar = fmaxf(mstar, p.ws_ml[((size_t)slot_of(j, jbeg) * p.Mpad + row) * 2]);
        }
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
        for (int j = jcut - 1; j < Wg; ++j) {
            const int jbeg = slice_start(j), jend = slice_start(j + 1);
            if (jbeg >= item_end) break;
            if (jbeg == jend) continue;
            const size_t s = (size_t)slot_of(j, jbeg) * p.Mpad + row;
            const float m = p.ws_ml[s * 2];
            const float wgt = (m == -INFINITY) ? 0.f : fast_exp2(m - mstar);
            den += wgt * p.ws_ml[s * 2 + 1];
            acc += *reinterpret_cast<const f32x4*>(p.ws_o + s * 128 + d4 * 4) * wgt;
        }
        const float inv = 1.f / den;
        const int i = row / p.G, gq = row - i * p.G;
        uint16_t* op = p.out + ((size_t)(b * p.S + i) * p.Hq + kvh * p.G + gq) * 128 + d4 * 4;
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(acc[e] * inv);
        *reinterpret_cast<bf16x4*>(op) = o4;
    }
}

// ---- fp32 path (small correctness configurations): one wavefront per (sequence, row, head) ----
struct AttnParamsF32 {
    const float* q;
    const float* k;
    const float* v;
    const int32_t* table;
    const int32_t* ctx;
    float* out;
    int S, Hq, Hkv, G, P, max_pages;
    int64_t page_stride, head_stride, token_stride;
    float scale_log2;
};

template <int D>
__global__ __launch_bounds__(64) void isd_attention_f32_kernel(const AttnParamsF32 p)
{
    const int h = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x;
    const int ctx = min(p.ctx[b], p.max_pages * p.P);
    const int last = ctx - p.S + i;
    const int kvh = h / p.G;
    const float* qp = p.q + ((size_t)(b * p.S + i) * p.Hq + h) * D;
    const int32_t* tab = p.table + (size_t)b * p.max_pages;
    float o[D];
#pragma unroll
    for (int d = 0; d < D; ++d) o[d] = 0.f;
    float m = -INFINITY, l = 0.f;
    for (int t = lane; t <= last; t += 64) {
        const int pg = tab[t / p.P];
        const size_t off = (size_t)pg * p.page_stride + kvh * p.head_stride + (t % p.P) * p.token_stride;
        const float* kp = p.k + off;
        const float* vp = p.v + off;
        float dot = 0.f;
#pragma unroll
        for (int d = 0; d < D; d += 4) {
            const float4 kk = *reinterpret_cast<const float4*>(kp + d);
            const float4 qq = *reinterpret_cast<const float4*>(qp + d);
            dot += kk.x * qq.x + kk.y * qq.y + kk.z * qq.z + kk.w * qq.w;
        }
        const float s = dot * p.scale_log2;
        const float mnew = fmaxf(m, s);
        const float alpha = fast_exp2(m - mnew);   // m = -inf on the first key gives 0
        const float pv = fast_exp2(s - mnew);
        l = l * alpha + pv;
#pragma unroll
        for (int d = 0; d < D; d += 4) {
            const float4 vv = *reinterpret_cast<const float4*>(vp + d);
            o[d] = o[d] * alpha + pv * vv.x;
            o[d + 1] = o[d + 1] * alpha + pv * vv.y;
            o[d + 2] = o[d + 2] * alpha + pv * vv.z;
            o[d + 3] = o[d + 3] * alpha + pv * vv.w;
        }
        m = mnew;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off);
        const float l2 = __shfl_xor(l, off);
        const float mnew = fmaxf(m, m2);
        const float a1 = (m == -INFINITY) ? 0.f : fast_exp2(m - mnew);
        const float a2 = (m2 == -INFINITY) ? 0.f : fast_exp2(m2 - mnew);
        l = l * a1 + l2 * a2;
#pragma unroll
        for (int d = 0; d < D; ++d) o[d] = o[d] * a1 + __shfl_xor(o[d], off) * a2;
        m = mnew;
    }
    if (lane == 0) {
        const float inv = 1.f / l;
        float* op = p.out + ((size_t)(b * p.S + i) * p.Hq + h) * D;
#pragma unroll
        for (int d = 0; d < D; ++d) op[d] = o[d] * inv;
    }
}

// ---- host side ----------------------------------------------------------------------------

static bool shapes_ok(int32_t B, int32_t S, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                      int32_t max_pages, int32_t dtype, int* err)
{
    *err = IDLM_OK;
    if (dtype != IDLM_DTYPE_F32 && dtype != IDLM_DTYPE_BF16) { *err = IDLM_ERR_DTYPE; return false; }
    if (B < 0 || B > 65535 || S < 1 || S > 32 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || Hkv > 65535 ||
        P != 16 || max_pages < 1 || (int64_t)max_pages * P >= (1 << 30) ||
        (int64_t)B * max_pages >= (1LL << 31)) { *err = IDLM_ERR_SHAPE; return false; }
    const int G = Hq / Hkv;
    if (dtype == IDLM_DTYPE_BF16) {
        if (D != 128) { *err = IDLM_ERR_DTYPE; return false; }
        if (S * G > 256) { *err = IDLM_ERR_SHAPE; return false; }
    } else {
        if (D != 64 && D != 128) { *err = IDLM_ERR_DTYPE; return false; }
        if (Hq > 65535) { *err = IDLM_ERR_SHAPE; return false; }
    }
    return true;
}

static void row_tiling(int M, int* NB, int* RG)
{
    if (M <= 16) { *NB = 1; *RG = 1; }
    else if (M <= 32) { *NB = 2; *RG = 1; }
#ifdef IDLM_EXP_M64_22
    else if (M <= 64) { *NB = 2; *RG = 2; }
#else
    else if (M <= 64) { *NB = 4; *RG = 1; }
#endif
    else if (M <= 128) { *NB = 4; *RG = 2; }
    else { *NB = 4; *RG = 4; }
}

}  // namespace idlm

using namespace idlm;

extern "C" size_t idlm_isd_attention_workspace(int32_t B, int32_t S, int32_t Hq, int32_t Hkv, int32_t D,
                                               int32_t P, int32_t max_pages_per_seq, int32_t dtype)
{
    int err;
    if (!shapes_ok(B, S, Hq, Hkv, D, P, max_pages_per_seq, dtype, &err)) return 0;
    if (dtype != IDLM_DTYPE_BF16 || B == 0) return 0;
    int NB, RG;
    row_tiling(S * (Hq / Hkv), &NB, &RG);
    const size_t rows = (size_t)2 * kMaxWorkgroups * (16 * NB * RG);
    return rows * 128 * sizeof(float) + rows * 2 * sizeof(float);
}

extern "C" int idlm_isd_attention_ev(const void* q, const void* k_cache, const void* v_cache,
                                     const int32_t* block_table, const int32_t* ctx_lens, int32_t S, void* out,
                                     int32_t B, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                                     int32_t num_pages, int32_t max_pages_per_seq, int64_t page_stride,
                                     int64_t head_stride, int64_t token_stride, float scale, int32_t dtype,
                                     int32_t num_workgroups, void* workspace, size_t workspace_bytes, void* stream,
                                     void* const* events)
{
    int err;
    if (!shapes_ok(B, S, Hq, Hkv, D, P, max_pages_per_seq, dtype, &err)) return err;
    if (num_pages < 1 || page_stride < 1 || head_stride < 1 || token_stride < D) return IDLM_ERR_SHAPE;
    if (num_workgroups < 0 || num_workgroups > kMaxWorkgroups) return IDLM_ERR_SHAPE;
    if (B == 0) return IDLM_OK;
    if (!q || !k_cache || !v_cache || !block_table || !ctx_lens || !out) return IDLM_ERR_NULL;
    const size_t esz = dtype == IDLM_DTYPE_BF16 ? 2 : 4;
    if (!aligned(q, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(out, 16) ||
        !aligned(block_table, 4) || !aligned(ctx_lens, 4))
        return IDLM_ERR_ALIGN;
    if ((page_stride * esz) % 16 || (head_stride * esz) % 16 || (token_stride * esz) % 16) return IDLM_ERR_ALIGN;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)D);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int G = Hq / Hkv;

    if (dtype == IDLM_DTYPE_F32) {
        AttnParamsF32 p;
        p.q = static_cast<const float*>(q);
        p.k = static_cast<const float*>(k_cache);
        p.v = static_cast<const float*>(v_cache);
        p.table = block_table; p.ctx = ctx_lens; p.out = static_cast<float*>(out);
        p.S = S; p.Hq = Hq; p.Hkv = Hkv; p.G = G; p.P = P; p.max_pages = max_pages_per_seq;
        p.page_stride = page_stride; p.head_stride = head_stride; p.token_stride = token_stride;
        p.scale_log2 = scale * kLog2e;
        (void)hipGetLastError();
        dim3 grid(Hq, S, B);
        if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[0]), st);
        if (D == 64) hipLaunchKernelGGL(isd_attention_f32_kernel<64>, grid, dim3(64), 0, st, p);
        else hipLaunchKernelGGL(isd_attention_f32_kernel<128>, grid, dim3(64), 0, st, p);
        if (events) {
            (void)hipEventRecord(static_cast<hipEvent_t>(events[1]), st);
            (void)hipEventRecord(static_cast<hipEvent_t>(events[2]), st);
        }
        return launch_status();
    }

    const size_t need = idlm_isd_attention_workspace(B, S, Hq, Hkv, D, P, max_pages_per_seq, dtype);
    if (!workspace || workspace_bytes < need) return IDLM_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return IDLM_ERR_ALIGN;

    // one persistent workgroup per compute unit (a workgroup holds a whole CU's registers)
    int W = num_workgroups;
    if (W == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            return IDLM_ERR_LAUNCH;
        W = cus > kMaxWorkgroups ? kMaxWorkgroups : cus;
    }

    AttnParams p;
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k_cache);
    p.v = static_cast<const uint16_t*>(v_cache);
    p.out = static_cast<uint16_t*>(out);
    p.B = B; p.S = S; p.Hq = Hq; p.Hkv = Hkv; p.G = G; p.M = S * G; p.max_pages = max_pages_per_seq;
    int NB, RG;
    row_tiling(p.M, &NB, &RG);
    p.Mpad = 16 * NB * RG;
    const size_t rows = (size_t)2 * kMaxWorkgroups * p.Mpad;
    p.ws_o = static_cast<float*>(workspace);
    p.ws_ml = p.ws_o + rows * 128;
    p.page_stride = page_stride; p.head_stride = head_stride; p.token_stride = token_stride;
    p.scale_log2 = scale * kLog2e;

    (void)hipGetLastError();
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[0]), st);
    const int nreg = 32 * NB + 2 * NB;
#define IDLM_LAUNCH_ATTN(NB_, RG_, SLOTS_)                                                              \
    do {                                                                                                 \
        size_t shmem = (size_t)(SLOTS_) * nreg * 64 * sizeof(float);                                     \
        const size_t qbytes = (size_t)(RG_) * (NB_) * 4 * 64 * 16;                                       \
        if (qbytes > shmem) shmem = qbytes;                                                              \
        if (shmem > 65536 - sizeof(TilePlan))                                                            \
            (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&isd_attention_bf16_kernel<NB_, RG_>), \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);           \
        hipLaunchKernelGGL((isd_attention_bf16_kernel<NB_, RG_>), dim3(W), dim3(256), shmem, st, p,      \
                           block_table, ctx_lens);                                                      \
    } while (0)
    if (NB == 1) IDLM_LAUNCH_ATTN(1, 1, 2);
    else if (NB == 2 && RG == 1) IDLM_LAUNCH_ATTN(2, 1, 2);
    else if (NB == 2) IDLM_LAUNCH_ATTN(2, 2, 2);
    else if (RG == 1) IDLM_LAUNCH_ATTN(4, 1, 2);
    else if (RG == 2) IDLM_LAUNCH_ATTN(4, 2, 2);
    else IDLM_LAUNCH_ATTN(4, 4, 0);
#undef IDLM_LAUNCH_ATTN
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[1]), st);
    const int Wg = W >= Hkv ? W / Hkv : 1;   // slices per head, as in the main kernel
    if (Wg > 1)
        hipLaunchKernelGGL(isd_attention_merge_kernel, dim3((unsigned)((Wg - 1) * Hkv)), dim3(256), 0, st, p, Wg, ctx_lens);
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[2]), st);
    return launch_status();
}

extern "C" int idlm_isd_attention(const void* q, const void* k_cache, const void* v_cache,
                                  const int32_t* block_table, const int32_t* ctx_lens, int32_t S, void* out,
                                  int32_t B, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                                  int32_t num_pages, int32_t max_pages_per_seq, int64_t page_stride,
                                  int64_t head_stride, int64_t token_stride, float scale, int32_t dtype,
                                  int32_t num_workgroups, void* workspace, size_t workspace_bytes, void* stream)
{
    return idlm_isd_attention_ev(q, k_cache, v_cache, block_table, ctx_lens, S, out, B, Hq, Hkv, D, P,
                                 num_pages, max_pages_per_seq, page_stride, head_stride, token_stride,
                                 scale, dtype, num_workgroups, workspace, workspace_bytes, stream, nullptr);
}
