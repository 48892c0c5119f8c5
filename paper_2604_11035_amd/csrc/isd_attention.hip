// Paged causal attention of one ISD step's stride of S query rows per sequence
// (strict causal masking, Sec. 3.1; single paged kernel over prefix + stride, Sec. 3.3 (1),
// App. D) for gfx950.
//
// bf16 path.  Per KV head the work is the list of 32-token tiles of every sequence, in sequence
// order.  The launch is persistent (one workgroup of four wavefronts per compute unit) and the
// list is shared at wavefront level: wavefront v works on virtual head v % VH (a KV head and a
// group of up to 64 query rows) and owns slice v / VH of NW / VH equal contiguous slices
// ("stream-K"), which it finds with a block-wide prefix sum over ctx_lens: no host round trip,
// no empty workgroups, equal bytes per wavefront whatever the length mix, and no barrier after
// the prefix sum.  A sequence that lies wholly inside a slice is written out directly; one that
// a slice boundary cuts leaves a partial result (at most two per wavefront: row-scaled fp16 plus
// per-row reference exponent, denominator and scale) that a small second kernel joins.  Partials
// wait in the wavefront's LDS until it has read all its K/V: stores that mix into the stream of
// reads cost several times their share of the bytes on this memory system.
//
// For a tile the S*G query rows that share the KV head form the N side of every MFMA and
// everything is computed transposed, so that no cross-lane data movement is needed between
// the two contractions:
//     St[token][row] = K[token][:] . Qt[:][row]          v_mfma_f32_16x16x32_bf16, A = K, B = Q
//     Ot[d][row]    += Vt[d][token] . Pt[token][row]     A = V transposed, B = P
// The accumulator layout of St (lane = row, 4 consecutive tokens per register quad) is exactly
// the B-operand layout of the second MFMA once the contraction index is numbered accordingly.
// K rows are read from HBM directly in A-operand layout with 16-byte loads, and V rows are read
// with 16-byte loads of full 256-byte rows and transposed inside each lane (8 tokens x 8 dims of
// 16-bit values held by one lane).  Q operands of the wavefront's current sequence sit in LDS.
//
// HBM-bound for S*G below the machine's flop/byte ridge: algorithmic traffic is one read of
// the sequence's K and V rows (2 * Hkv * D * 2 bytes per context token).  This file holds the kernel for up to
// 64 query rows per KV head (any bf16 shape at D = 64), the kernel that joins partial results, the fp32 path and
// the entry points; more than 64 rows per KV head at D = 128 run on the kernel of isd_attention_shared.hip.
#include "isd_attention_plan.h"

namespace idlm {

// The block table and the context lengths are separate __restrict__ kernel arguments: nothing
// the kernel stores can alias them, so their wave-uniform loads stay on the scalar unit and do
// not tie up the vector-memory counter that the K/V prefetch relies on.
//
// Work is shared at WAVEFRONT level.  A "virtual head" is (KV head, group of 16*NB query rows);
// with NW wavefronts in the launch, wavefront v works on virtual head v % VH and owns slice
// v / VH of NW / VH equal contiguous slices of the per-head tile list.  After the common
// prefix sum the four wavefronts of a workgroup never synchronise again: each streams its
// slice tile by tile, switching sequence (new Q, fresh accumulators, output written) whenever
// the slice crosses into the next one, with the next tile's K/V always in flight - also across
// such a switch.
//
// LAYOUT fixes the strides inside a page at compile time, so that the eight loads of an operand share
// one address and differ in their immediate offsets: 0 = any strides (token-major pools, padded rows),
// 1 = contiguous slot-major pages (token_stride = 128), 2 = the same with the K pages in operand order.
//
// D is the head dimension, 64 or 128: D/32 contraction steps for St, D/16 sixteen-row blocks of Ot, and a lane's
// share of a V row (and of an output row) is a chunk of D/16 consecutive values, 8 or 16 bytes.
template <int NB, int LAYOUT, int D>
__global__ __launch_bounds__(256) void isd_attention_bf16_kernel(const AttnParams p,
                                                                 const int32_t* __restrict__ block_table,
                                                                 const int32_t* __restrict__ ctx_lens)
{
    constexpr int KS = D / 32;    // contraction steps of St = K Qt
    constexpr int E = D / 16;     // sixteen-row blocks of Ot = values per lane chunk
    typedef typename LaneChunk<D>::type chunk_t;
    extern __shared__ u32x4 qlds_all[];   // [wavefront][(nb*KS + s)*64 + lane] Q operands of the current item
    __shared__ TilePlan plan;

    const unsigned long long t_start = p.wave_trace ? __builtin_amdgcn_s_memrealtime() : 0ull;
    int traced_tiles = 0, traced_parts = 0;
    const int total_weight = plan_scan(p, ctx_lens, plan);
    if (total_weight == kSeqCost * p.B) return;   // no tiles at all
    const int lane = threadIdx.x & 63;
    const int w = wave_id();
    const int NW = gridDim.x * 4;
    const int VH = p.Hkv * p.RG;
    const int Wg = NW >= VH ? NW / VH : 1;
    auto slice_of = [&](int v) { return NW >= VH ? v / VH : 0; };

    const int wv = blockIdx.x * 4 + w;
    const int slice = slice_of(wv);
    if (slice >= Wg) return;
    // Under saturation the wavefronts on odd XCDs (workgroup number odd) get about 6 % less of the memory system than those on
    // even ones.  With a multiple of eight virtual heads the parity of a wavefront's XCD is bit 2 of its virtual head, the same
    // for all slices of a head; so odd slices take the head whose number differs in bit 2 (the slices of every head then
    // alternate between the two kinds of XCD) and the slices on even XCDs are made longer by the share p.xcd_bias / 1024.
    const bool balanced = p.xcd_bias != 0;
    const int vh0 = NW >= VH ? (wv % VH) ^ (balanced ? 4 * (slice & 1) : 0) : wv;
    const int vstep = NW >= VH ? VH : NW;
    int b0 = 0, pre0 = 0, b_end, pre_end;   // first sequence of the slice and the tiles before it
    const int slice_begin = slice_first_tile(p, ctx_lens, plan, total_weight, Wg, slice, vh0, b0, pre0);
    const int slice_end = slice_first_tile(p, ctx_lens, plan, total_weight, Wg, slice + 1, vh0, b_end, pre_end);
    if (slice_begin >= slice_end) return;

    const int n = lane & 15, g = lane >> 4;
    const int S = p.S, G = p.G, M = p.M;
    const float cs = p.scale_log2;
    u32x4* const qlds = qlds_all + (size_t)w * (NB * KS * 64) + lane;
    // a partial result waits here, in this wavefront's own LDS, until the wavefront has read all its K/V
    chunk_t* const stash_o = reinterpret_cast<chunk_t*>(qlds_all + (size_t)4 * (NB * KS * 64)) + (size_t)w * (NB * 4 * 64);
    f32x4* const stash_ml = reinterpret_cast<f32x4*>(reinterpret_cast<chunk_t*>(qlds_all + (size_t)4 * (NB * KS * 64)) +
                                                     (size_t)4 * (NB * 4 * 64)) + w * (NB * 16);
    auto flush_stash = [&](int slot) {
        chunk_t* dst = static_cast<chunk_t*>(p.ws_o) + (size_t)slot * (NB * 4 * 64) + lane;
#pragma unroll
        for (int q = 0; q < NB * 4; ++q) dst[q * 64] = stash_o[q * 64 + lane];
        if (lane < NB * 16) p.ws_ml[(size_t)slot * (NB * 16) + lane] = stash_ml[lane];
    };

    for (int vh = vh0; vh < VH; vh += vstep) {
        const int kvh = vh / p.RG;
        const int rowbase = (vh - kvh * p.RG) * 16 * NB;
        int qpos[NB];   // stride position i of this lane's row in each 16-row block
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) qpos[nb] = (rowbase + 16 * nb + n) / G;
        const uint16_t* kh = p.k + kvh * p.head_stride;
        const uint16_t* vhp = p.v + kvh * p.head_stride;

        // Page ids of tile kt of sequence b (two 16-token pages).  The second id is only read when
        // that page belongs to the sequence; otherwise the first page is read again and masked out.
        auto page_ids = [&](int b, int kt, int& pg0, int& pg1) {
            const int32_t* __restrict__ tab = block_table + (size_t)b * p.max_pages;
            const int npages = (min(ctx_lens[b], p.max_pages * 16) + 15) >> 4;
            pg0 = tab[2 * kt];
            pg1 = (2 * kt + 1 < npages) ? tab[2 * kt + 1] : pg0;
            // a page id outside the pool breaks the caller's side of the contract; the read stays inside the
            // pool anyway (two scalar instructions)
            pg0 = min(max(pg0, 0), p.num_pages - 1);
            pg1 = min(max(pg1, 0), p.num_pages - 1);
        };
        // next tile of the slice: the next tile of the sequence, or tile 0 of the next non-empty one
        auto advance = [&](int& b, int& kt, int& nt) {
            if (++kt == nt) {
                kt = 0;
                do { ++b; nt = seq_tiles(p, ctx_lens, b); } while (nt == 0);
            }
        };
        bf16x8 tk[2][KS];  // K of the current tile: [16-token block][k-step], A operand of St
        chunk_t tv[8];     // V of the current tile: slot j' = token 16*(j'/4) + 4*g + j'%4, dims E*n .. E*n+E-1
        // Addresses are a wave-uniform 64-bit page base (scalar registers) plus a 32-bit lane offset in bytes
        // (the host checks that it fits) plus, for the fixed layouts, an immediate: one address per operand and
        // page instead of one per load.
        // K pages in operand order: the 16 bytes that lane l needs for k-step s sit at entry 64*s + l of the
        // page's 4 KB block, so a load instruction reads 1 KB of whole cache lines instead of 16 rows x 64 bytes
        typedef const __attribute__((address_space(1))) char* gbytes;
        typedef const __attribute__((address_space(1))) u32x4* gvec;
        typedef const __attribute__((address_space(1))) chunk_t* gchunk;
        const int tstride = LAYOUT == 0 ? (int)p.token_stride : D;
        const uint32_t klane = LAYOUT == 2 ? (uint32_t)(lane * 16) : (uint32_t)(2 * (n * tstride + g * 8));
        const int kstep = LAYOUT == 2 ? 1024 : 64;
        const uint32_t vlane = (uint32_t)(2 * (4 * g * tstride + n * E));
        const int vstep = 2 * tstride;
        auto page_base = [&](const uint16_t* pool, int pg) {
            const uint64_t a = reinterpret_cast<uint64_t>(pool) + 2 * (uint64_t)pg * (uint64_t)p.page_stride;
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
            const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
            return (gbytes)(((uint64_t)hi << 32) | lo);
        };
        auto load_k = [&](int pg0, int pg1) {
            const gbytes k0 = page_base(kh, pg0) + klane;
            const gbytes k1 = page_base(kh, pg1) + klane;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                tk[0][s] = __builtin_bit_cast(bf16x8, __builtin_nontemporal_load((gvec)(k0 + kstep * s)));
                tk[1][s] = __builtin_bit_cast(bf16x8, __builtin_nontemporal_load((gvec)(k1 + kstep * s)));
            }
        };
        auto load_v = [&](int pg0, int pg1) {
            const gbytes v0 = page_base(vhp, pg0) + vlane;
            const gbytes v1 = page_base(vhp, pg1) + vlane;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                tv[j] = __builtin_nontemporal_load((gchunk)(v0 + j * vstep));
                tv[4 + j] = __builtin_nontemporal_load((gchunk)(v1 + j * vstep));
            }
        };

        // cursors: current tile (b, kt of nt); c1 = next tile of the slice, whose page ids are held in
        // (npg0, npg1).  K/V loads are issued unconditionally (the compiler can then count the
        // outstanding loads exactly and waits for K without waiting for V and vice versa); the very
        // last tile of the slice simply requests itself again.
        int b = b0, nt = seq_tiles(p, ctx_lens, b), kt = slice_begin - pre0;
        const int remaining = slice_end - slice_begin;
        int c1b = b, c1kt = kt, c1nt = nt, npg0, npg1;
        page_ids(b, kt, npg0, npg1);
        load_k(npg0, npg1);
        load_v(npg0, npg1);
        if (remaining > 1) {
            advance(c1b, c1kt, c1nt);
            page_ids(c1b, c1kt, npg0, npg1);
        }

        // Q rows of sequence bq for this lane (row n of each 16-row block, dims 32s + 8g .. +7); rows
        // past the stride's last one read its last row instead and are zeroed on the way to LDS
        u32x4 qreg[NB][KS];
        auto load_q = [&](int bq) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int row = opaque(rowbase + 16 * nb + n);
                const int qi = row < M ? qpos[nb] : S - 1;
                const int gq = row < M ? row - qpos[nb] * G : G - 1;
                const uint16_t* qp = p.q + ((size_t)(bq * S + qi) * p.Hq + kvh * G + gq) * D + g * 8;
#pragma unroll
                for (int s = 0; s < KS; ++s) qreg[nb][s] = *reinterpret_cast<const u32x4*>(qp + 32 * s);
            }
        };
        auto store_q = [&]() {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const bool valid = opaque(rowbase + 16 * nb + n) < M;
#pragma unroll
                for (int s = 0; s < KS; ++s) qlds[(nb * KS + s) * 64] = valid ? qreg[nb][s] : u32x4{0u, 0u, 0u, 0u};
            }
        };
        load_q(b);
        store_q();

        int stash_slot = -1;   // slot of the partial held in LDS, if any
        // Output rows of whole sequences, ready to be stored (bf16, transposed for full-row stores), parked in accumulation
        // registers: stores that arrive in the middle of the K/V read stream cost many times their share of the bytes, so
        // the first whole sequences of a slice (two; one where 64 rows of 128 values leave no more registers) are written
        // only when the slice has been read.  [nb][j][dword of the chunk]
        constexpr int kParkWords = NB * 4 * (E / 2);
        constexpr int kParkSlots = (NB == 4 && D == 128) ? 1 : 2;
        uint32_t park0[kParkWords], park1[kParkWords];
        int park_b0 = 0, park_b1 = 0, nparked = 0;
        // stores the rows of 16-row block nb of sequence bb: c[j] is chunk 4g + n%4 of rows 4*(n/4) + j
        auto store_rows = [&](int bb, int nb, const chunk_t (&c)[4]) {
            const int row0 = opaque(rowbase + 16 * nb + (n & 12));
            int ip = row0 / G, gq = row0 - ip * G;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (row0 + j < M) {
                    uint16_t* op = p.out + ((size_t)(bb * S + ip) * p.Hq + kvh * G + gq) * D + (4 * g + (n & 3)) * E;
                    __builtin_nontemporal_store(c[j], reinterpret_cast<chunk_t*>(op));
                }
                if (++gq == G) { gq = 0; ++ip; }
            }
        };
        auto flush_parked = [&](const uint32_t (&park)[kParkWords], int bb) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                chunk_t c[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int k = 0; k < E / 2; ++k) c[j][k] = acc_fetch(park[(nb * 4 + j) * (E / 2) + k]);
                store_rows(bb, nb, c);
            }
        };
        traced_tiles += remaining;
        for (int i = 0; i < remaining;) {
            ++traced_parts;
            // ---- a sequence starts (or continues from an earlier slice); its Q is in this wavefront's
            //      LDS already, the accumulators restart ----
            const int n_in = min(nt - kt, remaining - i);   // tiles of this sequence inside the slice
            const bool first_of_slice = i == 0;
            const int ctx = min(ctx_lens[b], p.max_pages * 16);
            const int item_first_kt = kt;
            // Per sixteen-row block: output accumulators, the denominators (accumulated by the matrix unit as the
            // product of the weights with a matrix of ones: all four entries of a lane hold its row's sum over the
            // whole tile), the reference exponent, and two values derived from it that the tile loop uses in its
            // place: the score above which the reference has to be raised, and the addend of the exponent.
            f32x4 oacc[E][NB], lacc[NB];
            float mref[NB], over[NB], nref[NB];
            auto set_ref = [&](int nb, float m) {
                mref[nb] = m;
                over[nb] = (m + kRescaleSlack) / cs;            // -inf while the row has seen no key
                nref[nb] = (m == -INFINITY) ? 0.f : -m;
            };
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                set_ref(nb, -INFINITY);
                lacc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int e = 0; e < E; ++e) oacc[e][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            int pb = b, pkt = kt, pnt = nt;   // cursor of the tile after this sequence's last one

            // One tile in three parts, so that the loop below holds nothing but the common case: the running
            // reference exponent of a row is raised (and the row's accumulators rescaled) only when a score
            // overshoots it by kRescaleSlack powers of two, which after a row's first tile practically never
            // happens.  A first tile needs no rescale either (its accumulators are still zero), so the tile loop
            // leaves through its side exit only for a later overshoot, the rescale is done out there, and the loop
            // is entered again.  The accumulators are then loop-carried through matrix instructions alone and
            // stay in accumulation registers; with the rescale inside the loop they were copied out to vector
            // registers at the top of every tile.
            f32x4 sacc[NB][2];
            float smax[NB];   // largest raw score of this lane's eight entries per block
            auto scores = [&](int tb) {
                asm volatile("" ::: "memory");   // Q comes out of LDS anew for every tile instead of staying in registers
                // ---- St = K Qt ----
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    sacc[nb][0] = f32x4{0.f, 0.f, 0.f, 0.f};
                    sacc[nb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
                // The order of issue is pinned: kAhead Q operands are on their way from LDS before the first product
                // starts and every pair of products is followed by the read of the operand kAhead pairs later, so
                // that no product waits for LDS (left alone, the scheduler reads each operand right before its use).
                constexpr int kOps = NB * KS, kAhead = kOps < 4 ? kOps : 4;
                bf16x8 qb[kOps];
#pragma unroll
                for (int r = 0; r < kAhead; ++r) qb[r] = __builtin_bit_cast(bf16x8, qlds[r * 64]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < kOps; ++r) {
                    const int nb = r / KS, ks = r % KS;
                    sacc[nb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tk[0][ks], qb[r], sacc[nb][0], 0, 0, 0);
                    sacc[nb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tk[1][ks], qb[r], sacc[nb][1], 0, 0, 0);
                    if (r + kAhead < kOps) qb[r + kAhead] = __builtin_bit_cast(bf16x8, qlds[(r + kAhead) * 64]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                load_k(npg0, npg1);   // K registers are free again: next tile's K goes in flight
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
                        if (tb + 16 * (jj >> 2) + 4 * g + (jj & 3) >= ctx) tv[jj] = chunk_t(0u);
                }
                bool overshoot = false;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    // chains of three-operand maxima
                    float mx = fmaxf(fmaxf(sacc[nb][0][0], sacc[nb][0][1]), sacc[nb][0][2]);
                    mx = fmaxf(fmaxf(mx, sacc[nb][0][3]), sacc[nb][1][0]);
                    mx = fmaxf(fmaxf(mx, sacc[nb][1][1]), sacc[nb][1][2]);
                    smax[nb] = fmaxf(mx, sacc[nb][1][3]);
                    overshoot |= smax[nb] > over[nb];
                }
                return __any(overshoot) != 0;
            };
            // the largest score of each row of the tile (the four lanes that share a row agree on it)
            auto row_max = [&](float (&rm)[NB]) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    float x = smax[nb] * cs;
                    x = fmaxf(x, __shfl_xor(x, 16));
                    rm[nb] = fmaxf(x, __shfl_xor(x, 32));
                }
            };
            auto weights_and_values = [&]() {
                // ---- Pt = 2^(St*scale - ref), packed straight into B-operand order ----
                bf16x8 pt[NB];
                const bf16x8 ones = __builtin_bit_cast(bf16x8, u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u});
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
                    for (int tblk = 0; tblk < 2; ++tblk)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            pt[nb][4 * tblk + j] = (__bf16)fast_exp2(fmaf(sacc[nb][tblk][j], cs, nref[nb]));
                    // the denominator is the sum of the weights as the second product sees them (rounded)
                    lacc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pt[nb], lacc[nb], 0, 0, 0);
                }
                // ---- Vt: transpose the lane's 8 tokens x E dims, then Ot += Vt Pt ----
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    u32x4 vt;
#pragma unroll
                    for (int wp = 0; wp < 4; ++wp) {
                        const uint32_t x = tv[2 * wp][e >> 1], y = tv[2 * wp + 1][e >> 1];
                        vt[wp] = (e & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
                    }
                    const bf16x8 va = __builtin_bit_cast(bf16x8, vt);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        oacc[e][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pt[nb], oacc[e][nb], 0, 0, 0);
                }
                load_v(npg0, npg1);   // V registers are free again
                // ---- cursors: c1 becomes the tile in flight's successor (scalar work only) ----
                pb = c1b; pkt = c1kt; pnt = c1nt;
                if (i + 2 < remaining) {
                    advance(c1b, c1kt, c1nt);
                    page_ids(c1b, c1kt, npg0, npg1);
                }
            };


            if constexpr (NB == 4) {
                // ---- 64 rows per wavefront (NB = 4): one tile with the two halves of its rows interleaved ----
                // A wavefront of 64 rows is alone on its SIMD, and it issues in order: while its matrix instructions run
                // nothing else does unless the instruction stream itself puts vector work between them.  So the tile is
                // written as four phases whose order of issue is pinned step by step:
                //   1. scores of blocks 0, 1                         (matrix unit; Q operands four reads ahead)
                //   2. scores of blocks 2, 3  +  weights of 0, 1     (matrix unit and vector ALU side by side)
                //   3. values of blocks 0, 1  +  weights of 2, 3     (V is transposed block by block on the way)
                //   4. values of blocks 2, 3  +  the transposes again (cheaper than keeping 32 registers of transposed V)
                // The rescale of a late overshoot is ordinary arithmetic on the accumulators here (they are vector registers
                // in this file) inside a branch that is practically never taken.
                auto fix_refs = [&](int nb0) {
    #pragma unroll
                    for (int nb = nb0; nb < nb0 + 2; ++nb) {
                        float rm = smax[nb] * cs;
                        rm = fmaxf(rm, __shfl_xor(rm, 16));
                        rm = fmaxf(rm, __shfl_xor(rm, 32));
                        const bool fresh = mref[nb] == -INFINITY;
                        const bool late = !fresh && rm > mref[nb] + kRescaleSlack;
                        const float mnew = fmaxf(mref[nb], rm);
                        const float alpha = late ? fast_exp2(mref[nb] - mnew) : 1.f;
                        lacc[nb] *= alpha;
    #pragma unroll
                        for (int e = 0; e < E; ++e) oacc[e][nb] *= alpha;
                        set_ref(nb, (fresh || late) ? mnew : mref[nb]);
                    }
                };
                auto tile_interleaved = [&](int tb) {
                    asm volatile("" ::: "memory");   // Q comes out of LDS anew for every tile instead of staying in registers
                    constexpr int kOps = 2 * KS;     // Q operands of one half of the rows
                    constexpr int kAhead = kOps < 4 ? kOps : 4;
                    constexpr int kPer = 16 / kOps;  // weights of the other half computed per step of phase 2
                    constexpr int kPerE = 16 / E;    // ... per step of phase 3
                    const bool masked = tb + 32 > ctx - S + 1;
                    auto mask_half = [&](int nb0) {
    #pragma unroll
                        for (int nb = nb0; nb < nb0 + 2; ++nb) {
                            const int lim = ctx - S + qpos[nb];   // last key this row may see
    #pragma unroll
                            for (int tblk = 0; tblk < 2; ++tblk)
    #pragma unroll
                                for (int j = 0; j < 4; ++j)
                                    if (tb + 16 * tblk + 4 * g + j > lim) sacc[nb][tblk][j] = -INFINITY;
                        }
                    };
                    auto half_max = [&](int nb0) {
                        bool overshoot = false;
    #pragma unroll
                        for (int nb = nb0; nb < nb0 + 2; ++nb) {
                            float mx = fmaxf(fmaxf(sacc[nb][0][0], sacc[nb][0][1]), sacc[nb][0][2]);
                            mx = fmaxf(fmaxf(mx, sacc[nb][0][3]), sacc[nb][1][0]);
                            mx = fmaxf(fmaxf(mx, sacc[nb][1][1]), sacc[nb][1][2]);
                            smax[nb] = fmaxf(mx, sacc[nb][1][3]);
                            overshoot |= smax[nb] > over[nb];
                        }
                        return __any(overshoot) != 0;
                    };
                    // weight number w (0 .. 15) of the half that starts at block nb0: block nb0 + w/8, entry w%8
                    float pw[16];
                    auto weight = [&](int nb0, int w) {
                        const int nb = nb0 + (w >> 3), tblk = (w >> 2) & 1, j = w & 3;
                        pw[w] = fast_exp2(fmaf(sacc[nb][tblk][j], cs, nref[nb]));
                    };
                    bf16x8 pt[NB];
                    const bf16x8 ones = __builtin_bit_cast(bf16x8, u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u});
                    auto pack_half = [&](int nb0) {
    #pragma unroll
                        for (int w = 0; w < 16; ++w) pt[nb0 + (w >> 3)][w & 7] = (__bf16)pw[w];
                        lacc[nb0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pt[nb0], lacc[nb0], 0, 0, 0);
                        lacc[nb0 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pt[nb0 + 1], lacc[nb0 + 1], 0, 0, 0);
                    };
                    auto transposed_v = [&](int e) {
                        u32x4 vt;
    #pragma unroll
                        for (int wp = 0; wp < 4; ++wp) {
                            const uint32_t x = tv[2 * wp][e >> 1], y = tv[2 * wp + 1][e >> 1];
                            vt[wp] = (e & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
                        }
                        return __builtin_bit_cast(bf16x8, vt);
                    };
    #pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        sacc[nb][0] = f32x4{0.f, 0.f, 0.f, 0.f};
                        sacc[nb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                    }
                    // ---- phase 1 ----
                    bf16x8 qb[2 * kOps];
    #pragma unroll
                    for (int r = 0; r < kAhead; ++r) qb[r] = __builtin_bit_cast(bf16x8, qlds[r * 64]);
                    __builtin_amdgcn_sched_barrier(0);
    #pragma unroll
                    for (int r = 0; r < kOps; ++r) {
                        const int nb = r / KS, ks = r % KS;
                        sacc[nb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tk[0][ks], qb[r], sacc[nb][0], 0, 0, 0);
                        sacc[nb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tk[1][ks], qb[r], sacc[nb][1], 0, 0, 0);
                        qb[r + kAhead] = __builtin_bit_cast(bf16x8, qlds[(r + kAhead) * 64]);   // runs on into the second half
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (masked) mask_half(0);
                    if (half_max(0)) fix_refs(0);
                    // ---- phase 2 ----
    #pragma unroll
                    for (int r = 0; r < kOps; ++r) {
                        const int nb = 2 + r / KS, ks = r % KS;
                        sacc[nb][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tk[0][ks], qb[kOps + r], sacc[nb][0], 0, 0, 0);
                        sacc[nb][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tk[1][ks], qb[kOps + r], sacc[nb][1], 0, 0, 0);
                        if (r + kAhead < kOps) qb[kOps + r + kAhead] = __builtin_bit_cast(bf16x8, qlds[(kOps + r + kAhead) * 64]);
    #pragma unroll
                        for (int u = 0; u < kPer; ++u) weight(0, r * kPer + u);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    load_k(npg0, npg1);   // K registers are free again: next tile's K goes in flight
                    pack_half(0);
                    if (masked) {
                        mask_half(2);
                        // value rows beyond the context may hold anything (NaN included): zero them
    #pragma unroll
                        for (int jj = 0; jj < 8; ++jj)
                            if (tb + 16 * (jj >> 2) + 4 * g + (jj & 3) >= ctx) tv[jj] = chunk_t(0u);
                    }
                    if (half_max(2)) fix_refs(2);
                    // ---- phase 3 ----
                    __builtin_amdgcn_sched_barrier(0);
    #pragma unroll
                    for (int e = 0; e < E; ++e) {
                        const bf16x8 va = transposed_v(e);
                        oacc[e][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pt[0], oacc[e][0], 0, 0, 0);
                        oacc[e][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pt[1], oacc[e][1], 0, 0, 0);
    #pragma unroll
                        for (int u = 0; u < kPerE; ++u) weight(2, e * kPerE + u);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    pack_half(2);
                    // ---- phase 4 ----
    #pragma unroll
                    for (int e = 0; e < E; ++e) {
                        const bf16x8 va = transposed_v(e);
                        oacc[e][2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pt[2], oacc[e][2], 0, 0, 0);
                        oacc[e][3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pt[3], oacc[e][3], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    load_v(npg0, npg1);   // V registers are free again
                    // ---- cursors: c1 becomes the tile in flight's successor (scalar work only) ----
                    pb = c1b; pkt = c1kt; pnt = c1nt;
                    if (i + 2 < remaining) {
                        advance(c1b, c1kt, c1nt);
                        page_ids(c1b, c1kt, npg0, npg1);
                    }
                };

                for (int t = 0; t < n_in; ++t, ++i) tile_interleaved(32 * (kt + t));
            } else
            for (int t = 0; t < n_in;) {
                bool rescale = false;
                for (; t < n_in; ++t, ++i) {
                    if (scores(32 * (kt + t))) {
                        // rows that have not seen a key yet take the tile's maximum as their reference (their
                        // accumulators are zero); any other overshoot leaves the loop
                        float rm[NB];
                        row_max(rm);
                        bool late = false;
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            const bool fresh = mref[nb] == -INFINITY;
                            late |= !fresh && rm[nb] > mref[nb] + kRescaleSlack;
                            set_ref(nb, fresh ? rm[nb] : mref[nb]);
                        }
                        if (__any(late)) { rescale = true; break; }
                    }
                    weights_and_values();
                }
                if (rescale) {
                    float rm[NB];
                    row_max(rm);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const float mnew = fmaxf(mref[nb], rm[nb]);
                        const float alpha = (mnew == -INFINITY) ? 1.f : fast_exp2(mref[nb] - mnew);
                        lacc[nb] *= alpha;
#pragma unroll
                        for (int e = 0; e < E; ++e) oacc[e][nb] *= alpha;
                        set_ref(nb, mnew);
                    }
                    weights_and_values();
                    ++t; ++i;
                }
            }

            // ---- the sequence (or the slice) ends here.  The next sequence's Q is requested first:
            //      the memory counter retires in order, so Q can then be waited for without waiting
            //      for the acknowledgement of the stores below (after the last sequence the request
            //      repeats the current Q: unconditional requests keep the outstanding count exact). ----
            load_q(i < remaining ? pb : b);
            {
                const bool complete = item_first_kt == 0 && kt + n_in == nt;
                const size_t wslot = (size_t)(2 * wv + (first_of_slice ? 0 : 1));
                const int q4 = n & 3;
                // Stores that mix into the stream of K/V reads cost several times their share of the bytes
                // (the memory goes back and forth between reading and writing), so a partial result is
                // kept in LDS and written when the wavefront has no more K/V to read: the first sequence's
                // until then, the last one's at once - after the first one's has left the LDS.
                if (!complete && stash_slot >= 0) flush_stash(stash_slot);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    // denominator of this lane's row (already summed over the tile's 32 keys, hence over the four lanes
                    // that share the row)
                    const float l = lacc[nb][0];
                    if (complete) {
                        // Every store instruction should write whole 128-byte lines.  Lane (row n, group
                        // g) holds dims 4E g + E j + e as four chunks j of E values.  A 4x4 transpose between
                        // j and the four lanes of a quad leaves lane (n, g) with chunk 4g + n%4 of rows
                        // 4*(n/4) + j: store j then writes four complete rows of 2 D bytes.
                        const float inv = 1.f / l;
                        chunk_t c[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
#pragma unroll
                            for (int e = 0; e < E; e += 2) {
                                typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
                                const bf16x2 o2 = {(__bf16)(oacc[e][nb][j] * inv), (__bf16)(oacc[e + 1][nb][j] * inv)};
                                c[j][e >> 1] = __builtin_bit_cast(uint32_t, o2);
                            }
                        }
#pragma unroll
                        for (int stage = 1; stage <= 2; ++stage) {
                            const bool hi = (q4 & stage) != 0;
#pragma unroll
                            for (int pair = 0; pair < 2; ++pair) {
                                // stage 1 swaps chunks (0,1) and (2,3) with lane^1, stage 2 (0,2) and (1,3) with lane^2
                                const int lo_i = stage == 1 ? 2 * pair : pair, hi_i = lo_i + stage;
                                chunk_t send, recv;
#pragma unroll
                                for (int k = 0; k < E / 2; ++k) send[k] = hi ? c[lo_i][k] : c[hi_i][k];
#pragma unroll
                                for (int k = 0; k < E / 2; ++k) recv[k] = stage == 1 ? quad_xor<1>(send[k]) : quad_xor<2>(send[k]);
#pragma unroll
                                for (int k = 0; k < E / 2; ++k) {
                                    if (hi) c[lo_i][k] = recv[k]; else c[hi_i][k] = recv[k];
                                }
                            }
                        }
                        if (nparked == 0) {
#pragma unroll
                            for (int j = 0; j < 4; ++j)
#pragma unroll
                                for (int k = 0; k < E / 2; ++k) park0[(nb * 4 + j) * (E / 2) + k] = acc_park(c[j][k]);
                        } else if (kParkSlots > 1 && nparked == 1) {
#pragma unroll
                            for (int j = 0; j < 4; ++j)
#pragma unroll
                                for (int k = 0; k < E / 2; ++k) park1[(nb * 4 + j) * (E / 2) + k] = acc_park(c[j][k]);
                        } else {
                            store_rows(b, nb, c);   // no room left: written at once
                        }
                    } else {
                        // partial: each row scaled to a largest magnitude of 1 and kept as fp16, [nb][j][lane]
                        // entries of dims 4E g + E j .. + E-1 of local row 16nb + n (the merge kernel's unit of work)
                        float amax = 0.f;
#pragma unroll
                        for (int e = 0; e < E; ++e)
#pragma unroll
                            for (int j = 0; j < 4; ++j) amax = fmaxf(amax, fabsf(oacc[e][nb][j]));
                        amax = fmaxf(amax, __shfl_xor(amax, 16));
                        amax = fmaxf(amax, __shfl_xor(amax, 32));
                        const float inv = amax > 0.f ? 1.f / amax : 0.f;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            chunk_t hv;
#pragma unroll
                            for (int e = 0; e < E; e += 2) {
                                typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
                                const f16x2 h2 = {(_Float16)(oacc[e][nb][j] * inv), (_Float16)(oacc[e + 1][nb][j] * inv)};
                                hv[e >> 1] = __builtin_bit_cast(uint32_t, h2);
                            }
                            stash_o[(nb * 4 + j) * 64 + lane] = hv;
                        }
                        // l > 0 whenever the row saw a key; the merge kernel skips rows whose reference is -inf
                        if (g == 0) stash_ml[nb * 16 + n] = f32x4{mref[nb], l, l > 0.f ? amax / l : 0.f, 0.f};
                    }
                }
                if (!complete) stash_slot = (int)wslot;
                if (complete && nparked < kParkSlots) {
                    if (nparked == 0) park_b0 = b; else park_b1 = b;
                    ++nparked;
                }
            }
            store_q();
            b = pb; kt = pkt; nt = pnt;   // first tile of the next sequence (unused after the last one)
        }
        // the slice has been read: everything that waited is written now
        if (nparked > 0) flush_parked(park0, park_b0);
        if (kParkSlots > 1 && nparked > 1) flush_parked(park1, park_b1);
        if (stash_slot >= 0) flush_stash(stash_slot);
    }
    wave_trace_write(p, wv, t_start, traced_tiles, traced_parts);
}

// Joins the partials of sequences that span several wavefront slices.  Block (vh, j) looks at the
// cut between slices j-1 and j of virtual head vh (the main kernel's partition); the block of the
// first cut that falls inside a sequence merges all of that sequence's partials:
// out = sum_k 2^(m_k - m*) O_k / sum_k 2^(m_k - m*) l_k.
template <int D>
__global__ __launch_bounds__(256) void isd_attention_merge_kernel(const AttnParams p, int Wg, int rows_per_group,
                                                                  const int32_t* __restrict__ ctx_lens)
{
    __shared__ TilePlan plan;
    const int total_weight = plan_scan(p, ctx_lens, plan);
    const int total = total_weight - kSeqCost * p.B;
    if (total == 0) return;
    const int VH = p.Hkv * p.RG;
    const int vh = blockIdx.x % VH;
    const int jcut = blockIdx.x / VH + 1;          // cut = start of slice jcut
    // the main kernel's partition: slices of unequal length, and (streaming kernel) heads that alternate with the slice
    const bool balanced = p.xcd_bias != 0;
    auto slice_start = [&](int j) {
        int bb, pp;
        return slice_first_tile(p, ctx_lens, plan, total_weight, Wg, j, vh, bb, pp);
    };
    int b = 0, pre = 0;
    const int cut = slice_first_tile(p, ctx_lens, plan, total_weight, Wg, jcut, vh, b, pre);
    if (cut <= 0 || cut >= total) return;
    const int ntiles = seq_tiles(p, ctx_lens, b);
    if (cut == pre) return;                        // the cut coincides with the start of a sequence
    const int item_begin = pre, item_end = pre + ntiles;
    const int first_begin = slice_start(jcut - 1);
    if (first_begin > item_begin) return;          // an earlier cut is inside the same sequence
    // slices jcut-1 .. hold this sequence's partials, written by wavefront j*VH + vh into slot 2v if
    // the sequence is the first one of that slice (the slice starts inside it), 2v+1 if it is its last
    auto slot_of = [&](int j, int jbeg) {
        return 2 * (j * VH + (vh ^ (balanced ? 4 * (j & 1) : 0))) + (jbeg >= item_begin ? 0 : 1);
    };
    const int kvh = vh / p.RG;
    const int rowbase = (vh - kvh * p.RG) * rows_per_group;
    const int nrows = min(rows_per_group, p.M - rowbase);
    // partial layout: [slot][nb][j][lane = 16g+n] entries of E = D/16 fp16 = dims 4E g + E j .. + E-1 of local
    // row 16nb + n, each row scaled to a largest magnitude of 1; (reference exponent, denominator,
    // scale) at [slot][nb][n].  Thread (lane, j) handles one entry of every 16-row block: loads
    // contiguous across threads, one store, and one pass with a running reference keeps a single
    // round trip per partial.
    constexpr int E = D / 16;
    typedef typename LaneChunk<D>::type chunk_t;
    const chunk_t* const ws_o = static_cast<const chunk_t*>(p.ws_o);
    const int NBk = rows_per_group >> 4;
    const int j = threadIdx.x & 3, lane = threadIdx.x >> 2;
    const int n = lane & 15, g = lane >> 4;
    float acc[4][E], mrun[4], den[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
        mrun[nb] = -INFINITY;
        den[nb] = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[nb][e] = 0.f;
    }
    int knext = first_begin;                       // slice k is [kbeg, kend); slice jcut starts at the cut
    for (int k = jcut - 1; k < Wg; ++k) {
        const int kbeg = knext;
        if (kbeg >= item_end) break;
        const int kend = (k + 1 == jcut) ? cut : slice_start(k + 1);
        knext = kend;
        if (kbeg == kend) continue;
        const size_t slot = (size_t)slot_of(k, kbeg);
        f32x4 ml[4];
        chunk_t o[4];
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            if (nb < NBk) {
                const size_t sl = slot * NBk + nb;
                ml[nb] = p.ws_ml[sl * 16 + n];
                o[nb] = ws_o[(sl * 4 + j) * 64 + lane];
            }
        }
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            if (nb < NBk && ml[nb][0] != -INFINITY) {   // a part in which the row saw no key adds nothing
                const float mnew = fmaxf(mrun[nb], ml[nb][0]);
                const float aold = (mrun[nb] == -INFINITY) ? 0.f : fast_exp2(mrun[nb] - mnew);
                const float anew = fast_exp2(ml[nb][0] - mnew);
                den[nb] = den[nb] * aold + ml[nb][1] * anew;
                const float wo = anew * ml[nb][1] * ml[nb][2];
                typedef __attribute__((ext_vector_type(E))) _Float16 f16xE;
                const f16xE hv = __builtin_bit_cast(f16xE, o[nb]);
#pragma unroll
                for (int e = 0; e < E; ++e) acc[nb][e] = acc[nb][e] * aold + (float)hv[e] * wo;
                mrun[nb] = mnew;
            }
        }
    }
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
        const int lrow = 16 * nb + n;
        if (nb < NBk && lrow < nrows) {
            const float inv = 1.f / den[nb];
            const int row = rowbase + lrow;
            const int i = row / p.G, gq = row - i * p.G;
            typedef __attribute__((ext_vector_type(E))) __bf16 bf16xE;
            bf16xE ov;
#pragma unroll
            for (int e = 0; e < E; ++e) ov[e] = (__bf16)(acc[nb][e] * inv);
            uint16_t* orow = p.out + ((size_t)(b * p.S + i) * p.Hq + kvh * p.G + gq) * D;
            if (D == 128 && p.partial_layout == 1) {
                // entries of the shared-tile kernel: values 32 j + 4 g .. + 3 and 32 j + 16 + 4 g .. + 3
                typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
                *reinterpret_cast<bf16x4_t*>(orow + 32 * j + 4 * g) = bf16x4_t{ov[0], ov[1], ov[2], ov[3]};
                *reinterpret_cast<bf16x4_t*>(orow + 32 * j + 16 + 4 * g) = bf16x4_t{ov[E - 4], ov[E - 3], ov[E - 2], ov[E - 1]};
            } else {
                *reinterpret_cast<bf16xE*>(orow + 4 * E * g + E * j) = ov;
            }
        }
    }
}

// ---- plain path (fp32; small correctness configurations): one wavefront per (sequence, row, head),
// fp32 arithmetic ----
struct AttnParamsF32 {
    const void* q;
    const void* k;
    const void* v;
    const int32_t* table;
    const int32_t* ctx;
    void* out;
    int S, Hq, Hkv, G, P, max_pages, num_pages;
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
    const size_t qoff = ((size_t)(b * p.S + i) * p.Hq + h) * D;
    const int32_t* tab = p.table + (size_t)b * p.max_pages;
    float o[D];
#pragma unroll
    for (int d = 0; d < D; ++d) o[d] = 0.f;
    float m = -INFINITY, l = 0.f;
    for (int t = lane; t <= last; t += 64) {
        const int pg = min(max(tab[t / p.P], 0), p.num_pages - 1);   // never read outside the pool
        const size_t off = (size_t)pg * p.page_stride + kvh * p.head_stride + (t % p.P) * p.token_stride;
        float dot = 0.f;
#pragma unroll
        for (int d = 0; d < D; d += 4) {
            const float4 kk = *reinterpret_cast<const float4*>(static_cast<const float*>(p.k) + off + d);
            const float4 qq = *reinterpret_cast<const float4*>(static_cast<const float*>(p.q) + qoff + d);
            dot += kk.x * qq.x + kk.y * qq.y + kk.z * qq.z + kk.w * qq.w;
        }
        const float s = dot * p.scale_log2;
        const float mnew = fmaxf(m, s);
        const float alpha = fast_exp2(m - mnew);   // m = -inf on the first key gives 0
        const float pv = fast_exp2(s - mnew);
        l = l * alpha + pv;
#pragma unroll
        for (int d = 0; d < D; d += 4) {
            const float4 vv = *reinterpret_cast<const float4*>(static_cast<const float*>(p.v) + off + d);
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
        float* op = static_cast<float*>(p.out) + qoff;
#pragma unroll
        for (int d = 0; d < D; ++d) op[d] = o[d] * inv;
    }
}

// ---- host side ----------------------------------------------------------------------------

// bf16 (D = 64 or 128) runs on the MFMA kernels, fp32 on the plain one
static bool uses_mfma_path(int32_t D, int32_t dtype) { return dtype != IDLM_DTYPE_F32 && (D == 64 || D == 128); }

static bool shapes_ok(int32_t B, int32_t S, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                      int32_t max_pages, int32_t dtype, int* err)
{
    *err = IDLM_OK;
    if (dtype != IDLM_DTYPE_F32 && dtype != IDLM_DTYPE_BF16 && dtype != IDLM_DTYPE_BF16_KOP) {
        *err = IDLM_ERR_DTYPE;
        return false;
    }
    if (B < 0 || B > 65535 || S < 1 || S > 32 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || Hkv > 65535 ||
        P != 16 || max_pages < 1 || (int64_t)max_pages * P >= (1 << 30) ||
        (int64_t)B * max_pages >= (1LL << 31)) { *err = IDLM_ERR_SHAPE; return false; }
    const int G = Hq / Hkv;
    if ((D != 64 && D != 128) || (dtype == IDLM_DTYPE_BF16_KOP && D != 128)) { *err = IDLM_ERR_DTYPE; return false; }
    if (uses_mfma_path(D, dtype)) {
        if (S * G > 256) { *err = IDLM_ERR_SHAPE; return false; }
    } else {
        if (Hq > 65535) { *err = IDLM_ERR_SHAPE; return false; }
    }
    return true;
}

constexpr int kXcdBias = 48;

// More than 64 rows per KV head with 128-wide heads go to the kernel whose wavefronts share the K/V tiles through
// LDS (its tile is built for D = 128): workgroups of four wavefronts with 32 rows each, two workgroups per compute unit
static bool uses_shared_kernel(int M, int D) { return D == 128 && M > 64; }
static int default_workgroups(int M, int D) { return uses_shared_kernel(M, D) ? 2 * kDefaultWorkgroups : kDefaultWorkgroups; }

// 16-row blocks per wavefront (NB) and groups of 16*NB rows per KV head (RG) for M = S*G query rows
static void row_tiling(int M, int D, int* NB, int* RG)
{
    if (uses_shared_kernel(M, D)) { *NB = 2; *RG = M <= 128 ? 4 : 8; return; }
    if (M <= 16) { *NB = 1; *RG = 1; }
    else if (M <= 32) { *NB = 2; *RG = 1; }
    else if (M <= 64) { *NB = 4; *RG = 1; }
    else if (M <= 128) { *NB = 4; *RG = 2; }
    else { *NB = 4; *RG = 4; }
}

// Launches the main kernel of one page layout for NB sixteen-row blocks per wavefront.  The dynamic LDS
// of the larger variants is beyond the default 64 KB limit and has to be granted first.
template <int NB, int LAYOUT, int D>
static int launch_main_nb(int W, size_t shmem, hipStream_t st, const AttnParams& p, const int32_t* block_table,
                          const int32_t* ctx_lens)
{
    if (shmem > 48 * 1024 &&
        hipFuncSetAttribute(reinterpret_cast<const void*>(&isd_attention_bf16_kernel<NB, LAYOUT, D>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem) != hipSuccess) {
        (void)hipGetLastError();
        return IDLM_ERR_LAUNCH;
    }
    hipLaunchKernelGGL((isd_attention_bf16_kernel<NB, LAYOUT, D>), dim3(W), dim3(256), shmem, st, p, block_table, ctx_lens);
    return IDLM_OK;
}

template <int LAYOUT, int D>
static int launch_main(int NB, int W, size_t shmem, hipStream_t st, const AttnParams& p, const int32_t* block_table,
                       const int32_t* ctx_lens)
{
    if (NB == 1) return launch_main_nb<1, LAYOUT, D>(W, shmem, st, p, block_table, ctx_lens);
    if (NB == 2) return launch_main_nb<2, LAYOUT, D>(W, shmem, st, p, block_table, ctx_lens);
    return launch_main_nb<4, LAYOUT, D>(W, shmem, st, p, block_table, ctx_lens);
}

}  // namespace idlm

using namespace idlm;

// bytes of the partial-result slots of a grid of W workgroups: two slots of 16*NB rows per wavefront, each row
// as D fp16 values plus four fp32 row scalars
static size_t partial_slots_bytes(int NB, int W, int waves_per_workgroup, int D)
{
    const size_t slots = (size_t)2 * W * waves_per_workgroup;
    return slots * NB * (4 * 64 * (size_t)(D / 8) + 16 * sizeof(f32x4));
}

// per-wavefront trace records of the main kernel (idlm_isd_attention_wave_trace): a process-wide debug setting
static unsigned long long* g_wave_trace = nullptr;
static size_t g_wave_trace_records = 0;

extern "C" int idlm_isd_attention_wave_trace(uint64_t* records_out, size_t records)
{
    if ((records_out == nullptr) != (records == 0)) return IDLM_ERR_NULL;
    if (!aligned(records_out, 8)) return IDLM_ERR_ALIGN;
    g_wave_trace = reinterpret_cast<unsigned long long*>(records_out);
    g_wave_trace_records = records;
    return IDLM_OK;
}

extern "C" size_t idlm_isd_attention_workspace(int32_t B, int32_t S, int32_t Hq, int32_t Hkv, int32_t D,
                                               int32_t P, int32_t max_pages_per_seq, int32_t dtype,
                                               int32_t num_workgroups)
{
    int err;
    if (!shapes_ok(B, S, Hq, Hkv, D, P, max_pages_per_seq, dtype, &err)) return 0;
    if (num_workgroups < 0 || num_workgroups > kMaxWorkgroups) return 0;
    if (!uses_mfma_path(D, dtype) || B == 0) return 0;
    int NB, RG;
    const int M = S * (Hq / Hkv);
    row_tiling(M, D, &NB, &RG);
    return partial_slots_bytes(NB, num_workgroups ? num_workgroups : default_workgroups(M, D), 4, D);
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
    if (token_stride > (1 << 24)) return IDLM_ERR_SHAPE;   // lane offsets inside a page are 32-bit
    if (num_workgroups < 0 || num_workgroups > kMaxWorkgroups) return IDLM_ERR_SHAPE;
    if (B == 0) return IDLM_OK;
    if (!q || !k_cache || !v_cache || !block_table || !ctx_lens || !out) return IDLM_ERR_NULL;
    const size_t esz = dtype == IDLM_DTYPE_F32 ? 4 : 2;
    if (dtype == IDLM_DTYPE_BF16_KOP && token_stride != D) return IDLM_ERR_DTYPE;   // a page's 4 KB per head must be one block
    if (!aligned(q, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(out, 16) ||
        !aligned(block_table, 4) || !aligned(ctx_lens, 4))
        return IDLM_ERR_ALIGN;
    if ((page_stride * esz) % 16 || (head_stride * esz) % 16 || (token_stride * esz) % 16) return IDLM_ERR_ALIGN;
    if (!(scale > 0.f)) scale = 1.0f / sqrtf((float)D);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int G = Hq / Hkv;

    if (!uses_mfma_path(D, dtype)) {
        AttnParamsF32 p;
        p.q = q; p.k = k_cache; p.v = v_cache;
        p.table = block_table; p.ctx = ctx_lens; p.out = out;
        p.S = S; p.Hq = Hq; p.Hkv = Hkv; p.G = G; p.P = P; p.max_pages = max_pages_per_seq; p.num_pages = num_pages;
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

    const size_t need = idlm_isd_attention_workspace(B, S, Hq, Hkv, D, P, max_pages_per_seq, dtype, num_workgroups);
    if (!workspace || workspace_bytes < need) return IDLM_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return IDLM_ERR_ALIGN;

    // one persistent workgroup per compute unit (a workgroup holds a whole CU's registers)
    const bool shared = uses_shared_kernel(S * G, D);
    const int wpw = 4;   // wavefronts per workgroup
    int W = num_workgroups;
    if (W == 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            return IDLM_ERR_LAUNCH;
        W = cus > kDefaultWorkgroups ? kDefaultWorkgroups : cus;
        if (shared) W *= 2;
        // A batch that cannot hold more than a few tiles per wavefront gets a smaller grid: slices
        // shorter than about 16 tiles only multiply the partial results that have to be joined.  The
        // bound uses what the host knows (B and the width of the block table).
        int nb_, rg_;
        row_tiling(S * G, D, &nb_, &rg_);
        const int64_t max_tiles = (int64_t)B * ((max_pages_per_seq + 1) / 2);
        const int64_t wavefronts = (max_tiles / 16 > 0 ? max_tiles / 16 : 1) * Hkv * rg_;
        if ((wavefronts + wpw - 1) / wpw < W) W = (int)((wavefronts + wpw - 1) / wpw);
    }

    // the slots of the grid that is launched fit: it is never larger than the one the workspace was sized for
    int NB, RG_;
    row_tiling(S * G, D, &NB, &RG_);

    AttnParams p;
    p.q = static_cast<const uint16_t*>(q);
    p.k = static_cast<const uint16_t*>(k_cache);
    p.v = static_cast<const uint16_t*>(v_cache);
    p.out = static_cast<uint16_t*>(out);
    p.B = B; p.S = S; p.Hq = Hq; p.Hkv = Hkv; p.G = G; p.M = S * G; p.max_pages = max_pages_per_seq;
    p.num_pages = num_pages;
    p.RG = RG_;
    p.Mpad = 16 * NB;
    p.partial_layout = shared ? 1 : 0;
    p.wave_trace = (size_t)W * wpw <= g_wave_trace_records ? g_wave_trace : nullptr;
    {
        // With the K pages in operand order, slices on even XCDs take over 48 / 1024 of a slice from those on odd ones where the
        // mapping allows it (measured: the two kinds of wavefront then finish together; 40 .. 56 are equally good).  With
        // slot-major K pages the two kinds finish together as they are (and the kernel is not bound by the memory system alone).
        const int VHq = Hkv * p.RG, NWq = W * wpw;
        const int Wgq = NWq >= VHq ? NWq / VHq : 1;
        p.xcd_bias = (!shared && dtype == IDLM_DTYPE_BF16_KOP && VHq % 8 == 0 && NWq >= VHq && Wgq % 2 == 0) ? kXcdBias : 0;
    }
    const size_t slots = (size_t)2 * W * wpw;
    p.ws_o = workspace;
    p.ws_ml = reinterpret_cast<f32x4*>(static_cast<char*>(workspace) + slots * NB * 4 * 64 * (size_t)(D / 8));
    p.page_stride = page_stride; p.head_stride = head_stride; p.token_stride = token_stride;
    p.scale_log2 = scale * kLog2e;

    (void)hipGetLastError();
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[0]), st);
    // per wavefront: Q operands of its current sequence, one parked partial result, that partial's row scalars
    const size_t shmem = (size_t)4 * NB * ((D / 32) * 64 * 16 + 4 * 64 * (D / 8) + 16 * 16);
    const int layout = dtype == IDLM_DTYPE_BF16_KOP ? 2 : (token_stride == D ? 1 : 0);
    const int rc = shared ? launch_shared_kernel(layout, W, st, p, block_table, ctx_lens)
                 : D == 64 ? (layout == 1 ? launch_main<1, 64>(NB, W, shmem, st, p, block_table, ctx_lens)
                                          : launch_main<0, 64>(NB, W, shmem, st, p, block_table, ctx_lens))
                 : layout == 2 ? launch_main<2, 128>(NB, W, shmem, st, p, block_table, ctx_lens)
                 : layout == 1 ? launch_main<1, 128>(NB, W, shmem, st, p, block_table, ctx_lens)
                               : launch_main<0, 128>(NB, W, shmem, st, p, block_table, ctx_lens);
    if (rc != IDLM_OK) return rc;
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[1]), st);
    const int VH = Hkv * p.RG, NW = W * wpw;
    const int Wg = NW >= VH ? NW / VH : 1;   // slices per virtual head, as in the main kernel
    if (Wg > 1) {
        const dim3 mgrid((unsigned)((Wg - 1) * VH));
        if (D == 64) hipLaunchKernelGGL(isd_attention_merge_kernel<64>, mgrid, dim3(256), 0, st, p, Wg, p.Mpad, ctx_lens);
        else hipLaunchKernelGGL(isd_attention_merge_kernel<128>, mgrid, dim3(256), 0, st, p, Wg, p.Mpad, ctx_lens);
    }
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
