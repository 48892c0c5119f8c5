// Paged causal attention of one ISD step (strict causal masking, Sec. 3.1; single paged kernel over prefix +
// stride, Sec. 3.3 (1), App. D) for gfx950: the variant for MANY query rows per KV head (65 .. 256 rows = S * G,
// bf16, D = 128), where the arithmetic of a tile costs more time than its bytes.
//
// One wavefront cannot overlap its own matrix and vector work on this machine: it issues in order, and measured on
// one wavefront per SIMD a matrix instruction hides at most two vector instructions, a third one delays the next
// matrix instruction by a whole slot of 16 cycles.  The softmax between the two contractions is vector work of about
// the same length as the contractions, so with the 64 rows per wavefront of the streaming kernel the two simply add
// up.  Here a wavefront has 32 rows (NB = 2 sixteen-row blocks) and half the registers, and TWO workgroups of four
// wavefronts share a compute unit, two wavefronts per SIMD that know nothing of each other: while one is in its
// softmax the other one's matrix instructions run.  Half the rows per wavefront would double the K/V bytes that go
// from L2 into the compute unit, so the four wavefronts of a workgroup share every K/V tile through LDS:
//
//   * A workgroup-level virtual head is a KV head and a group of up to 128 query rows.  The tile list of a KV head
//     is cut into slices of equal cost exactly as in the streaming kernel, but at WORKGROUP level.
//   * K/V tiles go from global memory straight into an LDS ring of kRing tiles (global_load_lds_dwordx4: each
//     lane's 16 bytes land at LDS base + 16 * lane, no registers involved).  A tile is 16 blocks of 1 KB (K: 16-token
//     page x contraction step, in MFMA A-operand order; V: four 256-byte token rows); each wavefront requests the
//     four blocks of one 16-token page.
//   * Per tile one barrier, which runs one tile ahead: before tile i a wavefront waits until its own requests of tile
//     i + 1 have landed (the vector-memory counter retires in order; the requests of tile i + 2 stay in flight), and the
//     barrier then says that all sixteen blocks of tile i + 1 are there AND that everybody has finished tile i - 1,
//     whose ring slot takes the request of tile i + 3.  The K operands of tile i + 1 can so be read at the end of tile i.
//   * Every wavefront reads the whole tile from LDS: K operands with lane-contiguous 16-byte reads, V operands with
//     the transposing 8-byte read (ds_read_b64_tr_b16), which delivers Vt in A-operand order straight from token rows.
//     Its Q rows stay in registers for the whole sequence.
// The arithmetic of a tile (transposed formulation, lazily rescaled base-2 softmax, denominators from the matrix
// unit), the partial results of sequences that a slice boundary cuts and the kernel that joins them are those of the
// streaming kernel; a wavefront is numbered (slice, virtual head, index in the workgroup) for that.
#include "isd_attention_plan.h"

namespace idlm {

constexpr int kRing = 4;            // K/V tiles in a workgroup's LDS: one in use, up to three requested or landed
constexpr int kTileBytes = 16384;   // 32 tokens x 128 values x 2 bytes, K and V
constexpr int kSharedWaves = 4;     // wavefronts per workgroup, one per SIMD; two workgroups per compute unit

typedef __attribute__((address_space(3))) char* lds_bytes;
typedef __attribute__((ext_vector_type(4))) short s16x4;

// 16 bytes per lane from global memory (64-bit base in scalar registers + 32-bit byte offset per lane) straight
// into LDS at byte address lds_addr + 16 * lane.  The compiler does not know that this is a memory instruction: it
// neither counts it nor waits for it; dma_wait does, and everything it is ordered against is volatile as well.
__device__ __forceinline__ void dma16(uint64_t base, uint32_t lane_offset, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_offset), "s"(base) : "memory");
}
// waits until at most N vector-memory instructions of this wavefront are outstanding (they retire in order)
template <int N>
__device__ __forceinline__ void dma_wait()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
// workgroup barrier that the compiler moves no memory access across
__device__ __forceinline__ void ring_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int NB, int LAYOUT>
__global__ __launch_bounds__(256, 2) void isd_attention_shared_kernel(const AttnParams p,
                                                                   const int32_t* __restrict__ block_table,
                                                                   const int32_t* __restrict__ ctx_lens)
{
    constexpr int D = 128, KS = 4, E = 8;
    typedef u32x4 chunk_t;
    // the ring; its base is a multiple of 256 bytes, so that a token row starts at LDS bank 0
    extern __shared__ __attribute__((aligned(1024))) u32x4 smem[];   // [kRing] tiles of K (8 operand blocks of 1 KB) and V (32 rows of 256 bytes)
    __shared__ TilePlan plan;

    const unsigned long long t_start = p.wave_trace ? __builtin_amdgcn_s_memrealtime() : 0ull;
    int traced_tiles = 0, traced_parts = 0;
    const int total_weight = plan_scan(p, ctx_lens, plan);
    if (total_weight == kSeqCost * p.B) return;   // no tiles at all
    const int lane = threadIdx.x & 63;
    const int w = wave_id();
    // Workgroup-level virtual heads: (KV head, group of 64 NB rows).  The groups of one KV head and slice read the same
    // K/V at about the same time; workgroup numbers that differ by 8 run on the same XCD (one L2), so within every
    // block of 16 numbers bit 3 becomes the lowest bit of the number the work is derived from.
    const int NG = gridDim.x, Hkv = p.Hkv, RGW = p.RG / kSharedWaves;
    const int u = blockIdx.x;
    const int wg = (u | 15) < NG ? ((u & ~15) | ((u & 7) << 1) | ((u >> 3) & 1)) : u;
    const int VHW = Hkv * RGW;
    const int Wg = NG >= VHW ? NG / VHW : 1;
    const int slice = NG >= VHW ? wg / VHW : 0;
    if (slice >= Wg) return;
    // every wavefront looks the slice up for itself: the same values in all eight, so that they take the same
    // number of barriers
    int b0 = 0, pre0 = 0, b_end, pre_end;
    const int slice_begin = slice_first_tile(p, ctx_lens, plan, total_weight, Wg, slice, 0, b0, pre0);
    const int slice_end = slice_first_tile(p, ctx_lens, plan, total_weight, Wg, slice + 1, 0, b_end, pre_end);
    if (slice_begin >= slice_end) return;
    const int remaining = slice_end - slice_begin;
    const int vh0 = NG >= VHW ? wg % VHW : wg;
    const int vhstep = NG >= VHW ? VHW : NG;

    const int n = lane & 15, g = lane >> 4;
    const int S = p.S, G = p.G, M = p.M;
    const float cs = p.scale_log2;

    const lds_bytes ring = (lds_bytes)smem;
    const uint32_t ring_addr = (uint32_t)(size_t)ring;

    // ---- what this wavefront requests of every tile: four blocks of 1 KB, all of 16-token page w / 2 (one page id and
    //      one pair of page addresses per wavefront and tile) ----
    // K blocks: contraction steps 2 (w % 2) and 2 (w % 2) + 1 in A-operand order (lane (n, g): token n, values
    // 32 step + 8 g .. + 7).
    // V blocks: rows (tokens of the page) 8 (w % 2) .. + 3 and 8 (w % 2) + 4 .. + 7, 256 bytes each; lane l brings 16-byte
    // chunk (l % 16) ^ 2 (t % 8) of row t = first row + l / 16 to place l % 16 of that row.  The exclusive-or spreads the
    // rows over the LDS banks for the transposing reads below, which take 32 bytes of sixteen different rows at a time.
    const int tstride = LAYOUT == 0 ? (int)p.token_stride : D;
    const int pw = w >> 1, hw = w & 1;
    const uint32_t koff_a = LAYOUT == 2 ? (uint32_t)(lane * 16 + 1024 * (2 * hw)) : (uint32_t)(2 * (n * tstride + g * 8) + 64 * (2 * hw));
    const uint32_t koff_b = koff_a + (LAYOUT == 2 ? 1024u : 64u);
    const uint32_t voff_a = (uint32_t)(2 * ((8 * hw + g) * tstride + 8 * (n ^ (2 * g))));
    const uint32_t voff_b = (uint32_t)(2 * ((8 * hw + 4 + g) * tstride + 8 * (n ^ (2 * (4 + g)))));
    const uint32_t kdst = (uint32_t)((4 * pw + 2 * hw) * 1024), vdst = (uint32_t)(kTileBytes / 2 + (4 * pw + 2 * hw) * 1024);

    // ---- what this lane reads of every tile ----
    // K operand (page tblk, step ks): 16 bytes at (4 tblk + ks) * 1024 + 16 * lane.
    // V operand of output block e (values 16 e .. 16 e + 15 of Ot's rows), tokens 16 tblk + 4 g + j, j = 0 .. 3: the
    // transposing 8-byte read hands lane 16 g + m element j of what lane 16 g + (m / 4 + 4 j) points at, position m % 4.
    // So lane 16 g + m' (m' = q + 4 j) points at values 16 e + 4 q .. + 3 of token 16 tblk + 4 g + j, and lane 16 g + m
    // receives V[those four tokens][16 e + m]: the A operand of Ot += Vt Pt in the token order of Pt.
    // The chunk index of that address is exclusive-or'ed with the row's rotation: 32 e toggles bits 5 .. 7.
    const int vq = n & 3, vj = n >> 2;
    const uint32_t vread0 = (uint32_t)((4 * g + vj) * 256 + (((vq >> 1)) ^ (2 * ((4 * (g & 1) + vj) & 7))) * 16 + 8 * (vq & 1));

    for (int vh = vh0; vh < VHW; vh += vhstep) {
        const int kvh = vh / RGW;
        const int rowbase = ((vh - kvh * RGW) * kSharedWaves + w) * 16 * NB;
        const bool has_rows = rowbase < M;   // a wavefront without rows still requests its blocks and takes the barriers
        const size_t wv = ((size_t)slice * VHW + vh) * kSharedWaves + w;   // number of this wavefront's partial slots
        int qpos[NB];   // stride position i of this lane's row in each 16-row block
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) qpos[nb] = (rowbase + 16 * nb + n) / G;
        const uint64_t page_bytes = 2 * (uint64_t)p.page_stride;
        const uint64_t kh = reinterpret_cast<uint64_t>(p.k + kvh * p.head_stride);
        const uint64_t vhp = reinterpret_cast<uint64_t>(p.v + kvh * p.head_stride);

        auto seq_pages = [&](int b) { return (min(ctx_lens[b], p.max_pages * 16) + 15) >> 4; };
        // Id of this wavefront's page of tile kt of sequence b: page_word issues the read of the table, the request one
        // tile later is its first use.  The tile's second page is only read when it belongs to the sequence (np = its
        // number of pages); otherwise the first page is read again and masked out.
        auto page_word = [&](int b, int kt, int np) {
            const int32_t* __restrict__ tab = block_table + (size_t)b * p.max_pages;
            return tab[(pw && 2 * kt + 1 < np) ? 2 * kt + 1 : 2 * kt];
        };

        // ---- the request cursor: the next tile to be requested, the page ids of that tile and of its successor,
        //      the number of tiles requested so far ----
        int db = b0, dnt = seq_tiles(p, ctx_lens, db), dkt = slice_begin - pre0, dnp = seq_pages(db);
        int id, issued = 0, cpos = 0;
        auto cursor_step = [&]() {   // the cursor stays on the last tile of the slice
            if (cpos + 1 < remaining) {
                ++cpos;
                if (++dkt == dnt) {
                    dkt = 0;
                    do { ++db; dnt = seq_tiles(p, ctx_lens, db); } while (dnt == 0);
                    dnp = seq_pages(db);
                }
            }
        };
        // Requests this wavefront's blocks of the cursor's tile into ring slot issued % kRing and moves the cursor on.
        // Past the end of the slice the last tile is requested again (nobody reads it): the number of outstanding
        // requests is then the same for every tile, which is what dma_wait counts on.
        auto request_tile = [&]() {
            // a page id outside the pool breaks the caller's side of the contract; the read stays inside the pool anyway
            const int pg = min(max(id, 0), p.num_pages - 1);
            const uint32_t dst = ring_addr + (uint32_t)((issued & (kRing - 1)) * kTileBytes);
            const uint64_t pb = (uint64_t)(uint32_t)pg * page_bytes;
            dma16(kh + pb, koff_a, dst + kdst);
            dma16(kh + pb, koff_b, dst + kdst + 1024);
            dma16(vhp + pb, voff_a, dst + vdst);
            dma16(vhp + pb, voff_b, dst + vdst + 1024);
            ++issued;
            cursor_step();
        };
        // the read of the cursor's page id
        auto next_ids = [&]() { id = page_word(db, dkt, dnp); };
        static_assert((kRing & (kRing - 1)) == 0, "ring slots are taken modulo a power of two");
        next_ids();
#pragma unroll
        for (int r = 0; r < kRing - 1; ++r) {
            request_tile();
            next_ids();
        }

        // ---- Q rows of sequence bq for this lane (row n of each 16-row block, values 32 s + 8 g .. + 7), the B operands
        //      of St for the whole sequence; rows past the stride's last one are zero ----
        bf16x8 qreg[NB][KS];
        auto load_q = [&](int bq) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int row = rowbase + 16 * nb + n;
                const bool valid = row < M;
                const int qi = valid ? qpos[nb] : S - 1;
                const int gq = valid ? row - qpos[nb] * G : G - 1;
                const uint16_t* qp = p.q + ((size_t)(bq * S + qi) * p.Hq + kvh * G + gq) * D + g * 8;
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    const u32x4 x = *reinterpret_cast<const u32x4*>(qp + 32 * s);
                    qreg[nb][s] = __builtin_bit_cast(bf16x8, valid ? x : u32x4{0u, 0u, 0u, 0u});
                }
            }
        };

        int b = b0, nt = seq_tiles(p, ctx_lens, b), kt = slice_begin - pre0;
        if (has_rows) load_q(b);
        // K operands of the next tile (page tblk, step ks at [2 ks + tblk]): read from LDS one tile ahead, as soon as a
        // barrier has said that the tile is there, so that a tile starts with its first contraction
        bf16x8 kop[2 * KS];
        auto read_k = [&](int slot) {
            const lds_bytes kl = ring + slot * kTileBytes + lane * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int tblk = 0; tblk < 2; ++tblk)
                    kop[2 * ks + tblk] = __builtin_bit_cast(
                        bf16x8, *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(kl + (4 * tblk + ks) * 1024));
        };
        dma_wait<4 * (kRing - 2)>();   // tile 0 is there
        ring_barrier();
        if (has_rows) read_k(0);

        traced_tiles += remaining;
        for (int i = 0; i < remaining;) {
            ++traced_parts;
            // ---- a sequence starts (or continues from an earlier slice) ----
            const int n_in = min(nt - kt, remaining - i);   // tiles of this sequence inside the slice
            const bool first_of_slice = i == 0;
            const int ctx = min(ctx_lens[b], p.max_pages * 16);
            const int item_first_kt = kt;
            // Per sixteen-row block: output accumulators (lane (n, g), block e, entry j: value 16 e + 4 g + j of row n),
            // the denominators (accumulated by the matrix unit as the product of the weights with a matrix of ones), the
            // reference exponent, and two values derived from it that the tile uses in its place: the score above which
            // the reference has to be raised, and the addend of the exponent.
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

            // one tile from ring slot `slot`
            auto tile = [&](int tb, int slot) {
                const lds_bytes vl = ring + (slot * kTileBytes + kTileBytes / 2);
                u32x4 vt[E];
                __builtin_amdgcn_sched_barrier(0);
                // ---- St = K Qt ----
                f32x4 sacc[NB][2];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    sacc[nb][0] = f32x4{0.f, 0.f, 0.f, 0.f};
                    sacc[nb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                    for (int tblk = 0; tblk < 2; ++tblk) {
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            sacc[nb][tblk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[2 * ks + tblk], qreg[nb][ks], sacc[nb][tblk], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                // The next request goes out while the matrix unit works on the scores (scalar arithmetic and four
                // request instructions); then the V operands, which are on their way while the softmax runs.  V operand e:
                // tokens 16 tblk + 4 g + j of values 16 e + n.
                request_tile();
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const lds_bytes ve = vl + (vread0 ^ (uint32_t)(32 * e));
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)ve);
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(ve + 4096));
                    vt[e] = __builtin_bit_cast(u32x4, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
                __builtin_amdgcn_sched_barrier(0);
                // ---- causal mask and end of context ----
                // (the s_nop keeps the branches branches: as selects this work would run on every tile)
                const bool masked = tb + 32 > ctx - S + 1;
                if (masked) {
                    asm volatile("s_nop 0");
                    const int t0 = tb + 4 * opaque(g);   // first of this lane's tokens; hidden, or it is computed on every tile
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const int lim = ctx - S + qpos[nb];   // last key this row may see
#pragma unroll
                        for (int tblk = 0; tblk < 2; ++tblk)
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                if (t0 + 16 * tblk + j > lim) sacc[nb][tblk][j] = -INFINITY;
                    }
                }
                // ---- reference exponents: raised (and the accumulators rescaled) only when a score overshoots the
                //      running reference by kRescaleSlack powers of two, or for a row's first key ----
                float smax[NB];
                bool overshoot = false;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    float mx = fmaxf(fmaxf(sacc[nb][0][0], sacc[nb][0][1]), sacc[nb][0][2]);
                    mx = fmaxf(fmaxf(mx, sacc[nb][0][3]), sacc[nb][1][0]);
                    mx = fmaxf(fmaxf(mx, sacc[nb][1][1]), sacc[nb][1][2]);
                    smax[nb] = fmaxf(mx, sacc[nb][1][3]);
                    overshoot |= smax[nb] > over[nb];
                }
                if (__any(overshoot)) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
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
                }
                // ---- Pt = 2^(St*scale - ref), packed straight into B-operand order; the denominator is the sum of
                //      the weights as the second product sees them (rounded) ----
                bf16x8 pt[NB];
                const bf16x8 ones = __builtin_bit_cast(bf16x8, u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u});
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
                    for (int tblk = 0; tblk < 2; ++tblk)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            pt[nb][4 * tblk + j] = (__bf16)fast_exp2(fmaf(sacc[nb][tblk][j], cs, nref[nb]));
                    lacc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pt[nb], lacc[nb], 0, 0, 0);
                }
                // ---- Ot += Vt Pt.  Value rows beyond the context may hold anything (NaN included): on the tiles that
                //      reach the end of the context their entries are cleared (entry 4 tblk + j = token 16 tblk + 4 g + j) ----
                if (masked) {
                    asm volatile("s_nop 0");
                    u32x4 keep;
                    const int t0 = tb + 4 * opaque(g);
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const int tok = t0 + 16 * (d >> 1) + 2 * (d & 1);
                        keep[d] = (tok < ctx ? 0xffffu : 0u) | (tok + 1 < ctx ? 0xffff0000u : 0u);
                    }
#pragma unroll
                    for (int e = 0; e < E; ++e) vt[e] &= keep;
                }
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const bf16x8 va = __builtin_bit_cast(bf16x8, vt[e]);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        oacc[e][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pt[nb], oacc[e][nb], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                read_k((slot + 1) & (kRing - 1));   // the barrier before this tile has said that the next one is there
            };

            for (int t = 0; t < n_in; ++t, ++i) {
                dma_wait<4 * (kRing - 3)>();   // this wavefront's blocks of tile i + 1 have landed
                ring_barrier();                // everybody's have, and everybody has finished tile i - 1, whose slot takes
                if (has_rows) tile(32 * (kt + t), i & (kRing - 1));   // tile i + kRing - 1 (requested inside)
                else request_tile();
                next_ids();                    // first used behind the next barrier
            }

            // ---- the sequence (or the slice) ends here ----
            const bool last = i >= remaining;
            int nb_ = b, nkt = kt + n_in, nnt = nt;
            if (!last) {
                nkt = 0;
                do { ++nb_; nnt = seq_tiles(p, ctx_lens, nb_); } while (nnt == 0);
            }
            if (has_rows) {
                const bool complete = item_first_kt == 0 && kt + n_in == nt;
                const size_t wslot = 2 * wv + (first_of_slice ? 0 : 1);
                // the next sequence's Q is requested before the stores below: the memory counter retires in order
                const int bcur = b;
                if (!last) load_q(nb_);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const float l = lacc[nb][0];   // denominator of this lane's row (summed over the tile's 32 keys by the matrix unit)
                    if (complete) {
                        const int row = rowbase + 16 * nb + n;
                        if (row < M) {
                            const float inv = 1.f / l;
                            uint16_t* op = p.out + ((size_t)(bcur * S + qpos[nb]) * p.Hq + kvh * G + (row - qpos[nb] * G)) * D + 4 * g;
#pragma unroll
                            for (int e = 0; e < E; ++e) {
                                typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
                                const bf16x4_t o4 = {(__bf16)(oacc[e][nb][0] * inv), (__bf16)(oacc[e][nb][1] * inv),
                                                     (__bf16)(oacc[e][nb][2] * inv), (__bf16)(oacc[e][nb][3] * inv)};
                                *reinterpret_cast<bf16x4_t*>(op + 16 * e) = o4;
                            }
                        }
                    } else {
                        // partial: each row scaled to a largest magnitude of 1 and kept as fp16; entry [nb][j][lane] holds
                        // values 32 j + 4 g .. + 3 and 32 j + 16 + 4 g .. + 3 of local row 16 nb + n (partial layout 1 of
                        // the kernel that joins them)
                        float amax = 0.f;
#pragma unroll
                        for (int e = 0; e < E; ++e)
#pragma unroll
                            for (int j = 0; j < 4; ++j) amax = fmaxf(amax, fabsf(oacc[e][nb][j]));
                        amax = fmaxf(amax, __shfl_xor(amax, 16));
                        amax = fmaxf(amax, __shfl_xor(amax, 32));
                        const float inv = amax > 0.f ? 1.f / amax : 0.f;
                        chunk_t* dst = static_cast<chunk_t*>(p.ws_o) + wslot * (NB * 4 * 64) + lane;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            chunk_t hv;
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
                                const int e = 2 * j + (k >> 1), x = 2 * (k & 1);
                                const f16x2 h2 = {(_Float16)(oacc[e][nb][x] * inv), (_Float16)(oacc[e][nb][x + 1] * inv)};
                                hv[k] = __builtin_bit_cast(uint32_t, h2);
                            }
                            dst[(nb * 4 + j) * 64] = hv;
                        }
                        // l > 0 whenever the row saw a key; the merge kernel skips rows whose reference is -inf
                        if (g == 0) p.ws_ml[wslot * (NB * 16) + nb * 16 + n] = f32x4{mref[nb], l, l > 0.f ? amax / l : 0.f, 0.f};
                    }
                }
            }
            b = nb_; kt = nkt; nt = nnt;
        }
        // The slice has been read.  The requests that ran past its end are waited for before anybody requests into the
        // ring again (or the workgroup gives its LDS back).
        dma_wait<0>();
        ring_barrier();
    }
    wave_trace_write(p, (int)blockIdx.x * kSharedWaves + w, t_start, traced_tiles, traced_parts);
}

// ---- host side ----

template <int NB, int LAYOUT>
static int launch_nb(int W, hipStream_t st, const AttnParams& p, const int32_t* block_table, const int32_t* ctx_lens)
{
    const size_t shmem = shared_kernel_lds_bytes();
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&isd_attention_shared_kernel<NB, LAYOUT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem) != hipSuccess) {
        (void)hipGetLastError();
        return IDLM_ERR_LAUNCH;
    }
    hipLaunchKernelGGL((isd_attention_shared_kernel<NB, LAYOUT>), dim3(W), dim3(64 * kSharedWaves), shmem, st, p, block_table,
                       ctx_lens);
    return IDLM_OK;
}

size_t shared_kernel_lds_bytes() { return (size_t)kRing * kTileBytes; }

int launch_shared_kernel(int layout, int W, hipStream_t st, const AttnParams& p, const int32_t* block_table,
                         const int32_t* ctx_lens)
{
    return layout == 2 ? launch_nb<2, 2>(W, st, p, block_table, ctx_lens)
         : layout == 1 ? launch_nb<2, 1>(W, st, p, block_table, ctx_lens)
                       : launch_nb<2, 0>(W, st, p, block_table, ctx_lens);
}

}  // namespace idlm
