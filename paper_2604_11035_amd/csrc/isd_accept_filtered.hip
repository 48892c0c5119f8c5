// Acceptance under the filtered sampling distribution of the paper's runs (App. H, ISD
// configuration table: temperature, top_k 50, top_p 0.95) with point-mass proposals, or with
// drafts drawn from the filtered distribution of the row that proposed them (Alg. 1 as printed,
// Sec. 3.2; that row's candidates are kept from the call that processed it, 512 bytes per row,
// so the proposer's logits are never read again):
//   1. one streaming pass per logit row that keeps the exact top_k (<= 64) elements, in
//      descending order, equal values by ascending index;
//   2. per sequence (one wavefront per row, lane = candidate): temperature, top-p cut, renormalisation,
//      accept tests, and every draw (fresh token, sampled proposals) as a Gumbel-max over the
//      at most 64 surviving candidates - no second pass over the logits.
// HBM-bound: one read of the logits.
#include "isd_accept_common.h"

namespace idlm {

constexpr int kTopKMax = 64;       // candidates per row (one per lane of the second kernel)
constexpr int kBufCap = 2048;      // candidate buffer of the streaming pass (keys in LDS)

// (value, index) as one 64-bit key whose unsigned order is "larger value first, then lower index".
__device__ __forceinline__ unsigned long long cand_key(float v, int idx)
{
    const uint32_t bits = __float_as_uint(v);
    const uint32_t ordered = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
    return ((unsigned long long)ordered << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)idx);
}
__device__ __forceinline__ float key_value(unsigned long long key)
{
    const uint32_t o = (uint32_t)(key >> 32);
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}
__device__ __forceinline__ int key_index(unsigned long long key) { return (int)(0xFFFFFFFFu - (uint32_t)key); }

// Sorts buf[0..n) in descending order (bitonic network, 256 threads); n is a power of two that
// covers the entries in use, the others are 0.  All threads of the block call it.
__device__ void sort_buffer_desc(unsigned long long* buf, int n)
{
    const int tid = threadIdx.x;
    for (int k = 2; k <= n; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < n / 2; t += 256) {
                const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));   // lower partner: bit j clear
                const int l = i | j;
                const bool desc = (i & k) == 0;
                const unsigned long long a = buf[i], b = buf[l];
                if ((a < b) == desc) { buf[i] = b; buf[l] = a; }
            }
            __syncthreads();
        }
}

// One workgroup per row, exact top K as sorted keys.
//
// Fast path (rows in no particular order).  The first batch gives a threshold without sorting
// anything: every thread takes the maximum of its 64 elements, and the K-th largest of the 256
// thread maxima is a lower bound of the row's K-th largest element (the K maxima above it are K
// elements of the row).  About K/256 of the threads, hence a fraction ~ K/(256*64) of the elements,
// reach it: a few hundred of a 150k row.  The row is then streamed without any barrier; whoever
// holds such an element appends its key to the buffer through one LDS atomic.  One sort at the end.
//
// If the buffer overflows (ascending rows, long runs of equal values), the row is done again by
// the robust path: elements above the current threshold (the K-th largest key seen so far, 0
// before K elements have been seen) are appended batch by batch; when the buffer cannot take the
// next batch it is sorted and cut back to its K largest, which raises the threshold.
template <int UNROLL, bool BF16>
__global__ __launch_bounds__(256) void isd_row_topk_kernel(const void* __restrict__ logits, int V, int K,
                                                           unsigned long long* __restrict__ out_keys)
{
    typedef LogitVec<BF16> LV;
    typedef typename LV::raw raw_t;
    constexpr int N = LV::N;
    __shared__ unsigned long long buf[kBufCap];
    __shared__ float s_max[256];
    __shared__ int s_count, s_want, s_overflow;
    __shared__ unsigned long long s_thr;
    __shared__ float s_first;
    const int row = blockIdx.x, tid = threadIdx.x;
    const raw_t* __restrict__ pv = reinterpret_cast<const raw_t*>(static_cast<const char*>(logits) + (size_t)row * V * (16 / N));
    const int fend = V / N;
    const raw_t none = LV::minus_inf();
    for (int t = tid; t < kBufCap; t += 256) buf[t] = 0ull;
    if (tid == 0) { s_count = 0; s_thr = 0ull; s_overflow = 0; s_first = -INFINITY; }

    auto prune = [&]() {           // every thread; buffer -> its K largest, threshold raised
        const int used = s_count;
        int n2 = 64;
        while (n2 < used) n2 <<= 1;
        sort_buffer_desc(buf, n2);
        const int kept = min(used, K);
        for (int t = kept + tid; t < n2; t += 256) buf[t] = 0ull;
        if (tid == 0) {
            s_count = kept;
            s_thr = kept == K ? buf[K - 1] : 0ull;
        }
        __syncthreads();
    };
    auto write_out = [&]() {
        if (tid < kTopKMax) out_keys[(size_t)row * kTopKMax + tid] = tid < s_count ? buf[tid] : 0ull;
    };

    // ---- fast path ----
    {
        raw_t v[UNROLL];
        float tmax = -INFINITY;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int f = u * 256 + tid;
            v[u] = f < fend ? __builtin_nontemporal_load(pv + f) : none;
            float e[N];
            LV::unpack(v[u], e);
#pragma unroll
            for (int i = 0; i < N; ++i) tmax = fmaxf(tmax, e[i]);
        }
        s_max[tid] = tmax;
        __syncthreads();
        // position of this thread's maximum among the 256 (equal values: lower thread first), by counting
        int rank = 0;
        for (int j = 0; j < 256; ++j) {
            const float o = s_max[j];
            rank += (o > tmax || (o == tmax && j < tid)) ? 1 : 0;
        }
        if (rank == K - 1) s_first = tmax;
        __syncthreads();
        const float thr_v = s_first;
        const volatile int* overflow = &s_overflow;
        for (int base = 0; base < fend; base += UNROLL * 256) {
            if (base) {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) {
                    const int f = base + u * 256 + tid;
                    v[u] = f < fend ? __builtin_nontemporal_load(pv + f) : none;
                }
            }
            int mine = 0;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const bool in_row = base + u * 256 + tid < fend;
                float e[N];
                LV::unpack(v[u], e);
#pragma unroll
                for (int i = 0; i < N; ++i) mine += (in_row && e[i] >= thr_v) ? 1 : 0;
            }
            if (mine) {
                int slot = atomicAdd(&s_count, mine);
                if (slot + mine <= kBufCap) {
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) {
                        const int f = base + u * 256 + tid;
                        if (f < fend) {
                            // unpacked again from the loaded vector: keeping the counting loop's values alive
                            // until here would double the registers of the bf16 form
                            asm volatile("" : "+v"(v[u]));
                            float e[N];
                            LV::unpack(v[u], e);
#pragma unroll
                            for (int i = 0; i < N; ++i)
                                if (e[i] >= thr_v) buf[slot++] = cand_key(e[i], f * N + i);
                        }
                    }
                } else {
                    s_overflow = 1;
                }
            }
            if (*overflow) break;          // someone ran out of room: the rest of this pass is void
        }
        __syncthreads();
        if (!s_overflow) {
            prune();
            write_out();
            return;
        }
        __syncthreads();
        for (int t = tid; t < kBufCap; t += 256) buf[t] = 0ull;
        if (tid == 0) { s_count = 0; s_thr = 0ull; }
        __syncthreads();
    }

    // ---- robust path (rare; four loads at a time keeps its registers below the fast path's) ----
    constexpr int RU = 4;
    for (int base = 0; base < fend; base += RU * 256) {
        raw_t v[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            const int f = base + u * 256 + tid;
            v[u] = f < fend ? __builtin_nontemporal_load(pv + f) : none;
        }
        const unsigned long long thr = s_thr;
        const float thr_v = thr ? key_value(thr) : -INFINITY;
        // candidates by value alone (elements beyond the row read as -inf and never pass once a
        // threshold exists; before that the exact test below drops them); the exact (value, index)
        // test is only paid by the few that get this far
        int mine = 0;
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            float e[N];
            LV::unpack(v[u], e);
#pragma unroll
            for (int i = 0; i < N; ++i) mine += (e[i] >= thr_v) ? 1 : 0;
        }
        if (tid == 0) s_want = 0;
        if (!__syncthreads_or(mine)) continue;       // nothing in this batch reaches the threshold
        if (mine) atomicAdd(&s_want, mine);
        __syncthreads();
        if (s_count + s_want <= kBufCap) {
            // the common case: everything that passes fits
            if (mine) {
                int exact = 0;
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const int f = base + u * 256 + tid;
                    if (f < fend) {
                        float e[N];
                        LV::unpack(v[u], e);
#pragma unroll
                        for (int i = 0; i < N; ++i)
                            exact += (e[i] >= thr_v && cand_key(e[i], f * N + i) > thr) ? 1 : 0;
                    }
                }
                int slot = exact ? atomicAdd(&s_count, exact) : 0;
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const int f = base + u * 256 + tid;
                    if (f < fend) {
                        float e[N];
                        LV::unpack(v[u], e);
#pragma unroll
                        for (int i = 0; i < N; ++i) {
                            const unsigned long long key = cand_key(e[i], f * N + i);
                            if (e[i] >= thr_v && key > thr) buf[slot++] = key;
                        }
                    }
                }
            }
            __syncthreads();
        } else {
            // too many for the buffer (the first batch of a row, or adversarially ordered data): 1024
            // elements at a time, cutting the buffer back as soon as it holds 1024 keys
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                float e[N];
                LV::unpack(v[u], e);
                const int f = base + u * 256 + tid;
#pragma unroll
                for (int h = 0; h < N / 4; ++h) {     // 1024 elements per round
                    if (s_count >= 1024) prune();
                    else __syncthreads();
                    const unsigned long long t2 = s_thr;
                    if (f < fend) {
#pragma unroll
                        for (int i = 4 * h; i < 4 * h + 4; ++i) {
                            const unsigned long long key = cand_key(e[i], f * N + i);
                            if (key > t2) buf[atomicAdd(&s_count, 1)] = key;
                        }
                    }
                    __syncthreads();
                }
            }
        }
    }
    prune();
    write_out();
}

struct FilteredParams {
    const int32_t* draft_tokens;
    const unsigned long long* cand;     // [rows][64] keys in descending order, 0 = none
    const unsigned long long* q_cand;   // the same record of the step that proposed the drafts, or null (point mass)
    const int32_t* q_row;               // [B] row of q_cand that proposed draft 0
    float* draft_q;
    int32_t* accept_len;
    int32_t* new_tokens;
    const int32_t* n_draft;
    const uint8_t* greedy;
    float* draft_probs;
    int32_t* kept;
    uint2 key;
    int S, V, n_draft_uniform, sample_proposals;
    uint32_t rng_offset;
    float k;              // log2(e) / T
    float one_plus_tau;
    float top_p;
};

// The filtered distribution of one row over the wavefront's lanes: lane c holds candidate c.
// Returns the number of candidates kept; pf = renormalised probability (0 for lanes not kept).
__device__ __forceinline__ int filtered_row(const FilteredParams& p, const unsigned long long* __restrict__ cand, int row,
                                            int lane, int& idx, float& pf)
{
    const unsigned long long key = cand[(size_t)row * kTopKMax + lane];
    const int n = __builtin_popcountll(__ballot(key != 0ull));
    idx = key ? key_index(key) : -1;
    const float val = key ? key_value(key) : -INFINITY;
    const float top = __shfl(val, 0);
    const float w = key ? fast_exp2((val - top) * p.k) : 0.f;
    float cum = w;                          // inclusive prefix sum over the lanes
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float y = __shfl_up(cum, off);
        if (lane >= off) cum += y;
    }
    const float total = __shfl(cum, 63);
    const unsigned long long reached = __ballot(lane < n && cum >= p.top_p * total);
    const int keep = reached ? min(n, (int)__builtin_ctzll(reached) + 1) : n;
    const float s2 = __shfl(cum, keep - 1);
    pf = lane < keep ? w / s2 : 0.f;
    return keep;
}

// Gumbel-max draw among the candidates of a row with weight > 0 (noise of the candidates'
// vocabulary ids): argmax of ln(weight) + g; returns -1 if nothing qualifies.
__device__ __forceinline__ int draw(const FilteredParams& p, int row, int stream, int idx, float weight)
{
    float score = -INFINITY;
    if (weight > 0.f) {
        const uint4 w = philox4x32_10(make_uint4((uint32_t)idx >> 2, (uint32_t)row, (uint32_t)stream, p.rng_offset), p.key);
        const uint32_t word = (idx & 3) == 0 ? w.x : (idx & 3) == 1 ? w.y : (idx & 3) == 2 ? w.z : w.w;
        score = logf(weight) + gumbel(word);
    }
    int best = score > -INFINITY ? idx : INT_MAX;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float s2 = __shfl_xor(score, off);
        const int i2 = __shfl_xor(best, off);
        combine_best(score, best, s2, i2);
    }
    return best == INT_MAX ? -1 : best;
}

constexpr int kChainWaves = 8;     // wavefronts per sequence; rows are dealt out to them in turn

__global__ __launch_bounds__(64 * kChainWaves) void isd_accept_filtered_chain_kernel(const FilteredParams p)
{
    __shared__ int s_ok[64];        // accept decision of every draft (S <= 64)
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int S = p.S, ncol = S - 1;
    const bool is_greedy = p.greedy ? (p.greedy[b] != 0) : false;
    int D = p.n_draft ? p.n_draft[b] : p.n_draft_uniform;
    D = max(0, min(D, S - 1));
    const bool has_q = p.q_cand != nullptr;
    // first proposing row, kept inside the sequence's S rows whatever the array holds
    const int q0 = has_q ? b * S + max(0, min(p.q_row[b], S - D)) : 0;

    // accept tests of the drafts, every row on its own
    for (int j = wave; j < S; j += kChainWaves) {
        const int row = b * S + j;
        if (j >= D && !p.kept) {        // nothing of this row is needed here
            if (j < ncol && lane == 0) {
                if (p.draft_probs) p.draft_probs[(size_t)b * ncol + j] = 0.f;
                if (p.draft_q) p.draft_q[(size_t)b * ncol + j] = 0.f;
            }
            continue;
        }
        int idx;
        float pf;
        const int keep = filtered_row(p, p.cand, row, lane, idx, pf);
        if (p.kept && lane == 0) p.kept[row] = keep;
        if (j < ncol) {
            float px = 0.f, qx = 0.f;
            bool ok = true;
            if (j < D) {
                const int x = p.draft_tokens[(size_t)b * ncol + j];
                const unsigned long long hit = __ballot(idx == x && pf > 0.f);
                px = hit ? __shfl(pf, (int)__builtin_ctzll(hit)) : 0.f;
                qx = 1.f;
                if (has_q) {
                    int qi;
                    float qf;
                    filtered_row(p, p.q_cand, q0 + j, lane, qi, qf);
                    const unsigned long long qhit = __ballot(qi == x && qf > 0.f);
                    qx = qhit ? __shfl(qf, (int)__builtin_ctzll(qhit)) : 0.f;
                }
                if (is_greedy) {
                    ok = (x == __shfl(idx, 0));
                } else {
                    const uint4 w = philox4x32_10(make_uint4(0u, (uint32_t)row, 0u, p.rng_offset), p.key);
                    // a draft outside the proposer's support cannot have been drawn from it: the
                    // ratio is taken as infinite if the anchor keeps the token, as zero otherwise
                    const float thr = qx > 0.f ? fminf(1.f, p.one_plus_tau * px / qx) : (px > 0.f ? 1.f : 0.f);
                    ok = unit_uniform(w.x) < thr;
                }
                if (lane == 0) s_ok[j] = ok ? 1 : 0;
            }
            if (lane == 0) {
                if (p.draft_probs) p.draft_probs[(size_t)b * ncol + j] = px;
                if (p.draft_q) p.draft_q[(size_t)b * ncol + j] = qx;
            }
        }
    }
    __syncthreads();
    int r = D;                      // first failure
    for (int j = D - 1; j >= 0; --j)
        if (!s_ok[j]) r = j;
    if (threadIdx.x == 0) p.accept_len[b] = r;

    // tokens
    for (int j = wave; j < S; j += kChainWaves) {
        const int row = b * S + j;
        int tok;
        if (j < r) tok = p.draft_tokens[(size_t)b * ncol + j];
        else if (j > r && j <= D) tok = -1;
        else if (is_greedy || (j != r && !p.sample_proposals)) {
            tok = key_index(p.cand[(size_t)row * kTopKMax]);        // the arg-max: first key of the row
        } else {
            int idx;
            float pf;
            filtered_row(p, p.cand, row, lane, idx, pf);
            tok = __shfl(idx, 0);
            if (j == r) {
                // bonus token: a draw from pf; after a rejection: from max(0, pf - qf)
                // (point mass: pf without the draft)
                float weight = pf;
                if (r < D && has_q) {
                    int qi;
                    float qf;
                    filtered_row(p, p.q_cand, q0 + r, lane, qi, qf);
                    float mine = 0.f;
                    for (int t = 0; t < kTopKMax; ++t) {
                        const int id = __shfl(qi, t);
                        const float v = __shfl(qf, t);
                        if (id == idx && id >= 0) mine = v;
                    }
                    weight = pf - mine;
                } else if (r < D) {
                    if (idx == p.draft_tokens[(size_t)b * ncol + r]) weight = 0.f;
                }
                const int got = draw(p, row, 1, idx, weight);
                if (got >= 0) tok = got;
            } else {
                const int got = draw(p, row, 2, idx, pf);
                if (got >= 0) tok = got;
            }
        }
        if (lane == 0) p.new_tokens[row] = tok;
    }
}

}  // namespace idlm

using namespace idlm;

extern "C" size_t idlm_isd_accept_filtered_workspace(int32_t B, int32_t S, int32_t V)
{
    if (B < 0 || S < 1 || S > 64 || V < 4 || (V & 3) || (int64_t)B * S >= INT32_MAX) return 0;
    if (B == 0) return 0;
    return align256((size_t)B * S * kTopKMax * sizeof(unsigned long long));
}

static int accept_filtered_impl(const void* logits, int32_t logits_dtype, const int32_t* draft_tokens, const uint64_t* q_cand,
                                const int32_t* q_row, uint64_t rng_seed, int32_t* accept_len, int32_t* new_tokens,
                                int32_t B, int32_t S, int32_t V, int32_t n_draft_uniform, const int32_t* n_draft,
                                const uint8_t* greedy, uint32_t rng_offset, float temperature, float tau, int32_t top_k,
                                float top_p, int32_t sample_proposals, float* draft_probs, float* draft_q, int32_t* kept,
                                uint64_t* cand_out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (logits_dtype != IDLM_DTYPE_F32 && logits_dtype != IDLM_DTYPE_BF16) return IDLM_ERR_DTYPE;
    const int per_vec = logits_dtype == IDLM_DTYPE_BF16 ? 8 : 4;     // elements per 16-byte load
    if (B < 0 || S < 1 || S > 64 || V < per_vec || (V % per_vec) || (int64_t)B * S >= INT32_MAX) return IDLM_ERR_SHAPE;
    if (!n_draft && (n_draft_uniform < 0 || n_draft_uniform > S - 1)) return IDLM_ERR_SHAPE;
    if (!(temperature > 0.f) || !(tau >= 0.f) || !(temperature < INFINITY) || !(tau < INFINITY)) return IDLM_ERR_SHAPE;
    if (top_k < 1 || top_k > kTopKMax || !(top_p > 0.f) || !(top_p <= 1.f)) return IDLM_ERR_SHAPE;
    if (B == 0) return IDLM_OK;
    if (!logits || !accept_len || !new_tokens) return IDLM_ERR_NULL;
    if (S > 1 && !draft_tokens) return IDLM_ERR_NULL;
    if (q_cand && !q_row) return IDLM_ERR_NULL;
    if (!aligned(logits, 16) || !aligned(q_cand, 8) || !aligned(cand_out, 8)) return IDLM_ERR_ALIGN;
    if (q_cand && q_cand == cand_out) return IDLM_ERR_SHAPE;     // the proposer's record is read while this one is written
    unsigned long long* cand = reinterpret_cast<unsigned long long*>(cand_out);
    if (!cand) {
        const size_t need = idlm_isd_accept_filtered_workspace(B, S, V);
        if (!workspace || workspace_bytes < need) return IDLM_ERR_WORKSPACE;
        if (!aligned(workspace, 256)) return IDLM_ERR_ALIGN;
        cand = static_cast<unsigned long long*>(workspace);
    }

    FilteredParams p;
    p.draft_tokens = draft_tokens;
    p.cand = cand;
    p.q_cand = reinterpret_cast<const unsigned long long*>(q_cand);
    p.q_row = q_row;
    p.draft_q = draft_q;
    p.accept_len = accept_len; p.new_tokens = new_tokens; p.n_draft = n_draft; p.greedy = greedy;
    p.draft_probs = draft_probs; p.kept = kept;
    p.key = make_uint2((uint32_t)rng_seed, (uint32_t)(rng_seed >> 32));
    p.S = S; p.V = V; p.n_draft_uniform = n_draft_uniform; p.sample_proposals = sample_proposals ? 1 : 0;
    p.rng_offset = rng_offset;
    p.k = kLog2e / temperature;
    p.one_plus_tau = 1.f + tau;
    p.top_p = top_p;
    hipStream_t st = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    if (logits_dtype == IDLM_DTYPE_BF16)
        hipLaunchKernelGGL((isd_row_topk_kernel<16, true>), dim3((unsigned)(B * S)), dim3(256), 0, st, logits, V,
                           top_k < V ? top_k : V, cand);
    else
        hipLaunchKernelGGL((isd_row_topk_kernel<16, false>), dim3((unsigned)(B * S)), dim3(256), 0, st, logits, V,
                           top_k < V ? top_k : V, cand);
    hipLaunchKernelGGL(isd_accept_filtered_chain_kernel, dim3((unsigned)B), dim3(64 * kChainWaves), 0, st, p);
    return launch_status();
}

extern "C" int idlm_isd_accept_filtered(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                                        int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S, int32_t V,
                                        int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                                        uint32_t rng_offset, float temperature, float tau, int32_t top_k, float top_p,
                                        int32_t sample_proposals, float* draft_probs, int32_t* kept,
                                        void* workspace, size_t workspace_bytes, void* stream)
{
    return accept_filtered_impl(logits, IDLM_DTYPE_F32, draft_tokens, nullptr, nullptr, rng_seed, accept_len, new_tokens, B, S, V,
                                n_draft_uniform, n_draft, greedy, rng_offset, temperature, tau, top_k, top_p,
                                sample_proposals, draft_probs, nullptr, kept, nullptr, workspace, workspace_bytes, stream);
}

extern "C" int idlm_isd_accept_filtered_q(const void* logits, int32_t logits_dtype, const int32_t* draft_tokens, const uint64_t* q_cand,
                                          const int32_t* q_row, uint64_t rng_seed, int32_t* accept_len,
                                          int32_t* new_tokens, int32_t B, int32_t S, int32_t V, int32_t n_draft_uniform,
                                          const int32_t* n_draft, const uint8_t* greedy, uint32_t rng_offset,
                                          float temperature, float tau, int32_t top_k, float top_p,
                                          int32_t sample_proposals, float* draft_probs, float* draft_q, int32_t* kept,
                                          uint64_t* cand_out, void* workspace, size_t workspace_bytes, void* stream)
{
    return accept_filtered_impl(logits, logits_dtype, draft_tokens, q_cand, q_row, rng_seed, accept_len, new_tokens, B, S, V,
                                n_draft_uniform, n_draft, greedy, rng_offset, temperature, tau, top_k, top_p,
                                sample_proposals, draft_probs, draft_q, kept, cand_out, workspace, workspace_bytes, stream);
}
