// Introspective acceptance pass of one ISD step (Alg. 1, introspection loop; fused
// verification of Sec. 3.3 (3)) as four launches (the last three are tiny):
//   1. row statistics: one streaming pass over every logit row (16-byte loads, online
//      max / sum-of-exponentials / arg-max per thread, wavefront + LDS reductions);
//   2. per sequence (one wavefront): accept tests, accepted-prefix length, proposals;
//   3. only for stochastic sequences: a Gumbel-max pass over the single row that emits the
//      fresh token, split over several workgroups that combine with one 64-bit atomic max;
//   4. decode of the winning keys into new_tokens.
// HBM-bound: the algorithmic traffic is one read of the logits (4*V bytes per row).
#include "isd_accept_common.h"
#include <mutex>

namespace idlm {

struct ChainResult {   // what the sampling pass needs to know about a sequence
    int row;           // stride row r that emits the fresh token, or -1 (greedy: nothing to sample)
    int excluded;      // token id removed from the sample (the rejected draft), or -1
    float floor;       // a score that the winner of row r's Gumbel-max reaches or exceeds (-inf: none known)
    int pad;
};

struct AcceptWorkspace {
    size_t stats_off, keys_off, chain_off, total;
};

static AcceptWorkspace layout(int32_t B, int32_t S, const AcceptPlan& p)
{
    AcceptWorkspace w;
    w.stats_off = 0;
    size_t stats = (size_t)B * S * p.nsplit * sizeof(RowPartial);
    w.keys_off = align256(stats);
    w.chain_off = w.keys_off + align256((size_t)B * sizeof(unsigned long long));   // one arg-max key per sequence
    w.total = w.chain_off + align256((size_t)B * sizeof(ChainResult));
    return w;
}

// ---- pass 2: accept chain and proposals, one wavefront per sequence ---------------------------



template <bool BF16>
__global__ __launch_bounds__(64) void isd_accept_chain_kernel(
    const void* __restrict__ logits, const int32_t* __restrict__ draft_tokens, uint2 key,
    int32_t* __restrict__ accept_len, int32_t* __restrict__ new_tokens, int S, int V,
    int n_draft_uniform, const int32_t* __restrict__ n_draft, const uint8_t* __restrict__ greedy,
    uint32_t rng_offset, float* __restrict__ draft_probs, const RowPartial* __restrict__ stats,
    int nsplit, ChainResult* __restrict__ chain, unsigned long long* __restrict__ keys)
{
    const int b = blockIdx.x;
    const int tid = threadIdx.x;      // one lane per stride row (S <= 64)
    const bool is_greedy = greedy ? (greedy[b] != 0) : false;
    int n_d = n_draft ? n_draft[b] : n_draft_uniform;
    n_d = max(0, min(n_d, S - 1));
    const int ncol = S - 1;

    int a = 0, ok = 1, x = -1;
    float p = 0.f, m_row = -INFINITY, m2_row = -INFINITY;
    if (tid < S) {
        const int row = b * S + tid;
        const RowPartial* sp = stats + (size_t)row * nsplit;
        float m = sp[0].m, z = sp[0].z, second = sp[0].m2;
        a = sp[0].arg;
        for (int k = 1; k < nsplit; ++k) {
            second = combine_second(m, second, sp[k].m, sp[k].m2);
            combine_stats(m, z, a, sp[k].m, sp[k].z, sp[k].arg);
        }
        m_row = m;
        m2_row = second;
        if (tid < n_d) {
            x = draft_tokens[(size_t)b * ncol + tid];
            if (x >= 0 && x < V) {
                const float lx = LogitVec<BF16>::element(logits, (size_t)row * V + x);
                p = fast_exp2(fmaf(lx, kLog2e, -ref_log2(m))) / z;
            }
            if (is_greedy) {
                ok = (x == a);
            } else {
                const uint4 w = philox4x32_10(make_uint4(0u, (uint32_t)row, 0u, rng_offset), key);
                ok = unit_uniform(w.x) < p;
            }
        }
        if (draft_probs && tid < ncol) draft_probs[(size_t)b * ncol + tid] = p;
    }
    // accepted prefix = rows below the first failed test
    const unsigned long long failed = __ballot(tid < n_d && !ok);
    const int r = failed ? (int)__builtin_ctzll(failed) : n_d;
    const int a_r = __shfl(a, r);
    const int x_r = __shfl(x, r);
    const float m_r = __shfl(m_row, r);
    const float m2_r = __shfl(m2_row, r);
    if (tid < S) {
        int tok;
        if (tid < r) tok = x;
        else if (tid == r) tok = a_r;
        else if (tid <= n_d) tok = -1;
        else tok = a;
        if (tid != r || is_greedy) new_tokens[(size_t)b * S + tid] = tok;
    }
    if (tid == 0) {
        accept_len[b] = r;
        ChainResult cr;
        cr.row = is_greedy ? -1 : r;
        cr.excluded = (r < n_d) ? x_r : -1;
        cr.floor = -INFINITY;
        if (!is_greedy && m_r > -INFINITY) {
            if (cr.excluded == a_r) {
                cr.floor = m2_r + kGumbelMin;
            } else {   // the arg-max element's own score, as the sampling pass will compute it
                const uint4 w = philox4x32_10(make_uint4((uint32_t)(a_r >> 2), (uint32_t)(b * S + r), 1u, rng_offset), key);
                const int k = a_r & 3;
                cr.floor = m_r + gumbel(k == 0 ? w.x : k == 1 ? w.y : k == 2 ? w.z : w.w);
            }
        }
        cr.pad = 0;
        chain[b] = cr;
        keys[b] = 0ull;   // "nothing sampled yet"
    }
}

// ---- pass 3: Gumbel-max sample of the one row per stochastic sequence -------------------------

template <bool BF16>
__global__ __launch_bounds__(256) void isd_accept_sample_kernel(
    const void* __restrict__ logits, uint2 key, int S, int V, uint32_t rng_offset,
    const ChainResult* __restrict__ chain, unsigned long long* keys, int nsb, int gchunk)
{
    typedef LogitVec<BF16> LV;
    typedef typename LV::raw raw_t;
    constexpr int N = LV::N;
    const int b = blockIdx.x / nsb;
    const int c = blockIdx.x - b * nsb;
    const int tid = threadIdx.x;
    const ChainResult cr = chain[b];
    if (cr.row < 0) return;           // greedy sequence: the chain kernel wrote everything

    __shared__ float s_best[4];
    __shared__ int s_bidx[4];

    // Gumbel-max over slice c of row r: argmax_i (l_i + g_i), the rejected draft excluded
    const int excluded = cr.excluded;
    const uint32_t row = (uint32_t)(b * S + cr.row);
    const raw_t* __restrict__ pv = reinterpret_cast<const raw_t*>(
        static_cast<const char*>(logits) + (size_t)row * V * (16 / N));
    const int fbeg = (c * gchunk) / N;
    const int fend = min(V, (c + 1) * gchunk) / N;
    float best = -INFINITY;
    int bidx = INT_MAX;
    const float floor0 = cr.floor;
    float thr = floor0;   // max(floor, this thread's best so far)
    auto may_win = [&](float l, uint32_t word) {
        return one_minus_uniform(word) < fast_exp2(fmaf(l - thr, kLog2e, 0.01f));
    };
    auto evaluate = [&](float l, uint32_t word, int idx) {
        const float s = l + gumbel(word);
        if (idx != excluded && s > best) { best = s; bidx = idx; }
    };
    for (int f0 = fbeg + tid; f0 < fend; f0 += 4 * 256) {   // four loads in flight, then the noise of what can win
        raw_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int f = f0 + u * 256;
            v[u] = pv[f < fend ? f : f0];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int f = f0 + u * 256;
            if (f >= fend) break;
            float e[N];
            LV::unpack(v[u], e);
#pragma unroll
            for (int h = 0; h < N / 4; ++h) {   // one Philox block per four consecutive elements
                if (fmaxf(fmaxf(e[h * 4], e[h * 4 + 1]), fmaxf(e[h * 4 + 2], e[h * 4 + 3])) < thr - kNoiseMax) continue;
                const int i0 = f * N + h * 4;
                const uint4 w = philox4x32_10(make_uint4((uint32_t)(i0 >> 2), row, 1u, rng_offset), key);
                const bool p0 = may_win(e[h * 4], w.x), p1 = may_win(e[h * 4 + 1], w.y);
                const bool p2 = may_win(e[h * 4 + 2], w.z), p3 = may_win(e[h * 4 + 3], w.w);
                // a branch of the whole wavefront (rarely taken), so that the logarithms are not computed
                // speculatively for everything
                if (__ballot(p0 || p1 || p2 || p3) != 0ull) {
                    if (p0) evaluate(e[h * 4], w.x, i0);
                    if (p1) evaluate(e[h * 4 + 1], w.y, i0 + 1);
                    if (p2) evaluate(e[h * 4 + 2], w.z, i0 + 2);
                    if (p3) evaluate(e[h * 4 + 3], w.w, i0 + 3);
                    thr = fmaxf(best, floor0);
                }
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float s2 = __shfl_xor(best, off);
        const int i2 = __shfl_xor(bidx, off);
        combine_best(best, bidx, s2, i2);
    }
    const int wv = tid >> 6;
    if ((tid & 63) == 0) { s_best[wv] = best; s_bidx[wv] = bidx; }
    __syncthreads();
    if (tid == 0) {
        for (int k = 1; k < 4; ++k) combine_best(best, bidx, s_best[k], s_bidx[k]);
        if (bidx != INT_MAX) atomicMax(&keys[b], sample_key(best, bidx));
    }
}

// ---- pass 4: decode the winning key of every stochastic sequence into its fresh token ----------

__global__ __launch_bounds__(256) void isd_accept_emit_kernel(const ChainResult* __restrict__ chain,
                                                              const unsigned long long* __restrict__ keys,
                                                              int32_t* __restrict__ new_tokens, int B, int S)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    const ChainResult cr = chain[b];
    if (cr.row < 0) return;
    const unsigned long long k = keys[b];
    new_tokens[(size_t)b * S + cr.row] = k ? (int32_t)(0xFFFFFFFFu - (uint32_t)k) : -1;
}

}  // namespace idlm

using namespace idlm;

extern "C" size_t idlm_isd_accept_workspace(int32_t B, int32_t S, int32_t V)
{
    if (B < 0 || S < 1 || S > 64 || V < 4 || (V & 3) || (int64_t)B * S >= INT32_MAX) return 0;
    if (B == 0) return 0;
    return layout(B, S, make_plan(B, S, V)).total;
}

namespace idlm {

template <bool BF16>
static int accept_impl(const void* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                       int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S, int32_t V,
                       int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                       uint32_t rng_offset, float* draft_probs, void* workspace, size_t workspace_bytes,
                       void* stream, void* const* events)
{
    constexpr int N = LogitVec<BF16>::N;   // elements per 16-byte vector
    if (B < 0 || S < 1 || S > 64 || V < N || (V % N) || (int64_t)B * S >= INT32_MAX) return IDLM_ERR_SHAPE;
    if (!n_draft && (n_draft_uniform < 0 || n_draft_uniform > S - 1)) return IDLM_ERR_SHAPE;
    if (B == 0) return IDLM_OK;
    if (!logits || !accept_len || !new_tokens) return IDLM_ERR_NULL;
    if (S > 1 && !draft_tokens) return IDLM_ERR_NULL;
    if (!aligned(logits, 16)) return IDLM_ERR_ALIGN;
    const AcceptPlan plan = make_plan(B, S, V);
    const AcceptWorkspace w = layout(B, S, plan);
    if (!workspace || workspace_bytes < w.total) return IDLM_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return IDLM_ERR_ALIGN;
    if ((int64_t)B * S * plan.nsplit >= INT32_MAX || (int64_t)B * plan.nsb >= INT32_MAX) return IDLM_ERR_SHAPE;

    char* ws = static_cast<char*>(workspace);
    RowPartial* stats = reinterpret_cast<RowPartial*>(ws + w.stats_off);
    unsigned long long* keys = reinterpret_cast<unsigned long long*>(ws + w.keys_off);
    hipStream_t st = static_cast<hipStream_t>(stream);

    (void)hipGetLastError();
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[0]), st);
    hipLaunchKernelGGL((isd_row_stats_kernel<16, BF16>), dim3((unsigned)(B * S * plan.nsplit)), dim3(256), 0, st,
                       logits, V, plan.chunk, plan.nsplit, S, stats, kLog2e);
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[1]), st);
    const uint2 key = make_uint2((uint32_t)rng_seed, (uint32_t)(rng_seed >> 32));
    ChainResult* chain = reinterpret_cast<ChainResult*>(ws + w.chain_off);
    hipLaunchKernelGGL(isd_accept_chain_kernel<BF16>, dim3((unsigned)B), dim3(64), 0, st, logits, draft_tokens,
                       key, accept_len, new_tokens, S, V, n_draft_uniform, n_draft, greedy, rng_offset,
                       draft_probs, stats, plan.nsplit, chain, keys);
    hipLaunchKernelGGL(isd_accept_sample_kernel<BF16>, dim3((unsigned)(B * plan.nsb)), dim3(256), 0, st, logits,
                       key, S, V, rng_offset, chain, keys, plan.nsb, plan.gchunk);
    hipLaunchKernelGGL(isd_accept_emit_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, st, chain, keys,
                       new_tokens, B, S);
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[2]), st);
    return launch_status();
}

}  // namespace idlm

extern "C" int idlm_isd_accept_ev(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                                  int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S,
                                  int32_t V, int32_t n_draft_uniform, const int32_t* n_draft,
                                  const uint8_t* greedy, uint32_t rng_offset, float* draft_probs,
                                  void* workspace, size_t workspace_bytes, void* stream,
                                  void* const* events)
{
    return accept_impl<false>(logits, draft_tokens, rng_seed, accept_len, new_tokens, B, S, V,
                              n_draft_uniform, n_draft, greedy, rng_offset, draft_probs, workspace,
                              workspace_bytes, stream, events);
}

extern "C" int idlm_isd_accept(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                               int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S,
                               int32_t V, int32_t n_draft_uniform, const int32_t* n_draft,
                               const uint8_t* greedy, uint32_t rng_offset, float* draft_probs,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    return accept_impl<false>(logits, draft_tokens, rng_seed, accept_len, new_tokens, B, S, V,
                              n_draft_uniform, n_draft, greedy, rng_offset, draft_probs, workspace,
                              workspace_bytes, stream, nullptr);
}

extern "C" int idlm_isd_accept_bf16_ev(const uint16_t* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                                       int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S,
                                       int32_t V, int32_t n_draft_uniform, const int32_t* n_draft,
                                       const uint8_t* greedy, uint32_t rng_offset, float* draft_probs,
                                       void* workspace, size_t workspace_bytes, void* stream,
                                       void* const* events)
{
    return accept_impl<true>(logits, draft_tokens, rng_seed, accept_len, new_tokens, B, S, V,
                             n_draft_uniform, n_draft, greedy, rng_offset, draft_probs, workspace,
                             workspace_bytes, stream, events);
}

extern "C" int idlm_isd_accept_bf16(const uint16_t* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                                    int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S,
                                    int32_t V, int32_t n_draft_uniform, const int32_t* n_draft,
                                    const uint8_t* greedy, uint32_t rng_offset, float* draft_probs,
                                    void* workspace, size_t workspace_bytes, void* stream)
{
    return accept_impl<true>(logits, draft_tokens, rng_seed, accept_len, new_tokens, B, S, V,
                             n_draft_uniform, n_draft, greedy, rng_offset, draft_probs, workspace,
                             workspace_bytes, stream, nullptr);
}

// ---- the same call for callers that cannot allocate -------------------------------------------
// The workspace of idlm_isd_accept (slice statistics, one arg-max key and one chain record per
// sequence) lives in a fixed array in device memory instead of a caller's buffer.  Every GPU the
// library runs on holds its own copy of the array, at its own address, until the process ends.

namespace idlm {

constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// In host code `scratch` is only a handle for the runtime, not an address a kernel could use: the
// array's device address on the current device is asked for once per device and kept.
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];

static int static_scratch(void** ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return IDLM_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return IDLM_ERR_LAUNCH;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return IDLM_OK;
}

}  // namespace idlm

extern "C" size_t idlm_isd_accept_static_max_bytes(void) { return kStaticScratchBytes; }

extern "C" int idlm_isd_accept_static(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                                      int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S,
                                      int32_t V, int32_t n_draft_uniform, const int32_t* n_draft,
                                      const uint8_t* greedy, uint32_t rng_offset, float* draft_probs,
                                      void* stream)
{
    // shapes first, so that a rejected shape is reported as such and an oversized one as IDLM_ERR_WORKSPACE
    if (B < 0 || S < 1 || S > 64 || V < 4 || (V & 3) || (int64_t)B * S >= INT32_MAX) return IDLM_ERR_SHAPE;
    if (B == 0) return IDLM_OK;
    if (idlm_isd_accept_workspace(B, S, V) > kStaticScratchBytes) return IDLM_ERR_WORKSPACE;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != IDLM_OK) return rc;
    // every word of the scratch that a kernel of the call reads is written earlier in the same call (slice
    // statistics by the streaming pass, keys and chain records by the chain kernel), so nothing has to be cleared
    return accept_impl<false>(logits, draft_tokens, rng_seed, accept_len, new_tokens, B, S, V, n_draft_uniform,
                              n_draft, greedy, rng_offset, draft_probs, ws, kStaticScratchBytes, stream, nullptr);
}
