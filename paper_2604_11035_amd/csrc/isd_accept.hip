// Introspective acceptance pass of one ISD step (Alg. 1, introspection loop; fused
// verification of Sec. 3.3 (3)) as two launches:
//   1. row statistics: one streaming pass over every logit row (16-byte loads, online
//      max / sum-of-exponentials / arg-max per thread, wavefront + LDS reductions);
//   2. per sequence: accept tests, accepted-prefix length, proposals, and - only for
//      stochastic sequences - a Gumbel-max pass over the single row that emits the fresh
//      token, split over several workgroups and joined by the last one to finish.
// HBM-bound: the algorithmic traffic is one read of the logits (4*V bytes per row).
#include "idlm_common.h"
#include <limits.h>

namespace idlm {

typedef __attribute__((ext_vector_type(4))) float f32x4;

struct RowPartial {   // statistics of one slice of one logit row
    float m;          // maximum (true value, compared exactly)
    float z;          // sum of 2^(l*log2e - ref_log2(m))
    int arg;          // lowest index attaining m (INT_MAX if the slice is empty)
    int pad;
};

struct SamplePartial {
    float score;
    int idx;
};

struct AcceptPlan {
    int chunk;    // vocabulary elements per workgroup in pass 1 (multiple of 1024)
    int nsplit;   // slices per row in pass 1
    int gchunk;   // vocabulary elements per workgroup in the Gumbel pass (multiple of 1024)
    int nsb;      // workgroups per sequence in pass 2
};

static AcceptPlan make_plan(int32_t B, int32_t S, int32_t V)
{
    AcceptPlan p;
    const int64_t rows = (int64_t)B * S;
    // Enough workgroups to fill 256 CUs several times over, slices of at most 32K elements
    // (128 KB) so that the tail of the launch stays short, at least 4K elements each.
    int64_t want = (4096 + rows - 1) / (rows > 0 ? rows : 1);
    int64_t by_size = ((int64_t)V + 32767) / 32768;
    int64_t nsplit = want > by_size ? want : by_size;
    int64_t max_split = ((int64_t)V + 4095) / 4096;
    if (nsplit > max_split) nsplit = max_split;
    if (nsplit < 1) nsplit = 1;
    int64_t chunk = (((int64_t)V + nsplit - 1) / nsplit + 1023) / 1024 * 1024;
    p.chunk = (int)chunk;
    p.nsplit = (int)(((int64_t)V + chunk - 1) / chunk);
    int64_t nsb = ((int64_t)V + 16383) / 16384;   // 16K elements of Philox + logs per workgroup
    if (nsb > 32) nsb = 32;
    int64_t gchunk = (((int64_t)V + nsb - 1) / nsb + 1023) / 1024 * 1024;
    p.gchunk = (int)gchunk;
    p.nsb = (int)(((int64_t)V + gchunk - 1) / gchunk);
    return p;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct AcceptWorkspace {
    size_t stats_off, gpart_off, counter_off, total;
};

static AcceptWorkspace layout(int32_t B, int32_t S, const AcceptPlan& p)
{
    AcceptWorkspace w;
    w.stats_off = 0;
    size_t stats = (size_t)B * S * p.nsplit * sizeof(RowPartial);
    w.gpart_off = align256(stats);
    size_t gpart = (size_t)B * p.nsb * sizeof(SamplePartial);
    w.counter_off = w.gpart_off + align256(gpart);
    w.total = w.counter_off + align256((size_t)B * sizeof(uint32_t));
    return w;
}

// ---- reductions ---------------------------------------------------------------------------

__device__ __forceinline__ void combine_stats(float& m, float& z, int& a, float m2, float z2, int a2)
{
    const float mm = fmaxf(m, m2);
    const float r = ref_log2(mm);
    z = z * rescale_factor(m, r) + z2 * rescale_factor(m2, r);
    a = (m2 > m) ? a2 : ((m > m2) ? a : min(a, a2));
    m = mm;
}

__device__ __forceinline__ void combine_best(float& s, int& i, float s2, int i2)
{
    if (s2 > s || (s2 == s && i2 < i)) { s = s2; i = i2; }
}

// ---- pass 1: row statistics ---------------------------------------------------------------

template <int UNROLL>
__global__ __launch_bounds__(256) void isd_row_stats_kernel(const float* __restrict__ logits, int V,
                                                            int chunk, int nsplit, int S,
                                                            RowPartial* __restrict__ stats,
                                                            uint32_t* __restrict__ counters)
{
    const int row = blockIdx.x / nsplit;
    const int c = blockIdx.x - row * nsplit;
    const int tid = threadIdx.x;
    const f32x4* __restrict__ p4 = reinterpret_cast<const f32x4*>(logits + (size_t)row * V);
    const int fbeg = (c * chunk) >> 2;
    const int fend = min(V, (c + 1) * chunk) >> 2;

    if (c == 0 && tid == 0 && row % S == 0) counters[row / S] = 0u;

    float m = -INFINITY;   // running maximum of this thread's elements
    float z = 0.f;         // sum of 2^(l*log2e - ref_log2(m))
    int arg4 = -1;         // float4 index that holds the first occurrence of m

    int f = fbeg + tid;
    for (; f + (UNROLL - 1) * 256 < fend; f += UNROLL * 256) {
        f32x4 v[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(p4 + f + u * 256);
        float newm = m;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const float bm = fmaxf(fmaxf(v[u].x, v[u].y), fmaxf(v[u].z, v[u].w));
            if (bm > newm) { newm = bm; arg4 = f + u * 256; }
        }
        const float r = ref_log2(newm);
        float acc = z * rescale_factor(m, r);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            acc += fast_exp2(fmaf(v[u].x, kLog2e, -r));
            acc += fast_exp2(fmaf(v[u].y, kLog2e, -r));
            acc += fast_exp2(fmaf(v[u].z, kLog2e, -r));
            acc += fast_exp2(fmaf(v[u].w, kLog2e, -r));
        }
        z = acc;
        m = newm;
    }
    for (; f < fend; f += 256) {
        const f32x4 v = __builtin_nontemporal_load(p4 + f);
        const float bm = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
        float newm = m;
        if (bm > newm) { newm = bm; arg4 = f; }
        const float r = ref_log2(newm);
        float acc = z * rescale_factor(m, r);
        acc += fast_exp2(fmaf(v.x, kLog2e, -r));
        acc += fast_exp2(fmaf(v.y, kLog2e, -r));
        acc += fast_exp2(fmaf(v.z, kLog2e, -r));
        acc += fast_exp2(fmaf(v.w, kLog2e, -r));
        z = acc;
        m = newm;
    }

    // which of the four components was first to reach m
    int arg = INT_MAX;
    if (arg4 >= 0) {
        const f32x4 v = p4[arg4];
        const int lane = (v.x == m) ? 0 : (v.y == m) ? 1 : (v.z == m) ? 2 : 3;
        arg = arg4 * 4 + lane;
    }

    // wavefront reduction, then the four wavefronts through LDS
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off);
        const float z2 = __shfl_xor(z, off);
        const int a2 = __shfl_xor(arg, off);
        combine_stats(m, z, arg, m2, z2, a2);
    }
    __shared__ float sm[4], sz[4];
    __shared__ int sa[4];
    const int w = tid >> 6;
    if ((tid & 63) == 0) { sm[w] = m; sz[w] = z; sa[w] = arg; }
    __syncthreads();
    if (tid == 0) {
        for (int k = 1; k < 4; ++k) combine_stats(m, z, arg, sm[k], sz[k], sa[k]);
        RowPartial out;
        out.m = m; out.z = z; out.arg = arg; out.pad = 0;
        stats[(size_t)row * nsplit + c] = out;
    }
}

// ---- counter-based random numbers (Philox4x32-10, Salmon et al. SC'11) --------------------

__device__ __forceinline__ uint4 philox4x32_10(uint4 ctr, uint2 key)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, ctr.x), lo0 = 0xD2511F53u * ctr.x;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, ctr.z), lo1 = 0xCD9E8D57u * ctr.z;
        ctr = make_uint4(hi1 ^ ctr.y ^ key.x, lo1, hi0 ^ ctr.w ^ key.y, lo0);
        key.x += 0x9E3779B9u;
        key.y += 0xBB67AE85u;
    }
    return ctr;
}

// 32 bits -> u = (2*(x>>9)+1) * 2^-24: an odd 24-bit numerator, exact in fp32, inside (0,1)
__device__ __forceinline__ float unit_uniform(uint32_t x)
{
    return (float)(2u * (x >> 9) + 1u) * 5.9604644775390625e-8f;
}

__device__ __forceinline__ float gumbel(uint32_t x) { return -logf(-logf(unit_uniform(x))); }

// ---- pass 2: accept chain, proposals, Gumbel-max sample -------------------------------------

__global__ __launch_bounds__(256) void isd_accept_finalize_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ draft_tokens, uint2 key,
    int32_t* __restrict__ accept_len, int32_t* __restrict__ new_tokens, int S, int V,
    int n_draft_uniform, const int32_t* __restrict__ n_draft, const uint8_t* __restrict__ greedy,
    uint32_t rng_offset, float* __restrict__ draft_probs, const RowPartial* __restrict__ stats,
    int nsplit, SamplePartial* gpart, uint32_t* counters, int nsb, int gchunk)
{
    const int b = blockIdx.x / nsb;
    const int c = blockIdx.x - b * nsb;
    const int tid = threadIdx.x;
    const bool is_greedy = greedy ? (greedy[b] != 0) : false;
    if (is_greedy && c != 0) return;
    int n_d = n_draft ? n_draft[b] : n_draft_uniform;
    n_d = max(0, min(n_d, S - 1));
    const int ncol = S - 1;

    __shared__ int s_arg[64];
    __shared__ int s_ok[64];
    __shared__ int s_r;
    __shared__ float s_best[4];
    __shared__ int s_bidx[4];

    if (tid < S) {
        const int row = b * S + tid;
        const RowPartial* sp = stats + (size_t)row * nsplit;
        float m = sp[0].m, z = sp[0].z;
        int a = sp[0].arg;
        for (int k = 1; k < nsplit; ++k) combine_stats(m, z, a, sp[k].m, sp[k].z, sp[k].arg);
        int ok = 1;
        float p = 0.f;
        if (tid < n_d) {
            const int x = draft_tokens[(size_t)b * ncol + tid];
            if (x >= 0 && x < V) {
                const float lx = logits[(size_t)row * V + x];
                p = fast_exp2(fmaf(lx, kLog2e, -ref_log2(m))) / z;
            }
            if (is_greedy) {
                ok = (x == a);
            } else {
                const uint4 w = philox4x32_10(make_uint4(0u, (uint32_t)row, 0u, rng_offset), key);
                ok = unit_uniform(w.x) < p;
            }
        }
        if (c == 0 && draft_probs && tid < ncol) draft_probs[(size_t)b * ncol + tid] = p;
        s_arg[tid] = a;
        s_ok[tid] = ok;
    }
    __syncthreads();
    if (tid == 0) {
        int r = n_d;
        for (int j = 0; j < n_d; ++j)
            if (!s_ok[j]) { r = j; break; }
        s_r = r;
    }
    __syncthreads();
    const int r = s_r;
    if (c == 0) {
        if (tid < S) {
            int tok;
            if (tid < r) tok = draft_tokens[(size_t)b * ncol + tid];
            else if (tid == r) tok = s_arg[r];
            else if (tid <= n_d) tok = -1;
            else tok = s_arg[tid];
            if (tid != r || is_greedy) new_tokens[(size_t)b * S + tid] = tok;
        }
        if (tid == 0) accept_len[b] = r;
    }
    if (is_greedy) return;

    // Gumbel-max over slice c of row r: argmax_i (l_i + g_i), the rejected draft excluded
    const int excluded = (r < n_d) ? draft_tokens[(size_t)b * ncol + r] : -1;
    const uint32_t row = (uint32_t)(b * S + r);
    const float4* __restrict__ p4 = reinterpret_cast<const float4*>(logits + (size_t)row * V);
    const int fbeg = (c * gchunk) >> 2;
    const int fend = min(V, (c + 1) * gchunk) >> 2;
    float best = -INFINITY;
    int bidx = INT_MAX;
    for (int f = fbeg + tid; f < fend; f += 256) {
        const float4 v = p4[f];
        const uint4 w = philox4x32_10(make_uint4((uint32_t)f, row, 1u, rng_offset), key);
        const float s0 = v.x + gumbel(w.x), s1 = v.y + gumbel(w.y);
        const float s2 = v.z + gumbel(w.z), s3 = v.w + gumbel(w.w);
        const int i0 = f * 4;
        if (i0 != excluded && s0 > best) { best = s0; bidx = i0; }
        if (i0 + 1 != excluded && s1 > best) { best = s1; bidx = i0 + 1; }
        if (i0 + 2 != excluded && s2 > best) { best = s2; bidx = i0 + 2; }
        if (i0 + 3 != excluded && s3 > best) { best = s3; bidx = i0 + 3; }
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
        SamplePartial sp;
        sp.score = best; sp.idx = bidx;
        gpart[(size_t)b * nsb + c] = sp;
        __threadfence();                                  // publish the partial ...
        const uint32_t ticket = atomicAdd(&counters[b], 1u);   // ... then take a ticket
        if (ticket == (uint32_t)(nsb - 1)) {
            __threadfence();                              // last to finish: see everyone's partial
            float fs = -INFINITY;
            int fi = INT_MAX;
            const volatile SamplePartial* gp = gpart + (size_t)b * nsb;
            for (int k = 0; k < nsb; ++k) combine_best(fs, fi, gp[k].score, gp[k].idx);
            new_tokens[(size_t)b * S + r] = (fi == INT_MAX) ? -1 : fi;
            counters[b] = 0u;
        }
    }
}

}  // namespace idlm

using namespace idlm;

extern "C" size_t idlm_isd_accept_workspace(int32_t B, int32_t S, int32_t V)
{
    if (B < 0 || S < 1 || S > 64 || V < 4 || (V & 3) || (int64_t)B * S >= INT32_MAX) return 0;
    if (B == 0) return 0;
    return layout(B, S, make_plan(B, S, V)).total;
}

extern "C" int idlm_isd_accept_ev(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                                  int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S,
                                  int32_t V, int32_t n_draft_uniform, const int32_t* n_draft,
                                  const uint8_t* greedy, uint32_t rng_offset, float* draft_probs,
                                  void* workspace, size_t workspace_bytes, void* stream,
                                  void* const* events)
{
    if (B < 0 || S < 1 || S > 64 || V < 4 || (V & 3) || (int64_t)B * S >= INT32_MAX) return IDLM_ERR_SHAPE;
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
    SamplePartial* gpart = reinterpret_cast<SamplePartial*>(ws + w.gpart_off);
    uint32_t* counters = reinterpret_cast<uint32_t*>(ws + w.counter_off);
    hipStream_t st = static_cast<hipStream_t>(stream);

    (void)hipGetLastError();
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[0]), st);
    hipLaunchKernelGGL(isd_row_stats_kernel<8>, dim3((unsigned)(B * S * plan.nsplit)), dim3(256), 0, st,
                       logits, V, plan.chunk, plan.nsplit, S, stats, counters);
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[1]), st);
    const uint2 key = make_uint2((uint32_t)rng_seed, (uint32_t)(rng_seed >> 32));
    hipLaunchKernelGGL(isd_accept_finalize_kernel, dim3((unsigned)(B * plan.nsb)), dim3(256), 0, st,
                       logits, draft_tokens, key, accept_len, new_tokens, S, V, n_draft_uniform,
                       n_draft, greedy, rng_offset, draft_probs, stats, plan.nsplit, gpart, counters,
                       plan.nsb, plan.gchunk);
    if (events) (void)hipEventRecord(static_cast<hipEvent_t>(events[2]), st);
    return launch_status();
}

extern "C" int idlm_isd_accept(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                               int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S,
                               int32_t V, int32_t n_draft_uniform, const int32_t* n_draft,
                               const uint8_t* greedy, uint32_t rng_offset, float* draft_probs,
                               void* workspace, size_t workspace_bytes, void* stream)
{
    return idlm_isd_accept_ev(logits, draft_tokens, rng_seed, accept_len, new_tokens, B, S, V,
                              n_draft_uniform, n_draft, greedy, rng_offset, draft_probs, workspace,
                              workspace_bytes, stream, nullptr);
}
