// Acceptance with general proposal distributions, sampling temperature, relaxed threshold and
// sampled proposals (Alg. 1 as printed: drafts drawn from q, accepted with probability
// min(1, p/q), resampled from normalize(max(0, p - q)) at the first rejection; Sec. 3.2; the
// threshold relaxation of Sec. 5; temperature as in the sampling set-up of App. H).  The
// deployed point-mass setting is the fast path in isd_accept.hip; this file is the general one:
//   1. row statistics of the step's logits at temperature T (and of the proposal rows, unless
//      the caller kept their log-sum-exp from the call that produced them);
//   2. per sequence (one wavefront): accept tests against min(1, (1+tau) p/q), accepted prefix,
//      and one "job" per row that still needs a Gumbel-max pass (the fresh token's row; every
//      MASK row when proposals are sampled);
//   3. the Gumbel-max passes, split over several workgroups per row that combine with one
//      64-bit atomic max;
//   4. decode of the winning keys.
#include "isd_accept_common.h"

namespace idlm {

constexpr float kLn2 = 0.69314718056f;

enum { JOB_NONE = 0, JOB_PLAIN = 1, JOB_RESID_POINT = 2, JOB_RESID_Q = 3 };

struct SampleJob {     // one row that needs a Gumbel-max pass
    int mode;          // JOB_*
    int stream;        // random stream: 1 fresh token, 2 proposal
    int excluded;      // JOB_RESID_POINT: the rejected draft
    int fallback;      // token if no element qualifies (arg-max of the row)
    float lse2;        // log2 sum 2^(l*k) of the row
    int q_row;         // JOB_RESID_Q: row of q_logits (inside the sequence)
    float q_lse2;      // ... and its log2-sum
    float floor;       // JOB_PLAIN / JOB_RESID_POINT: a score the winner reaches or exceeds (-inf: none known)
};

struct GeneralParams {
    const float* logits;
    const int32_t* draft_tokens;
    const float* q_logits;
    const int32_t* q_row;
    const float* q_lse;          // natural-log lse of the q rows, or NULL (then q_stats is used)
    const RowPartial* stats;
    const RowPartial* q_stats;
    int32_t* accept_len;
    int32_t* new_tokens;
    const int32_t* n_draft;
    const uint8_t* greedy;
    float* draft_probs;
    float* draft_q;
    float* row_lse;
    SampleJob* jobs;
    unsigned long long* keys;
    uint2 key;
    int S, V, n_draft_uniform, nsplit, sample_proposals;
    uint32_t rng_offset;
    float k;        // log2(e) / T
    float inv_t;    // 1 / T
    float one_plus_tau;
};

__device__ __forceinline__ void merged_stats(const RowPartial* sp, int nsplit, float k, float& m, float& z, int& a,
                                             float& m2)
{
    m = sp[0].m; z = sp[0].z; a = sp[0].arg; m2 = sp[0].m2;
    for (int q = 1; q < nsplit; ++q) {
        m2 = combine_second(m, m2, sp[q].m, sp[q].m2);
        combine_stats(m, z, a, sp[q].m, sp[q].z, sp[q].arg, k);
    }
}

__global__ __launch_bounds__(64) void isd_accept_general_chain_kernel(const GeneralParams p)
{
    const int b = blockIdx.x;
    const int tid = threadIdx.x;      // one lane per stride row (S <= 64)
    const int S = p.S, V = p.V;
    const bool is_greedy = p.greedy ? (p.greedy[b] != 0) : false;
    int n_d = p.n_draft ? p.n_draft[b] : p.n_draft_uniform;
    n_d = max(0, min(n_d, S - 1));
    const int ncol = S - 1;
    int qr0 = p.q_logits ? p.q_row[b] : 0;
    qr0 = max(0, min(qr0, S - n_d));          // the q rows of the drafts stay inside the sequence

    int a = 0, ok = 1, x = -1, my_qrow = 0;
    float pr = 0.f, qv = 0.f, lse2 = 0.f, q_lse2 = 0.f, m = -INFINITY, m2 = -INFINITY;
    if (tid < S) {
        const int row = b * S + tid;
        float z;
        merged_stats(p.stats + (size_t)row * p.nsplit, p.nsplit, p.k, m, z, a, m2);
        lse2 = ref_k(m, p.k) + __builtin_amdgcn_logf(z);       // log2 of the row's sum of 2^(l*k)
        if (p.row_lse) p.row_lse[row] = lse2 * kLn2;
        if (tid < n_d) {
            x = p.draft_tokens[(size_t)b * ncol + tid];
            const bool valid = x >= 0 && x < V;
            if (valid) pr = fast_exp2(fmaf(p.logits[(size_t)row * V + x], p.k, -lse2));
            qv = 1.f;
            if (p.q_logits) {
                my_qrow = qr0 + tid;
                const int qrow = b * S + my_qrow;
                if (p.q_lse) {
                    q_lse2 = p.q_lse[qrow] * kLog2e;
                } else {
                    float mq, zq, m2q;
                    int aq;
                    merged_stats(p.q_stats + (size_t)qrow * p.nsplit, p.nsplit, p.k, mq, zq, aq, m2q);
                    q_lse2 = ref_k(mq, p.k) + __builtin_amdgcn_logf(zq);
                }
                qv = valid ? fast_exp2(fmaf(p.q_logits[(size_t)qrow * V + x], p.k, -q_lse2)) : 0.f;
            }
            if (is_greedy) {
                ok = (x == a);
            } else {
                const uint4 w = philox4x32_10(make_uint4(0u, (uint32_t)row, 0u, p.rng_offset), p.key);
                // q(x) = 0: a draft the proposer could not have drawn passes iff the anchor gives it any mass (p/q = inf),
                // and fails when the anchor gives it none (0/0: the output must stay on the anchor distribution)
                const float thr = qv > 0.f ? fminf(1.f, p.one_plus_tau * pr / qv) : (pr > 0.f ? 1.f : 0.f);
                ok = unit_uniform(w.x) < thr;
            }
        }
        if (tid < ncol) {
            if (p.draft_probs) p.draft_probs[(size_t)b * ncol + tid] = tid < n_d ? pr : 0.f;
            if (p.draft_q) p.draft_q[(size_t)b * ncol + tid] = tid < n_d ? qv : 0.f;
        }
    }
    const unsigned long long failed = __ballot(tid < n_d && !ok);
    const int r = failed ? (int)__builtin_ctzll(failed) : n_d;
    if (tid < S) {
        SampleJob job;
        job.mode = JOB_NONE; job.stream = 1; job.excluded = -1; job.fallback = a; job.lse2 = lse2;
        job.q_row = my_qrow; job.q_lse2 = q_lse2; job.floor = -INFINITY;
        int tok;
        if (tid < r) tok = x;
        else if (tid == r) {
            tok = a;
            if (!is_greedy) {
                if (r < n_d) {
                    job.mode = p.q_logits ? JOB_RESID_Q : JOB_RESID_POINT;
                    job.excluded = x;
                } else {
                    job.mode = JOB_PLAIN;
                }
            }
        } else if (tid <= n_d) tok = -1;
        else {
            tok = a;
            if (p.sample_proposals && !is_greedy) { job.mode = JOB_PLAIN; job.stream = 2; }
        }
        const int row = b * S + tid;
        if ((job.mode == JOB_PLAIN || job.mode == JOB_RESID_POINT) && m > -INFINITY) {
            // floor of the Gumbel-max over l/T + g: the arg-max element's own score, or, when that element is
            // the excluded one, the second-largest bound with the smallest possible noise
            if (job.excluded == a) {
                job.floor = m2 * p.inv_t + kGumbelMin;
            } else {
                const uint4 w = philox4x32_10(make_uint4((uint32_t)(a >> 2), (uint32_t)row, (uint32_t)job.stream, p.rng_offset),
                                              p.key);
                const int k4 = a & 3;
                job.floor = m * p.inv_t + gumbel(k4 == 0 ? w.x : k4 == 1 ? w.y : k4 == 2 ? w.z : w.w);
            }
        }
        p.jobs[row] = job;
        p.keys[row] = 0ull;
        if (job.mode == JOB_NONE) p.new_tokens[row] = tok;
    }
    if (tid == 0) p.accept_len[b] = r;
}

__global__ __launch_bounds__(256) void isd_accept_general_sample_kernel(const GeneralParams p, int nsb, int gchunk)
{
    const int row = blockIdx.x / nsb;           // b*S + j
    const int c = blockIdx.x - row * nsb;
    const int tid = threadIdx.x;
    const SampleJob job = p.jobs[row];
    if (job.mode == JOB_NONE) return;

    __shared__ float s_best[4];
    __shared__ int s_bidx[4];
    const int V = p.V;
    const float4* __restrict__ l4 = reinterpret_cast<const float4*>(p.logits + (size_t)row * V);
    const int b = row / p.S;
    const float4* __restrict__ q4 = job.mode == JOB_RESID_Q
        ? reinterpret_cast<const float4*>(p.q_logits + ((size_t)b * p.S + job.q_row) * V) : l4;
    const int fbeg = (c * gchunk) >> 2;
    const int fend = min(V, (c + 1) * gchunk) >> 2;
    float best = -INFINITY;
    int bidx = INT_MAX;
    if (job.mode == JOB_RESID_Q) {
        for (int f = fbeg + tid; f < fend; f += 256) {
            const float4 v = l4[f];
            const float4 t = q4[f];
            const uint4 w = philox4x32_10(make_uint4((uint32_t)f, (uint32_t)row, (uint32_t)job.stream, p.rng_offset), p.key);
            const float lv[4] = {v.x, v.y, v.z, v.w};
            const float qv[4] = {t.x, t.y, t.z, t.w};
            const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // ln(p_i - q_i) + g_i over the elements where the anchor exceeds the proposal
                const float pi = fast_exp2(fmaf(lv[e], p.k, -job.lse2));
                const float qi = fast_exp2(fmaf(qv[e], p.k, -job.q_lse2));
                if (!(pi > qi)) continue;
                const float s = logf(pi - qi) + gumbel(wv[e]);
                if (s > best) { best = s; bidx = f * 4 + e; }
            }
        }
    } else {
        // l/T + g with the exact pruning of the Gumbel-max (see isd_accept_common.h): an element is evaluated
        // only if 1 - u < e^(l/T - floor), behind a branch of the whole wavefront
        const float floor0 = job.floor;
        float thr = floor0;
        auto may_win = [&](float l, uint32_t word) {
            return one_minus_uniform(word) < fast_exp2(fmaf(l, p.k, fmaf(-thr, kLog2e, 0.01f)));
        };
        for (int f = fbeg + tid; f < fend; f += 256) {
            const float4 v = l4[f];
            if (fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)) * p.inv_t < thr - kNoiseMax) continue;
            const uint4 w = philox4x32_10(make_uint4((uint32_t)f, (uint32_t)row, (uint32_t)job.stream, p.rng_offset), p.key);
            const float lv[4] = {v.x, v.y, v.z, v.w};
            const uint32_t wv[4] = {w.x, w.y, w.z, w.w};
            bool pass[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) pass[e] = may_win(lv[e], wv[e]);
            if (__ballot(pass[0] || pass[1] || pass[2] || pass[3]) != 0ull) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = f * 4 + e;
                    if (!pass[e] || i == job.excluded) continue;
                    const float s = lv[e] * p.inv_t + gumbel(wv[e]);
                    if (s > best) { best = s; bidx = i; }
                }
                thr = fmaxf(best, floor0);
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float s2 = __shfl_xor(best, off);
        const int i2 = __shfl_xor(bidx, off);
        combine_best(best, bidx, s2, i2);
    }
    const int wvid = tid >> 6;
    if ((tid & 63) == 0) { s_best[wvid] = best; s_bidx[wvid] = bidx; }
    __syncthreads();
    if (tid == 0) {
        for (int q = 1; q < 4; ++q) combine_best(best, bidx, s_best[q], s_bidx[q]);
        if (bidx != INT_MAX) atomicMax(&p.keys[row], sample_key(best, bidx));
    }
}

__global__ __launch_bounds__(256) void isd_accept_general_emit_kernel(const GeneralParams p, int rows)
{
    const int row = blockIdx.x * 256 + threadIdx.x;
    if (row >= rows) return;
    const SampleJob job = p.jobs[row];
    if (job.mode == JOB_NONE) return;
    const unsigned long long key = p.keys[row];
    p.new_tokens[row] = key ? (int32_t)(0xFFFFFFFFu - (uint32_t)key) : job.fallback;
}

struct GeneralLayout {
    size_t stats_off, q_stats_off, keys_off, jobs_off, total;
};

static GeneralLayout general_layout(int32_t B, int32_t S, const AcceptPlan& plan)
{
    GeneralLayout w;
    const size_t stats = align256((size_t)B * S * plan.nsplit * sizeof(RowPartial));
    w.stats_off = 0;
    w.q_stats_off = stats;
    w.keys_off = 2 * stats;
    w.jobs_off = w.keys_off + align256((size_t)B * S * sizeof(unsigned long long));
    w.total = w.jobs_off + align256((size_t)B * S * sizeof(SampleJob));
    return w;
}

}  // namespace idlm

using namespace idlm;

extern "C" size_t idlm_isd_accept_general_workspace(int32_t B, int32_t S, int32_t V)
{
    if (B < 0 || S < 1 || S > 64 || V < 4 || (V & 3) || (int64_t)B * S >= INT32_MAX) return 0;
    if (B == 0) return 0;
    return general_layout(B, S, make_plan(B, S, V)).total;
}

extern "C" int idlm_isd_accept_general(const float* logits, const int32_t* draft_tokens, const float* q_logits,
                                       const int32_t* q_row, const float* q_lse, uint64_t rng_seed,
                                       int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S, int32_t V,
                                       int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                                       uint32_t rng_offset, float temperature, float tau, int32_t sample_proposals,
                                       float* draft_probs, float* draft_q, float* row_lse, void* workspace,
                                       size_t workspace_bytes, void* stream)
{
    if (B < 0 || S < 1 || S > 64 || V < 4 || (V & 3) || (int64_t)B * S >= INT32_MAX) return IDLM_ERR_SHAPE;
    if (!n_draft && (n_draft_uniform < 0 || n_draft_uniform > S - 1)) return IDLM_ERR_SHAPE;
    if (!(temperature > 0.f) || !(tau >= 0.f) || !(temperature < INFINITY) || !(tau < INFINITY)) return IDLM_ERR_SHAPE;
    if (B == 0) return IDLM_OK;
    if (!logits || !accept_len || !new_tokens) return IDLM_ERR_NULL;
    if (S > 1 && !draft_tokens) return IDLM_ERR_NULL;
    if (q_logits && !q_row) return IDLM_ERR_NULL;
    if (!aligned(logits, 16) || (q_logits && !aligned(q_logits, 16))) return IDLM_ERR_ALIGN;
    const AcceptPlan plan = make_plan(B, S, V);
    const GeneralLayout w = general_layout(B, S, plan);
    if (!workspace || workspace_bytes < w.total) return IDLM_ERR_WORKSPACE;
    if (!aligned(workspace, 256)) return IDLM_ERR_ALIGN;
    if ((int64_t)B * S * plan.nsplit >= INT32_MAX || (int64_t)B * S * plan.nsb >= INT32_MAX) return IDLM_ERR_SHAPE;

    char* ws = static_cast<char*>(workspace);
    GeneralParams p;
    p.logits = logits; p.draft_tokens = draft_tokens; p.q_logits = q_logits; p.q_row = q_row; p.q_lse = q_lse;
    p.stats = reinterpret_cast<RowPartial*>(ws + w.stats_off);
    p.q_stats = reinterpret_cast<RowPartial*>(ws + w.q_stats_off);
    p.accept_len = accept_len; p.new_tokens = new_tokens; p.n_draft = n_draft; p.greedy = greedy;
    p.draft_probs = draft_probs; p.draft_q = draft_q; p.row_lse = row_lse;
    p.jobs = reinterpret_cast<SampleJob*>(ws + w.jobs_off);
    p.keys = reinterpret_cast<unsigned long long*>(ws + w.keys_off);
    p.key = make_uint2((uint32_t)rng_seed, (uint32_t)(rng_seed >> 32));
    p.S = S; p.V = V; p.n_draft_uniform = n_draft_uniform; p.nsplit = plan.nsplit;
    p.sample_proposals = sample_proposals ? 1 : 0;
    p.rng_offset = rng_offset;
    p.inv_t = 1.f / temperature;
    p.k = kLog2e / temperature;
    p.one_plus_tau = 1.f + tau;
    hipStream_t st = static_cast<hipStream_t>(stream);

    (void)hipGetLastError();
    const unsigned rows_grid = (unsigned)(B * S * plan.nsplit);
    hipLaunchKernelGGL(isd_row_stats_kernel<16>, dim3(rows_grid), dim3(256), 0, st, logits, V, plan.chunk,
                       plan.nsplit, S, const_cast<RowPartial*>(p.stats), p.k);
    if (q_logits && !q_lse)
        hipLaunchKernelGGL(isd_row_stats_kernel<16>, dim3(rows_grid), dim3(256), 0, st, q_logits, V, plan.chunk,
                           plan.nsplit, S, const_cast<RowPartial*>(p.q_stats), p.k);
    hipLaunchKernelGGL(isd_accept_general_chain_kernel, dim3((unsigned)B), dim3(64), 0, st, p);
    hipLaunchKernelGGL(isd_accept_general_sample_kernel, dim3((unsigned)(B * S * plan.nsb)), dim3(256), 0, st, p,
                       plan.nsb, plan.gchunk);
    hipLaunchKernelGGL(isd_accept_general_emit_kernel, dim3((unsigned)((B * S + 255) / 256)), dim3(256), 0, st, p,
                       B * S);
    return launch_status();
}
