/*
 * CPU oracle for one introspective-strided-decoding (ISD) step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, double-precision
 * statement of what the two hot-path calls compute.  It is used by tests/, by
 * the smoke check and by the benchmark's cpu_baseline leg, never by the product
 * path, and it shares no code, header, table or helper with the HIP library.
 *
 * What is written out here:
 *   - attention:  the definition of causal softmax attention of S query rows
 *     per sequence over a paged KV cache (strict causal masking, Sec. 3.1
 *     "Causal training with logit shift": key i visible to query j iff i <= j;
 *     one paged extend of the stride's rows, Sec. 3.3 (1) and App. D).
 *   - acceptance: Alg. 1's introspection loop, specialised to point-mass
 *     (arg-max) proposals as deployed in Sec. 3.3 (3): accept test, accepted
 *     prefix, resample from the residual on the first rejection, bonus token
 *     when every draft passes, arg-max proposals from the MASK rows.
 *   - acceptance with general proposal distributions (Alg. 1 as printed: drafts
 *     sampled from q, accept with probability min(1, p/q), residual
 *     normalize(max(0, p - q))), sampling temperature and the relaxed threshold.
 *   - acceptance under the filtered sampling distribution of the paper's runs (App. H:
 *     temperature, top-k, top-p), with point-mass proposals or with drafts drawn from the
 *     filtered distribution of the row that proposed them.
 *   - the counter-based generator Philox4x32-10 (Salmon et al., SC'11) that
 *     supplies the uniforms of the accept test and of the Gumbel-max sampler.
 *   - the two steps that close the loop between consecutive ISD steps (Sec. 3.3
 *     (2): forward -> verify -> trim -> prepare -> forward): the batched scatter
 *     of the stride's K/V rows into the pages (kv_append), and trim-and-commit
 *     plus preparation of the next stride (commit) after Alg. 1's last line.
 *   - one linear layer of the lossless variant (App. G): base projection for
 *     every token, low-rank residual only at MASK positions (gated_lora_linear).
 *
 * Pins (tests that check this file against something other than itself) are in
 * tests/test_oracle_*.py; every function here has at least one.
 *
 * No blocking, fusion or reordering: loops follow the definitions.  OpenMP is
 * used only to run independent (sequence, head) / (sequence) items in parallel.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_TABLE (-2) /* a block-table entry that had to be read is out of range */

/* ------------------------------------------------------------------------ */
/* Philox4x32-10                                                              */
/* ------------------------------------------------------------------------ */

/* One call: 128-bit counter ctr[4], 64-bit key key[2] -> 4 output words.
 * Ten rounds; each round multiplies counter words 0 and 2 by fixed odd
 * constants, mixes high/low halves with the other words and the key, and the
 * key is bumped by the Weyl constants between rounds. */
void isd_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)M0 * c0;
        uint64_t p1 = (uint64_t)M1 * c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* 32 random bits -> u in (0,1): u = (2*(x>>9) + 1) * 2^-24.  The numerator is an
 * odd 24-bit integer, so u is exact in fp32 and never 0 or 1. */
static double uniform_from_bits(uint32_t x)
{
    return (double)(2u * (x >> 9) + 1u) * (1.0 / 16777216.0);
}

/* Random word for vocabulary element i of logit row `row`:
 * counter = (i>>2, row, stream, offset), key = (seed lo, seed hi), word i&3.
 * stream 0 = accept-test uniform (element 0 only), stream 1 = Gumbel noise. */
static uint32_t rng_word(uint64_t seed, uint32_t offset, uint32_t stream, uint32_t row, uint32_t i)
{
    uint32_t ctr[4] = { i >> 2, row, stream, offset };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    isd_oracle_philox4x32_10(ctr, key, out);
    return out[i & 3u];
}

/* The uniforms (and, if asked, the Gumbel noise -ln(-ln u)) of elements 0..V-1 of rows
 * row0..row0+n_rows-1 under a stream tag, one by one through rng_word. */
void isd_oracle_rng_dump(uint64_t seed, uint32_t offset, uint32_t stream, uint32_t row0, int32_t n_rows, int32_t V,
                         double* uniforms, double* gumbels)
{
    for (int r = 0; r < n_rows; ++r)
        for (int i = 0; i < V; ++i) {
            const double u = uniform_from_bits(rng_word(seed, offset, stream, row0 + (uint32_t)r, (uint32_t)i));
            if (uniforms) uniforms[(int64_t)r * V + i] = u;
            if (gumbels) gumbels[(int64_t)r * V + i] = -log(-log(u));
        }
}

double isd_oracle_accept_uniform(uint64_t seed, uint32_t offset, uint32_t row)
{
    return uniform_from_bits(rng_word(seed, offset, 0u, row, 0u));
}

double isd_oracle_gumbel(uint64_t seed, uint32_t offset, uint32_t row, uint32_t i)
{
    double u = uniform_from_bits(rng_word(seed, offset, 1u, row, i));
    return -log(-log(u));
}

/* ------------------------------------------------------------------------ */
/* Attention                                                                  */
/* ------------------------------------------------------------------------ */

static double load_elem(const void* base, int64_t idx, int dtype)
{
    if (dtype == 0) return (double)((const float*)base)[idx];
    /* bf16: the upper 16 bits of an IEEE fp32 */
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/*
 * out[b,i,h,:] = sum_t softmax_t(scale * <q[b,i,h,:], k_t[h/G,:]>) * v_t[h/G,:]
 * over keys t = 0 .. ctx_lens[b]-S+i  (query row i sits at absolute position
 * ctx_lens[b]-S+i; ctx_lens counts the S rows of this step, whose K/V are
 * already in the pages).  Key t lives in page block_table[b][t/P], slot t%P.
 *
 * q   [B,S,Hq,D] contiguous; k_cache / v_cache: element (page,hk,slot,d) at
 * page*page_stride + hk*head_stride + slot*token_stride + d (in elements).
 * dtype 0 = fp32, 1 = bf16 bit patterns.  out is double [B,S,Hq,D].
 * Only sequences/heads with sel==NULL or sel[b*Hkv+hk]!=0 are computed (others
 * are left untouched) so that large workloads can be spot-checked.
 */
int isd_oracle_attention(const void* q, const void* k_cache, const void* v_cache,
                         const int32_t* block_table, const int32_t* ctx_lens, int32_t S,
                         double* out, int32_t B, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                         int32_t num_pages, int32_t max_pages_per_seq, int64_t page_stride,
                         int64_t head_stride, int64_t token_stride, double scale, int32_t dtype,
                         const uint8_t* sel)
{
    if (!q || !k_cache || !v_cache || !block_table || !ctx_lens || !out) return ORACLE_ERR_ARG;
    if (B < 0 || S < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || D < 1 || P < 1) return ORACLE_ERR_ARG;
    if (dtype != 0 && dtype != 1) return ORACLE_ERR_ARG;
    const int G = Hq / Hkv;
    if (!(scale > 0.0)) scale = 1.0 / sqrt((double)D);
    int status = ORACLE_OK;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int hk = 0; hk < Hkv; ++hk) {
            if (sel && !sel[b * Hkv + hk]) continue;
            const int ctx = ctx_lens[b];
            if (ctx < S || (ctx + P - 1) / P > max_pages_per_seq) {
#pragma omp critical
                status = ORACLE_ERR_ARG;
                continue;
            }
            double* score = (double*)malloc((size_t)ctx * sizeof(double));
            for (int i = 0; i < S; ++i) {
                const int last = ctx - S + i; /* last visible key */
                for (int g = 0; g < G; ++g) {
                    const int h = hk * G + g;
                    const int64_t qoff = (((int64_t)b * S + i) * Hq + h) * D;
                    double smax = -INFINITY;
                    int bad = 0;
                    for (int t = 0; t <= last; ++t) {
                        const int page = block_table[(int64_t)b * max_pages_per_seq + t / P];
                        if (page < 0 || page >= num_pages) { bad = 1; break; }
                        const int64_t koff = page * page_stride + hk * head_stride + (t % P) * token_stride;
                        double dot = 0.0;
                        for (int d = 0; d < D; ++d)
                            dot += load_elem(q, qoff + d, dtype) * load_elem(k_cache, koff + d, dtype);
                        score[t] = scale * dot;
                        if (score[t] > smax) smax = score[t];
                    }
                    if (bad) {
#pragma omp critical
                        status = ORACLE_ERR_TABLE;
                        continue;
                    }
                    double denom = 0.0;
                    for (int t = 0; t <= last; ++t) {
                        score[t] = exp(score[t] - smax);
                        denom += score[t];
                    }
                    double* o = out + qoff;
                    for (int d = 0; d < D; ++d) o[d] = 0.0;
                    for (int t = 0; t <= last; ++t) {
                        const int page = block_table[(int64_t)b * max_pages_per_seq + t / P];
                        const int64_t voff = page * page_stride + hk * head_stride + (t % P) * token_stride;
                        const double w = score[t] / denom;
                        for (int d = 0; d < D; ++d) o[d] += w * load_elem(v_cache, voff + d, dtype);
                    }
                }
            }
            free(score);
        }
    }
    return status;
}

/* ------------------------------------------------------------------------ */
/* Introspective acceptance                                                   */
/* ------------------------------------------------------------------------ */

/*
 * One sequence b has S logit rows.  Row j < n_d is the causal anchor of drafted
 * token j (the model's own next-token distribution at the position before that
 * draft), row n_d is the anchor after the last draft (bonus token), rows > n_d
 * come from MASK positions and propose next step's drafts.
 *
 * Steps, in Alg. 1's order, with the proposal distribution a point mass on the
 * draft (arg-max proposals, Sec. 3.3 (3)), so min(1, p/q) = p(draft) and the
 * residual normalize(max(0, p - q)) is p with the draft removed:
 *   1. every row: m = max, Z = sum exp(l - m), a = lowest index attaining m
 *   2. j < n_d: p_j = exp(l[draft_j] - m_j) / Z_j           -> draft_probs
 *   3. accept test j < n_d: greedy: draft_j == a_j ; else u_j < p_j (strict)
 *   4. accept_len r = number of leading accepted drafts
 *   5. the one fresh token comes from row r:
 *        greedy:      a_r
 *        stochastic:  argmax_i (l_r[i] + gumbel_i), excluding i == draft_r iff r < n_d
 *   6. new_tokens[j] = draft_j (j < r) | fresh token (j == r) | -1 (r < j <= n_d)
 *                      | a_j (j > n_d)
 *
 * Diagnostic outputs (may be NULL) let a test decide whether a floating-point
 * decision is far enough from its threshold to be compared bit-for-bit with a
 * single-precision implementation:
 *   accept_margin[b,j] = |u_j - p_j| for stochastic j < n_d (INFINITY otherwise)
 *   sample_gap[b]      = best minus second-best perturbed score in row r
 *                        (INFINITY for greedy sequences)
 *   runner_up[b]       = index of that second-best element (-1 for greedy)
 */
int isd_oracle_accept(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                      int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S, int32_t V,
                      int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                      uint32_t rng_offset, double* draft_probs, double* accept_margin,
                      double* sample_gap, int32_t* runner_up)
{
    if (!logits || !accept_len || !new_tokens) return ORACLE_ERR_ARG;
    if (B < 0 || S < 1 || V < 1) return ORACLE_ERR_ARG;
    if (S > 1 && !draft_tokens) return ORACLE_ERR_ARG;
    const int ncol = S - 1;
    int status = ORACLE_OK;

#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int n_d = n_draft ? n_draft[b] : n_draft_uniform;
        if (n_d < 0 || n_d > S - 1) {
#pragma omp critical
            status = ORACLE_ERR_ARG;
            continue;
        }
        const int is_greedy = greedy ? (greedy[b] != 0) : 0;
        double* m = (double*)malloc(sizeof(double) * S);
        double* Z = (double*)malloc(sizeof(double) * S);
        int32_t* a = (int32_t*)malloc(sizeof(int32_t) * S);

        /* step 1 */
        for (int j = 0; j < S; ++j) {
            const float* l = logits + ((int64_t)b * S + j) * V;
            double mx = -INFINITY;
            int arg = 0;
            for (int i = 0; i < V; ++i)
                if ((double)l[i] > mx) { mx = (double)l[i]; arg = i; }
            double z = 0.0;
            for (int i = 0; i < V; ++i) z += exp((double)l[i] - mx);
            m[j] = mx; Z[j] = z; a[j] = arg;
        }

        /* steps 2-4 */
        int r = n_d;
        int open = 1; /* still inside the accepted prefix */
        for (int j = 0; j < ncol; ++j) {
            if (draft_probs) draft_probs[(int64_t)b * ncol + j] = 0.0;
            if (accept_margin) accept_margin[(int64_t)b * ncol + j] = INFINITY;
        }
        for (int j = 0; j < n_d; ++j) {
            const float* l = logits + ((int64_t)b * S + j) * V;
            const int x = draft_tokens[(int64_t)b * ncol + j];
            if (x < 0 || x >= V) {
#pragma omp critical
                status = ORACLE_ERR_ARG;
                continue;
            }
            const double p = exp((double)l[x] - m[j]) / Z[j];
            if (draft_probs) draft_probs[(int64_t)b * ncol + j] = p;
            int ok;
            if (is_greedy) {
                ok = (x == a[j]);
            } else {
                const double u = isd_oracle_accept_uniform(rng_seed, rng_offset, (uint32_t)(b * S + j));
                ok = (u < p);
                if (accept_margin) accept_margin[(int64_t)b * ncol + j] = fabs(u - p);
            }
            if (open && !ok) { r = j; open = 0; }
        }
        accept_len[b] = r;

        /* step 5 */
        int fresh;
        double gap = INFINITY;
        int second = -1;
        if (is_greedy) {
            fresh = a[r];
        } else {
            const float* l = logits + ((int64_t)b * S + r) * V;
            const int excluded = (r < n_d) ? draft_tokens[(int64_t)b * ncol + r] : -1;
            double best = -INFINITY, next = -INFINITY;
            fresh = -1;
            for (int i = 0; i < V; ++i) {
                if (i == excluded) continue;
                const double s = (double)l[i] + isd_oracle_gumbel(rng_seed, rng_offset, (uint32_t)(b * S + r), (uint32_t)i);
                if (s > best) { next = best; second = fresh; best = s; fresh = i; }
                else if (s > next) { next = s; second = i; }
            }
            gap = best - next;
        }
        if (sample_gap) sample_gap[b] = gap;
        if (runner_up) runner_up[b] = second;

        /* step 6 */
        for (int j = 0; j < S; ++j) {
            int32_t tok;
            if (j < r) tok = draft_tokens[(int64_t)b * ncol + j];
            else if (j == r) tok = fresh;
            else if (j <= n_d) tok = -1;
            else tok = a[j];
            new_tokens[(int64_t)b * S + j] = tok;
        }
        free(m); free(Z); free(a);
    }
    return status;
}

/* ------------------------------------------------------------------------ */
/* Acceptance with general proposal distributions                            */
/* ------------------------------------------------------------------------ */

/* Gumbel noise of the proposal sampler: stream tag 2 of the same generator. */
static double proposal_gumbel(uint64_t seed, uint32_t offset, uint32_t row, uint32_t i)
{
    double u = uniform_from_bits(rng_word(seed, offset, 2u, row, i));
    return -log(-log(u));
}

/* log-sum-exp of row l / T (max subtracted first) and the lowest arg-max index */
static void row_lse(const float* l, int V, double T, double* lse, int32_t* arg)
{
    double mx = -INFINITY;
    int a = 0;
    for (int i = 0; i < V; ++i)
        if ((double)l[i] > mx) { mx = (double)l[i]; a = i; }
    double z = 0.0;
    for (int i = 0; i < V; ++i) z += exp(((double)l[i] - mx) / T);
    *lse = mx / T + log(z);
    *arg = a;
}

/*
 * Alg. 1 in full: drafts x_j drawn from proposal distributions q_j, accepted with
 * probability min(1, p_j(x_j)/q_j(x_j)), resampled from normalize(max(0, p_j - q_j)) at
 * the first rejection (Sec. 3.2 "Adaptive stride via p/q acceptance"), with the two
 * knobs the paper's runs use on top: sampling temperature T (App. H: all runs at
 * T = 1, here any T > 0: p = softmax(l/T), q = softmax(l'/T)) and the relaxed
 * threshold that Sec. 5 names as a way to trade exactness for speed: accept iff
 * u < min(1, (1+tau) * p/q).
 *
 * q_logits == NULL is the deployed setting (point-mass proposals, q_j(x_j) = 1).
 * Otherwise q_j = softmax(q_logits[b, q_row[b] + j, :] / T): the previous step's logits
 * of the MASK row that proposed draft j.
 *
 * For sequence b with D drafts:
 *   1. every row j: lse_j of l_j/T, arg-max a_j.
 *   2. j < D: p_j = exp(l_j[x_j]/T - lse_j); q_j likewise from the q row (1 for point mass).
 *   3. accept_j: greedy ? x_j == a_j : u_{b,j} < min(1, (1+tau) p_j/q_j)   (q_j = 0: accepted iff p_j > 0).
 *   4. r = accepted prefix.
 *   5. fresh token of row r: greedy: a_r.  Otherwise, after a rejection (r < D):
 *        argmax_i [ln(p_r(i) - q_r(i)) + g_{b,r,i}] over i with p_r(i) > q_r(i)
 *        (point mass: q_r = delta at x_r); a_r if no such i exists;
 *      with all accepted (r = D): argmax_i [l_r[i]/T + g_{b,r,i}].
 *   6. new_tokens: x_j (j < r) | fresh (j = r) | -1 (r < j <= D) | proposal (j > D):
 *      sample_proposals ? argmax_i [l_j[i]/T + g2_{b,j,i}] (stream 2) : a_j.
 * Outputs draft_probs (p_j), draft_q (q_j), row_lse [B,S]; diagnostics as in
 * isd_oracle_accept, accept_margin = |u - min(1,(1+tau)p/q)|, plus proposal_gap [B,S]
 * (top-two gap of the perturbed scores of every sampled proposal row, INFINITY elsewhere).
 */
int isd_oracle_accept_general(const float* logits, const int32_t* draft_tokens, const float* q_logits,
                              const int32_t* q_row, uint64_t rng_seed, int32_t* accept_len,
                              int32_t* new_tokens, int32_t B, int32_t S, int32_t V, int32_t n_draft_uniform,
                              const int32_t* n_draft, const uint8_t* greedy, uint32_t rng_offset,
                              double temperature, double tau, int32_t sample_proposals,
                              double* draft_probs, double* draft_q, double* row_lse_out,
                              double* accept_margin, double* sample_gap, int32_t* runner_up,
                              double* proposal_gap)
{
    if (!logits || !accept_len || !new_tokens) return ORACLE_ERR_ARG;
    if (B < 0 || S < 1 || V < 1 || !(temperature > 0.0) || !(tau >= 0.0)) return ORACLE_ERR_ARG;
    if (S > 1 && !draft_tokens) return ORACLE_ERR_ARG;
    if (q_logits && !q_row) return ORACLE_ERR_ARG;
    const int ncol = S - 1;
    const double T = temperature;
    int status = ORACLE_OK;

#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int D = n_draft ? n_draft[b] : n_draft_uniform;
        int bad = (D < 0 || D > S - 1);
        if (!bad && q_logits && D > 0 && (q_row[b] < 0 || q_row[b] + D > S)) bad = 1;
        for (int j = 0; !bad && j < D; ++j) {
            const int x = draft_tokens[(int64_t)b * ncol + j];
            if (x < 0 || x >= V) bad = 1;
        }
        if (bad) {
#pragma omp critical
            status = ORACLE_ERR_ARG;
            continue;
        }
        const int is_greedy = greedy ? (greedy[b] != 0) : 0;
        double* lse = (double*)malloc(sizeof(double) * S);
        int32_t* a = (int32_t*)malloc(sizeof(int32_t) * S);
        for (int j = 0; j < S; ++j) {
            row_lse(logits + ((int64_t)b * S + j) * V, V, T, &lse[j], &a[j]);
            if (row_lse_out) row_lse_out[(int64_t)b * S + j] = lse[j];
        }
        for (int j = 0; j < ncol; ++j) {
            if (draft_probs) draft_probs[(int64_t)b * ncol + j] = 0.0;
            if (draft_q) draft_q[(int64_t)b * ncol + j] = 0.0;
            if (accept_margin) accept_margin[(int64_t)b * ncol + j] = INFINITY;
        }
        int r = D, open = 1;
        for (int j = 0; j < D; ++j) {
            const float* l = logits + ((int64_t)b * S + j) * V;
            const int x = draft_tokens[(int64_t)b * ncol + j];
            const double p = exp((double)l[x] / T - lse[j]);
            double q = 1.0;
            if (q_logits) {
                const float* lq = q_logits + ((int64_t)b * S + q_row[b] + j) * V;
                double lse_q;
                int32_t aq;
                row_lse(lq, V, T, &lse_q, &aq);
                q = exp((double)lq[x] / T - lse_q);
            }
            if (draft_probs) draft_probs[(int64_t)b * ncol + j] = p;
            if (draft_q) draft_q[(int64_t)b * ncol + j] = q;
            int ok;
            if (is_greedy) {
                ok = (x == a[j]);
            } else {
                const double u = isd_oracle_accept_uniform(rng_seed, rng_offset, (uint32_t)(b * S + j));
                /* q = 0: p/q is infinite for p > 0 (accepted); p = q = 0 is rejected, so that no token
                 * of zero anchor probability is ever finalised (Sec. 3.2: the output follows p) */
                double thr = (q > 0.0) ? (1.0 + tau) * p / q : (p > 0.0 ? INFINITY : 0.0);
                if (thr > 1.0) thr = 1.0;
                ok = (u < thr);
                if (accept_margin) accept_margin[(int64_t)b * ncol + j] = fabs(u - thr);
            }
            if (open && !ok) { r = j; open = 0; }
        }
        accept_len[b] = r;

        int fresh;
        double gap = INFINITY;
        int second = -1;
        if (is_greedy) {
            fresh = a[r];
        } else {
            const float* l = logits + ((int64_t)b * S + r) * V;
            const uint32_t row = (uint32_t)(b * S + r);
            double best = -INFINITY, next = -INFINITY;
            fresh = -1;
            if (r < D) {
                const int x = draft_tokens[(int64_t)b * ncol + r];
                const float* lq = q_logits ? q_logits + ((int64_t)b * S + q_row[b] + r) * V : NULL;
                double lse_q = 0.0;
                int32_t aq;
                if (lq) row_lse(lq, V, T, &lse_q, &aq);
                for (int i = 0; i < V; ++i) {
                    const double pi = exp((double)l[i] / T - lse[r]);
                    const double qi = lq ? exp((double)lq[i] / T - lse_q) : (i == x ? 1.0 : 0.0);
                    if (!(pi > qi)) continue;
                    const double sc = log(pi - qi) + isd_oracle_gumbel(rng_seed, rng_offset, row, (uint32_t)i);
                    if (sc > best) { next = best; second = fresh; best = sc; fresh = i; }
                    else if (sc > next) { next = sc; second = i; }
                }
                if (fresh < 0) { fresh = a[r]; best = INFINITY; }
            } else {
                for (int i = 0; i < V; ++i) {
                    const double sc = (double)l[i] / T + isd_oracle_gumbel(rng_seed, rng_offset, row, (uint32_t)i);
                    if (sc > best) { next = best; second = fresh; best = sc; fresh = i; }
                    else if (sc > next) { next = sc; second = i; }
                }
            }
            gap = best - next;
        }
        if (sample_gap) sample_gap[b] = gap;
        if (runner_up) runner_up[b] = second;

        for (int j = 0; j < S; ++j) {
            int32_t tok;
            double pg = INFINITY;
            if (j < r) tok = draft_tokens[(int64_t)b * ncol + j];
            else if (j == r) tok = fresh;
            else if (j <= D) tok = -1;
            else if (!sample_proposals || is_greedy) tok = a[j];
            else {
                const float* l = logits + ((int64_t)b * S + j) * V;
                double best = -INFINITY, next = -INFINITY;
                tok = -1;
                for (int i = 0; i < V; ++i) {
                    const double sc = (double)l[i] / T + proposal_gumbel(rng_seed, rng_offset, (uint32_t)(b * S + j), (uint32_t)i);
                    if (sc > best) { next = best; best = sc; tok = i; }
                    else if (sc > next) next = sc;
                }
                pg = best - next;
            }
            new_tokens[(int64_t)b * S + j] = tok;
            if (proposal_gap) proposal_gap[(int64_t)b * S + j] = pg;
        }
        free(lse); free(a);
    }
    return status;
}

/* ------------------------------------------------------------------------ */
/* Acceptance under a filtered sampling distribution (top-k, top-p)          */
/* ------------------------------------------------------------------------ */

typedef struct { double v; int32_t i; } cand_t;

static int cand_cmp(const void* a, const void* b)
{
    const cand_t* x = (const cand_t*)a;
    const cand_t* y = (const cand_t*)b;
    if (x->v > y->v) return -1;
    if (x->v < y->v) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

/* The sampling distribution of a row under the set-up the paper's runs use (App. H, ISD
 * configuration table: temperature 1.0, top_k 50, top_p 0.95), applied in the usual order:
 * temperature, then the top_k largest logits (equal values: lowest index first), then the
 * shortest prefix of those, in descending order, whose renormalised probability mass reaches
 * top_p (at least one element).  Returns the number kept; idx[] their vocabulary ids in
 * descending order, prob[] their renormalised probabilities. */
static int filtered_row(const float* l, int V, double T, int top_k, double top_p, cand_t* work,
                        int32_t* idx, double* prob, double* cut_margin)
{
    for (int i = 0; i < V; ++i) { work[i].v = (double)l[i]; work[i].i = i; }
    qsort(work, (size_t)V, sizeof(cand_t), cand_cmp);
    int n = top_k < V ? top_k : V;
    double sum = 0.0;
    for (int c = 0; c < n; ++c) { prob[c] = exp((work[c].v - work[0].v) / T); sum += prob[c]; }
    double cum = 0.0, margin = INFINITY;
    int keep = n;
    for (int c = 0; c < n; ++c) {
        cum += prob[c] / sum;
        if (c + 1 < n && fabs(cum - top_p) < margin) margin = fabs(cum - top_p);   /* the last prefix is kept anyway */
        if (cum >= top_p) { keep = c + 1; break; }
    }
    if (cut_margin) *cut_margin = margin;
    double s2 = 0.0;
    for (int c = 0; c < keep; ++c) s2 += prob[c];
    for (int c = 0; c < keep; ++c) { prob[c] /= s2; idx[c] = work[c].i; }
    return keep;
}

/* Probability of vocabulary id x under a filtered row (0 outside the kept set). */
static double filtered_prob_of(const int32_t* idx, const double* prob, int cnt, int x)
{
    for (int c = 0; c < cnt; ++c)
        if (idx[c] == x) return prob[c];
    return 0.0;
}

/*
 * Alg. 1 under the filtered sampling distribution pf_j of every row (see filtered_row), with
 * point-mass proposals (q_logits == NULL: the deployed setting, q_j(x_j) = 1) or with proposals
 * drawn from the filtered distribution qf_j of the row that proposed them (Alg. 1 as printed,
 * Sec. 3.2 "Adaptive stride via p/q acceptance", under the sampler of App. H:
 * qf_j = filter(q_logits[b, q_row[b] + j, :]) with the same temperature, top_k and top_p):
 *   accept draft x_j iff u < min(1, (1+tau) pf_j(x_j) / qf_j(x_j)); a draft outside qf_j's
 *   support (it cannot have been drawn from it) is accepted iff pf_j(x_j) > 0;
 *   greedy sequences: x_j == arg-max;
 *   on the first rejection, row r resamples from normalize(max(0, pf_r - qf_r)) (point mass:
 *   pf_r without x_r); the bonus token after D acceptances is a draw from pf_D;
 *   proposals of the rows after the drafts: arg-max, or (sample_proposals) a draw from pf_j
 *   with random stream 2.
 * Draws are Gumbel-max over the kept elements with the noise of their vocabulary ids, so that
 * the unfiltered case (top_k >= V, top_p = 1) reproduces isd_oracle_accept_general.
 * Outputs as isd_oracle_accept; kept[b,j] = number of elements of row j that survive the filter;
 * draft_q[b,j] = qf_j(x_j) (1 for point mass); cut_margin[b,j] (and q_cut_margin[b,j] for the
 * proposing row of draft j) = distance of the closest cumulative probability from top_p (a
 * single-precision implementation may cut such a row one element earlier or later when this is
 * tiny); resid_small[b] = the smaller of pf - qf at the winner and the runner-up of a residual
 * draw (the difference cancels in single precision when it is tiny), INFINITY otherwise.
 * A rejection with an empty residual cannot happen for tau = 0 (it needs pf_r <= qf_r
 * everywhere, hence pf_r == qf_r and a ratio of 1); should rounding or tau produce it, row r's
 * arg-max is emitted.
 */
static int accept_filtered_impl(const float* logits, const int32_t* draft_tokens, const float* q_logits,
                                const int32_t* q_row, uint64_t rng_seed,
                                int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S, int32_t V,
                                int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                                uint32_t rng_offset, double temperature, double tau, int32_t top_k,
                                double top_p, int32_t sample_proposals, double* draft_probs, double* draft_q,
                                int32_t* kept, double* accept_margin, double* sample_gap, int32_t* runner_up,
                                double* proposal_gap, double* cut_margin, double* q_cut_margin,
                                double* resid_small)
{
    if (!logits || !accept_len || !new_tokens) return ORACLE_ERR_ARG;
    if (B < 0 || S < 1 || V < 1 || !(temperature > 0.0) || !(tau >= 0.0)) return ORACLE_ERR_ARG;
    if (top_k < 1 || !(top_p > 0.0) || !(top_p <= 1.0)) return ORACLE_ERR_ARG;
    if (S > 1 && !draft_tokens) return ORACLE_ERR_ARG;
    if (q_logits && !q_row) return ORACLE_ERR_ARG;
    const int ncol = S - 1;
    const int K = top_k < V ? top_k : V;
    int status = ORACLE_OK;

#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int D = n_draft ? n_draft[b] : n_draft_uniform;
        int bad = (D < 0 || D > S - 1);
        if (!bad && q_logits && D > 0 && (q_row[b] < 0 || q_row[b] + D > S)) bad = 1;
        for (int j = 0; !bad && j < D; ++j) {
            const int x = draft_tokens[(int64_t)b * ncol + j];
            if (x < 0 || x >= V) bad = 1;
        }
        if (bad) {
#pragma omp critical
            status = ORACLE_ERR_ARG;
            continue;
        }
        const int is_greedy = greedy ? (greedy[b] != 0) : 0;
        cand_t* work = (cand_t*)malloc(sizeof(cand_t) * (size_t)V);
        int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)S * K);
        double* prob = (double*)malloc(sizeof(double) * (size_t)S * K);
        int* cnt = (int*)malloc(sizeof(int) * S);
        int32_t* qidx = (int32_t*)malloc(sizeof(int32_t) * (size_t)S * K);   /* proposing row of draft j */
        double* qprob = (double*)malloc(sizeof(double) * (size_t)S * K);
        int* qcnt = (int*)malloc(sizeof(int) * S);
        for (int j = 0; j < S; ++j) {
            cnt[j] = filtered_row(logits + ((int64_t)b * S + j) * V, V, temperature, top_k, top_p, work,
                                  idx + (size_t)j * K, prob + (size_t)j * K,
                                  cut_margin ? cut_margin + (int64_t)b * S + j : NULL);
            if (kept) kept[(int64_t)b * S + j] = cnt[j];
        }
        for (int j = 0; j < ncol; ++j) {
            if (draft_probs) draft_probs[(int64_t)b * ncol + j] = 0.0;
            if (draft_q) draft_q[(int64_t)b * ncol + j] = 0.0;
            if (accept_margin) accept_margin[(int64_t)b * ncol + j] = INFINITY;
            if (q_cut_margin) q_cut_margin[(int64_t)b * ncol + j] = INFINITY;
        }
        for (int j = 0; q_logits && j < D; ++j)
            qcnt[j] = filtered_row(q_logits + ((int64_t)b * S + q_row[b] + j) * V, V, temperature, top_k, top_p, work,
                                   qidx + (size_t)j * K, qprob + (size_t)j * K,
                                   q_cut_margin ? q_cut_margin + (int64_t)b * ncol + j : NULL);
        int r = D, open = 1;
        for (int j = 0; j < D; ++j) {
            const int x = draft_tokens[(int64_t)b * ncol + j];
            const double pf = filtered_prob_of(idx + (size_t)j * K, prob + (size_t)j * K, cnt[j], x);
            const double qf = q_logits ? filtered_prob_of(qidx + (size_t)j * K, qprob + (size_t)j * K, qcnt[j], x) : 1.0;
            if (draft_probs) draft_probs[(int64_t)b * ncol + j] = pf;
            if (draft_q) draft_q[(int64_t)b * ncol + j] = qf;
            int ok;
            if (is_greedy) {
                ok = (x == idx[(size_t)j * K]);
            } else {
                const double u = isd_oracle_accept_uniform(rng_seed, rng_offset, (uint32_t)(b * S + j));
                double thr = (qf > 0.0) ? (1.0 + tau) * pf / qf : (pf > 0.0 ? INFINITY : 0.0);
                if (thr > 1.0) thr = 1.0;
                ok = (u < thr);
                if (accept_margin) accept_margin[(int64_t)b * ncol + j] = fabs(u - thr);
            }
            if (open && !ok) { r = j; open = 0; }
        }
        accept_len[b] = r;

        int fresh = idx[(size_t)r * K];
        double gap = INFINITY, small = INFINITY;
        int second = -1;
        if (!is_greedy) {
            const int x = (r < D) ? draft_tokens[(int64_t)b * ncol + r] : -1;
            double best = -INFINITY, next = -INFINITY, w_best = INFINITY, w_next = INFINITY;
            int found = -1;
            for (int c = 0; c < cnt[r]; ++c) {
                const int i = idx[(size_t)r * K + c];
                double w = prob[(size_t)r * K + c];            /* bonus token: pf_D itself */
                if (r < D) {                                   /* residual max(0, pf_r - qf_r) */
                    const double qv = q_logits ? filtered_prob_of(qidx + (size_t)r * K, qprob + (size_t)r * K, qcnt[r], i)
                                               : (i == x ? 1.0 : 0.0);
                    w -= qv;
                    if (!(w > 0.0)) continue;
                }
                const double sc = log(w) + isd_oracle_gumbel(rng_seed, rng_offset, (uint32_t)(b * S + r), (uint32_t)i);
                if (sc > best || (sc == best && i < found)) { next = best; second = found; w_next = w_best; best = sc; found = i; w_best = w; }
                else if (sc > next) { next = sc; second = i; w_next = w; }
            }
            if (found >= 0) { fresh = found; gap = best - next; }
            if (r < D && q_logits && found >= 0) small = w_best < w_next ? w_best : w_next;
        }
        if (sample_gap) sample_gap[b] = gap;
        if (runner_up) runner_up[b] = second;
        if (resid_small) resid_small[b] = small;

        for (int j = 0; j < S; ++j) {
            int32_t tok;
            double pg = INFINITY;
            if (j < r) tok = draft_tokens[(int64_t)b * ncol + j];
            else if (j == r) tok = fresh;
            else if (j <= D) tok = -1;
            else if (!sample_proposals || is_greedy) tok = idx[(size_t)j * K];
            else {
                double best = -INFINITY, next = -INFINITY;
                tok = -1;
                for (int c = 0; c < cnt[j]; ++c) {
                    const int i = idx[(size_t)j * K + c];
                    const double sc = log(prob[(size_t)j * K + c]) + proposal_gumbel(rng_seed, rng_offset, (uint32_t)(b * S + j), (uint32_t)i);
                    if (sc > best || (sc == best && i < tok)) { next = best; best = sc; tok = i; }
                    else if (sc > next) next = sc;
                }
                pg = best - next;
            }
            new_tokens[(int64_t)b * S + j] = tok;
            if (proposal_gap) proposal_gap[(int64_t)b * S + j] = pg;
        }
        free(work); free(idx); free(prob); free(cnt); free(qidx); free(qprob); free(qcnt);
    }
    return status;
}

/* Point-mass proposals (the deployed setting). */
int isd_oracle_accept_filtered(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                               int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S, int32_t V,
                               int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                               uint32_t rng_offset, double temperature, double tau, int32_t top_k,
                               double top_p, int32_t sample_proposals, double* draft_probs, int32_t* kept,
                               double* accept_margin, double* sample_gap, int32_t* runner_up,
                               double* proposal_gap, double* cut_margin)
{
    return accept_filtered_impl(logits, draft_tokens, NULL, NULL, rng_seed, accept_len, new_tokens, B, S, V,
                                n_draft_uniform, n_draft, greedy, rng_offset, temperature, tau, top_k, top_p,
                                sample_proposals, draft_probs, NULL, kept, accept_margin, sample_gap, runner_up,
                                proposal_gap, cut_margin, NULL, NULL);
}

/* Proposals drawn from the filtered distribution of q_logits[b, q_row[b] + j, :] (NULL: point mass). */
int isd_oracle_accept_filtered_q(const float* logits, const int32_t* draft_tokens, const float* q_logits,
                                 const int32_t* q_row, uint64_t rng_seed,
                                 int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S, int32_t V,
                                 int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                                 uint32_t rng_offset, double temperature, double tau, int32_t top_k,
                                 double top_p, int32_t sample_proposals, double* draft_probs, double* draft_q,
                                 int32_t* kept, double* accept_margin, double* sample_gap, int32_t* runner_up,
                                 double* proposal_gap, double* cut_margin, double* q_cut_margin,
                                 double* resid_small)
{
    return accept_filtered_impl(logits, draft_tokens, q_logits, q_row, rng_seed, accept_len, new_tokens, B, S, V,
                                n_draft_uniform, n_draft, greedy, rng_offset, temperature, tau, top_k, top_p,
                                sample_proposals, draft_probs, draft_q, kept, accept_margin, sample_gap, runner_up,
                                proposal_gap, cut_margin, q_cut_margin, resid_small);
}

/* ------------------------------------------------------------------------ */
/* Between two steps: KV append, trim-and-commit, next stride                */
/* ------------------------------------------------------------------------ */

/*
 * Batched scatter of the stride's K/V rows into the paged cache (Sec. 3.3 (1):
 * each ISD step appends its 2N-1 tokens in extend mode; (2): the stride's KV slots
 * are filled by one scatter for the whole batch).  Row i of sequence b belongs to
 * absolute position t = ctx_lens[b]-S+i (ctx_lens counts the S rows) and goes to
 * page block_table[b][t/P], slot t%P, for every KV head.
 * k_new / v_new [B,S,Hkv,D] contiguous; cache addressing as in attention.
 * dtype 0 = 4-byte elements, 1 = 2-byte elements (bit patterns are copied).
 * A position outside the table or a page id outside the pool is an error here
 * (the oracle refuses; nothing more is written).
 */
int isd_oracle_kv_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                         const int32_t* block_table, const int32_t* ctx_lens, int32_t S, int32_t B,
                         int32_t Hkv, int32_t D, int32_t P, int32_t num_pages, int32_t max_pages_per_seq,
                         int64_t page_stride, int64_t head_stride, int64_t token_stride, int32_t dtype)
{
    if (!k_new || !v_new || !k_cache || !v_cache || !block_table || !ctx_lens) return ORACLE_ERR_ARG;
    if (B < 0 || S < 1 || Hkv < 1 || D < 1 || P < 1 || (dtype != 0 && dtype != 1)) return ORACLE_ERR_ARG;
    const size_t esz = dtype == 0 ? 4 : 2;
    for (int b = 0; b < B; ++b)
        for (int i = 0; i < S; ++i) {
            const int64_t t = (int64_t)ctx_lens[b] - S + i;
            if (t < 0 || t / P >= max_pages_per_seq) return ORACLE_ERR_ARG;
            const int32_t page = block_table[(int64_t)b * max_pages_per_seq + t / P];
            if (page < 0 || page >= num_pages) return ORACLE_ERR_TABLE;
            const int slot = (int)(t % P);
            for (int h = 0; h < Hkv; ++h) {
                const int64_t src = (((int64_t)b * S + i) * Hkv + h) * D;
                const int64_t dst = page * page_stride + h * head_stride + slot * token_stride;
                memcpy((char*)k_cache + dst * esz, (const char*)k_new + src * esz, D * esz);
                memcpy((char*)v_cache + dst * esz, (const char*)v_new + src * esz, D * esz);
            }
        }
    return ORACLE_OK;
}

/*
 * Trim-and-commit after verification, and the next stride (Alg. 1, last line:
 * the accepted tokens join the prefix and their KV entries are committed; Sec. 3.2:
 * after a rejection everything behind it is dropped and the next step only proposes,
 * with nothing to introspect; Sec. 3.3 (2): the trim-and-commit cycle gives back the
 * slots of rejected and MASK positions after every verification).
 *
 * For sequence b with D = n_draft[b] drafts verified this step and r =
 * accept_len[b] of them accepted (0 <= r <= D <= S-1):
 *   - the step finalises r+1 tokens, new_tokens[b][0..r] (the accepted drafts and
 *     the freshly sampled token), appended to out_tokens[b] (at most out_cap kept);
 *   - of the stride's S KV slots the first r+1 stay (the step's first input token
 *     and the accepted drafts); the rest - rejected drafts and MASK positions - are
 *     given back: the context shrinks to ctx-S+r+1;
 *   - the next stride starts with the fresh token.  If nothing was rejected (r = D)
 *     it carries nd = min(n_draft_steady, S-1-D) drafts, the arg-max proposals of
 *     the MASK rows new_tokens[b][D+1 .. D+nd]; after a rejection it carries none.
 *     The remaining positions hold mask_token.  draft_tokens_next[b][0..nd) repeats
 *     the drafts in the layout the acceptance pass reads ([B,S-1]), -1 beyond;
 *   - the next stride's S positions are appended at once: ctx_lens[b] becomes
 *     ctx-S+r+1+S = ctx+r+1, and pages for positions that have none yet are popped
 *     from the top of free_list (entries free_list[0 .. *free_top)), sequence by
 *     sequence in index order, each sequence's pages in ascending position order.
 * If the free list cannot cover the whole batch (*status = 1) or a sequence would
 * outgrow its block-table row (*status = 2) nothing at all is changed.
 * Returns ORACLE_ERR_ARG for malformed arguments (including r or D out of range).
 */
int isd_oracle_commit(const int32_t* accept_len, const int32_t* new_tokens, int32_t* n_draft,
                      int32_t* ctx_lens, int32_t* stride_tokens, int32_t* draft_tokens_next,
                      int32_t* out_tokens, int32_t* out_lens, int32_t out_cap, int32_t* block_table,
                      int32_t* pages_used, const int32_t* free_list, int32_t* free_top, int32_t* status,
                      int32_t n_draft_steady, int32_t mask_token, int32_t B, int32_t S, int32_t P,
                      int32_t max_pages_per_seq)
{
    if (!accept_len || !new_tokens || !n_draft || !ctx_lens || !stride_tokens || !out_tokens ||
        !out_lens || !block_table || !pages_used || !free_list || !free_top || !status)
        return ORACLE_ERR_ARG;
    if (S > 1 && !draft_tokens_next) return ORACLE_ERR_ARG;
    if (B < 0 || S < 1 || P < 1 || max_pages_per_seq < 1 || out_cap < 0 || n_draft_steady < 0) return ORACLE_ERR_ARG;
    int64_t need = 0;
    for (int b = 0; b < B; ++b) {
        const int r = accept_len[b], D = n_draft[b];
        if (D < 0 || D > S - 1 || r < 0 || r > D) return ORACLE_ERR_ARG;
        const int64_t pages = ((int64_t)ctx_lens[b] + r + 1 + P - 1) / P;
        if (pages > max_pages_per_seq) { *status = 2; return ORACLE_OK; }
        if (pages > pages_used[b]) need += pages - pages_used[b];
    }
    if (need > *free_top) { *status = 1; return ORACLE_OK; }
    int32_t top = *free_top;
    for (int b = 0; b < B; ++b) {
        const int r = accept_len[b], D = n_draft[b];
        const int32_t* nt = new_tokens + (int64_t)b * S;
        for (int j = 0; j <= r; ++j)
            if (out_lens[b] < out_cap) out_tokens[(int64_t)b * out_cap + out_lens[b]++] = nt[j];
        int nd = 0;
        if (r == D) nd = n_draft_steady < S - 1 - D ? n_draft_steady : S - 1 - D;
        int32_t* st = stride_tokens + (int64_t)b * S;
        st[0] = nt[r];
        for (int k = 0; k < nd; ++k) st[1 + k] = nt[D + 1 + k];
        for (int k = 1 + nd; k < S; ++k) st[k] = mask_token;
        for (int k = 0; k < S - 1; ++k) draft_tokens_next[(int64_t)b * (S - 1) + k] = k < nd ? st[1 + k] : -1;
        const int32_t ctx_next = ctx_lens[b] + r + 1;
        const int32_t pages = (ctx_next + P - 1) / P;
        while (pages_used[b] < pages) block_table[(int64_t)b * max_pages_per_seq + pages_used[b]++] = free_list[--top];
        n_draft[b] = nd;
        ctx_lens[b] = ctx_next;
    }
    *free_top = top;
    *status = 0;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Segment-gated LoRA projection (lossless residual ISD)                      */
/* ------------------------------------------------------------------------ */

/*
 * One linear layer of the gated-LoRA model (App. G "Per-position computation";
 * Sec. 3.2 "Lossless ISD with residual adaptation"): token j gets
 *     h_j = W x_j + 1[j is a MASK position] * B (A x_j)
 * i.e. the base projection for every token and the low-rank residual only where
 * the per-token binary gate is set.
 *
 * x [T,d_in], W [d_out,d_in], A [r,d_in], Bm [d_out,r], all row-major
 * contiguous, dtype 0 = fp32, 1 = bf16 bit patterns; gate uint8 [T] (non-zero =
 * MASK position); h double [T,d_out].  Rows with sel != NULL && sel[t] == 0 are
 * skipped (left untouched) so that large workloads can be spot-checked.
 * The low-rank intermediate u = A x_j is kept in double: the paper fixes no
 * precision for it.
 */
int isd_oracle_gated_lora_linear(const void* x, const void* W, const void* A, const void* Bm,
                                 const uint8_t* gate, double* h, int32_t T, int32_t d_in,
                                 int32_t d_out, int32_t r, int32_t dtype, const uint8_t* sel)
{
    if (T < 0 || d_in < 1 || d_out < 1 || r < 0 || (dtype != 0 && dtype != 1)) return ORACLE_ERR_ARG;
    if (T == 0) return ORACLE_OK;
    if (!x || !W || !h || !gate || (r > 0 && (!A || !Bm))) return ORACLE_ERR_ARG;
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        if (sel && !sel[t]) continue;
        double* u = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
        if (gate[t]) {
            for (int rho = 0; rho < r; ++rho) {          /* u = A x_t */
                double acc = 0.0;
                for (int k = 0; k < d_in; ++k)
                    acc += load_elem(A, (int64_t)rho * d_in + k, dtype) * load_elem(x, (int64_t)t * d_in + k, dtype);
                u[rho] = acc;
            }
        }
        for (int o = 0; o < d_out; ++o) {
            double base = 0.0;                            /* (W x_t)_o */
            for (int k = 0; k < d_in; ++k)
                base += load_elem(W, (int64_t)o * d_in + k, dtype) * load_elem(x, (int64_t)t * d_in + k, dtype);
            double resid = 0.0;                           /* (B u)_o, MASK positions only */
            if (gate[t])
                for (int rho = 0; rho < r; ++rho) resid += load_elem(Bm, (int64_t)o * r + rho, dtype) * u[rho];
            h[(int64_t)t * d_out + o] = base + resid;
        }
        free(u);
    }
    return ORACLE_OK;
}

/*
 * The per-token gate of one ISD stride (App. G, table of position types): of the
 * S rows of sequence b, rows 0 .. n_draft[b] are fed clean tokens (the exact token
 * and the drafts under introspection: base weights only, gate 0) and rows beyond
 * are fed MASK (proposal positions: base + LoRA, gate 1).  gate uint8 [B*S].
 */
int isd_oracle_segment_gate(const int32_t* n_draft, uint8_t* gate, int32_t B, int32_t S)
{
    if (B < 0 || S < 1 || (B > 0 && (!n_draft || !gate))) return ORACLE_ERR_ARG;
    for (int b = 0; b < B; ++b) {
        int nd = n_draft[b];
        if (nd < 0) nd = 0;
        if (nd > S - 1) nd = S - 1;
        for (int j = 0; j < S; ++j) gate[(int64_t)b * S + j] = (uint8_t)(j > nd);
    }
    return ORACLE_OK;
}

/* Number of threads the parallel loops use from now on (timing the oracle on one core); no
 * effect on results: every item is computed by one thread. */
void isd_oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int isd_oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
