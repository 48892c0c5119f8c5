/*
 * idlm.h - C ABI of the MI355X (gfx950) hot path of one introspective strided
 * decoding (ISD) step: paged causal attention of a stride of S query rows per
 * sequence, and the introspective acceptance pass over the step's logits.
 *
 * Conventions shared by every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller unless stated
 *     otherwise.  The library never allocates, frees or keeps a pointer past the
 *     call; temporary storage comes from the caller's `workspace`.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream).  Outputs are valid once the caller has synchronised
 *     that stream.  Two calls that share a workspace must be ordered by the
 *     caller (same stream, or an event).
 *   - Return value: IDLM_OK (0) or a negative IDLM_ERR_* code.  All arguments
 *     that are visible to the host (pointers being NULL, shapes, strides,
 *     alignment, workspace size) are checked before anything is launched, and
 *     nothing is launched or written when a check fails.  The CONTENTS of device
 *     arrays are preconditions that are not checked: ctx_lens[b] >= S and
 *     ceil(ctx_lens[b]/P) <= max_pages_per_seq; block_table[b][p] in
 *     [0,num_pages) for p < ceil(ctx_lens[b]/P) (entries beyond that are never
 *     read); draft token ids in [0,V); n_draft[b] in [0,S-1]; logits hold no NaN.
 *     (idlm_isd_validate checks them on request).
 *     A broken precondition gives meaningless results, never an access outside
 *     the caller's buffers as far as the sizes passed on the host allow to tell
 *     (context lengths are cut at the table row, page ids are forced into the pool).
 *   - No global mutable state; entry points may be called from several host
 *     threads.  No C++ exception crosses this boundary.
 */
#ifndef IDLM_H
#define IDLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IDLM_VERSION 202 /* major*10000 + minor*100 + patch */

enum {
    IDLM_OK = 0,
    IDLM_ERR_NULL = -1,      /* a required pointer is NULL */
    IDLM_ERR_SHAPE = -2,     /* a size is out of the supported range */
    IDLM_ERR_DTYPE = -3,     /* unknown dtype code, or dtype/shape combination not supported */
    IDLM_ERR_ALIGN = -4,     /* a pointer or stride breaks the alignment the kernels need */
    IDLM_ERR_WORKSPACE = -5, /* workspace missing or smaller than the *_workspace() size */
    IDLM_ERR_LAUNCH = -6,    /* the HIP runtime refused the launch (no device, bad stream, ...) */
    IDLM_ERR_CONTENT = -7    /* idlm_isd_validate only: a device array breaks a precondition */
};

/* Bits of report[0] of idlm_isd_validate. */
enum {
    IDLM_BAD_CTX_SHORT = 1,  /* ctx_lens[b] < S */
    IDLM_BAD_CTX_LONG = 2,   /* ctx_lens[b] > max_pages_per_seq * P */
    IDLM_BAD_PAGE_ID = 4,    /* a block-table entry the step reads is outside [0, num_pages) */
    IDLM_BAD_N_DRAFT = 8,    /* n_draft[b] outside [0, S-1] */
    IDLM_BAD_DRAFT_ID = 16   /* a draft token id the step reads is outside [0, V) */
};

enum {
    IDLM_DTYPE_F32 = 0,
    IDLM_DTYPE_BF16 = 1,
    /* bf16 with the K pool's pages in operand order: inside the 4 KB block of a (page, KV head),
     * the 16-byte chunk c (dims 8c .. 8c+7) of slot t is stored at 16-byte entry
     * 64*(c/4) + 16*(c%4) + t instead of 16*t + c.  The attention kernel then reads K in whole
     * cache lines (it matters when more than 64 query rows share a KV head, S*G > 64, and K/V are
     * read by several wavefronts).  Needs token_stride = D = 128, P = 16; the V pool is unchanged.
     * idlm_isd_kv_append writes this layout when given the same code. */
    IDLM_DTYPE_BF16_KOP = 2
};

/*
 * idlm_isd_attention - causal attention of the step's S query rows over each
 * sequence's paged KV cache and within the stride.
 *
 * Definition (strict causal masking: key position i is visible to query
 * position j iff i <= j, Sec. 3.1 "Causal training with logit shift"; each ISD
 * step is one paged "extend" of the stride's rows whose K/V are already in the
 * pages, Sec. 3.3 (1) and App. D):
 *   query row i of sequence b sits at absolute position ctx_lens[b]-S+i and
 *   out[b,i,h,:] = sum_{t=0}^{ctx_lens[b]-S+i} softmax_t(scale * <q[b,i,h,:], K_t[h/G,:]>) * V_t[h/G,:]
 *   with G = Hq/Hkv and key/value t of sequence b stored in page
 *   block_table[b][t/P], slot t%P.  S = 1 is ordinary paged decode attention.
 *
 * q, out      [B,S,Hq,D] contiguous, element type `dtype`; 16-byte aligned.
 * k_cache,    page pools; element (page, kv head, slot, d) is at
 * v_cache     page*page_stride + head*head_stride + slot*token_stride + d (strides in
 *             elements, the same for both pools).  [num_pages,Hkv,P,D] contiguous is
 *             (Hkv*P*D, P*D, D); a token-major pool is (P*Hkv*D, D, Hkv*D).  16-byte
 *             aligned base and strides.
 * block_table int32 [B,max_pages_per_seq].
 * ctx_lens    int32 [B]: KV length of each sequence INCLUDING this step's S rows.
 * scale       softmax scale; <= 0 selects 1/sqrt(D).
 * dtype       IDLM_DTYPE_BF16 with D in {64,128}, IDLM_DTYPE_BF16_KOP with D = 128 (MFMA path; fp32
 *             accumulation; G = Hq/Hkv and S with S*G <= 256), or IDLM_DTYPE_F32 with D in {64,128}
 *             (plain path, one wavefront per (row, head) with fp32 arithmetic, for correctness
 *             rather than speed).
 * num_workgroups  size of the persistent grid that shares the batch's 32-token tiles evenly;
 *             0 = one workgroup per compute unit of the current device (at most 256; two per compute unit, at
 *             most 512, when D = 128 and more than 64 query rows share a KV head, S*G > 64), fewer when B and
 *             the width of the block table bound the work to a few tiles per wavefront (the setting to use);
 *             1..1024 forces a grid (testing, or leaving compute units to other streams).
 * workspace   at least idlm_isd_attention_workspace(..., num_workgroups) bytes, 256-byte aligned (MFMA path:
 *             partial results of the sequences that a slice boundary cuts;
 *             the plain path needs none and accepts NULL).
 * Supported: P = 16, 1 <= S <= 32, 0 <= B <= 65535 (B = 0 is a no-op), B*max_pages_per_seq < 2^31.
 */
int idlm_isd_attention(const void* q, const void* k_cache, const void* v_cache,
                       const int32_t* block_table, const int32_t* ctx_lens, int32_t S, void* out,
                       int32_t B, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                       int32_t num_pages, int32_t max_pages_per_seq,
                       int64_t page_stride, int64_t head_stride, int64_t token_stride,
                       float scale, int32_t dtype, int32_t num_workgroups,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace idlm_isd_attention needs for these shapes and this num_workgroups (the value
 * that will be passed to the call; 0 = the library's own choice, at most 256 workgroups, or 512 of half the rows
 * each for D = 128 and S*G > 64): two partial-result slots per wavefront of the grid, 35 MB for the default grid
 * at D = 128 and S*G >= 33 query rows per KV head.  Host-only, no GPU needed.  Returns 0 for shapes that are rejected anyway. */
size_t idlm_isd_attention_workspace(int32_t B, int32_t S, int32_t Hq, int32_t Hkv, int32_t D,
                                    int32_t P, int32_t max_pages_per_seq, int32_t dtype,
                                    int32_t num_workgroups);

/*
 * idlm_isd_accept - introspective acceptance over the step's logits.
 *
 * Sequence b has S logit rows.  Row j < n_d (n_d = its number of drafted tokens) is the
 * model's own next-token distribution p_j ("causal anchor") for drafted token x_j, row n_d is
 * the anchor after the last draft, rows > n_d come from MASK positions.  Following Alg. 1
 * (introspection loop) with arg-max, i.e. point-mass, proposals as deployed in Sec. 3.3 (3),
 * so that the accept probability min(1, p/q) is p_j(x_j) and the residual
 * normalize(max(0, p - q)) is p_j with x_j removed (Sec. 3.2 "Adaptive stride via p/q
 * acceptance"):
 *   p_j        = softmax(logits[b,j,:])[x_j]                               (j < n_d)
 *   accept_j   = greedy[b] ? (x_j == argmax logits[b,j,:]) : (u_{b,j} < p_j)
 *   accept_len = number of leading accepted drafts, r in [0, n_d]
 *   fresh token (row r): greedy: argmax of row r; otherwise Gumbel-max sample of row r,
 *               with x_r excluded iff r < n_d (rejection); r = n_d is the bonus token
 *   new_tokens[b,j] = x_j (j < r) | fresh token (j = r) | -1 (r < j <= n_d, discarded)
 *                     | argmax logits[b,j,:] (j > n_d, next step's proposals)
 * arg-max ties go to the lowest index.  Random numbers: Philox4x32-10 with key = (rng_seed
 * low word, high word) and counter = (i >> 2, b*S+j, stream, rng_offset); element i uses
 * output word i & 3; stream 0 word 0 of counter (0, row, 0, rng_offset) is the accept
 * uniform, stream 1 feeds the Gumbel noise of vocabulary element i.  A 32-bit word x maps to
 * u = (2*(x >> 9) + 1) * 2^-24 and g = -ln(-ln u).
 *
 * logits       fp32 [B,S,V] contiguous, 16-byte aligned; V % 4 == 0.
 * draft_tokens int32 [B,S-1] (row stride S-1); entries j < n_d are read.  May be NULL iff S = 1.
 * accept_len   int32 [B]   out.
 * new_tokens   int32 [B,S] out.
 * n_draft      int32 [B], or NULL to use n_draft_uniform (0 <= n_draft_uniform <= S-1) for all.
 * greedy       uint8 [B] (non-zero = greedy), or NULL = every sequence stochastic.
 * rng_offset   step counter; vary it between steps that reuse a seed.
 * draft_probs  fp32 [B,S-1] out (p_j for j < n_d, 0 beyond), or NULL.
 * workspace    at least idlm_isd_accept_workspace(B,S,V) bytes, 256-byte aligned.
 * Supported: 1 <= S <= 64, 4 <= V < 2^31, B*S < 2^31; B = 0 is a no-op.
 */
int idlm_isd_accept(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                    int32_t* accept_len, int32_t* new_tokens,
                    int32_t B, int32_t S, int32_t V,
                    int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                    uint32_t rng_offset, float* draft_probs,
                    void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace idlm_isd_accept needs (host-only). Returns 0 for rejected shapes. */
size_t idlm_isd_accept_workspace(int32_t B, int32_t S, int32_t V);

/*
 * idlm_isd_accept_static - idlm_isd_accept for callers that cannot allocate or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same
 * arguments, results (bit for bit) and error behaviour as idlm_isd_accept, without `workspace`:
 * the scratch memory is a fixed array of idlm_isd_accept_static_max_bytes() bytes (1 MiB) in the
 * library's device image, one copy per GPU, held until the process ends.  The call allocates and
 * frees nothing (no hipMalloc / hipFree, no allocating library routine) and does not synchronise.
 * Limit: idlm_isd_accept_workspace(B,S,V) must not exceed idlm_isd_accept_static_max_bytes()
 * (about 60 000 logit rows per call; the benchmark's B=256, S=16 needs 72 KB); beyond it the call
 * returns IDLM_ERR_WORKSPACE and launches nothing.
 * All calls on one GPU share that GPU's array: two calls whose kernels can overlap on one GPU
 * (different streams without an ordering event, several host threads) race on it - order them,
 * or use idlm_isd_accept with separate workspaces.  The array keeps the last call's contents;
 * every word a call reads it has written before, so nothing needs clearing between calls.
 */
int idlm_isd_accept_static(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                           int32_t* accept_len, int32_t* new_tokens,
                           int32_t B, int32_t S, int32_t V,
                           int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                           uint32_t rng_offset, float* draft_probs, void* stream);

/* Size in bytes of the fixed scratch array idlm_isd_accept_static uses (host-only). */
size_t idlm_isd_accept_static_max_bytes(void);

/*
 * idlm_isd_accept_bf16 - the same acceptance (Alg. 1, introspection loop; Sec. 3.3 (3)) over
 * logits stored as bf16, which halves the bytes the pass has to read.  Every logit widens
 * exactly to fp32 and all arithmetic after the load is that of idlm_isd_accept, so the results
 * are those of idlm_isd_accept called on the widened values: same rules, same random streams,
 * same tie rule (bf16 rows hold many equal values; arg-max ties go to the lowest index).
 *
 * logits  bf16 (raw 16-bit patterns) [B,S,V] contiguous, 16-byte aligned; V % 8 == 0, V >= 8.
 * All other arguments, the workspace size (idlm_isd_accept_workspace) and the error behaviour
 * are those of idlm_isd_accept.
 */
int idlm_isd_accept_bf16(const uint16_t* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                         int32_t* accept_len, int32_t* new_tokens,
                         int32_t B, int32_t S, int32_t V,
                         int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                         uint32_t rng_offset, float* draft_probs,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * idlm_isd_accept_general - acceptance with general proposal distributions, sampling
 * temperature, relaxed threshold and sampled proposals: Alg. 1 as printed (drafts drawn from
 * q_j, accepted with probability min(1, p_j(x_j)/q_j(x_j)), resampled from
 * normalize(max(0, p_j - q_j)) at the first rejection, Sec. 3.2 "Adaptive stride via p/q
 * acceptance"), the threshold relaxation discussed in Sec. 5 (accept iff
 * u < min(1, (1+tau) p/q)) and a sampling temperature T (App. H lists the sampling set-up of
 * the paper's runs): p_j = softmax(logits[b,j,:]/T), q_j = softmax(q_logits[b, q_row[b]+j, :]/T).
 * idlm_isd_accept is the deployed special case (point-mass proposals, T = 1, tau = 0) and the
 * one to use on the hot path; outputs and conventions are the same, with these additions:
 *
 * q_logits     fp32 [B,S,V] or NULL: the logits of the step that proposed the drafts (the
 *              caller keeps the previous step's buffer); NULL = point-mass proposals, q = 1.
 * q_row        int32 [B] (required with q_logits): row of q_logits that proposed draft 0 of
 *              sequence b; draft j came from row q_row[b]+j (forced into the sequence).
 * q_lse        fp32 [B,S] or NULL: natural-log sum of exp(q_logits[b,i,:]/T) per row - the
 *              row_lse output of the call that processed q_logits at the same T.  NULL with
 *              q_logits given costs one more streaming pass over q_logits.
 * temperature  T > 0.  tau >= 0.
 *              q_j(x_j) = 0: the draft is accepted iff p_j(x_j) > 0 (p = q = 0 is rejected).
 * sample_proposals  non-zero: rows after the drafts propose argmax_i(l_i/T + Gumbel noise of
 *              random stream 2) instead of the arg-max (greedy sequences always use the arg-max).
 * fresh token  after a rejection: argmax_i [ln(p(i) - q(i)) + g_i] over i with p(i) > q(i)
 *              (point mass: q = delta at the draft), the row's arg-max if there is no such i;
 *              with every draft accepted: argmax_i [l_i/T + g_i] (random stream 1).
 * draft_probs  fp32 [B,S-1] out or NULL: p_j(x_j);  draft_q: q_j(x_j) (1 for point mass).
 * row_lse      fp32 [B,S] out or NULL.
 * workspace    at least idlm_isd_accept_general_workspace(B,S,V) bytes, 256-byte aligned.
 * Same shape limits as idlm_isd_accept.
 */
int idlm_isd_accept_general(const float* logits, const int32_t* draft_tokens, const float* q_logits,
                            const int32_t* q_row, const float* q_lse, uint64_t rng_seed,
                            int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S, int32_t V,
                            int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                            uint32_t rng_offset, float temperature, float tau, int32_t sample_proposals,
                            float* draft_probs, float* draft_q, float* row_lse, void* workspace,
                            size_t workspace_bytes, void* stream);

size_t idlm_isd_accept_general_workspace(int32_t B, int32_t S, int32_t V);

/*
 * idlm_isd_accept_filtered - acceptance under the filtered sampling distribution of the paper's
 * runs (App. H, ISD configuration table: temperature 1.0, top_k 50, top_p 0.95), with point-mass
 * proposals (the deployed setting).  The distribution pf_j of row j is built in the usual order:
 * logits / T, the top_k largest (equal values: lowest index first), then the shortest prefix of
 * those, in descending order, whose renormalised probability mass reaches top_p (at least one
 * element), renormalised again.  Then, as in idlm_isd_accept with p replaced by pf:
 *   accept_j = greedy[b] ? (x_j == argmax) : (u_{b,j} < min(1, (1+tau) pf_j(x_j)))
 *   fresh token of row r: greedy: arg-max; otherwise a draw from pf_r, without x_r after a
 *               rejection (the arg-max if nothing else survives the filter)
 *   proposals of the rows after the drafts: arg-max, or (sample_proposals, non-greedy) a draw
 *               from pf_j with random stream 2.
 * A draw is argmax over the surviving ids i of ln pf(i) + Gumbel noise of id i (the noise
 * idlm_isd_accept uses), so top_k >= V with top_p = 1 reproduces the unfiltered results.
 *
 * top_k        1 .. 64.   top_p in (0, 1].   temperature > 0.   tau >= 0.
 * draft_probs  fp32 [B,S-1] out or NULL: pf_j(x_j) (0 for a draft outside the support).
 * kept         int32 [B,S] out or NULL: number of ids that survive the filter in each row.
 * workspace    at least idlm_isd_accept_filtered_workspace(B,S,V) bytes, 256-byte aligned.
 * One streaming pass over the logits (exact top_k per row), then one small kernel: there is no
 * second pass.  Same shape limits as idlm_isd_accept.
 */
int idlm_isd_accept_filtered(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                             int32_t* accept_len, int32_t* new_tokens, int32_t B, int32_t S, int32_t V,
                             int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                             uint32_t rng_offset, float temperature, float tau, int32_t top_k, float top_p,
                             int32_t sample_proposals, float* draft_probs, int32_t* kept,
                             void* workspace, size_t workspace_bytes, void* stream);

size_t idlm_isd_accept_filtered_workspace(int32_t B, int32_t S, int32_t V);

/*
 * idlm_isd_accept_filtered_q - idlm_isd_accept_filtered for drafts that were DRAWN from the
 * filtered distribution of the row that proposed them (sample_proposals of the previous call):
 * Alg. 1 as printed (Sec. 3.2 "Adaptive stride via p/q acceptance") under the sampler of App. H.
 * With qf_j the filtered distribution (same temperature, top_k, top_p) of the proposing row of
 * draft j:
 *   accept_j = greedy[b] ? (x_j == argmax) : (u_{b,j} < min(1, (1+tau) pf_j(x_j) / qf_j(x_j)));
 *               a draft outside qf_j's support (it cannot have been drawn from it) is accepted
 *               iff pf_j(x_j) > 0
 *   fresh token after a rejection at row r: a draw from normalize(max(0, pf_r - qf_r)), i.e.
 *               argmax over the ids kept in pf_r with pf_r(i) > qf_r(i) of
 *               ln(pf_r(i) - qf_r(i)) + Gumbel noise of id i; the arg-max if there is none
 *   everything else as idlm_isd_accept_filtered, which is the case q_cand == NULL.
 * For tau = 0 the emitted token is distributed as pf_r whatever qf_r was.
 *
 * The proposer is not passed as logits but as the record this call keeps of every row: the
 * row's top_k (value, id) pairs, 64 x 8 bytes per row, so the previous step's logits are never
 * read again.
 * logits, logits_dtype  IDLM_DTYPE_F32: fp32 [B,S,V], V % 4 == 0; IDLM_DTYPE_BF16: raw bf16 [B,S,V],
 *            V % 8 == 0 - half the bytes to stream; every value widens exactly to fp32 and the
 *            results are those of the fp32 call on the widened values (as idlm_isd_accept_bf16).
 * cand_out   uint64 [B,S,64] out or NULL: the record of this call's rows (opaque; entries beyond
 *            top_k are 0).  Given, it also replaces the workspace (which may then be NULL).
 * q_cand     uint64 [B,S,64] or NULL: cand_out of the call that proposed the drafts, made with
 *            the same top_k; must not be the buffer passed as cand_out.  NULL = point mass.
 * q_row      int32 [B] (required with q_cand): row of q_cand that proposed draft 0 of sequence
 *            b; draft j came from row q_row[b]+j (forced into the sequence's S rows).
 * draft_q    fp32 [B,S-1] out or NULL: qf_j(x_j) (1 for point mass, 0 outside the support).
 * Single precision: pf - qf cancels when the two are close, so a residual draw whose winner
 * has a tiny residual may differ from double-precision arithmetic.
 */
int idlm_isd_accept_filtered_q(const void* logits, int32_t logits_dtype, const int32_t* draft_tokens, const uint64_t* q_cand,
                               const int32_t* q_row, uint64_t rng_seed, int32_t* accept_len,
                               int32_t* new_tokens, int32_t B, int32_t S, int32_t V, int32_t n_draft_uniform,
                               const int32_t* n_draft, const uint8_t* greedy, uint32_t rng_offset,
                               float temperature, float tau, int32_t top_k, float top_p,
                               int32_t sample_proposals, float* draft_probs, float* draft_q, int32_t* kept,
                               uint64_t* cand_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * idlm_isd_kv_append - batched scatter of the stride's K/V rows into the paged cache, before the
 * step's attention (Sec. 3.3 (1): every ISD step appends its stride in extend mode; (2): the stride's
 * KV slots are filled by one scatter for the whole batch).
 *
 * Row i of sequence b belongs to absolute position t = ctx_lens[b]-S+i (ctx_lens counts the S
 * rows, as in idlm_isd_attention) and is copied, for every KV head, to page block_table[b][t/P],
 * slot t%P of both pools.  Slots of a previous stride that were given back are simply overwritten.
 * A row whose position is negative or beyond the table row, or whose page id is outside
 * [0,num_pages), is skipped (nothing is written for it).
 *
 * k_new, v_new [B,S,Hkv,D] contiguous, element type `dtype`, 16-byte aligned; D*sizeof(element) a
 *              multiple of 16.
 * k_cache,     page pools addressed as in idlm_isd_attention (strides in elements).
 * v_cache
 * Supported: 0 <= B <= 65535, 1 <= S <= 64, any P >= 1.  Bit patterns are copied unchanged.
 */
int idlm_isd_kv_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                       const int32_t* block_table, const int32_t* ctx_lens, int32_t S, int32_t B,
                       int32_t Hkv, int32_t D, int32_t P, int32_t num_pages, int32_t max_pages_per_seq,
                       int64_t page_stride, int64_t head_stride, int64_t token_stride, int32_t dtype,
                       void* stream);

/*
 * idlm_isd_commit - trim-and-commit after idlm_isd_accept, and the next stride (Alg. 1, last
 * line: the accepted tokens join the prefix and the KV cache is committed; Sec. 3.2 "Adaptive
 * stride via p/q acceptance": after a rejection the rest is discarded and the next step is a pure
 * stride; Sec. 3.3 (2): the trim-and-commit cycle frees rejected and MASK positions).
 *
 * For sequence b with D = n_draft[b] and r = accept_len[b] (0 <= r <= D <= S-1):
 *   - new_tokens[b][0..r] (accepted drafts, then the fresh token) are appended to out_tokens[b]
 *     (row stride out_cap; tokens beyond out_cap are dropped) and out_lens[b] grows accordingly;
 *   - the stride's first r+1 KV slots stay, the others are given back, and the next stride's S
 *     positions are appended at once: ctx_lens[b] += r+1;
 *   - stride_tokens[b] = fresh token, then nd drafts, then mask_token; nd = min(n_draft_steady,
 *     S-1-D) arg-max proposals new_tokens[b][D+1 .. D+nd] if nothing was rejected (r = D), else 0;
 *     draft_tokens_next[b] ([B,S-1], the layout idlm_isd_accept reads) repeats the drafts, -1
 *     beyond; n_draft[b] = nd;
 *   - positions that have no page yet get one: block_table[b][pages_used[b]++] = free_list[--top],
 *     sequences in index order, starting from top = *free_top; *free_top is updated.
 * *status: 0 done; 1 the free list cannot cover the batch; 2 a sequence would outgrow its table
 * row; 3 an accept_len / n_draft pair is out of range.  For a non-zero status NOTHING is changed.
 * All arrays int32 on the device, 4-byte aligned; n_draft, ctx_lens, out_lens, block_table,
 * pages_used, free_top are updated in place.  draft_tokens_next may be NULL iff S = 1.
 * Supported: 0 <= B <= 65535, 1 <= S <= 64.  One small launch; asynchronous on `stream`.
 */
int idlm_isd_commit(const int32_t* accept_len, const int32_t* new_tokens, int32_t* n_draft,
                    int32_t* ctx_lens, int32_t* stride_tokens, int32_t* draft_tokens_next,
                    int32_t* out_tokens, int32_t* out_lens, int32_t out_cap, int32_t* block_table,
                    int32_t* pages_used, const int32_t* free_list, int32_t* free_top, int32_t* status,
                    int32_t n_draft_steady, int32_t mask_token, int32_t B, int32_t S, int32_t P,
                    int32_t max_pages_per_seq, void* stream);

/*
 * idlm_gated_lora_linear - one linear layer of the lossless variant with its low-rank adapter
 * gated per token (App. G "Per-position computation"; Sec. 3.2 "Lossless ISD with residual
 * adaptation"):
 *     h[t,:] = W x[t,:] + gate_t * Bm (A x[t,:])
 * gate_t = 1 at MASK (proposal) positions, 0 at clean positions (the exact token and the drafts
 * under introspection), whose outputs are therefore those of the base layer alone, bit for bit:
 * h[t,:] of a clean token does not depend on A, Bm or on the gates of other tokens.
 * bf16 operands, fp32 accumulation on the matrix cores, u = A x rounded to bf16 between the two
 * products, h rounded to bf16 once at the end.
 *
 * x        bf16 [T,d_in]      contiguous, 16-byte aligned (all matrices: raw 16-bit patterns).
 * W        bf16 [d_out,d_in]  base weight, one output feature per row.
 * A        bf16 [r,d_in]      adapter down-projection; Bm bf16 [d_out,r] its up-projection.
 *                             Both must be finite.  May be NULL iff r = 0 (plain base layer).
 * gate     uint8 [T] (non-zero = MASK position), or NULL: then token t = b*S + j of a batch of
 *          strides of S rows is a MASK position iff j > n_draft[b] (int32 [T/S], clamped to
 *          [0,S-1]; T % S == 0), the row order of idlm_isd_attention / idlm_isd_accept.
 * h        bf16 [T,d_out] out.
 * tile_tokens  0 = choose (with k_splits = 0: the pair that a small cost model of the launch -
 *          rounds of workgroups over the compute units, cost of a reduction step per tile
 *          size, traffic of the partial sums - rates cheapest), or 64 / 128 / 256 to force it.
 * k_splits     0 = choose, or 1..16: the reduction over d_in is cut into this many parts, one
 *          workgroup each, summed in a fixed order by a second kernel (few tokens: more
 *          workgroups for the same weight traffic).  Results do not depend on the number of
 *          compute units; they may differ in the last bit between different (tile_tokens,
 *          k_splits), and clean tokens equal the base layer run with the same two values.
 * workspace    at least idlm_gated_lora_linear_workspace(T,d_in,d_out,r,tile_tokens,k_splits)
 *          bytes (u and the fp32 partial sums), 256-byte aligned; may be NULL when that is 0.
 * Supported: d_in a multiple of 64, d_out a multiple of 8, r a multiple of 64 up to 4096 (the
 * paper's adapters: 128 and 1024); T = 0 is a no-op.  Errors and stream as for the other calls.
 */
int idlm_gated_lora_linear(const uint16_t* x, const uint16_t* W, const uint16_t* A, const uint16_t* Bm,
                           const uint8_t* gate, const int32_t* n_draft, int32_t S, uint16_t* h,
                           int32_t T, int32_t d_in, int32_t d_out, int32_t r, int32_t tile_tokens,
                           int32_t k_splits, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace idlm_gated_lora_linear needs (host-only); 0 when none is needed or the
 * shape is rejected anyway. */
size_t idlm_gated_lora_linear_workspace(int32_t T, int32_t d_in, int32_t d_out, int32_t r,
                                        int32_t tile_tokens, int32_t k_splits);

/*
 * idlm_isd_validate - debug aid: checks the CONTENTS of the device arrays that the calls of one
 * step (idlm_isd_attention, idlm_isd_kv_append, the idlm_isd_accept family) take as
 * preconditions, and WAITS for the result (it synchronises `stream`; not for graph capture or
 * the serving loop).
 *
 * block_table, ctx_lens, S, B, P, num_pages, max_pages_per_seq: as for idlm_isd_attention; either
 *          pointer may be NULL to skip the checks that need it.
 * draft_tokens int32 [B,S-1], n_draft int32 [B] or NULL (n_draft_uniform), V: as for
 *          idlm_isd_accept; draft_tokens may be NULL to skip the id check.
 * report   DEVICE int32[4], written: [0] = OR of the IDLM_BAD_* bits found, [1] = lowest sequence
 *          index with a finding (-1: none), [2], [3] = 0.
 * host_report  HOST int32[4] or NULL: receives the same four words.
 * Returns IDLM_OK when nothing was found, IDLM_ERR_CONTENT otherwise (or the usual codes for bad
 * host-visible arguments; S up to 64 as for the acceptance calls).
 */
int idlm_isd_validate(const int32_t* block_table, const int32_t* ctx_lens, int32_t S, int32_t B, int32_t P,
                      int32_t num_pages, int32_t max_pages_per_seq, const int32_t* draft_tokens,
                      const int32_t* n_draft, int32_t n_draft_uniform, int32_t V, int32_t* report,
                      int32_t* host_report, void* stream);

/* Static, NUL-terminated description of a return code (host pointer, never NULL). */
const char* idlm_strerror(int code);

/* IDLM_VERSION of the loaded library. */
int idlm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* IDLM_H */
