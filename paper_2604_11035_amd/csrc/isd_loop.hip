// Between two ISD steps (Sec. 3.3 (2): forward -> verify -> trim -> prepare -> forward): the batched
// scatter of the stride's K/V rows into the paged cache, and trim-and-commit with the
// preparation of the next stride.  gfx950 only.
#include "idlm_common.h"

namespace idlm {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// ---- KV append ------------------------------------------------------------------------------

struct AppendParams {
    const char* k_new;   // [B,S,Hkv,D] rows of row_bytes each
    const char* v_new;
    char* k_cache;
    char* v_cache;
    const int32_t* block_table;
    const int32_t* ctx_lens;
    int B, S, Hkv, P, num_pages, max_pages;
    int chunks;          // 16-byte chunks per row (D * element size / 16)
    int k_operand_order; // K pages hold their 16-byte chunks in the attention kernel's operand order
    int64_t page_bytes, head_bytes, token_bytes;
};

// One thread per 16 bytes of one (K or V, sequence, stride row, KV head) row.  A row whose
// position or page id is not usable is skipped: nothing is ever written outside the pools.
__global__ __launch_bounds__(256) void isd_kv_append_kernel(const AppendParams p)
{
    const int64_t rows = (int64_t)p.B * p.S * p.Hkv;
    const int64_t per_pool = rows * p.chunks;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < 2 * per_pool; idx += (int64_t)gridDim.x * 256) {
        const bool is_v = idx >= per_pool;
        const int64_t rem = is_v ? idx - per_pool : idx;
        const int64_t row = rem / p.chunks;
        const int c = (int)(rem - row * p.chunks);
        const int h = (int)(row % p.Hkv);
        const int64_t bi = row / p.Hkv;
        const int i = (int)(bi % p.S);
        const int b = (int)(bi / p.S);
        const int64_t t = (int64_t)p.ctx_lens[b] - p.S + i;
        if (t < 0 || t / p.P >= p.max_pages) continue;
        const int page = p.block_table[(int64_t)b * p.max_pages + t / p.P];
        if (page < 0 || page >= p.num_pages) continue;
        int64_t dst = page * p.page_bytes + h * p.head_bytes;
        if (p.k_operand_order && !is_v)   // chunk c of slot t%16 is entry 64*(c/4) + 16*(c%4) + slot of the 4 KB block
            dst += (int64_t)(64 * (c >> 2) + 16 * (c & 3) + (int)(t % p.P)) * 16;
        else
            dst += (t % p.P) * p.token_bytes + (int64_t)c * 16;
        const int64_t src = (row * p.chunks + c) * 16;
        const u32x4 val = *reinterpret_cast<const u32x4*>((is_v ? p.v_new : p.k_new) + src);
        *reinterpret_cast<u32x4*>((is_v ? p.v_cache : p.k_cache) + dst) = val;
    }
}

// ---- trim-and-commit, next stride -----------------------------------------------------------

struct CommitParams {
    const int32_t* accept_len;
    const int32_t* new_tokens;
    int32_t* n_draft;
    int32_t* ctx_lens;
    int32_t* stride_tokens;
    int32_t* draft_tokens_next;
    int32_t* out_tokens;
    int32_t* out_lens;
    int32_t* block_table;
    int32_t* pages_used;
    const int32_t* free_list;
    int32_t* free_top;
    int32_t* status;
    int out_cap, n_draft_steady, mask_token, B, S, P, max_pages;
};

// One workgroup of 1024 threads for the whole batch; thread t owns the sequences
// [t*per, (t+1)*per), so that a prefix sum over threads is a prefix sum over sequences and the
// pages come off the free list in sequence order, as the definition says.  Nothing is written
// before every sequence has been checked.
__global__ __launch_bounds__(1024) void isd_commit_kernel(const CommitParams p)
{
    __shared__ int wave_need[16];
    __shared__ int flags;     // bit 0: a table row would overflow, bit 1: accept_len / n_draft out of range
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (tid == 0) flags = 0;
    __syncthreads();
    const int per = (p.B + 1023) >> 10;
    const int b0 = tid * per, b1 = min(p.B, b0 + per);
    int need = 0, bad = 0;
    for (int b = b0; b < b1; ++b) {
        const int r = p.accept_len[b], D = p.n_draft[b];
        if (D < 0 || D > p.S - 1 || r < 0 || r > D) { bad |= 2; continue; }
        const int64_t pages = ((int64_t)p.ctx_lens[b] + r + 1 + p.P - 1) / p.P;
        if (pages > p.max_pages) { bad |= 1; continue; }
        need += max(0, (int)pages - p.pages_used[b]);
    }
    if (bad) atomicOr(&flags, bad);
    int x = need;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off);
        if (lane >= off) x += y;
    }
    if (lane == 63) wave_need[w] = x;
    const int top0 = *p.free_top;       // read by everybody before anybody may write it
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int s = wave_need[k];
        before += (k < w) ? s : 0;
        total += s;
    }
    const int f = flags;
    if (f || total > top0) {
        if (tid == 0) *p.status = (f & 2) ? 3 : (f & 1) ? 2 : 1;
        return;
    }
    int top = top0 - (before + x - need);   // this thread's first page is free_list[top - 1]
    const int S = p.S;
    for (int b = b0; b < b1; ++b) {
        const int r = p.accept_len[b], D = p.n_draft[b];
        const int32_t* nt = p.new_tokens + (int64_t)b * S;
        int ol = p.out_lens[b];
        for (int j = 0; j <= r; ++j)
            if (ol < p.out_cap) p.out_tokens[(int64_t)b * p.out_cap + ol++] = nt[j];
        p.out_lens[b] = ol;
        const int nd = (r == D) ? min(p.n_draft_steady, S - 1 - D) : 0;
        int32_t* st = p.stride_tokens + (int64_t)b * S;
        st[0] = nt[r];
        for (int k = 1; k < S; ++k) {
            const int tok = (k <= nd) ? nt[D + k] : p.mask_token;
            st[k] = tok;
            p.draft_tokens_next[(int64_t)b * (S - 1) + k - 1] = (k <= nd) ? tok : -1;
        }
        const int ctx_next = p.ctx_lens[b] + r + 1;
        const int pages = (ctx_next + p.P - 1) / p.P;
        int used = p.pages_used[b];
        while (used < pages) p.block_table[(int64_t)b * p.max_pages + used++] = p.free_list[--top];
        p.pages_used[b] = used;
        p.n_draft[b] = nd;
        p.ctx_lens[b] = ctx_next;
    }
    if (tid == 0) {
        *p.free_top = top0 - total;
        *p.status = 0;
    }
}

}  // namespace idlm

using namespace idlm;

extern "C" int idlm_isd_kv_append(const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                                  const int32_t* block_table, const int32_t* ctx_lens, int32_t S, int32_t B,
                                  int32_t Hkv, int32_t D, int32_t P, int32_t num_pages, int32_t max_pages_per_seq,
                                  int64_t page_stride, int64_t head_stride, int64_t token_stride, int32_t dtype,
                                  void* stream)
{
    if (dtype != IDLM_DTYPE_F32 && dtype != IDLM_DTYPE_BF16 && dtype != IDLM_DTYPE_BF16_KOP) return IDLM_ERR_DTYPE;
    if (B < 0 || B > 65535 || S < 1 || S > 64 || Hkv < 1 || Hkv > 1024 || D < 1 || D > 1024 || P < 1 || P > 1024)
        return IDLM_ERR_SHAPE;
    if (dtype == IDLM_DTYPE_BF16_KOP && (D != 128 || P != 16 || token_stride != 128)) return IDLM_ERR_DTYPE;
    if (num_pages < 1 || max_pages_per_seq < 1 || page_stride < 1 || head_stride < 1 || token_stride < D)
        return IDLM_ERR_SHAPE;
    if (B == 0) return IDLM_OK;
    if (!k_new || !v_new || !k_cache || !v_cache || !block_table || !ctx_lens) return IDLM_ERR_NULL;
    const int64_t esz = dtype == IDLM_DTYPE_F32 ? 4 : 2;
    if ((D * esz) % 16 || (page_stride * esz) % 16 || (head_stride * esz) % 16 || (token_stride * esz) % 16)
        return IDLM_ERR_ALIGN;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) ||
        !aligned(block_table, 4) || !aligned(ctx_lens, 4))
        return IDLM_ERR_ALIGN;
    AppendParams p;
    p.k_new = static_cast<const char*>(k_new);
    p.v_new = static_cast<const char*>(v_new);
    p.k_cache = static_cast<char*>(k_cache);
    p.v_cache = static_cast<char*>(v_cache);
    p.block_table = block_table;
    p.ctx_lens = ctx_lens;
    p.B = B; p.S = S; p.Hkv = Hkv; p.P = P; p.num_pages = num_pages; p.max_pages = max_pages_per_seq;
    p.chunks = (int)(D * esz / 16);
    p.k_operand_order = dtype == IDLM_DTYPE_BF16_KOP;
    p.page_bytes = page_stride * esz; p.head_bytes = head_stride * esz; p.token_bytes = token_stride * esz;
    const int64_t threads = (int64_t)2 * B * S * Hkv * p.chunks;
    int64_t blocks = (threads + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    (void)hipGetLastError();
    hipLaunchKernelGGL(isd_kv_append_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), p);
    return launch_status();
}

extern "C" int idlm_isd_commit(const int32_t* accept_len, const int32_t* new_tokens, int32_t* n_draft,
                               int32_t* ctx_lens, int32_t* stride_tokens, int32_t* draft_tokens_next,
                               int32_t* out_tokens, int32_t* out_lens, int32_t out_cap, int32_t* block_table,
                               int32_t* pages_used, const int32_t* free_list, int32_t* free_top, int32_t* status,
                               int32_t n_draft_steady, int32_t mask_token, int32_t B, int32_t S, int32_t P,
                               int32_t max_pages_per_seq, void* stream)
{
    if (B < 0 || B > 65535 || S < 1 || S > 64 || P < 1 || P > 1024 || max_pages_per_seq < 1 || out_cap < 0 ||
        n_draft_steady < 0)
        return IDLM_ERR_SHAPE;
    if (B == 0) return IDLM_OK;
    if (!accept_len || !new_tokens || !n_draft || !ctx_lens || !stride_tokens || !out_tokens || !out_lens ||
        !block_table || !pages_used || !free_list || !free_top || !status)
        return IDLM_ERR_NULL;
    if (S > 1 && !draft_tokens_next) return IDLM_ERR_NULL;
    const void* ptrs[] = {accept_len, new_tokens, n_draft, ctx_lens, stride_tokens, draft_tokens_next, out_tokens,
                          out_lens, block_table, pages_used, free_list, free_top, status};
    for (const void* q : ptrs)
        if (!aligned(q, 4)) return IDLM_ERR_ALIGN;
    CommitParams p;
    p.accept_len = accept_len; p.new_tokens = new_tokens; p.n_draft = n_draft; p.ctx_lens = ctx_lens;
    p.stride_tokens = stride_tokens; p.draft_tokens_next = draft_tokens_next; p.out_tokens = out_tokens;
    p.out_lens = out_lens; p.block_table = block_table; p.pages_used = pages_used; p.free_list = free_list;
    p.free_top = free_top; p.status = status;
    p.out_cap = out_cap; p.n_draft_steady = n_draft_steady; p.mask_token = mask_token;
    p.B = B; p.S = S; p.P = P; p.max_pages = max_pages_per_seq;
    (void)hipGetLastError();
    hipLaunchKernelGGL(isd_commit_kernel, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(stream), p);
    return launch_status();
}
