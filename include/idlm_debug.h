/*
 * idlm_debug.h - measurement and inspection aids of the ISD hot-path library.  Nothing here is part
 * of an ISD step: these calls exist so that a benchmark can time each kernel of a call on the
 * stream it runs on, so that hardware byte counters can be calibrated against a copy of known
 * size, and so that the random numbers of the acceptance pass can be compared number by number
 * with another implementation.  Conventions (device pointers, stream, return codes) are those of
 * idlm.h.
 */
#ifndef IDLM_DEBUG_H
#define IDLM_DEBUG_H

#include "idlm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * idlm_isd_attention with timing hooks: `events`, when not NULL, is a HOST array of three hipEvent_t
 * (as void*) created by the caller; they are recorded on `stream` before the main kernel,
 * between the main kernel and the kernel that joins partial results, and after the latter, so that a
 * benchmark can time each kernel of the call without a profiler.  events == NULL is exactly
 * idlm_isd_attention.  For the fp32 path events[1] and events[2] are both recorded after its
 * single kernel.
 */
int idlm_isd_attention_ev(const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* block_table, const int32_t* ctx_lens, int32_t S, void* out,
                          int32_t B, int32_t Hq, int32_t Hkv, int32_t D, int32_t P,
                          int32_t num_pages, int32_t max_pages_per_seq,
                          int64_t page_stride, int64_t head_stride, int64_t token_stride,
                          float scale, int32_t dtype, int32_t num_workgroups,
                          void* workspace, size_t workspace_bytes, void* stream, void* const* events);


/* idlm_isd_accept with timing hooks (see idlm_isd_attention_ev): three events, recorded before the
 * row-statistics kernel, between it and the accept/sample kernel, and after the latter. */
int idlm_isd_accept_ev(const float* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                       int32_t* accept_len, int32_t* new_tokens,
                       int32_t B, int32_t S, int32_t V,
                       int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                       uint32_t rng_offset, float* draft_probs,
                       void* workspace, size_t workspace_bytes, void* stream, void* const* events);


/* idlm_isd_accept_bf16 with the same three events. */
int idlm_isd_accept_bf16_ev(const uint16_t* logits, const int32_t* draft_tokens, uint64_t rng_seed,
                            int32_t* accept_len, int32_t* new_tokens,
                            int32_t B, int32_t S, int32_t V,
                            int32_t n_draft_uniform, const int32_t* n_draft, const uint8_t* greedy,
                            uint32_t rng_offset, float* draft_probs,
                            void* workspace, size_t workspace_bytes, void* stream, void* const* events);

/*
 * idlm_isd_rng_dump - the random numbers of the acceptance pass, written out (a check, not part
 * of the step): for r < n_rows and i < V, the uniform u = (2 (x >> 9) + 1) 2^-24 and the Gumbel
 * noise g = -ln(-ln u) that vocabulary element i of logit row row0 + r draws, x being word i & 3
 * of Philox4x32-10 at counter (i >> 2, row0 + r, stream_tag, rng_offset) with key (rng_seed low,
 * high) - the generator Sec. 3.3 (3) leaves open ("Gumbel-max"); stream tags: 0 accept-test
 * uniform (element 0 of the row), 1 Gumbel noise of the fresh token, 2 of sampled proposals.
 * uniforms, gumbels  fp32 [n_rows, V] device, out; either may be NULL (not both).
 * The uniforms are exact (24-bit numerators); the noise is evaluated in single precision.
 * n_rows <= 65535.  Asynchronous on `stream`; errors as the other calls.
 */
int idlm_isd_rng_dump(uint64_t rng_seed, uint32_t rng_offset, int32_t stream_tag, int32_t row0, int32_t n_rows,
                      int32_t V, float* uniforms, float* gumbels, void* stream);

/*
 * idlm_isd_attention_wave_trace - measurement aid: from this call on every idlm_isd_attention of the process (bf16 path)
 * whose grid has at most `records` wavefronts writes, per wavefront v of its main kernel, four 64-bit words to
 * records_out[4 v ..]: the time the wavefront started and the time it finished (the device's constant 100 MHz clock,
 * common to all compute units), the number of 32-token tiles it worked on and the number of sequence parts they
 * belonged to.  Wavefronts without tiles write nothing: clear the array before the call.  Wavefront v belongs to
 * workgroup v / 4.  records_out is device memory of 32 * records bytes that stays valid until tracing is switched
 * off with (NULL, 0).  Not part of a step and not thread-safe: a process-wide setting, read when a call is launched.
 */
int idlm_isd_attention_wave_trace(uint64_t* records_out, size_t records);

/*
 * Measurement aid: copies n_bytes from src to dst with 16-byte loads and stores (n_bytes a
 * multiple of 16, both 16-byte aligned).  Used to calibrate hardware byte counters and to
 * measure the streaming bandwidth actually reachable on the device.  Same stream / error
 * conventions as above.
 */
int idlm_stream_copy(const void* src, void* dst, size_t n_bytes, void* stream);

/* Measurement aid: reads n_bytes (multiple of 16, 16-byte aligned) and writes one 4-byte
 * checksum word to *sink (device pointer): a read-only streaming pass. */
int idlm_stream_read(const void* src, size_t n_bytes, uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* IDLM_DEBUG_H */
