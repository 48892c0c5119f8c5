"""ctypes binding of libidlm_isd.so (same names as the C entry points)."""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import Optional

import torch

_HERE = Path(__file__).resolve().parent
_LIB_PATH = _HERE / "libidlm_isd.so"
_lib = None

IDLM_DTYPE_F32 = 0
IDLM_DTYPE_BF16 = 1


class IdlmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %d (%s)" % (where, code, idlm_strerror(code)))


def lib_path() -> Path:
    return _LIB_PATH


def lib() -> C.CDLL:
    """Loads the HIP library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise FileNotFoundError(
                "%s is missing: build it with `python -m paper_2604_11035_amd.build` "
                "(or __graft_entry__.build())" % _LIB_PATH)
        L = C.CDLL(str(_LIB_PATH))
        i32, i64, vp = C.c_int32, C.c_int64, C.c_void_p
        L.idlm_isd_attention.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i32, i32, i32,
                                         i64, i64, i64, C.c_float, i32, i32, vp, C.c_size_t, vp]
        L.idlm_isd_attention.restype = C.c_int
        L.idlm_isd_attention_ev.argtypes = L.idlm_isd_attention.argtypes + [vp]
        L.idlm_isd_attention_ev.restype = C.c_int
        L.idlm_isd_attention_workspace.argtypes = [i32] * 9
        L.idlm_isd_attention_workspace.restype = C.c_size_t
        L.idlm_isd_accept.argtypes = [vp, vp, C.c_uint64, vp, vp, i32, i32, i32, i32, vp, vp, C.c_uint32,
                                      vp, vp, C.c_size_t, vp]
        L.idlm_isd_accept.restype = C.c_int
        L.idlm_isd_accept_ev.argtypes = L.idlm_isd_accept.argtypes + [vp]
        L.idlm_isd_accept_ev.restype = C.c_int
        L.idlm_isd_accept_static.argtypes = [vp, vp, C.c_uint64, vp, vp, i32, i32, i32, i32, vp, vp, C.c_uint32, vp, vp]
        L.idlm_isd_accept_static.restype = C.c_int
        L.idlm_isd_accept_static_max_bytes.argtypes = []
        L.idlm_isd_accept_static_max_bytes.restype = C.c_size_t
        L.idlm_isd_accept_bf16.argtypes = L.idlm_isd_accept.argtypes
        L.idlm_isd_accept_bf16.restype = C.c_int
        L.idlm_isd_accept_bf16_ev.argtypes = L.idlm_isd_accept_ev.argtypes
        L.idlm_isd_accept_bf16_ev.restype = C.c_int
        L.idlm_isd_validate.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, i32, i32, vp, vp, vp]
        L.idlm_isd_validate.restype = C.c_int
        L.idlm_gated_lora_linear.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, i32, i32, i32, i32, i32, i32, vp,
                                             C.c_size_t, vp]
        L.idlm_gated_lora_linear.restype = C.c_int
        L.idlm_gated_lora_linear_workspace.argtypes = [i32] * 6
        L.idlm_gated_lora_linear_workspace.restype = C.c_size_t
        L.idlm_isd_accept_workspace.argtypes = [i32, i32, i32]
        L.idlm_isd_accept_workspace.restype = C.c_size_t
        L.idlm_isd_accept_general.argtypes = [vp, vp, vp, vp, vp, C.c_uint64, vp, vp, i32, i32, i32, i32, vp, vp,
                                              C.c_uint32, C.c_float, C.c_float, i32, vp, vp, vp, vp, C.c_size_t, vp]
        L.idlm_isd_accept_general.restype = C.c_int
        L.idlm_isd_accept_general_workspace.argtypes = [i32, i32, i32]
        L.idlm_isd_accept_general_workspace.restype = C.c_size_t
        L.idlm_isd_accept_filtered.argtypes = [vp, vp, C.c_uint64, vp, vp, i32, i32, i32, i32, vp, vp, C.c_uint32,
                                               C.c_float, C.c_float, i32, C.c_float, i32, vp, vp, vp, C.c_size_t, vp]
        L.idlm_isd_accept_filtered.restype = C.c_int
        L.idlm_isd_accept_filtered_q.argtypes = [vp, i32, vp, vp, vp, C.c_uint64, vp, vp, i32, i32, i32, i32, vp, vp, C.c_uint32,
                                                 C.c_float, C.c_float, i32, C.c_float, i32, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.idlm_isd_accept_filtered_q.restype = C.c_int
        L.idlm_isd_rng_dump.argtypes = [C.c_uint64, C.c_uint32, i32, i32, i32, i32, vp, vp, vp]
        L.idlm_isd_rng_dump.restype = C.c_int
        L.idlm_isd_accept_filtered_workspace.argtypes = [i32, i32, i32]
        L.idlm_isd_accept_filtered_workspace.restype = C.c_size_t
        L.idlm_isd_kv_append.argtypes = [vp] * 6 + [i32] * 7 + [i64] * 3 + [i32, vp]
        L.idlm_isd_kv_append.restype = C.c_int
        L.idlm_isd_commit.argtypes = [vp] * 8 + [i32] + [vp] * 5 + [i32] * 6 + [vp]
        L.idlm_isd_commit.restype = C.c_int
        L.idlm_strerror.argtypes = [C.c_int]
        L.idlm_strerror.restype = C.c_char_p
        L.idlm_version.restype = C.c_int
        L.idlm_stream_copy.argtypes = [vp, vp, C.c_size_t, vp]
        L.idlm_stream_copy.restype = C.c_int
        L.idlm_isd_attention_wave_trace.argtypes = [vp, C.c_size_t]
        L.idlm_isd_attention_wave_trace.restype = C.c_int
        L.idlm_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
        L.idlm_stream_read.restype = C.c_int
        _lib = L
    return _lib


def idlm_strerror(code: int) -> str:
    return lib().idlm_strerror(int(code)).decode()


def idlm_version() -> int:
    return int(lib().idlm_version())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return IDLM_DTYPE_BF16
    if t.dtype == torch.float32:
        return IDLM_DTYPE_F32
    raise TypeError("q/k/v must be bfloat16 or float32, got %s" % t.dtype)


def idlm_isd_attention_workspace(B, S, Hq, Hkv, D, P, max_pages_per_seq, dtype, num_workgroups=0) -> int:
    return int(lib().idlm_isd_attention_workspace(B, S, Hq, Hkv, D, P, max_pages_per_seq, dtype, num_workgroups))


def _events_arg(events):
    """Three hipEvent_t handles (ints) -> a host void*[3] for the *_ev entry points."""
    if events is None:
        return None
    assert len(events) == 3
    return (C.c_void_p * 3)(*[C.c_void_p(int(e)) for e in events])


def idlm_isd_attention(q, k_cache, v_cache, block_table, ctx_lens, S, out, *, scale=0.0, num_workgroups=0,
                       workspace=None, stream=None, events=None, k_operand_order=False):
    """out[b,i,h,:] = causal attention of stride row i over the paged KV cache (see idlm.h).

    q, out: [B,S,Hq,D]; k_cache, v_cache: [num_pages,Hkv,P,D] (any strides with a contiguous
    last dimension); block_table int32 [B,max_pages]; ctx_lens int32 [B].  `workspace` is a
    uint8 device tensor of at least idlm_isd_attention_workspace(...) bytes (may be None when
    that is 0); num_workgroups = 0 means one persistent workgroup per compute unit.  Asynchronous on `stream` (default: torch's current stream).  `events`: optional
    three hipEvent_t handles recorded around the call's kernels (idlm_isd_attention_ev).
    """
    B, S_, Hq, D = q.shape
    assert S_ == S and out.shape == q.shape and out.dtype == q.dtype
    assert q.is_contiguous() and out.is_contiguous()
    num_pages, Hkv, P, Dk = k_cache.shape
    assert Dk == D and v_cache.shape == k_cache.shape and v_cache.stride() == k_cache.stride()
    assert k_cache.stride(3) == 1 and k_cache.dtype == q.dtype and v_cache.dtype == q.dtype
    assert block_table.dtype == torch.int32 and ctx_lens.dtype == torch.int32
    assert block_table.is_contiguous() and ctx_lens.is_contiguous() and block_table.shape[0] == B
    args = (_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table), _ptr(ctx_lens), S, _ptr(out),
            B, Hq, Hkv, D, P, num_pages, block_table.shape[1],
            k_cache.stride(0), k_cache.stride(1), k_cache.stride(2), float(scale),
            2 if k_operand_order else _dtype_code(q),
            int(num_workgroups), _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
            _stream(stream))
    rc = lib().idlm_isd_attention(*args) if events is None else lib().idlm_isd_attention_ev(*args, _events_arg(events))
    if rc != 0:
        raise IdlmError(rc, "idlm_isd_attention")
    return out


def idlm_isd_accept_workspace(B, S, V) -> int:
    return int(lib().idlm_isd_accept_workspace(B, S, V))


def idlm_isd_accept(logits, draft_tokens, rng_seed, accept_len, new_tokens, *, n_draft, greedy=None,
                    rng_offset=0, draft_probs=None, workspace=None, stream=None, events=None):
    """Introspective acceptance over fp32 logits [B,S,V] (see idlm.h).

    n_draft: int (uniform) or int32 device tensor [B]; greedy: uint8 device tensor [B] or None.
    accept_len int32 [B] and new_tokens int32 [B,S] are written; draft_probs fp32 [B,S-1] optional.
    """
    return _accept(_with_or_without_events(lib().idlm_isd_accept, lib().idlm_isd_accept_ev), "idlm_isd_accept", torch.float32, logits, draft_tokens, rng_seed,
                   accept_len, new_tokens, n_draft, greedy, rng_offset, draft_probs, workspace, stream, events)


def idlm_isd_accept_bf16(logits, draft_tokens, rng_seed, accept_len, new_tokens, *, n_draft, greedy=None,
                         rng_offset=0, draft_probs=None, workspace=None, stream=None, events=None):
    """The same acceptance over bf16 logits [B,S,V] (half the bytes per row; see idlm.h)."""
    return _accept(_with_or_without_events(lib().idlm_isd_accept_bf16, lib().idlm_isd_accept_bf16_ev), "idlm_isd_accept_bf16", torch.bfloat16, logits, draft_tokens,
                   rng_seed, accept_len, new_tokens, n_draft, greedy, rng_offset, draft_probs, workspace, stream,
                   events)


def _with_or_without_events(plain, hooked):
    """The entry point of idlm.h unless timing events are given (then its *_ev form of idlm_debug.h)."""
    def fn(*a):
        return plain(*a[:16]) if a[16] is None else hooked(*a)
    return fn


def idlm_isd_accept_static_max_bytes() -> int:
    return int(lib().idlm_isd_accept_static_max_bytes())


def idlm_isd_accept_static(logits, draft_tokens, rng_seed, accept_len, new_tokens, *, n_draft, greedy=None,
                           rng_offset=0, draft_probs=None, stream=None):
    """idlm_isd_accept without a workspace argument: the scratch is a fixed array inside the library (see idlm.h)."""
    def fn(*a):
        return lib().idlm_isd_accept_static(*a[:13], a[15])      # no workspace, no workspace size, no events
    return _accept(fn, "idlm_isd_accept_static", torch.float32, logits, draft_tokens, rng_seed, accept_len, new_tokens,
                   n_draft, greedy, rng_offset, draft_probs, None, stream, None)


def _accept(fn, name, dtype, logits, draft_tokens, rng_seed, accept_len, new_tokens, n_draft, greedy,
            rng_offset, draft_probs, workspace, stream, events):
    B, S, V = logits.shape
    assert logits.dtype == dtype and logits.is_contiguous()
    assert accept_len.dtype == torch.int32 and new_tokens.dtype == torch.int32
    assert accept_len.numel() == B and new_tokens.shape == (B, S) and new_tokens.is_contiguous()
    if draft_tokens is not None:
        assert draft_tokens.dtype == torch.int32 and draft_tokens.is_contiguous()
        assert S == 1 or draft_tokens.shape == (B, S - 1)
    nd_ptr, nd_uni = None, 0
    if isinstance(n_draft, torch.Tensor):
        assert n_draft.dtype == torch.int32 and n_draft.numel() == B
        nd_ptr = _ptr(n_draft)
    else:
        nd_uni = int(n_draft)
    if greedy is not None:
        assert greedy.dtype == torch.uint8 and greedy.numel() == B
    if draft_probs is not None:
        assert draft_probs.dtype == torch.float32 and draft_probs.is_contiguous()
        assert draft_probs.numel() == B * (S - 1)
    rc = fn(
        _ptr(logits), _ptr(draft_tokens), int(rng_seed), _ptr(accept_len), _ptr(new_tokens),
        B, S, V, nd_uni, nd_ptr, _ptr(greedy), int(rng_offset), _ptr(draft_probs),
        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream(stream), _events_arg(events))
    if rc != 0:
        raise IdlmError(rc, name)
    return accept_len, new_tokens


def idlm_stream_copy(src, dst, stream=None):
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n
    rc = lib().idlm_stream_copy(_ptr(src), _ptr(dst), n, _stream(stream))
    if rc != 0:
        raise IdlmError(rc, "idlm_stream_copy")


def idlm_isd_attention_wave_trace(records=None):
    """Switches the per-wavefront trace of the attention main kernel on (records: int64 device tensor [n, 4], kept
    alive by the caller while tracing is on) or off (None)."""
    if records is None:
        rc = lib().idlm_isd_attention_wave_trace(None, 0)
    else:
        assert records.dtype == torch.int64 and records.is_contiguous() and records.dim() == 2 and records.shape[1] == 4
        rc = lib().idlm_isd_attention_wave_trace(_ptr(records), records.shape[0])
    if rc != 0:
        raise IdlmError(rc, "idlm_isd_attention_wave_trace")


def idlm_stream_read(src, sink, stream=None):
    rc = lib().idlm_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream))
    if rc != 0:
        raise IdlmError(rc, "idlm_stream_read")


def idlm_isd_kv_append(k_new, v_new, k_cache, v_cache, block_table, ctx_lens, S, *, stream=None,
                       k_operand_order=False):
    """Scatters the stride's K/V rows [B,S,Hkv,D] into the paged pools (see idlm.h)."""
    B, S_, Hkv, D = k_new.shape
    assert S_ == S and v_new.shape == k_new.shape and k_new.is_contiguous() and v_new.is_contiguous()
    num_pages, Hkv_c, P, Dk = k_cache.shape
    assert Hkv_c == Hkv and Dk == D and v_cache.shape == k_cache.shape and v_cache.stride() == k_cache.stride()
    assert k_cache.stride(3) == 1 and k_cache.dtype == k_new.dtype == v_new.dtype == v_cache.dtype
    assert block_table.dtype == torch.int32 and ctx_lens.dtype == torch.int32
    assert block_table.is_contiguous() and ctx_lens.is_contiguous() and block_table.shape[0] == B
    rc = lib().idlm_isd_kv_append(_ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                  _ptr(ctx_lens), S, B, Hkv, D, P, num_pages, block_table.shape[1],
                                  k_cache.stride(0), k_cache.stride(1), k_cache.stride(2),
                                  2 if k_operand_order else _dtype_code(k_new),
                                  _stream(stream))
    if rc != 0:
        raise IdlmError(rc, "idlm_isd_kv_append")


def idlm_isd_commit(accept_len, new_tokens, state, *, n_draft_steady, mask_token, P, stream=None):
    """Trim-and-commit plus the next stride, in place on `state`: a dict of int32 device tensors
    n_draft [B], ctx_lens [B], stride_tokens [B,S], draft_tokens [B,S-1], out_tokens [B,cap],
    out_lens [B], block_table [B,max_pages], pages_used [B], free_list [F], free_top [1],
    status [1] (see idlm.h).  Asynchronous: read state["status"] after synchronising."""
    B, S = new_tokens.shape
    for k, v in state.items():
        assert v.dtype == torch.int32 and v.is_contiguous(), k
    assert accept_len.dtype == torch.int32 and new_tokens.dtype == torch.int32 and new_tokens.is_contiguous()
    rc = lib().idlm_isd_commit(_ptr(accept_len), _ptr(new_tokens), _ptr(state["n_draft"]), _ptr(state["ctx_lens"]),
                               _ptr(state["stride_tokens"]), _ptr(state["draft_tokens"]) if S > 1 else None,
                               _ptr(state["out_tokens"]), _ptr(state["out_lens"]), state["out_tokens"].shape[1],
                               _ptr(state["block_table"]), _ptr(state["pages_used"]), _ptr(state["free_list"]),
                               _ptr(state["free_top"]), _ptr(state["status"]), int(n_draft_steady), int(mask_token),
                               B, S, P, state["block_table"].shape[1], _stream(stream))
    if rc != 0:
        raise IdlmError(rc, "idlm_isd_commit")


def idlm_isd_accept_general_workspace(B, S, V) -> int:
    return int(lib().idlm_isd_accept_general_workspace(B, S, V))


def idlm_isd_accept_general(logits, draft_tokens, rng_seed, accept_len, new_tokens, *, n_draft, q_logits=None,
                            q_row=None, q_lse=None, greedy=None, rng_offset=0, temperature=1.0, tau=0.0,
                            sample_proposals=False, draft_probs=None, draft_q=None, row_lse=None, workspace=None,
                            stream=None):
    """Acceptance with general proposal distributions, temperature and relaxed threshold (see idlm.h)."""
    B, S, V = logits.shape
    assert logits.dtype == torch.float32 and logits.is_contiguous()
    if S > 1:
        assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (B, S - 1) and draft_tokens.is_contiguous()
    if q_logits is not None:
        assert q_logits.shape == logits.shape and q_logits.dtype == torch.float32 and q_logits.is_contiguous()
        assert q_row is not None and q_row.dtype == torch.int32 and q_row.shape == (B,)
    if q_lse is not None:
        assert q_lse.dtype == torch.float32 and q_lse.shape == (B, S) and q_lse.is_contiguous()
    nd_uni, nd_arr = (int(n_draft), None) if isinstance(n_draft, int) else (0, n_draft)
    if nd_arr is not None:
        assert nd_arr.dtype == torch.int32 and nd_arr.shape == (B,)
    for t, shape in ((draft_probs, (B, S - 1)), (draft_q, (B, S - 1)), (row_lse, (B, S))):
        if t is not None:
            assert t.dtype == torch.float32 and tuple(t.shape) == shape and t.is_contiguous()
    rc = lib().idlm_isd_accept_general(
        _ptr(logits), _ptr(draft_tokens) if S > 1 else None, _ptr(q_logits), _ptr(q_row), _ptr(q_lse), int(rng_seed),
        _ptr(accept_len), _ptr(new_tokens), B, S, V, nd_uni, _ptr(nd_arr), _ptr(greedy), int(rng_offset),
        float(temperature), float(tau), 1 if sample_proposals else 0, _ptr(draft_probs), _ptr(draft_q), _ptr(row_lse),
        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != 0:
        raise IdlmError(rc, "idlm_isd_accept_general")


def idlm_isd_accept_filtered_workspace(B, S, V) -> int:
    return int(lib().idlm_isd_accept_filtered_workspace(B, S, V))


def idlm_isd_accept_filtered(logits, draft_tokens, rng_seed, accept_len, new_tokens, *, n_draft, top_k, top_p=1.0,
                             greedy=None, rng_offset=0, temperature=1.0, tau=0.0, sample_proposals=False,
                             draft_probs=None, kept=None, workspace=None, stream=None):
    """Acceptance under the temperature / top-k / top-p sampling distribution (see idlm.h)."""
    B, S, V = logits.shape
    assert logits.dtype == torch.float32 and logits.is_contiguous()
    if S > 1:
        assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (B, S - 1) and draft_tokens.is_contiguous()
    nd_uni, nd_arr = (int(n_draft), None) if isinstance(n_draft, int) else (0, n_draft)
    if nd_arr is not None:
        assert nd_arr.dtype == torch.int32 and nd_arr.shape == (B,)
    if draft_probs is not None:
        assert draft_probs.dtype == torch.float32 and tuple(draft_probs.shape) == (B, S - 1) and draft_probs.is_contiguous()
    if kept is not None:
        assert kept.dtype == torch.int32 and tuple(kept.shape) == (B, S) and kept.is_contiguous()
    rc = lib().idlm_isd_accept_filtered(
        _ptr(logits), _ptr(draft_tokens) if S > 1 else None, int(rng_seed), _ptr(accept_len), _ptr(new_tokens), B, S, V,
        nd_uni, _ptr(nd_arr), _ptr(greedy), int(rng_offset), float(temperature), float(tau), int(top_k), float(top_p),
        1 if sample_proposals else 0, _ptr(draft_probs), _ptr(kept), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream))
    if rc != 0:
        raise IdlmError(rc, "idlm_isd_accept_filtered")


def idlm_isd_accept_filtered_q(logits, draft_tokens, rng_seed, accept_len, new_tokens, *, n_draft, top_k, top_p=1.0,
                               q_cand=None, q_row=None, greedy=None, rng_offset=0, temperature=1.0, tau=0.0,
                               sample_proposals=False, draft_probs=None, draft_q=None, kept=None, cand_out=None,
                               workspace=None, stream=None):
    """Filtered acceptance for drafts drawn from the proposing rows' filtered distributions (see idlm.h);
    logits fp32 or bf16 [B,S,V]; q_cand / cand_out are int64 tensors [B,S,64] (the 64-bit records, opaque)."""
    B, S, V = logits.shape
    assert logits.dtype in (torch.float32, torch.bfloat16) and logits.is_contiguous()
    if S > 1:
        assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (B, S - 1) and draft_tokens.is_contiguous()
    nd_uni, nd_arr = (int(n_draft), None) if isinstance(n_draft, int) else (0, n_draft)
    if nd_arr is not None:
        assert nd_arr.dtype == torch.int32 and nd_arr.shape == (B,)
    for a in (draft_probs, draft_q):
        if a is not None:
            assert a.dtype == torch.float32 and tuple(a.shape) == (B, S - 1) and a.is_contiguous()
    if kept is not None:
        assert kept.dtype == torch.int32 and tuple(kept.shape) == (B, S) and kept.is_contiguous()
    for a in (q_cand, cand_out):
        if a is not None:
            assert a.dtype == torch.int64 and tuple(a.shape) == (B, S, 64) and a.is_contiguous()
    if q_cand is not None:
        assert q_row is not None and q_row.dtype == torch.int32 and q_row.shape == (B,)
    rc = lib().idlm_isd_accept_filtered_q(
        _ptr(logits), 1 if logits.dtype == torch.bfloat16 else 0, _ptr(draft_tokens) if S > 1 else None, _ptr(q_cand), _ptr(q_row), int(rng_seed), _ptr(accept_len),
        _ptr(new_tokens), B, S, V, nd_uni, _ptr(nd_arr), _ptr(greedy), int(rng_offset), float(temperature), float(tau),
        int(top_k), float(top_p), 1 if sample_proposals else 0, _ptr(draft_probs), _ptr(draft_q), _ptr(kept),
        _ptr(cand_out), _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream(stream))
    if rc != 0:
        raise IdlmError(rc, "idlm_isd_accept_filtered_q")


def idlm_isd_rng_dump(rng_seed, rng_offset, stream_tag, row0, n_rows, V, *, uniforms=None, gumbels=None, stream=None):
    """The uniforms / Gumbel noise the acceptance pass draws for rows row0 .. row0+n_rows-1 (see idlm_debug.h)."""
    for a in (uniforms, gumbels):
        if a is not None:
            assert a.dtype == torch.float32 and tuple(a.shape) == (n_rows, V) and a.is_contiguous()
    rc = lib().idlm_isd_rng_dump(int(rng_seed), int(rng_offset), int(stream_tag), int(row0), int(n_rows), int(V),
                                 _ptr(uniforms), _ptr(gumbels), _stream(stream))
    if rc != 0:
        raise IdlmError(rc, "idlm_isd_rng_dump")


def idlm_gated_lora_linear_workspace(T, d_in, d_out, r, tile_tokens=0, k_splits=0) -> int:
    return int(lib().idlm_gated_lora_linear_workspace(T, d_in, d_out, r, tile_tokens, k_splits))


def idlm_gated_lora_linear(x, W, A, Bm, h, *, gate=None, n_draft=None, S=1, tile_tokens=0, k_splits=0,
                           workspace=None, stream=None):
    """h[t] = W x[t] + gate[t] * Bm (A x[t]) over bf16 tensors x [T,d_in], W [d_out,d_in], A [r,d_in],
    Bm [d_out,r], h [T,d_out] (see idlm.h).  The gate is a uint8 tensor [T], or the MASK rows of every
    stride of S rows given int32 n_draft [T/S].  A / Bm may be None for a layer without adapter."""
    T, d_in = x.shape
    d_out = W.shape[0]
    r = 0 if A is None else A.shape[0]
    assert x.dtype == W.dtype == h.dtype == torch.bfloat16 and x.is_contiguous() and W.is_contiguous()
    assert W.shape == (d_out, d_in) and h.shape == (T, d_out) and h.is_contiguous()
    if r:
        assert A.dtype == Bm.dtype == torch.bfloat16 and A.is_contiguous() and Bm.is_contiguous()
        assert A.shape == (r, d_in) and Bm.shape == (d_out, r)
    if gate is not None:
        assert gate.dtype == torch.uint8 and gate.numel() == T and gate.is_contiguous()
    if n_draft is not None:
        assert n_draft.dtype == torch.int32 and n_draft.numel() * S == T and n_draft.is_contiguous()
    rc = lib().idlm_gated_lora_linear(_ptr(x), _ptr(W), _ptr(A), _ptr(Bm), _ptr(gate), _ptr(n_draft), S, _ptr(h),
                                      T, d_in, d_out, r, tile_tokens, k_splits, _ptr(workspace),
                                      0 if workspace is None else workspace.numel() * workspace.element_size(),
                                      _stream(stream))
    if rc != 0:
        raise IdlmError(rc, "idlm_gated_lora_linear")
    return h


def idlm_isd_validate(block_table, ctx_lens, S, *, P, num_pages, draft_tokens=None, n_draft=None, V=1, report=None,
                      stream=None):
    """Checks the device arrays of one step against the calls' preconditions and waits for the answer
    (see idlm.h).  Returns (return code, [bits, first bad sequence, 0, 0])."""
    B = int(ctx_lens.numel()) if ctx_lens is not None else int(n_draft.numel() if isinstance(n_draft, torch.Tensor)
                                                               else draft_tokens.shape[0])
    max_pages = 0 if block_table is None else block_table.shape[1]
    for t in (block_table, ctx_lens, draft_tokens):
        assert t is None or (t.dtype == torch.int32 and t.is_contiguous())
    nd_ptr, nd_uni = None, 0
    if isinstance(n_draft, torch.Tensor):
        assert n_draft.dtype == torch.int32 and n_draft.numel() == B
        nd_ptr = _ptr(n_draft)
    elif n_draft is not None:
        nd_uni = int(n_draft)
    if report is None:
        dev = next(t for t in (ctx_lens, block_table, draft_tokens) if t is not None).device
        report = torch.empty(4, dtype=torch.int32, device=dev)
    host = (C.c_int32 * 4)()
    rc = lib().idlm_isd_validate(_ptr(block_table), _ptr(ctx_lens), S, B, P, num_pages, max_pages, _ptr(draft_tokens),
                                 nd_ptr, nd_uni, V, _ptr(report), host, _stream(stream))
    return rc, list(host)
