"""CPU oracle of one ISD step (test infrastructure only).

Thin ctypes wrapper over `isd_oracle.c` (plain C, fp64).  Only tests/, the smoke
check and the benchmark's cpu_baseline leg may import this package; the product
path (paper_2604_11035_amd) never does.  Nothing here imports the product either.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_DIR = Path(__file__).resolve().parent
_SRC = _DIR / "isd_oracle.c"
_LIB = _DIR / "libisd_oracle.so"
_lib = None


# ISD_ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (CPU only; the process that loads it must have libasan preloaded,
# see tests/test_oracle_sanitized.py).
_SANITIZE = os.environ.get("ISD_ORACLE_SANITIZE", "") not in ("", "0")
if _SANITIZE:
    _LIB = _DIR / "libisd_oracle_san.so"


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP; or -O1 with the sanitizers)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=undefined"] if _SANITIZE else ["-O2"]
        subprocess.check_call(["gcc", *opt, "-std=c11", "-fopenmp", "-shared", "-fPIC",
                               "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(str(_LIB))
        L.isd_oracle_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.isd_oracle_philox4x32_10.restype = None
        L.isd_oracle_accept_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        L.isd_oracle_accept_uniform.restype = C.c_double
        L.isd_oracle_gumbel.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
        L.isd_oracle_gumbel.restype = C.c_double
        L.isd_oracle_attention.argtypes = [C.c_void_p] * 5 + [C.c_int32, C.c_void_p] + [C.c_int32] * 7 + \
            [C.c_int64] * 3 + [C.c_double, C.c_int32, C.c_void_p]
        L.isd_oracle_attention.restype = C.c_int
        L.isd_oracle_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p,
                                        C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                        C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p]
        L.isd_oracle_accept.restype = C.c_int
        L.isd_oracle_num_threads.restype = C.c_int
        L.isd_oracle_rng_dump.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.isd_oracle_rng_dump.restype = None
        L.isd_oracle_set_num_threads.argtypes = [C.c_int]
        L.isd_oracle_set_num_threads.restype = None
        L.isd_oracle_accept_general.argtypes = [C.c_void_p] * 4 + [C.c_uint64, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                                C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_uint32, C.c_double,
                                                C.c_double, C.c_int32] + [C.c_void_p] * 7
        L.isd_oracle_accept_general.restype = C.c_int
        L.isd_oracle_accept_filtered.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_int32,
                                                 C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_uint32,
                                                 C.c_double, C.c_double, C.c_int32, C.c_double, C.c_int32] + [C.c_void_p] * 7
        L.isd_oracle_accept_filtered.restype = C.c_int
        L.isd_oracle_accept_filtered_q.argtypes = [C.c_void_p] * 4 + [C.c_uint64, C.c_void_p, C.c_void_p, C.c_int32,
                                                   C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_uint32,
                                                   C.c_double, C.c_double, C.c_int32, C.c_double, C.c_int32] + [C.c_void_p] * 10
        L.isd_oracle_accept_filtered_q.restype = C.c_int
        L.isd_oracle_kv_append.argtypes = [C.c_void_p] * 6 + [C.c_int32] * 7 + [C.c_int64] * 3 + [C.c_int32]
        L.isd_oracle_kv_append.restype = C.c_int
        L.isd_oracle_commit.argtypes = [C.c_void_p] * 8 + [C.c_int32] + [C.c_void_p] * 5 + [C.c_int32] * 6
        L.isd_oracle_commit.restype = C.c_int
        L.isd_oracle_gated_lora_linear.argtypes = [C.c_void_p] * 6 + [C.c_int32] * 5 + [C.c_void_p]
        L.isd_oracle_gated_lora_linear.restype = C.c_int
        L.isd_oracle_segment_gate.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32]
        L.isd_oracle_segment_gate.restype = C.c_int
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(lib().isd_oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads used by the oracle's parallel loops from now on (results do not depend on it)."""
    lib().isd_oracle_set_num_threads(int(n))


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().isd_oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def rng_dump(seed: int, offset: int, stream: int, row0: int, n_rows: int, V: int):
    """(uniforms, gumbels), float64 [n_rows, V]: what element i of row row0 + r draws under a stream tag."""
    u = np.zeros((n_rows, V)); g = np.zeros((n_rows, V))
    lib().isd_oracle_rng_dump(int(seed), int(offset), int(stream), int(row0), n_rows, V, _ptr(u), _ptr(g))
    return u, g


def accept_uniform(seed: int, offset: int, row: int) -> float:
    return float(lib().isd_oracle_accept_uniform(seed, offset, row))


def gumbel(seed: int, offset: int, row: int, i: int) -> float:
    return float(lib().isd_oracle_gumbel(seed, offset, row, i))


def attention(q, k_cache, v_cache, block_table, ctx_lens, S, *, Hq, Hkv, D, P,
              scale=0.0, dtype=None, strides=None, sel=None, out=None) -> np.ndarray:
    """Paged causal attention of S query rows per sequence; returns float64 [B,S,Hq,D].

    q / k_cache / v_cache: float32 arrays, or uint16 arrays holding bf16 bits.
    strides = (page_stride, head_stride, token_stride) in elements; default is the
    contiguous [num_pages,Hkv,P,D] layout.
    """
    q = np.ascontiguousarray(q)
    k_cache = np.ascontiguousarray(k_cache)
    v_cache = np.ascontiguousarray(v_cache)
    if dtype is None:
        dtype = 1 if q.dtype == np.uint16 else 0
    want = np.uint16 if dtype == 1 else np.float32
    assert q.dtype == want and k_cache.dtype == want and v_cache.dtype == want
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    B = ctx_lens.shape[0]
    assert q.size == B * S * Hq * D
    max_pages = block_table.shape[1]
    if strides is None:
        num_pages = k_cache.size // (Hkv * P * D)
        strides = (Hkv * P * D, P * D, D)
    else:
        num_pages = (k_cache.size - 1) // strides[0] + 1
    if out is None:
        out = np.full((B, S, Hq, D), np.nan, dtype=np.float64)
    if sel is not None:
        sel = np.ascontiguousarray(sel, dtype=np.uint8)
        assert sel.size == B * Hkv
    rc = lib().isd_oracle_attention(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                    _ptr(ctx_lens), S, _ptr(out), B, Hq, Hkv, D, P, num_pages,
                                    max_pages, strides[0], strides[1], strides[2], float(scale),
                                    dtype, _ptr(sel))
    if rc != 0:
        raise ValueError("isd_oracle_attention failed: %d" % rc)
    return out


def accept(logits, draft_tokens, rng_seed, *, n_draft, greedy=None, rng_offset=0):
    """Introspective acceptance over logits [B,S,V].

    n_draft: int (same for every sequence) or int array [B].  greedy: None (all
    stochastic) or uint8 [B].  Returns a dict with accept_len [B], new_tokens
    [B,S], draft_probs [B,S-1] (float64) and the decision margins.
    """
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    B, S, V = logits.shape
    ncol = S - 1
    dt = None
    if S > 1:
        dt = np.ascontiguousarray(draft_tokens, dtype=np.int32)[:, :ncol]
        dt = np.ascontiguousarray(dt)
        assert dt.shape == (B, ncol)
    nd_arr, nd_uni = None, 0
    if np.isscalar(n_draft):
        nd_uni = int(n_draft)
    else:
        nd_arr = np.ascontiguousarray(n_draft, dtype=np.int32)
        assert nd_arr.shape == (B,)
    g = None if greedy is None else np.ascontiguousarray(greedy, dtype=np.uint8)
    accept_len = np.zeros(B, dtype=np.int32)
    new_tokens = np.zeros((B, S), dtype=np.int32)
    probs = np.zeros((B, max(ncol, 0)), dtype=np.float64)
    margin = np.zeros((B, max(ncol, 0)), dtype=np.float64)
    gap = np.zeros(B, dtype=np.float64)
    runner = np.zeros(B, dtype=np.int32)
    rc = lib().isd_oracle_accept(_ptr(logits), _ptr(dt), int(rng_seed), _ptr(accept_len),
                                 _ptr(new_tokens), B, S, V, nd_uni, _ptr(nd_arr), _ptr(g),
                                 int(rng_offset), _ptr(probs) if ncol else None,
                                 _ptr(margin) if ncol else None, _ptr(gap), _ptr(runner))
    if rc != 0:
        raise ValueError("isd_oracle_accept failed: %d" % rc)
    return dict(accept_len=accept_len, new_tokens=new_tokens, draft_probs=probs,
                accept_margin=margin, sample_gap=gap, runner_up=runner)


def kv_append(k_new, v_new, k_cache, v_cache, block_table, ctx_lens, S, *, Hkv, D, P, strides=None):
    """Scatters the stride's K/V rows [B,S,Hkv,D] into the paged caches IN PLACE (numpy arrays
    of uint16 bit patterns or float32, C-contiguous storage).  Raises on a broken precondition."""
    dtype = 1 if k_new.dtype == np.uint16 else 0
    want = np.uint16 if dtype == 1 else np.float32
    for a in (k_new, v_new, k_cache, v_cache):
        assert a.dtype == want and a.flags["C_CONTIGUOUS"]
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    B = ctx_lens.shape[0]
    assert k_new.size == B * S * Hkv * D and v_new.size == k_new.size
    if strides is None:
        num_pages = k_cache.size // (Hkv * P * D)
        strides = (Hkv * P * D, P * D, D)
    else:
        num_pages = (k_cache.size - 1) // strides[0] + 1
    rc = lib().isd_oracle_kv_append(_ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                    _ptr(ctx_lens), S, B, Hkv, D, P, num_pages, block_table.shape[1],
                                    strides[0], strides[1], strides[2], dtype)
    if rc != 0:
        raise ValueError("isd_oracle_kv_append failed: %d" % rc)


def commit(state, accept_len, new_tokens, *, n_draft_steady, mask_token, P):
    """Trim-and-commit plus preparation of the next stride, IN PLACE on `state`, a dict of int32
    numpy arrays: n_draft [B], ctx_lens [B], stride_tokens [B,S], draft_tokens [B,S-1],
    out_tokens [B,cap], out_lens [B], block_table [B,max_pages], pages_used [B], free_list [F],
    free_top [1].  Returns the status word (0 done, 1 free list too short, 2 table row too short)."""
    for k, v in state.items():
        assert v.dtype == np.int32 and v.flags["C_CONTIGUOUS"], k
    accept_len = np.ascontiguousarray(accept_len, dtype=np.int32)
    new_tokens = np.ascontiguousarray(new_tokens, dtype=np.int32)
    B, S = new_tokens.shape
    status = np.full(1, -1, dtype=np.int32)
    rc = lib().isd_oracle_commit(_ptr(accept_len), _ptr(new_tokens), _ptr(state["n_draft"]), _ptr(state["ctx_lens"]),
                                 _ptr(state["stride_tokens"]), _ptr(state["draft_tokens"]) if S > 1 else None,
                                 _ptr(state["out_tokens"]), _ptr(state["out_lens"]), state["out_tokens"].shape[1],
                                 _ptr(state["block_table"]), _ptr(state["pages_used"]), _ptr(state["free_list"]),
                                 _ptr(state["free_top"]), _ptr(status), int(n_draft_steady), int(mask_token),
                                 B, S, P, state["block_table"].shape[1])
    if rc != 0:
        raise ValueError("isd_oracle_commit failed: %d" % rc)
    return int(status[0])


def accept_general(logits, draft_tokens, rng_seed, *, n_draft, q_logits=None, q_row=None, greedy=None, rng_offset=0,
                   temperature=1.0, tau=0.0, sample_proposals=False):
    """Acceptance with general proposal distributions, temperature and relaxed threshold
    (isd_oracle_accept_general).  q_logits [B,S,V] + q_row [B] give the proposal
    distributions (None = point mass).  Returns the outputs of `accept` plus draft_q,
    row_lse [B,S] and proposal_gap [B,S]."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    B, S, V = logits.shape
    ncol = S - 1
    dt = None
    if S > 1:
        dt = np.ascontiguousarray(np.ascontiguousarray(draft_tokens, dtype=np.int32)[:, :ncol])
        assert dt.shape == (B, ncol)
    ql = qr = None
    if q_logits is not None:
        ql = np.ascontiguousarray(q_logits, dtype=np.float32)
        assert ql.shape == logits.shape
        qr = np.ascontiguousarray(q_row, dtype=np.int32)
        assert qr.shape == (B,)
    nd_arr, nd_uni = None, 0
    if np.isscalar(n_draft):
        nd_uni = int(n_draft)
    else:
        nd_arr = np.ascontiguousarray(n_draft, dtype=np.int32)
    g = None if greedy is None else np.ascontiguousarray(greedy, dtype=np.uint8)
    accept_len = np.zeros(B, dtype=np.int32)
    new_tokens = np.zeros((B, S), dtype=np.int32)
    probs = np.zeros((B, max(ncol, 0))); dq = np.zeros((B, max(ncol, 0))); margin = np.zeros((B, max(ncol, 0)))
    lse = np.zeros((B, S)); gap = np.zeros(B); runner = np.zeros(B, dtype=np.int32); pgap = np.zeros((B, S))
    rc = lib().isd_oracle_accept_general(_ptr(logits), _ptr(dt), _ptr(ql), _ptr(qr), int(rng_seed), _ptr(accept_len),
                                         _ptr(new_tokens), B, S, V, nd_uni, _ptr(nd_arr), _ptr(g), int(rng_offset),
                                         float(temperature), float(tau), 1 if sample_proposals else 0,
                                         _ptr(probs) if ncol else None, _ptr(dq) if ncol else None, _ptr(lse),
                                         _ptr(margin) if ncol else None, _ptr(gap), _ptr(runner), _ptr(pgap))
    if rc != 0:
        raise ValueError("isd_oracle_accept_general failed: %d" % rc)
    return dict(accept_len=accept_len, new_tokens=new_tokens, draft_probs=probs, draft_q=dq, row_lse=lse,
                accept_margin=margin, sample_gap=gap, runner_up=runner, proposal_gap=pgap)


def accept_filtered(logits, draft_tokens, rng_seed, *, n_draft, top_k, top_p=1.0, greedy=None, rng_offset=0,
                    temperature=1.0, tau=0.0, sample_proposals=False):
    """Acceptance under the filtered sampling distribution (temperature, top-k, top-p) with
    point-mass proposals (isd_oracle_accept_filtered).  Returns the outputs of `accept` plus
    kept [B,S] and proposal_gap [B,S]."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    B, S, V = logits.shape
    ncol = S - 1
    dt = None
    if S > 1:
        dt = np.ascontiguousarray(np.ascontiguousarray(draft_tokens, dtype=np.int32)[:, :ncol])
    nd_arr, nd_uni = None, 0
    if np.isscalar(n_draft):
        nd_uni = int(n_draft)
    else:
        nd_arr = np.ascontiguousarray(n_draft, dtype=np.int32)
    g = None if greedy is None else np.ascontiguousarray(greedy, dtype=np.uint8)
    accept_len = np.zeros(B, dtype=np.int32); new_tokens = np.zeros((B, S), dtype=np.int32)
    probs = np.zeros((B, max(ncol, 0))); margin = np.zeros((B, max(ncol, 0)))
    kept = np.zeros((B, S), dtype=np.int32); gap = np.zeros(B); runner = np.zeros(B, dtype=np.int32); pgap = np.zeros((B, S))
    cut = np.zeros((B, S))
    rc = lib().isd_oracle_accept_filtered(_ptr(logits), _ptr(dt), int(rng_seed), _ptr(accept_len), _ptr(new_tokens), B, S, V,
                                          nd_uni, _ptr(nd_arr), _ptr(g), int(rng_offset), float(temperature), float(tau),
                                          int(top_k), float(top_p), 1 if sample_proposals else 0,
                                          _ptr(probs) if ncol else None, _ptr(kept), _ptr(margin) if ncol else None,
                                          _ptr(gap), _ptr(runner), _ptr(pgap), _ptr(cut))
    if rc != 0:
        raise ValueError("isd_oracle_accept_filtered failed: %d" % rc)
    return dict(accept_len=accept_len, new_tokens=new_tokens, draft_probs=probs, kept=kept, accept_margin=margin,
                sample_gap=gap, runner_up=runner, proposal_gap=pgap, cut_margin=cut)


def accept_filtered_q(logits, draft_tokens, rng_seed, *, n_draft, top_k, top_p=1.0, q_logits=None, q_row=None, greedy=None,
                      rng_offset=0, temperature=1.0, tau=0.0, sample_proposals=False):
    """Acceptance under the filtered sampling distribution with drafts drawn from the filtered distribution
    of q_logits[b, q_row[b] + j, :] (isd_oracle_accept_filtered_q; q_logits None: point mass).  Returns the
    outputs of `accept_filtered` plus draft_q [B,S-1], q_cut_margin [B,S-1] and resid_small [B]."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    B, S, V = logits.shape
    ncol = S - 1
    dt = None
    if S > 1:
        dt = np.ascontiguousarray(np.ascontiguousarray(draft_tokens, dtype=np.int32)[:, :ncol])
    nd_arr, nd_uni = None, 0
    if np.isscalar(n_draft):
        nd_uni = int(n_draft)
    else:
        nd_arr = np.ascontiguousarray(n_draft, dtype=np.int32)
    ql = qr = None
    if q_logits is not None:
        ql = np.ascontiguousarray(q_logits, dtype=np.float32)
        assert ql.shape == logits.shape
        qr = np.ascontiguousarray(q_row, dtype=np.int32)
        assert qr.shape == (B,)
    g = None if greedy is None else np.ascontiguousarray(greedy, dtype=np.uint8)
    accept_len = np.zeros(B, dtype=np.int32); new_tokens = np.zeros((B, S), dtype=np.int32)
    probs = np.zeros((B, max(ncol, 0))); dq = np.zeros((B, max(ncol, 0))); margin = np.zeros((B, max(ncol, 0)))
    kept = np.zeros((B, S), dtype=np.int32); gap = np.zeros(B); runner = np.zeros(B, dtype=np.int32); pgap = np.zeros((B, S))
    cut = np.zeros((B, S)); qcut = np.zeros((B, max(ncol, 0))); small = np.zeros(B)
    rc = lib().isd_oracle_accept_filtered_q(_ptr(logits), _ptr(dt), _ptr(ql), _ptr(qr), int(rng_seed), _ptr(accept_len),
                                            _ptr(new_tokens), B, S, V, nd_uni, _ptr(nd_arr), _ptr(g), int(rng_offset),
                                            float(temperature), float(tau), int(top_k), float(top_p),
                                            1 if sample_proposals else 0, _ptr(probs) if ncol else None,
                                            _ptr(dq) if ncol else None, _ptr(kept), _ptr(margin) if ncol else None,
                                            _ptr(gap), _ptr(runner), _ptr(pgap), _ptr(cut), _ptr(qcut) if ncol else None,
                                            _ptr(small))
    if rc != 0:
        raise ValueError("isd_oracle_accept_filtered_q failed: %d" % rc)
    return dict(accept_len=accept_len, new_tokens=new_tokens, draft_probs=probs, draft_q=dq, kept=kept, accept_margin=margin,
                sample_gap=gap, runner_up=runner, proposal_gap=pgap, cut_margin=cut, q_cut_margin=qcut, resid_small=small)


def gated_lora_linear(x, W, A, Bm, gate, *, sel=None) -> np.ndarray:
    """h[t] = W x[t] + gate[t] * Bm (A x[t]) in float64 (App. G).  x [T,d_in], W [d_out,d_in], A [r,d_in],
    Bm [d_out,r]: float32 arrays, or uint16 arrays holding bf16 bits (all the same kind); gate [T].
    Rows with sel[t] == 0 are not computed (NaN)."""
    x, W, A, Bm = (np.ascontiguousarray(a) for a in (x, W, A, Bm))
    dtype = 1 if x.dtype == np.uint16 else 0
    want = np.uint16 if dtype else np.float32
    assert all(a.dtype == want for a in (x, W, A, Bm))
    T, d_in = x.shape
    d_out, r = Bm.shape
    assert W.shape == (d_out, d_in) and A.shape == (r, d_in)
    gate = np.ascontiguousarray(gate, dtype=np.uint8)
    assert gate.shape == (T,)
    if sel is not None:
        sel = np.ascontiguousarray(sel, dtype=np.uint8)
        assert sel.shape == (T,)
    h = np.full((T, d_out), np.nan, dtype=np.float64)
    rc = lib().isd_oracle_gated_lora_linear(_ptr(x), _ptr(W), _ptr(A), _ptr(Bm), _ptr(gate), _ptr(h), T, d_in,
                                            d_out, r, dtype, _ptr(sel))
    if rc != 0:
        raise ValueError("isd_oracle_gated_lora_linear failed: %d" % rc)
    return h


def segment_gate(n_draft, S) -> np.ndarray:
    """uint8 [B*S]: 1 at the MASK rows (j > n_draft[b]) of every sequence's stride (App. G)."""
    n_draft = np.ascontiguousarray(n_draft, dtype=np.int32)
    gate = np.zeros(n_draft.shape[0] * S, dtype=np.uint8)
    rc = lib().isd_oracle_segment_gate(_ptr(n_draft), _ptr(gate), n_draft.shape[0], S)
    if rc != 0:
        raise ValueError("isd_oracle_segment_gate failed: %d" % rc)
    return gate
