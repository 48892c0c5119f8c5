"""Shared plumbing of the GPU parity tests: run the HIP path through the C ABI binding, run
the CPU oracle on the same seeded inputs, and compare to the stated bars."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2604_11035_amd as idlm
from isd_inputs import to_numpy

ATTN_REL_TOL = 1e-2      # max relative error per output vector, bf16 inputs / fp32 accumulation
ATTN_REL_TOL_F32 = 1e-4  # fp32 path
PROB_ABS_TOL = 1e-5      # draft probabilities
ACCEPT_MARGIN = 1e-5     # |u - p| below this: the accept decision is within fp32 evaluation error
GAP_MARGIN = 1e-4        # top-2 gap of perturbed scores below this: either candidate is valid


def bf16_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def gpu_attention(inp, num_workgroups=0, scale=0.0, k_operand_order=False):
    """Runs idlm_isd_attention on `inp` (tensors must live on the GPU); returns float64 numpy.
    k_operand_order: hand the K pool over in the kernel's operand-order page layout (a permuted copy)."""
    cfg = inp.cfg
    out = torch.full_like(inp.q, float("nan"))
    dcode = 1 if inp.q.dtype == torch.bfloat16 else 0
    B, S, Hq, D = inp.q.shape
    Hkv, P = inp.k_cache.shape[1], inp.k_cache.shape[2]
    nbytes = idlm.idlm_isd_attention_workspace(B, S, Hq, Hkv, D, P, inp.block_table.shape[1], dcode, num_workgroups)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=inp.q.device)
    k_cache = inp.k_cache
    if k_operand_order:
        from isd_inputs import k_pages_in_operand_order
        k_cache = k_pages_in_operand_order(inp.k_cache)
    idlm.idlm_isd_attention(inp.q, k_cache, inp.v_cache, inp.block_table, inp.ctx_lens, S, out,
                            scale=scale, num_workgroups=num_workgroups, workspace=ws, k_operand_order=k_operand_order)
    torch.cuda.synchronize()
    return bf16_to_f64(out)


def oracle_attention(inp, sel=None, scale=0.0):
    cfg = inp.cfg
    B, S, Hq, D = inp.q.shape
    Hkv, P = inp.k_cache.shape[1], inp.k_cache.shape[2]
    st = inp.k_cache.stride()
    return oracle.attention(to_numpy(inp.q), _storage_numpy(inp.k_cache), _storage_numpy(inp.v_cache),
                            to_numpy(inp.block_table), to_numpy(inp.ctx_lens), S, Hq=Hq, Hkv=Hkv, D=D, P=P,
                            scale=scale, strides=(st[0], st[1], st[2]), sel=sel)


def _storage_numpy(t: torch.Tensor) -> np.ndarray:
    """Host copy of the tensor's memory in storage order (handles permuted page pools)."""
    if t.is_contiguous():
        return to_numpy(t)
    # tests build non-contiguous pools as permuted views of a contiguous base
    base = t._base if t._base is not None else t
    assert base.is_contiguous() and base.numel() == t.numel()
    return to_numpy(base)


def attention_errors(got: np.ndarray, ref: np.ndarray):
    """Max over output vectors (one per sequence, stride row and head) of
    ||got - ref||_inf / ||ref||_inf, and the number of vectors compared.  NaN rows of `ref`
    (pairs the oracle was not asked to compute) are skipped."""
    mask = ~np.isnan(ref).any(axis=-1)
    g, r = got[mask], ref[mask]
    assert np.isfinite(g).all(), "non-finite attention output"
    num = np.abs(g - r).max(axis=-1)
    den = np.abs(r).max(axis=-1)
    return float((num / den).max()), int(mask.sum())


def attention_elementwise_excess(got: np.ndarray, ref: np.ndarray) -> float:
    """The element-wise view of the same comparison: the smallest c with
    |got - ref| <= 1e-2 |ref| + c rms(ref) for every element (rms over the element's output vector)."""
    mask = ~np.isnan(ref).any(axis=-1)
    g, r = got[mask], ref[mask]
    rms = np.sqrt((r * r).mean(axis=-1, keepdims=True))
    return float(((np.abs(g - r) - 1e-2 * np.abs(r)) / rms).max())


def as_bf16(logits: torch.Tensor) -> torch.Tensor:
    """The logits as stored by a model that emits bf16 (round to nearest even): input preparation
    for the bf16 entry point; the oracle gets these values widened back to fp32, which is exact."""
    return logits.to(torch.bfloat16)


def gpu_accept(inp, n_draft=None, greedy="cfg", rng_offset=None, want_probs=True, bf16=False):
    B, S, V = inp.logits.shape
    dev = inp.logits.device
    accept_len = torch.full((B,), -7, dtype=torch.int32, device=dev)
    new_tokens = torch.full((B, S), -7, dtype=torch.int32, device=dev)
    probs = torch.full((B, max(S - 1, 1)), -7.0, dtype=torch.float32, device=dev) if want_probs else None
    ws = torch.empty(max(idlm.idlm_isd_accept_workspace(B, S, V), 256), dtype=torch.uint8, device=dev)
    nd = inp.n_draft if n_draft is None else n_draft
    gr = inp.greedy if isinstance(greedy, str) else greedy
    drafts = inp.draft_tokens[:, :S - 1].contiguous() if S > 1 else None
    fn = idlm.idlm_isd_accept_bf16 if bf16 else idlm.idlm_isd_accept
    fn(as_bf16(inp.logits) if bf16 else inp.logits, drafts, inp.rng_seed, accept_len, new_tokens, n_draft=nd,
       greedy=gr, rng_offset=inp.rng_offset if rng_offset is None else rng_offset,
       draft_probs=probs if S > 1 else None, workspace=ws)
    torch.cuda.synchronize()
    return dict(accept_len=accept_len.cpu().numpy(), new_tokens=new_tokens.cpu().numpy(),
                draft_probs=None if probs is None else probs.cpu().numpy()[:, :S - 1].astype(np.float64))


def oracle_accept(inp, n_draft=None, greedy="cfg", rng_offset=None, bf16=False):
    S = inp.logits.shape[1]
    nd = inp.n_draft if n_draft is None else n_draft
    nd = to_numpy(nd) if isinstance(nd, torch.Tensor) else nd
    gr = inp.greedy if isinstance(greedy, str) else greedy
    gr = None if gr is None else to_numpy(gr)
    drafts = to_numpy(inp.draft_tokens)[:, :S - 1] if S > 1 else None
    logits = as_bf16(inp.logits).float() if bf16 else inp.logits
    return oracle.accept(to_numpy(logits), drafts, inp.rng_seed, n_draft=nd, greedy=gr,
                         rng_offset=inp.rng_offset if rng_offset is None else rng_offset)


def compare_accept(got, ref, n_draft, strict=True):
    """Bit-exact comparison of accept_len / new_tokens wherever the oracle's decision margins
    exceed the single-precision evaluation error; returns the number of sequences whose
    decisions were too close to call (0 is required when `strict`)."""
    B, S = ref["new_tokens"].shape
    if S > 1 and got["draft_probs"] is not None:
        err = np.abs(got["draft_probs"] - ref["draft_probs"]).max()
        assert err <= PROB_ABS_TOL, "draft_probs off by %g" % err
    nd = np.broadcast_to(np.asarray(n_draft), (B,))
    close = np.zeros(B, dtype=bool)
    if S > 1:
        col = np.arange(S - 1)[None, :]
        # only decisions inside the accepted prefix (and the first failing one) matter
        relevant = col <= ref["accept_len"][:, None]
        close |= ((ref["accept_margin"] < ACCEPT_MARGIN) & relevant & (col < nd[:, None])).any(axis=1)
    close_gap = ref["sample_gap"] < GAP_MARGIN
    if strict:
        assert not close.any() and not close_gap.any(), "inputs have decisions within fp32 error; pick another seed"
    ok = ~close
    assert np.array_equal(got["accept_len"][ok], ref["accept_len"][ok])
    for b in np.nonzero(ok)[0]:
        g, r = got["new_tokens"][b], ref["new_tokens"][b]
        if close_gap[b]:
            k = ref["accept_len"][b]
            assert g[k] in (r[k], ref["runner_up"][b])
            g = g.copy(); g[k] = r[k]
        assert np.array_equal(g, r), (b, g, r)
    return int(close.sum() + (close_gap & ok).sum())
