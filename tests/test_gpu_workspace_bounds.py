"""Every entry point that takes a workspace stays inside the size its *_workspace() function
reports: the workspace is a slice of a larger buffer whose remainder holds a pattern that must
survive the call, and the results must equal those of a call with a roomy workspace (which a
kernel reading past the end of the reported size would not reproduce from the pattern)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2604_11035_amd as idlm  # noqa: E402
from isd_inputs import get_config, make_accept_inputs, make_attention_inputs, make_lora_inputs  # noqa: E402

DEV = "cuda"
GUARD = 1 << 16


def _guarded(nbytes, fill):
    nbytes = max(nbytes, 256)
    full = torch.full((nbytes + GUARD,), fill, dtype=torch.uint8, device=DEV)
    return full, full[:nbytes]


def _check(call, nbytes, outputs):
    """call(ws) runs the entry point; outputs() returns the tensors to compare."""
    results = []
    for fill in (0x00, 0xFF):
        full, ws = _guarded(nbytes, fill)
        call(ws)
        torch.cuda.synchronize()
        assert bool((full[ws.numel():] == fill).all()), "the call wrote past the reported workspace size"
        results.append([t.clone() for t in outputs()])
    for a, b in zip(*results):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), "results depend on bytes the call did not write"


@pytest.mark.parametrize("name", ["small", "8b"])
def test_accept_entry_points(name):
    cfg = get_config(name, B=37) if name == "small" else get_config(name)
    acc = make_accept_inputs(cfg, device=DEV)
    B, S, V = acc.logits.shape
    al = torch.empty(B, dtype=torch.int32, device=DEV)
    nt = torch.empty(B, S, dtype=torch.int32, device=DEV)
    pr = torch.empty(B, S - 1, dtype=torch.float32, device=DEV)
    drafts = acc.draft_tokens[:, :S - 1].contiguous()
    outs = lambda: (al, nt, pr)
    kw = dict(n_draft=acc.n_draft, greedy=acc.greedy, draft_probs=pr)
    _check(lambda ws: idlm.idlm_isd_accept(acc.logits, drafts, 5, al, nt, workspace=ws, **kw),
           idlm.idlm_isd_accept_workspace(B, S, V), outs)
    lg16 = acc.logits.to(torch.bfloat16)
    _check(lambda ws: idlm.idlm_isd_accept_bf16(lg16, drafts, 5, al, nt, workspace=ws, **kw),
           idlm.idlm_isd_accept_workspace(B, S, V), outs)
    _check(lambda ws: idlm.idlm_isd_accept_general(acc.logits, drafts, 5, al, nt, temperature=0.9, tau=0.1, workspace=ws,
                                                   **kw),
           idlm.idlm_isd_accept_general_workspace(B, S, V), outs)
    _check(lambda ws: idlm.idlm_isd_accept_filtered(acc.logits, drafts, 5, al, nt, top_k=50, top_p=0.95, workspace=ws, **kw),
           idlm.idlm_isd_accept_filtered_workspace(B, S, V), outs)


# the last shape has 128 query rows per KV head: the kernel that shares the K/V tiles of a workgroup, two workgroups per CU
@pytest.mark.parametrize("name,kw", [("small", {}), ("small", {"B": 3}), ("8b", {}), ("small", {"S": 32, "B": 6})])
def test_attention(name, kw):
    cfg = get_config(name, **kw)
    att = make_attention_inputs(cfg, device=DEV)
    B, S, Hq, D = att.q.shape
    Hkv, P = att.k_cache.shape[1], att.k_cache.shape[2]
    out = torch.empty_like(att.q)
    for nwg in (0, 5, 300):
        n = idlm.idlm_isd_attention_workspace(B, S, Hq, Hkv, D, P, att.block_table.shape[1], 1, nwg)
        _check(lambda ws: idlm.idlm_isd_attention(att.q, att.k_cache, att.v_cache, att.block_table, att.ctx_lens, S, out,
                                                  num_workgroups=nwg, workspace=ws), n, lambda: (out,))
    # a workspace sized for a smaller grid than the one asked for is refused
    small = torch.empty(max(256, idlm.idlm_isd_attention_workspace(B, S, Hq, Hkv, D, P, att.block_table.shape[1], 1, 5)),
                        dtype=torch.uint8, device=DEV)
    with pytest.raises(idlm.IdlmError) as e:
        idlm.idlm_isd_attention(att.q, att.k_cache, att.v_cache, att.block_table, att.ctx_lens, S, out,
                                num_workgroups=300, workspace=small)
    assert e.value.code == -5


@pytest.mark.parametrize("B,S,d_in,d_out,r,tile,splits", [(23, 7, 320, 328, 64, 0, 0), (40, 9, 576, 264, 192, 128, 3),
                                                          (64, 7, 1024, 1024, 128, 0, 0), (5, 16, 128, 1032, 128, 64, 2)])
def test_gated_lora(B, S, d_in, d_out, r, tile, splits):
    li = make_lora_inputs(B, S, d_in, d_out, r, device=DEV, seed=2)
    h = torch.empty(B * S, d_out, dtype=torch.bfloat16, device=DEV)
    n = idlm.idlm_gated_lora_linear_workspace(B * S, d_in, d_out, r, tile, splits)
    _check(lambda ws: idlm.idlm_gated_lora_linear(li.x, li.W, li.A, li.Bm, h, n_draft=li.n_draft, S=S, tile_tokens=tile,
                                                  k_splits=splits, workspace=ws), n, lambda: (h,))
