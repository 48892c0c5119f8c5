"""idlm_isd_accept_static, the acceptance entry point that allocates nothing (its scratch memory is a fixed
array inside the library), against idlm_isd_accept with a caller's workspace, through the C ABI: the same
kernels run on the same inputs, so every output must be equal bit for bit - on two calls in a row, the second
on a smaller input (the array keeps the first call's contents), and the first call is also checked against the
CPU oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2604_11035_amd as idlm  # noqa: E402
from isd_inputs import get_config, make_accept_inputs  # noqa: E402

DEV = "cuda"


def _both(inp, rng_offset):
    B, S, V = inp.logits.shape
    drafts = inp.draft_tokens[:, :S - 1].contiguous()
    outs = []
    for static in (False, True):
        al = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        nt = torch.full((B, S), -7, dtype=torch.int32, device=DEV)
        pr = torch.full((B, S - 1), -7.0, dtype=torch.float32, device=DEV)
        kw = dict(n_draft=inp.n_draft, greedy=inp.greedy, rng_offset=rng_offset, draft_probs=pr)
        if static:
            idlm.idlm_isd_accept_static(inp.logits, drafts, inp.rng_seed, al, nt, **kw)
        else:
            ws = torch.empty(idlm.idlm_isd_accept_workspace(B, S, V), dtype=torch.uint8, device=DEV)
            idlm.idlm_isd_accept(inp.logits, drafts, inp.rng_seed, al, nt, workspace=ws, **kw)
        torch.cuda.synchronize()
        outs.append((al.cpu().numpy(), nt.cpu().numpy(), pr.cpu().numpy()))
    return outs


def test_static_scratch_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    import helpers as h
    big = make_accept_inputs(get_config("8b"), device=DEV)                   # 512 rows cut into slices
    small = make_accept_inputs(get_config("small", B=5), device=DEV)          # fewer, shorter rows
    assert idlm.idlm_isd_accept_workspace(*big.logits.shape) <= idlm.idlm_isd_accept_static_max_bytes()
    for inp, off in ((big, 3), (small, 4)):
        (al0, nt0, pr0), (al1, nt1, pr1) = _both(inp, off)
        assert (al0 >= 0).all() and (nt1 != -7).all()
        assert np.array_equal(al0, al1) and np.array_equal(nt0, nt1) and np.array_equal(pr0, pr1)
    # the first call's results against the oracle, to the bar of the parity tests
    (al0, nt0, pr0), (al1, nt1, pr1) = _both(big, 3)
    ref = h.oracle_accept(big, rng_offset=3)
    got = dict(accept_len=al1, new_tokens=nt1, draft_probs=pr1.astype(np.float64))
    assert h.compare_accept(got, ref, big.cfg.drafts, strict=False) <= 1


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    B, S, V = 8192, 16, 1024                              # 131 072 rows: beyond the fixed array
    assert idlm.idlm_isd_accept_workspace(B, S, V) > idlm.idlm_isd_accept_static_max_bytes()
    logits = torch.zeros(1, S, V, device=DEV)             # never read: the call must refuse before launching
    al = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    nt = torch.full((B, S), -7, dtype=torch.int32, device=DEV)
    dr = torch.zeros(B, S - 1, dtype=torch.int32, device=DEV)
    rc = idlm.lib().idlm_isd_accept_static(logits.data_ptr(), dr.data_ptr(), 1, al.data_ptr(), nt.data_ptr(), B, S, V, 1,
                                           None, None, 0, None, None)
    torch.cuda.synchronize()
    assert rc == -5 and "workspace" in idlm.idlm_strerror(rc)
    assert (al == -7).all() and (nt == -7).all()
