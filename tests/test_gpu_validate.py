"""idlm_isd_validate against the preconditions written out in numpy: every kind of broken device
array is found, with the lowest offending sequence, and clean inputs pass."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2604_11035_amd as idlm  # noqa: E402
from isd_inputs import get_config, make_accept_inputs, make_attention_inputs  # noqa: E402

DEV = "cuda"
CTX_SHORT, CTX_LONG, PAGE_ID, N_DRAFT, DRAFT_ID = 1, 2, 4, 8, 16


def expected(table, ctx, S, P, num_pages, drafts, n_draft, V):
    B = len(ctx)
    bits, first = 0, -1
    for b in range(B):
        bad = 0
        if ctx[b] < S:
            bad |= CTX_SHORT
        if ctx[b] > table.shape[1] * P:
            bad |= CTX_LONG
        npages = min(table.shape[1], -(-max(int(ctx[b]), 0) // P))
        if ((table[b, :npages] < 0) | (table[b, :npages] >= num_pages)).any():
            bad |= PAGE_ID
        nd = int(n_draft[b])
        if nd < 0 or nd > S - 1:
            bad |= N_DRAFT
        nd = max(0, min(nd, S - 1))
        if ((drafts[b, :nd] < 0) | (drafts[b, :nd] >= V)).any():
            bad |= DRAFT_ID
        if bad and first < 0:
            first = b
        bits |= bad
    return bits, first


def _state():
    cfg = get_config("small", B=40)
    att = make_attention_inputs(cfg, device=DEV)
    acc = make_accept_inputs(cfg, device=DEV)
    S = cfg.S
    return dict(table=att.block_table.clone(), ctx=att.ctx_lens.clone(), drafts=acc.draft_tokens[:, :S - 1].contiguous(),
                nd=acc.n_draft.clone(), S=S, P=cfg.P, num_pages=att.k_cache.shape[0], V=cfg.V)


def _run(st):
    rc, rep = idlm.idlm_isd_validate(st["table"], st["ctx"], st["S"], P=st["P"], num_pages=st["num_pages"],
                                     draft_tokens=st["drafts"], n_draft=st["nd"], V=st["V"])
    want = expected(st["table"].cpu().numpy(), st["ctx"].cpu().numpy(), st["S"], st["P"], st["num_pages"],
                    st["drafts"].cpu().numpy(), st["nd"].cpu().numpy(), st["V"])
    assert (rep[0], rep[1]) == want and rep[2:] == [0, 0]
    assert rc == (-7 if want[0] else 0)
    return rep


def test_clean_inputs_pass():
    assert _run(_state()) == [0, -1, 0, 0]


@pytest.mark.parametrize("kind", ["ctx_short", "ctx_long", "page_neg", "page_big", "n_draft_neg", "n_draft_big",
                                  "draft_neg", "draft_big", "several"])
def test_each_violation_is_found(kind):
    st = _state()
    if kind == "ctx_short":
        st["ctx"][17] = st["S"] - 1
    elif kind == "ctx_long":
        st["ctx"][5] = st["table"].shape[1] * st["P"] + 1
    elif kind == "page_neg":
        st["table"][9, 0] = -1                      # entries beyond the sequence's pages are -1 already and are fine
    elif kind == "page_big":
        npages = (int(st["ctx"][30]) + st["P"] - 1) // st["P"]
        st["table"][30, npages - 1] = st["num_pages"]
    elif kind == "n_draft_neg":
        st["nd"][3] = -1
    elif kind == "n_draft_big":
        st["nd"][39] = st["S"]
    elif kind == "draft_neg":
        st["drafts"][12, 0] = -5
    elif kind == "draft_big":
        st["drafts"][0, int(st["nd"][0]) - 1] = st["V"]
    else:
        st["ctx"][33] = 0
        st["drafts"][21, 1] = st["V"] + 7
        st["table"][25, 1] = 10 ** 9
    rep = _run(st)
    assert rep[0] != 0


def test_unread_entries_are_not_reported():
    st = _state()
    b = 7
    npages = (int(st["ctx"][b]) + st["P"] - 1) // st["P"]
    if npages < st["table"].shape[1]:
        st["table"][b, npages] = 10 ** 9            # beyond the sequence: never read
    st["drafts"][b, int(st["nd"][b]):] = -3         # beyond the drafts under verification: never read
    assert _run(st) == [0, -1, 0, 0]


def test_pointers_may_be_left_out_and_uniform_draft_count():
    st = _state()
    rc, rep = idlm.idlm_isd_validate(None, st["ctx"], st["S"], P=st["P"], num_pages=st["num_pages"], n_draft=st["S"] - 1)
    assert rc == 0 and rep[0] == 0
    rc, rep = idlm.idlm_isd_validate(None, st["ctx"], st["S"], P=st["P"], num_pages=st["num_pages"], n_draft=st["S"])
    assert rc == -7 and rep[:2] == [N_DRAFT, 0]
