"""Pins of the oracle's acceptance with general proposal distributions, temperature and the
relaxed threshold: the distribution of what a step emits is checked against closed forms
written with numpy / scipy (never against the oracle itself), with drafts drawn from q by numpy.
"""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax
from scipy.stats import chi2

import oracle


def chi2_ok(counts, probs, alpha=1e-4):
    n = counts.sum()
    keep = probs * n >= 5
    if (~keep).any():                       # pool the thin cells
        counts = np.append(counts[keep], counts[~keep].sum())
        probs = np.append(probs[keep], probs[~keep].sum())
    stat = ((counts - n * probs) ** 2 / (n * probs)).sum()
    return stat < chi2.ppf(1 - alpha, len(probs) - 1), stat


def run_first_row(l_p, l_q, T, tau, B, seed, rng):
    """B sequences with the same anchor logits l_p for row 0 and the same proposal logits l_q;
    draft 0 ~ softmax(l_q / T) drawn by numpy.  S = 2, one draft.  Returns emitted tokens of row 0
    (the accepted draft or the resample), accept flags, and the oracle's result."""
    V = len(l_p)
    q = softmax(np.asarray(l_q, np.float64) / T)
    drafts = rng.choice(V, size=(B, 1), p=q).astype(np.int32)
    logits = np.zeros((B, 2, V), np.float32)
    logits[:, 0] = l_p
    logits[:, 1] = rng.standard_normal(V)
    q_logits = np.zeros((B, 2, V), np.float32)
    q_logits[:, 1] = l_q                       # the proposal came from row 1 of the previous step
    r = oracle.accept_general(logits, drafts, seed, n_draft=1, q_logits=q_logits, q_row=np.ones(B, np.int32),
                              temperature=T, tau=tau)
    return r["new_tokens"][:, 0], r["accept_len"] == 1, r, drafts[:, 0]


@pytest.mark.parametrize("T", [1.0, 0.7, 1.6])
def test_emitted_token_follows_the_anchor_distribution_for_any_proposal_distribution(T):
    rng = np.random.default_rng(int(T * 10))
    V, B = 12, 60000
    l_p = rng.standard_normal(V) * 2
    for l_q in (l_p + rng.standard_normal(V), rng.standard_normal(V) * 3, l_p.copy(), -l_p):
        tok, acc, r, drafts = run_first_row(l_p.astype(np.float32), l_q.astype(np.float32), T, 0.0, B, 77, rng)
        p = softmax(l_p.astype(np.float32).astype(np.float64) / T)
        q = softmax(l_q.astype(np.float32).astype(np.float64) / T)
        ok, stat = chi2_ok(np.bincount(tok, minlength=V).astype(float), p)
        assert ok, (T, stat)
        # acceptance rate: sum_x q(x) min(1, p(x)/q(x)) = 1 - total variation distance
        rate = np.minimum(p, q).sum()
        assert abs(acc.mean() - rate) < 4 * np.sqrt(rate * (1 - rate) / B) + 1e-9
        # a resampled token lies in the support of max(0, p - q)
        res = tok[~acc]
        assert (p[res] > q[res]).all()
        # the reported probabilities are the softmax values of the drafts
        assert np.allclose(r["draft_probs"][:, 0], p[drafts], rtol=1e-12, atol=0)
        assert np.allclose(r["draft_q"][:, 0], q[drafts], rtol=1e-12, atol=0)


@pytest.mark.parametrize("tau", [0.1, 0.5])
def test_relaxed_threshold_gives_the_stated_mixture(tau):
    rng = np.random.default_rng(3)
    V, B, T = 10, 60000, 1.0
    l_p = (rng.standard_normal(V) * 2).astype(np.float32)
    l_q = (rng.standard_normal(V) * 2).astype(np.float32)
    tok, acc, r, _ = run_first_row(l_p, l_q, T, tau, B, 5, rng)
    p, q = softmax(l_p.astype(np.float64)), softmax(l_q.astype(np.float64))
    a = np.minimum(1.0, (1 + tau) * p / q)                  # accept probability of draft x
    res = np.maximum(0.0, p - q); res /= res.sum()          # resample distribution
    expect = q * a + (1 - (q * a).sum()) * res
    ok, stat = chi2_ok(np.bincount(tok, minlength=V).astype(float), expect)
    assert ok, stat
    assert abs(acc.mean() - (q * a).sum()) < 4 * np.sqrt(0.25 / B)
    # and it is NOT the anchor distribution any more (the knob trades exactness for acceptance)
    assert not chi2_ok(np.bincount(tok, minlength=V).astype(float), p)[0]


def test_bonus_token_and_sampled_proposals_follow_their_rows_at_temperature():
    rng = np.random.default_rng(8)
    V, B, S, T = 9, 50000, 4, 1.3
    row = (rng.standard_normal((S, V)) * 2).astype(np.float32)
    logits = np.broadcast_to(row, (B, S, V)).copy()
    drafts = np.zeros((B, S - 1), np.int32)
    r = oracle.accept_general(logits, drafts, 21, n_draft=0, temperature=T, sample_proposals=True)
    assert (r["accept_len"] == 0).all()
    for j in range(S):              # row 0 = bonus / exact token, rows 1.. = sampled proposals
        ok, stat = chi2_ok(np.bincount(r["new_tokens"][:, j], minlength=V).astype(float),
                           softmax(row[j].astype(np.float64) / T))
        assert ok, (j, stat)
    assert np.isinf(r["proposal_gap"][:, 0]).all() and np.isfinite(r["proposal_gap"][:, 1:]).all()
    # different streams: the fresh token and the proposal of another row are not the same draw
    r2 = oracle.accept_general(logits[:, [1, 0, 2, 3]], drafts, 21, n_draft=0, temperature=T, sample_proposals=True)
    assert (r2["new_tokens"][:, 0] != r["new_tokens"][:, 1]).mean() > 0.3
    assert np.allclose(r["row_lse"], logsumexp(row.astype(np.float64) / T, axis=-1)[None], rtol=1e-12)


def test_point_mass_special_case_is_the_deployed_acceptance():
    rng = np.random.default_rng(4)
    B, S, V = 300, 6, 64
    logits = (rng.standard_normal((B, S, V)) * 3).astype(np.float32)
    drafts = np.where(rng.random((B, S - 1)) < 0.6, logits[:, :S - 1].argmax(-1), rng.integers(0, V, (B, S - 1))).astype(np.int32)
    nd = rng.integers(0, S, size=B).astype(np.int32)
    g = (rng.random(B) < 0.4).astype(np.uint8)
    a = oracle.accept(logits, drafts, 9, n_draft=nd, greedy=g, rng_offset=3)
    b = oracle.accept_general(logits, drafts, 9, n_draft=nd, greedy=g, rng_offset=3)
    assert np.array_equal(a["accept_len"], b["accept_len"]) and np.array_equal(a["new_tokens"], b["new_tokens"])
    assert np.allclose(a["draft_probs"], b["draft_probs"], rtol=1e-12) and (b["draft_q"][np.arange(S - 1)[None] < nd[:, None]] == 1).all()


def test_greedy_ignores_proposal_distribution_threshold_and_temperature():
    rng = np.random.default_rng(6)
    B, S, V = 200, 5, 40
    logits = (rng.standard_normal((B, S, V)) * 3).astype(np.float32)
    ql = (rng.standard_normal((B, S, V)) * 3).astype(np.float32)
    drafts = np.where(rng.random((B, S - 1)) < 0.7, logits[:, :S - 1].argmax(-1), rng.integers(0, V, (B, S - 1))).astype(np.int32)
    g = np.ones(B, np.uint8)
    a = oracle.accept_general(logits, drafts, 1, n_draft=2, greedy=g)
    b = oracle.accept_general(logits, drafts, 1, n_draft=2, greedy=g, q_logits=ql, q_row=np.full(B, 2, np.int32),
                              temperature=0.4, tau=0.7, sample_proposals=True)
    assert np.array_equal(a["accept_len"], b["accept_len"]) and np.array_equal(a["new_tokens"], b["new_tokens"])
    am = logits.argmax(-1)
    want = (drafts[:, 0] == am[:, 0]).astype(int) + ((drafts[:, 0] == am[:, 0]) & (drafts[:, 1] == am[:, 1])).astype(int)
    assert np.array_equal(a["accept_len"], want)


def test_draft_outside_the_proposers_support():
    """q(x) = 0 (the proposer could not have drawn x): min(1, p/q) of Alg. 1 is 1 when the anchor gives x any
    mass, and the draft is rejected when the anchor gives it none (0/0), so that a token of zero anchor
    probability is never finalised (Sec. 3.2: outputs follow the anchor distribution)."""
    V, B = 8, 64
    ninf = np.float32(-np.inf)
    lp = np.zeros((B, 2, V), np.float32)
    lp[:, 0] = np.linspace(-1, 1, V)            # a non-uniform anchor, so that {p > q} is not empty
    lq = np.zeros((B, 2, V), np.float32)
    lq[:, 1, 3] = ninf                          # q(3) = 0 for the draft of row 0
    drafts = np.full((B, 1), 3, np.int32)
    q_row = np.ones(B, np.int32)
    r = oracle.accept_general(lp, drafts, 5, n_draft=1, q_logits=lq, q_row=q_row)
    assert (r["accept_len"] == 1).all() and (r["new_tokens"][:, 0] == 3).all()      # p(3) > 0: always accepted
    lp[:, 0, 3] = ninf                          # now p(3) = 0 as well
    r = oracle.accept_general(lp, drafts, 5, n_draft=1, q_logits=lq, q_row=q_row)
    assert (r["accept_len"] == 0).all() and (r["draft_probs"][:, 0] == 0).all() and (r["draft_q"][:, 0] == 0).all()
    assert (r["new_tokens"][:, 0] != 3).all()   # the resample comes from {p > q}, which cannot hold 3
    assert set(np.unique(r["new_tokens"][:, 0])) == {5, 6, 7}   # p > q = 1/7 only for the three largest logits


def test_general_acceptance_refuses_malformed_input():
    l = np.zeros((1, 3, 8), np.float32)
    d = np.zeros((1, 2), np.int32)
    with pytest.raises(ValueError):
        oracle.accept_general(l, d, 1, n_draft=1, temperature=0.0)
    with pytest.raises(ValueError):
        oracle.accept_general(l, d, 1, n_draft=1, tau=-0.1)
    with pytest.raises(ValueError):
        oracle.accept_general(l, d, 1, n_draft=2, q_logits=l, q_row=np.array([2], np.int32))   # q rows 2,3: beyond S
