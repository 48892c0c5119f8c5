"""Pins of the oracle's acceptance under the filtered sampling distribution (temperature, top-k,
top-p; the sampling set-up of the paper's runs, App. H): an independent numpy construction of the
filtered distribution, hand-computed small cases, chi-square tests of what is emitted, and the
unfiltered special case."""
import numpy as np
import pytest
from scipy.stats import chi2

import oracle


def filtered_reference(l, T, top_k, top_p):
    """temperature -> top-k (ties: lowest index) -> shortest prefix reaching top_p, renormalised."""
    l = np.asarray(l, np.float64)
    order = np.lexsort((np.arange(len(l)), -l))[:top_k]
    w = np.exp((l[order] - l[order[0]]) / T)
    pr = w / w.sum()
    n = int(np.searchsorted(np.cumsum(pr), top_p - 1e-15) + 1)
    n = min(n, len(order))
    out = np.zeros(len(l))
    out[order[:n]] = w[:n] / w[:n].sum()
    return out


def chi2_ok(counts, probs, alpha=1e-4):
    n = counts.sum()
    assert counts[probs == 0].sum() == 0          # nothing outside the support
    counts, probs = counts[probs > 0], probs[probs > 0]
    keep = probs * n >= 5
    if (~keep).any():
        counts = np.append(counts[keep], counts[~keep].sum()); probs = np.append(probs[keep], probs[~keep].sum())
    if len(probs) < 2:
        return True
    stat = ((counts - n * probs) ** 2 / (n * probs)).sum()
    return stat < chi2.ppf(1 - alpha, len(probs) - 1)


def test_hand_computed_filter():
    # logits 2 1 0 -1, T = 1, top-3: e^0 e^-1 e^-2 -> 0.6652 0.2447 0.0900; cumulative 0.6652, 0.9100 >= 0.8: two
    # survive, renormalised 1/(1+e^-1) = 0.7310586 and 0.2689414
    l = np.array([[[2.0, 1.0, 0.0, -1.0]] * 2] * 4, np.float32)
    drafts = np.array([[0], [1], [2], [3]], np.int32)
    r = oracle.accept_filtered(l, drafts, 1, n_draft=1, top_k=3, top_p=0.8)
    assert (r["kept"] == 2).all()
    assert np.allclose(r["draft_probs"][:, 0], [0.7310585786300049, 0.2689414213699951, 0.0, 0.0], atol=1e-15)
    # equal logits at the cut: the lowest index stays
    l2 = np.array([[[1.0, 3.0, 1.0, 1.0, 0.0]] * 2] * 5, np.float32)
    r2 = oracle.accept_filtered(l2, np.arange(5, dtype=np.int32)[:, None], 1, n_draft=1, top_k=2, top_p=1.0)
    assert (r2["kept"] == 2).all()
    e = np.exp(-2.0)
    assert np.allclose(r2["draft_probs"][:, 0], [e / (1 + e), 1 / (1 + e), 0, 0, 0], atol=1e-15)
    # top_p so small that only the arg-max survives; top_p = 1 keeps all k
    assert (oracle.accept_filtered(l, drafts, 1, n_draft=1, top_k=4, top_p=1e-6)["kept"] == 1).all()
    assert (oracle.accept_filtered(l, drafts, 1, n_draft=1, top_k=4, top_p=1.0)["kept"] == 4).all()


@pytest.mark.parametrize("T,top_k,top_p", [(1.0, 50, 0.95), (0.7, 5, 0.9), (1.4, 20, 1.0), (1.0, 1, 0.5)])
def test_probabilities_and_support_against_an_independent_construction(T, top_k, top_p):
    rng = np.random.default_rng(top_k)
    V, S = 300, 3
    rows = (rng.standard_normal((S, V)) * 2.5).astype(np.float32)
    rows[1, 17] = rows[1, 200] = rows[1].max() + 0.5          # a tie at the top
    ref = np.stack([filtered_reference(rows[j], T, top_k, top_p) for j in range(S)])
    # one sequence per vocabulary id, drafting that id in rows 0 and 1
    logits = np.broadcast_to(rows, (V, S, V)).copy()
    drafts = np.stack([np.arange(V), np.arange(V)], 1).astype(np.int32)
    r = oracle.accept_filtered(logits, drafts, 3, n_draft=2, top_k=top_k, top_p=top_p, temperature=T)
    assert np.allclose(r["draft_probs"][:, 0], ref[0], atol=1e-14) and np.allclose(r["draft_probs"][:, 1], ref[1], atol=1e-14)
    assert (r["kept"] == (ref > 0).sum(-1)[None]).all()


def test_emitted_tokens_follow_the_filtered_distribution():
    rng = np.random.default_rng(9)
    V, S, B, T, K, P = 40, 3, 60000, 1.2, 8, 0.9
    rows = (rng.standard_normal((S, V)) * 2).astype(np.float32)
    ref = np.stack([filtered_reference(rows[j], T, K, P) for j in range(S)])
    logits = np.broadcast_to(rows, (B, S, V)).copy()
    # nothing to verify: row 0 emits the fresh token, rows 1.. sampled proposals
    r = oracle.accept_filtered(logits, np.zeros((B, S - 1), np.int32), 5, n_draft=0, top_k=K, top_p=P, temperature=T,
                               sample_proposals=True)
    for j in range(S):
        assert chi2_ok(np.bincount(r["new_tokens"][:, j], minlength=V).astype(float), ref[j]), j
    # arg-max draft in row 0: accepted with probability pf(arg-max); a rejection resamples from the rest of the support
    am = int(rows[0].argmax())
    drafts = np.full((B, S - 1), am, np.int32)
    r = oracle.accept_filtered(logits, drafts, 6, n_draft=1, top_k=K, top_p=P, temperature=T)
    acc = r["accept_len"] == 1
    pa = ref[0, am]
    assert abs(acc.mean() - pa) < 4 * np.sqrt(pa * (1 - pa) / B)
    rest = ref[0].copy(); rest[am] = 0; rest /= rest.sum()
    assert chi2_ok(np.bincount(r["new_tokens"][~acc, 0], minlength=V).astype(float), rest)
    # a draft outside the support is always rejected
    out = int(np.argmin(rows[0]))
    r = oracle.accept_filtered(logits[:2000], np.full((2000, S - 1), out, np.int32), 6, n_draft=1, top_k=K, top_p=P, temperature=T)
    assert (r["accept_len"] == 0).all() and (r["draft_probs"][:, 0] == 0).all()


def test_without_filter_it_is_the_general_acceptance():
    rng = np.random.default_rng(2)
    B, S, V = 200, 5, 64
    logits = (rng.standard_normal((B, S, V)) * 3).astype(np.float32)
    drafts = np.where(rng.random((B, S - 1)) < 0.6, logits[:, :S - 1].argmax(-1), rng.integers(0, V, (B, S - 1))).astype(np.int32)
    nd = rng.integers(0, S, size=B).astype(np.int32)
    g = (rng.random(B) < 0.3).astype(np.uint8)
    a = oracle.accept_general(logits, drafts, 4, n_draft=nd, greedy=g, temperature=0.8, tau=0.2, sample_proposals=True)
    f = oracle.accept_filtered(logits, drafts, 4, n_draft=nd, greedy=g, temperature=0.8, tau=0.2, sample_proposals=True,
                               top_k=V, top_p=1.0)
    assert np.array_equal(a["accept_len"], f["accept_len"]) and np.array_equal(a["new_tokens"], f["new_tokens"])
    assert np.allclose(a["draft_probs"], f["draft_probs"], rtol=1e-12)


def test_filtered_acceptance_refuses_malformed_input():
    l = np.zeros((1, 2, 8), np.float32); d = np.zeros((1, 1), np.int32)
    for kw in (dict(top_k=0), dict(top_k=4, top_p=0.0), dict(top_k=4, top_p=1.5), dict(top_k=4, temperature=0.0)):
        with pytest.raises(ValueError):
            oracle.accept_filtered(l, d, 1, n_draft=1, **kw)


# ---- drafts drawn from the filtered distribution of the proposing row (Alg. 1 as printed, under the filter) ----

def run_first_row_q(l_p, l_q, T, top_k, top_p, tau, B, seed, rng):
    """B sequences with the same anchor row l_p and the same proposing row l_q; draft 0 is drawn by numpy from
    the filtered distribution of l_q (independent construction).  S = 2, one draft."""
    V = len(l_p)
    qf = filtered_reference(l_q, T, top_k, top_p)
    drafts = rng.choice(V, size=(B, 1), p=qf).astype(np.int32)
    logits = np.zeros((B, 2, V), np.float32)
    logits[:, 0] = l_p
    logits[:, 1] = rng.standard_normal(V)
    q_logits = np.zeros((B, 2, V), np.float32)
    q_logits[:, 1] = l_q
    r = oracle.accept_filtered_q(logits, drafts, seed, n_draft=1, q_logits=q_logits, q_row=np.ones(B, np.int32),
                                 temperature=T, tau=tau, top_k=top_k, top_p=top_p)
    return r["new_tokens"][:, 0], r["accept_len"] == 1, r, drafts[:, 0]


@pytest.mark.parametrize("T,top_k,top_p", [(1.0, 50, 0.95), (0.8, 6, 0.9), (1.5, 10, 1.0)])
def test_emitted_token_follows_the_filtered_anchor_for_any_filtered_proposal(T, top_k, top_p):
    """The point of the p/q test: whatever filtered distribution proposed the draft, what row 0 emits (the accepted
    draft or the residual resample) is distributed as the anchor's filtered distribution."""
    rng = np.random.default_rng(top_k + 100)
    V, B = 30, 60000
    l_p = (rng.standard_normal(V) * 2).astype(np.float32)
    for l_q in (l_p + rng.standard_normal(V).astype(np.float32), (rng.standard_normal(V) * 3).astype(np.float32), l_p.copy(), -l_p):
        tok, acc, r, drafts = run_first_row_q(l_p, l_q, T, top_k, top_p, 0.0, B, 91, rng)
        pf, qf = filtered_reference(l_p, T, top_k, top_p), filtered_reference(l_q, T, top_k, top_p)
        assert chi2_ok(np.bincount(tok, minlength=V).astype(float), pf)
        rate = np.minimum(pf, qf).sum()                     # 1 - total variation distance of the two filtered distributions
        assert abs(acc.mean() - rate) < 4 * np.sqrt(max(rate * (1 - rate), 1e-4) / B) + 1e-9
        res = tok[~acc]
        assert (pf[res] > qf[res]).all()                    # resamples lie in the support of max(0, pf - qf)
        assert np.allclose(r["draft_probs"][:, 0], pf[drafts], atol=1e-14) and np.allclose(r["draft_q"][:, 0], qf[drafts], atol=1e-14)
        if np.array_equal(l_q, l_p):
            assert acc.all()                                # identical distributions: ratio 1, never rejected


def test_filtered_proposals_hand_computed_residual():
    # pf = (0.5, 0.3, 0.2), qf = (0.2, 0.6, 0.2) over ids 0..2 (id 3 filtered out of both by top_k = 3):
    # residual max(0, pf - qf) = (0.3, 0, 0): every rejection resamples id 0; draft 1 passes with probability 0.5,
    # drafts 0 and 2 always pass (ratios 2.5 and 1)
    B = 4000
    l_p = np.log(np.array([0.5, 0.3, 0.2, 1e-3])).astype(np.float32)
    l_q = np.log(np.array([0.2, 0.6, 0.2, 1e-3])).astype(np.float32)
    logits = np.zeros((B, 2, 4), np.float32); logits[:, 0] = l_p
    q_logits = np.zeros((B, 2, 4), np.float32); q_logits[:, 1] = l_q
    for x, rate in ((0, 1.0), (1, 0.5), (2, 1.0)):
        r = oracle.accept_filtered_q(logits, np.full((B, 1), x, np.int32), 13, n_draft=1, q_logits=q_logits,
                                     q_row=np.ones(B, np.int32), top_k=3, top_p=1.0)
        acc = r["accept_len"] == 1
        assert abs(acc.mean() - rate) < 4 * np.sqrt(0.25 / B) * (rate < 1) + 1e-12
        assert (r["new_tokens"][~acc, 0] == 0).all()
        assert np.allclose(r["draft_probs"][:, 0], [0.5, 0.3, 0.2][x], atol=1e-6) and np.allclose(r["draft_q"][:, 0], [0.2, 0.6, 0.2][x], atol=1e-6)
    # a draft outside the proposer's support cannot have been drawn from it: accepted iff the anchor keeps it
    q2 = q_logits.copy(); q2[:, 1] = np.log(np.array([0.2, 0.6, 1e-3, 0.2])).astype(np.float32)      # proposer keeps 0, 1, 3
    r = oracle.accept_filtered_q(logits[:50], np.full((50, 1), 2, np.int32), 13, n_draft=1, q_logits=q2[:50],
                                 q_row=np.ones(50, np.int32), top_k=3, top_p=1.0)
    assert (r["accept_len"] == 1).all() and (r["draft_q"] == 0).all()
    r = oracle.accept_filtered_q(logits[:50], np.full((50, 1), 3, np.int32), 13, n_draft=1, q_logits=q2[:50],
                                 q_row=np.ones(50, np.int32), top_k=3, top_p=1.0)
    assert (r["accept_len"] == 0).all() and (r["draft_probs"] == 0).all()


@pytest.mark.parametrize("tau", [0.25])
def test_filtered_proposals_relaxed_threshold_mixture(tau):
    rng = np.random.default_rng(8)
    V, B, T, K, P = 16, 60000, 1.0, 8, 0.9
    l_p = (rng.standard_normal(V) * 2).astype(np.float32)
    l_q = (l_p + rng.standard_normal(V)).astype(np.float32)
    tok, acc, r, _ = run_first_row_q(l_p, l_q, T, K, P, tau, B, 5, rng)
    pf, qf = filtered_reference(l_p, T, K, P), filtered_reference(l_q, T, K, P)
    a = np.where(qf > 0, np.minimum(1.0, (1 + tau) * pf / np.where(qf > 0, qf, 1)), 0.0)
    res = np.maximum(0.0, pf - qf); res /= res.sum()
    expect = qf * a + (1 - (qf * a).sum()) * res
    assert chi2_ok(np.bincount(tok, minlength=V).astype(float), expect)
    assert abs(acc.mean() - (qf * a).sum()) < 4 * np.sqrt(0.25 / B)


def test_filtered_q_special_cases_reduce_to_the_pinned_functions():
    rng = np.random.default_rng(21)
    B, S, V = 150, 5, 48
    logits = (rng.standard_normal((B, S, V)) * 3).astype(np.float32)
    q_logits = (logits + rng.standard_normal((B, S, V))).astype(np.float32)
    drafts = np.where(rng.random((B, S - 1)) < 0.6, logits[:, :S - 1].argmax(-1), rng.integers(0, V, (B, S - 1))).astype(np.int32)
    nd = rng.integers(0, S, size=B).astype(np.int32)
    q_row = (S - nd).astype(np.int32) * (nd > 0)              # the last n_draft rows of the previous step
    g = (rng.random(B) < 0.3).astype(np.uint8)
    kw = dict(n_draft=nd, greedy=g, temperature=0.8, tau=0.2, sample_proposals=True, rng_offset=4)
    # no proposal logits: the point-mass function
    a = oracle.accept_filtered(logits, drafts, 4, top_k=7, top_p=0.9, **kw)
    f = oracle.accept_filtered_q(logits, drafts, 4, top_k=7, top_p=0.9, **kw)
    for k in ("accept_len", "new_tokens", "kept", "draft_probs", "sample_gap"):
        assert np.array_equal(a[k], f[k]), k
    assert (f["draft_q"][np.arange(S - 1)[None] < nd[:, None]] == 1).all()
    # no filter: Alg. 1 with full proposal distributions
    a = oracle.accept_general(logits, drafts, 4, q_logits=q_logits, q_row=q_row, **kw)
    f = oracle.accept_filtered_q(logits, drafts, 4, q_logits=q_logits, q_row=q_row, top_k=V, top_p=1.0, **kw)
    assert np.array_equal(a["accept_len"], f["accept_len"]) and np.array_equal(a["new_tokens"], f["new_tokens"])
    assert np.allclose(a["draft_probs"], f["draft_probs"], rtol=1e-12) and np.allclose(a["draft_q"], f["draft_q"], rtol=1e-12)
    assert (a["accept_len"] < nd).sum() > 20 and (a["accept_len"] == nd).sum() > 20
    with pytest.raises(ValueError):
        oracle.accept_filtered_q(logits, drafts, 4, n_draft=nd, q_logits=q_logits, q_row=np.full(B, S, np.int32), top_k=5)
