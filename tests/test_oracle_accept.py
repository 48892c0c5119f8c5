"""Pins for the oracle's introspective acceptance pass.

Library routine (scipy softmax, numpy argmax), closed forms for the accepted
prefix length, chi-square tests of the emitted token against the anchor
distribution (the exactness the acceptance rule is built to give, Sec. 3.2
"Adaptive stride via p/q acceptance"), forced accept / reject cases, and the
paper's worked example at N = 3.
"""
import os

import numpy as np
import pytest
from scipy import stats
from scipy.special import softmax

import oracle

GOLD = os.path.dirname(__file__) + "/golden/isd_worked_example_N3.txt"


def _logits(rng, B, S, V, sigma=2.0):
    return (rng.standard_normal((B, S, V)) * sigma).astype(np.float32)


def test_draft_probs_match_scipy_softmax():
    rng = np.random.default_rng(0)
    B, S, V = 5, 6, 97
    l = _logits(rng, B, S, V, 3.0)
    d = rng.integers(0, V, size=(B, S - 1)).astype(np.int32)
    r = oracle.accept(l, d, 1, n_draft=S - 1)
    sm = softmax(l.astype(np.float64), axis=-1)
    want = np.take_along_axis(sm[:, :S - 1], d[..., None].astype(np.int64), axis=-1)[..., 0]
    np.testing.assert_allclose(r["draft_probs"], want, rtol=1e-12)


def test_draft_probs_sum_to_one_over_the_vocabulary():
    rng = np.random.default_rng(1)
    V = 12
    l = np.repeat(_logits(rng, 1, 2, V), V, axis=0)          # same rows, V sequences
    d = np.arange(V, dtype=np.int32)[:, None]
    r = oracle.accept(l, d, 1, n_draft=1)
    assert abs(r["draft_probs"][:, 0].sum() - 1.0) < 1e-13


def test_probs_reported_for_every_draft_even_after_a_rejection_and_zero_beyond():
    rng = np.random.default_rng(2)
    l = _logits(rng, 4, 6, 50)
    d = rng.integers(0, 50, size=(4, 5)).astype(np.int32)
    r = oracle.accept(l, d, 1, n_draft=3, greedy=np.ones(4, np.uint8))
    assert (r["draft_probs"][:, :3] > 0).all()
    assert (r["draft_probs"][:, 3:] == 0).all()


@pytest.mark.parametrize("nd", [0, 1, 2, 3])
def test_greedy_is_argmax_prefix_comparison(nd):
    rng = np.random.default_rng(3 + nd)
    B, S, V = 64, 4, 40
    l = _logits(rng, B, S, V)
    am = l.argmax(-1)
    d = am[:, :S - 1].copy().astype(np.int32)
    wrong = rng.random((B, S - 1)) < 0.35
    d[wrong] = (d[wrong] + 1 + rng.integers(0, V - 1, size=wrong.sum())) % V
    r = oracle.accept(l, d, 1, n_draft=nd, greedy=np.ones(B, np.uint8))
    for b in range(B):
        k = 0
        while k < nd and d[b, k] == am[b, k]:
            k += 1
        assert r["accept_len"][b] == k <= nd
        exp = [d[b, j] for j in range(k)] + [am[b, k]] + [-1] * (nd - k) + [am[b, j] for j in range(nd + 1, S)]
        assert list(r["new_tokens"][b]) == exp
    assert np.isinf(r["sample_gap"]).all() and (r["runner_up"] == -1).all()


def test_argmax_ties_break_to_the_lowest_index():
    l = np.zeros((1, 3, 9), dtype=np.float32)
    l[0, 0, [2, 5]] = 4.0
    l[0, 1, [7, 3, 8]] = 1.5
    l[0, 2, :] = -1.0                      # whole row tied
    d = np.array([[5, 3]], dtype=np.int32)
    r = oracle.accept(l, d, 1, n_draft=1, greedy=np.ones(1, np.uint8))
    assert r["accept_len"][0] == 0          # draft 5 ties the max but is not the lowest index
    assert list(r["new_tokens"][0]) == [2, -1, 0]
    r = oracle.accept(l, np.array([[2, 3]], np.int32), 1, n_draft=2, greedy=np.ones(1, np.uint8))
    assert r["accept_len"][0] == 2 and list(r["new_tokens"][0]) == [2, 3, 0]


def test_minus_infinity_logits_get_zero_probability_and_are_never_sampled():
    l = np.full((200, 2, 6), -np.inf, dtype=np.float32)
    l[:, :, 1] = 0.0
    l[:, :, 4] = 0.0
    d = np.zeros((200, 1), dtype=np.int32)       # draft 0 has probability 0 -> always rejected
    r = oracle.accept(l, d, 5, n_draft=1)
    assert (r["draft_probs"] == 0).all() and (r["accept_len"] == 0).all()
    assert set(np.unique(r["new_tokens"][:, 0])) == {1, 4}


def _rows_with_draft_prob(pi, B, S, V, draft):
    """Logit rows whose softmax gives exactly `pi` to token `draft` (rest uniform)."""
    l = np.full((B, S, V), np.log((1 - pi) / (V - 1)) if pi < 1 else -np.inf, dtype=np.float32)
    l[:, :, draft] = np.log(pi) if pi > 0 else -np.inf
    return l


def test_forced_accept_and_forced_reject():
    B, S, V = 300, 4, 8
    d = np.full((B, S - 1), 3, dtype=np.int32)
    r = oracle.accept(_rows_with_draft_prob(1.0, B, S, V, 3), d, 9, n_draft=3)
    assert (r["accept_len"] == 3).all() and (r["new_tokens"][:, :3] == 3).all()
    assert (r["new_tokens"][:, 3] == 3).all()     # bonus from a point mass
    r = oracle.accept(_rows_with_draft_prob(0.0, B, S, V, 3), d, 9, n_draft=3)
    assert (r["accept_len"] == 0).all()
    assert (r["new_tokens"][:, 0] != 3).all() and (r["new_tokens"][:, 1:] == -1).all()


@pytest.mark.parametrize("pi,nd", [(0.7, 3), (0.5, 2), (0.9, 4)])
def test_accept_len_distribution_closed_form(pi, nd):
    """Independent accept tests with probability pi each: P(len >= k) = pi^k, so
    E[len] = sum_{k=1..D} pi^k and P(len = D) = pi^D (App. B, P-step all-pass)."""
    B, S, V = 40000, nd + 1, 8
    l = _rows_with_draft_prob(pi, B, S, V, 2)
    d = np.full((B, S - 1), 2, dtype=np.int32)
    r = oracle.accept(l, d, 1234, n_draft=nd)
    a = r["accept_len"]
    assert a.min() >= 0 and a.max() <= nd
    exp_mean = sum(pi ** k for k in range(1, nd + 1))
    se = 4 * nd / np.sqrt(B)
    assert abs(a.mean() - exp_mean) < se
    assert abs((a == nd).mean() - pi ** nd) < 4 * 0.5 / np.sqrt(B)
    for k in range(1, nd + 1):
        assert abs((a >= k).mean() - pi ** k) < 4 * 0.5 / np.sqrt(B)
    np.testing.assert_allclose(r["draft_probs"], pi, rtol=1e-6)


@pytest.mark.parametrize("draft", [0, 5, 11])
def test_emitted_token_follows_the_anchor_distribution_for_any_draft(draft):
    """Accept-or-resample at row 0 must reproduce softmax(row 0) whatever was drafted."""
    rng = np.random.default_rng(21)
    B, V = 120000, 12
    row = (rng.standard_normal(V) * 1.5).astype(np.float32)
    l = np.broadcast_to(row, (B, 2, V)).copy()
    d = np.full((B, 1), draft, dtype=np.int32)
    r = oracle.accept(l, d, 777, n_draft=1)
    first = r["new_tokens"][:, 0]
    assert ((first == draft) == (r["accept_len"] == 1)).all()
    p = softmax(row.astype(np.float64))
    counts = np.bincount(first, minlength=V)
    chi = stats.chisquare(counts, p * B)
    assert chi.pvalue > 1e-4, (chi, counts, p * B)
    # acceptance frequency itself = p(draft)
    assert abs((r["accept_len"] == 1).mean() - p[draft]) < 4 * 0.5 / np.sqrt(B)
    # on rejection the draft is excluded from the resample
    rej = r["accept_len"] == 0
    assert (first[rej] != draft).all()


def test_bonus_and_propose_only_samples_follow_softmax():
    rng = np.random.default_rng(22)
    B, V = 100000, 10
    row = (rng.standard_normal(V) * 2).astype(np.float32)
    l = np.broadcast_to(row, (B, 1, V)).copy()
    r = oracle.accept(l, None, 31337, n_draft=0)           # S = 1: plain AR decode + one sample
    assert (r["accept_len"] == 0).all()
    counts = np.bincount(r["new_tokens"][:, 0], minlength=V)
    assert stats.chisquare(counts, softmax(row.astype(np.float64)) * B).pvalue > 1e-4


def test_sampled_token_is_the_argmax_of_logit_plus_gumbel():
    rng = np.random.default_rng(23)
    B, S, V = 6, 3, 33
    l = _logits(rng, B, S, V)
    d = rng.integers(0, V, size=(B, S - 1)).astype(np.int32)
    seed, off = 99, 4
    r = oracle.accept(l, d, seed, n_draft=2, rng_offset=off)
    for b in range(B):
        k = r["accept_len"][b]
        g = np.array([oracle.gumbel(seed, off, b * S + k, i) for i in range(V)])
        s = l[b, k].astype(np.float64) + g
        if k < 2:
            s[d[b, k]] = -np.inf
        order = np.argsort(-s, kind="stable")
        assert r["new_tokens"][b, k] == order[0]
        assert r["runner_up"][b] == order[1]
        assert r["sample_gap"][b] == pytest.approx(s[order[0]] - s[order[1]], rel=1e-12)
        for j in range(2):
            u = oracle.accept_uniform(seed, off, b * S + j)
            assert r["accept_margin"][b, j] == pytest.approx(abs(u - r["draft_probs"][b, j]), rel=1e-12)
            if j < k:
                assert u < r["draft_probs"][b, j]
        if k < 2:
            assert not (oracle.accept_uniform(seed, off, b * S + k) < r["draft_probs"][b, k])


def test_rng_offset_and_seed_change_the_outcome_and_runs_are_repeatable():
    rng = np.random.default_rng(24)
    l = _logits(rng, 256, 4, 64, 1.0)
    d = rng.integers(0, 64, size=(256, 3)).astype(np.int32)
    a = oracle.accept(l, d, 5, n_draft=3, rng_offset=0)
    b = oracle.accept(l, d, 5, n_draft=3, rng_offset=0)
    c = oracle.accept(l, d, 5, n_draft=3, rng_offset=1)
    e = oracle.accept(l, d, 6, n_draft=3, rng_offset=0)
    assert np.array_equal(a["new_tokens"], b["new_tokens"])
    assert not np.array_equal(a["new_tokens"], c["new_tokens"])
    assert not np.array_equal(a["new_tokens"], e["new_tokens"])


def test_per_sequence_draft_counts_and_mixed_modes():
    rng = np.random.default_rng(25)
    B, S, V = 12, 5, 30
    l = _logits(rng, B, S, V)
    d = l.argmax(-1)[:, :S - 1].astype(np.int32)
    nd = np.array([0, 1, 2, 3, 4, 0, 1, 2, 3, 4, 2, 2], dtype=np.int32)
    gr = np.array([1, 1, 1, 1, 1, 0, 0, 0, 0, 0, 1, 0], dtype=np.uint8)
    r = oracle.accept(l, d, 3, n_draft=nd, greedy=gr)
    for b in range(B):
        assert 0 <= r["accept_len"][b] <= nd[b]
        if gr[b]:
            assert r["accept_len"][b] == nd[b]           # drafts are the arg-max -> all pass
            assert r["new_tokens"][b, nd[b]] == l[b, nd[b]].argmax()
        assert (r["new_tokens"][b, nd[b] + 1:] == l[b, nd[b] + 1:].argmax(-1)).all()
    with pytest.raises(ValueError):
        oracle.accept(l, d, 3, n_draft=S)                # more drafts than rows allow


def test_worked_example_stride_three():
    """App. F: (a) all three drafts pass -> bonus; (b) second draft fails -> resample, rest dropped."""
    cases = {}
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            cases[f[0]] = (int(f[1]), int(f[2]), int(f[3]), int(f[4]), f[5].split(","))
    V, S = 16, 6                                        # 1 exact + 3 drafts + 2 MASK rows
    for name, (nd, rej, alen, fresh_row, fate) in cases.items():
        drafts = np.array([[3, 7, 9, 0, 0]], dtype=np.int32)
        l = np.zeros((1, S, V), dtype=np.float32)
        for j in range(nd):
            l[0, j, drafts[0, j]] = -200.0 if j == rej else 200.0   # model endorses / rejects the draft
        l[0, nd, 11] = 5.0
        l[0, nd + 1, 12] = 5.0
        l[0, nd + 2, 13] = 5.0
        for mode in (None, np.ones(1, np.uint8)):
            r = oracle.accept(l, drafts, 2024, n_draft=nd, greedy=mode)
            assert r["accept_len"][0] == alen
            toks = r["new_tokens"][0]
            for j, what in enumerate(fate):
                if what == "draft":
                    assert toks[j] == drafts[0, j]
                elif what == "discarded":
                    assert toks[j] == -1
                else:
                    assert j == fresh_row and toks[j] >= 0
                    if rej >= 0:
                        assert toks[j] != drafts[0, j]
            assert list(toks[nd + 1:]) == [12, 13]      # MASK rows propose their arg-max
