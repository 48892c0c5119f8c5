"""Step semantics of the oracle against the paper's tokens-per-forward analysis.

Many sequences are driven through consecutive ISD steps with the oracle's accept
pass and synthetic logits that give every draft the same acceptance probability
p.  The state machine is the paper's renewal cycle (App. B "ISD (Ours)"): a
propose-only step after every rejection, verify+propose steps otherwise.  Tokens
finalised per forward and query rows per token must reproduce Eq. 3 and the
overhead formulas of App. B.
"""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.dirname(__file__) + "/golden/tpf_closed_form.txt"


def tpf(N, p):
    return sum([2.0] + [p ** k for k in range(1, N - 1)]) / (2 - p ** (N - 1))


def oh_var(N, p):
    return (3 * N - 1 - N * p ** (N - 1)) / sum([2.0] + [p ** k for k in range(1, N - 1)])


def oh_fix(N, p):
    return (2 * N - 1) * (2 - p ** (N - 1)) / sum([2.0] + [p ** k for k in range(1, N - 1)])


def test_closed_forms_reproduce_the_values_the_paper_states():
    for line in open(GOLD):
        if not line.strip() or line.startswith("#"):
            continue
        kind, N, p, val, tol = line.split()[:5]
        N, p, val, tol = int(N), float(p), float(val), float(tol)
        if kind == "tpf":
            assert abs(tpf(N, p) - val) <= tol
        elif kind == "breakeven_var":
            assert abs(tpf(N, p) / oh_var(N, p) - val) <= tol
        elif kind == "breakeven_fix":
            assert abs(tpf(N, p) / oh_fix(N, p) - val) <= tol
        else:
            raise AssertionError(kind)


def simulate(N, p, B=6000, steps=60, V=8, seed=5):
    """Returns (tokens per forward, query rows per token with variable-size propose steps)."""
    S = 2 * N - 1
    rng = np.random.default_rng(seed)
    n_draft = np.zeros(B, dtype=np.int32)          # first step: nothing to verify
    tokens = 0
    queries_var = 0
    for step in range(steps):
        drafts = rng.integers(0, V, size=(B, S - 1)).astype(np.int32)
        logits = np.full((B, S, V), np.log((1 - p) / (V - 1)) if p < 1 else -np.inf, dtype=np.float32)
        bi, ji = np.meshgrid(np.arange(B), np.arange(S - 1), indexing="ij")
        logits[bi, ji, drafts] = np.log(p) if p > 0 else -np.inf
        logits[:, S - 1, 0] = 0.0                  # last row is never an anchor of a draft
        r = oracle.accept(logits, drafts, 4242, n_draft=n_draft, rng_offset=step)
        alen = r["accept_len"]
        assert (alen <= n_draft).all()
        tokens += int((alen + 1).sum())            # accepted drafts + the one fresh token
        queries_var += int(np.where(n_draft == 0, N, S).sum())
        # all drafts passed (or nothing to verify) -> next step verifies N-1 new proposals;
        # a rejection -> next step is propose-only
        rejected = alen < n_draft
        n_draft = np.where(rejected, 0, N - 1).astype(np.int32)
    return tokens / (B * steps), queries_var / tokens


@pytest.mark.parametrize("N,p", [(2, 0.6), (3, 0.85), (4, 0.83), (4, 0.5), (5, 0.9)])
def test_simulated_tpf_and_overhead_match_the_closed_forms(N, p):
    got_tpf, got_oh = simulate(N, p)
    # the chain starts with a propose-only step, like a renewal cycle, so the finite-horizon
    # bias is O(1/steps); allow 2 %
    assert got_tpf == pytest.approx(tpf(N, p), rel=0.02)
    assert got_oh == pytest.approx(oh_var(N, p), rel=0.02)


@pytest.mark.parametrize("N", [2, 3, 4, 8])
def test_limits(N):
    t1, _ = simulate(N, 1.0, B=200, steps=40)
    t0, _ = simulate(N, 0.0, B=200, steps=40)
    # p = 1: one propose-only step, then N tokens per forward forever
    assert t1 == pytest.approx((1 + 39 * N) / 40, rel=1e-12)
    assert t0 == pytest.approx(1.0, rel=1e-12)
