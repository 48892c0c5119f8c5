"""Pins of the oracle's gated LoRA projection (App. G) against things other than itself: a case
worked by hand, numpy's matrix product on the two uniform gates (base only; merged weights
W + BA), closed forms, and the table of position types for the gate of a stride."""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.dirname(__file__) + "/golden/gated_lora_worked_example.txt"


def _rand(T=9, d_in=12, d_out=7, r=3, seed=0):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    return f(T, d_in), f(d_out, d_in), f(r, d_in), f(d_out, r)


def test_worked_example_by_hand():
    rows = [list(map(float, l.split())) for l in open(GOLD) if l.strip() and not l.startswith("#")]
    W = np.array([[2, 0], [1, -1]], dtype=np.float32)
    A = np.array([[1, 1]], dtype=np.float32)
    Bm = np.array([[3], [-2]], dtype=np.float32)
    x = np.array([r[:2] for r in rows], dtype=np.float32)
    gate = np.array([r[2] for r in rows], dtype=np.uint8)
    h = oracle.gated_lora_linear(x, W, A, Bm, gate)
    assert np.array_equal(h, np.array([r[3:] for r in rows]))


def test_gate_off_is_the_base_projection_and_gate_on_the_merged_weight():
    x, W, A, Bm = _rand()
    T = x.shape[0]
    X, Wd, Ad, Bd = (a.astype(np.float64) for a in (x, W, A, Bm))
    off = oracle.gated_lora_linear(x, W, A, Bm, np.zeros(T))
    on = oracle.gated_lora_linear(x, W, A, Bm, np.ones(T))
    np.testing.assert_allclose(off, X @ Wd.T, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(on, X @ (Wd + Bd @ Ad).T, rtol=1e-12, atol=1e-12)      # W -> W + BA
    assert np.abs(on - off).min() > 1e-6                                             # the residual is really there


def test_every_row_follows_its_own_gate_only():
    x, W, A, Bm = _rand(T=11, seed=3)
    T = x.shape[0]
    off = oracle.gated_lora_linear(x, W, A, Bm, np.zeros(T))
    on = oracle.gated_lora_linear(x, W, A, Bm, np.ones(T))
    gate = np.array([0, 1, 1, 0, 0, 1, 0, 1, 1, 1, 0], dtype=np.uint8)
    h = oracle.gated_lora_linear(x, W, A, Bm, gate)
    assert np.array_equal(h[gate == 0], off[gate == 0]) and np.array_equal(h[gate == 1], on[gate == 1])
    # base rows do not look at the adapter at all (lossless: identical to a model without it)
    h2 = oracle.gated_lora_linear(x, W, A * np.float32("nan"), Bm * np.float32("inf"), gate)
    assert np.array_equal(h2[gate == 0], off[gate == 0])
    # any non-zero gate byte counts as set
    assert np.array_equal(oracle.gated_lora_linear(x, W, A, Bm, gate * 255), h)


def test_closed_forms():
    T, d = 5, 6
    rng = np.random.default_rng(7)
    x = rng.standard_normal((T, d)).astype(np.float32)
    eye = np.eye(d, dtype=np.float32)
    gate = np.array([1, 0, 1, 0, 1], dtype=np.uint8)
    # W = I, A picks coordinate 2, B writes it to output 4 scaled by 3: h = x, and h[:,4] += 3*x[:,2] on MASK rows
    A = np.zeros((1, d), dtype=np.float32); A[0, 2] = 1
    Bm = np.zeros((d, 1), dtype=np.float32); Bm[4, 0] = 3
    h = oracle.gated_lora_linear(x, eye, A, Bm, gate)
    want = x.astype(np.float64).copy()
    want[:, 4] += 3.0 * x[:, 2].astype(np.float64) * gate
    assert np.array_equal(h, want)
    # a non-square, non-symmetric base weight: h[t,o] = sum_k W[o,k] x[t,k] with W[o,k] = 10*o + k
    W = (10 * np.arange(3)[:, None] + np.arange(d)[None, :]).astype(np.float32)
    ones = np.ones((2, d), dtype=np.float32)
    h = oracle.gated_lora_linear(ones, W, np.zeros((0, d), np.float32), np.zeros((3, 0), np.float32), [0, 1])
    assert np.array_equal(h, np.tile(W.sum(1).astype(np.float64), (2, 1)))           # rank 0: no residual
    # linear in x on both kinds of rows
    x2 = rng.standard_normal((T, d)).astype(np.float32)
    _, Wr, Ar, Br = _rand(T, d, 4, 2, seed=9)
    f = lambda v: oracle.gated_lora_linear(v, Wr, Ar, Br, gate)
    np.testing.assert_allclose(f(x) + f(x2), f((x.astype(np.float64) + x2).astype(np.float32)), atol=1e-5)


def test_bf16_bit_patterns_decode_exactly():
    import torch
    x, W, A, Bm = (torch.as_tensor(a).to(torch.bfloat16) for a in _rand(seed=5))
    bits = lambda t: t.view(torch.int16).numpy().view(np.uint16)
    gate = np.arange(x.shape[0]) % 2
    a = oracle.gated_lora_linear(bits(x), bits(W), bits(A), bits(Bm), gate)
    b = oracle.gated_lora_linear(x.float().numpy(), W.float().numpy(), A.float().numpy(), Bm.float().numpy(), gate)
    assert np.array_equal(a, b)


def test_selected_rows_only():
    x, W, A, Bm = _rand()
    T = x.shape[0]
    gate = np.arange(T) % 2
    sel = np.zeros(T, dtype=np.uint8); sel[[1, 4]] = 1
    full = oracle.gated_lora_linear(x, W, A, Bm, gate)
    part = oracle.gated_lora_linear(x, W, A, Bm, gate, sel=sel)
    assert np.array_equal(part[[1, 4]], full[[1, 4]]) and np.isnan(part[[0, 2, 3, 5, 6, 7, 8]]).all()


def test_segment_gate_follows_the_table_of_position_types():
    """App. G: the exact token and the drafts under introspection are clean inputs (base only);
    the MASK rows behind them carry the adapter.  N = 3: a propose step is 1 clean + 2 MASK rows,
    a full step 1 exact + 2 drafts + 2 MASK rows (App. B: 2N-1 rows)."""
    assert oracle.segment_gate([0], 3).tolist() == [0, 1, 1]
    assert oracle.segment_gate([2], 5).tolist() == [0, 0, 0, 1, 1]
    assert oracle.segment_gate([0, 2, 1], 5).tolist() == [0, 1, 1, 1, 1, 0, 0, 0, 1, 1, 0, 0, 1, 1, 1]
    assert oracle.segment_gate([4], 5).tolist() == [0] * 5          # every row verified, none proposed
    for S in (1, 2, 7, 16):
        for nd in range(S):
            g = oracle.segment_gate([nd], S)
            assert g.sum() == S - 1 - nd and (np.diff(g.astype(int)) >= 0).all()   # one clean segment, one MASK segment
