"""Pins for the oracle's paged causal stride attention.

Each test checks the C oracle against something it does not compute itself: a
hand-enumerated pure-Python evaluation, scipy's softmax on un-paged K/V, closed
forms (uniform scores -> running mean of V; one dominant key -> that key's V),
and invariants (prefix consistency of the causal mask, block-table permutation,
GQA sharing, layout strides).  A dropped scale, an off-by-one in the causal
window, a transposed head index or a wrong page walk fails at least one.
"""
import math

import numpy as np
import pytest
from scipy.special import softmax

import oracle


def _f32_to_bf16_bits(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)  # round to nearest even
    return r


def _bf16_bits_to_f64(b):
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _paged(K, V, ctx_lens, P, rng, identity=False, spare=3):
    """Scatter contiguous per-sequence K/V [B][ctx,Hkv,D] into a page pool."""
    B = len(K)
    Hkv, D = K[0].shape[1], K[0].shape[2]
    pages = [(c + P - 1) // P for c in ctx_lens]
    need = sum(pages)
    num_pages = need + spare
    order = np.arange(num_pages) if identity else rng.permutation(num_pages)
    kc = np.full((num_pages, Hkv, P, D), np.nan, dtype=np.float32)
    vc = np.full((num_pages, Hkv, P, D), np.nan, dtype=np.float32)
    table = np.full((B, max(pages) + 1), -1, dtype=np.int32)
    off = 0
    for b in range(B):
        for p in range(pages[b]):
            pg = order[off]
            off += 1
            table[b, p] = pg
            n = min(P, ctx_lens[b] - p * P)
            kc[pg, :, :n, :] = K[b][p * P:p * P + n].transpose(1, 0, 2)
            vc[pg, :, :n, :] = V[b][p * P:p * P + n].transpose(1, 0, 2)
    return kc, vc, table


def _dense_reference(q, K, V, ctx_lens, S, scale):
    """Textbook causal attention on contiguous K/V with scipy's softmax."""
    B = len(K)
    Hq, D = q.shape[2], q.shape[3]
    Hkv = K[0].shape[1]
    G = Hq // Hkv
    out = np.zeros((B, S, Hq, D))
    for b in range(B):
        for i in range(S):
            n = ctx_lens[b] - S + i + 1
            for h in range(Hq):
                s = (K[b][:n, h // G, :].astype(np.float64) @ q[b, i, h].astype(np.float64)) * scale
                out[b, i, h] = softmax(s) @ V[b][:n, h // G, :].astype(np.float64)
    return out


def test_hand_enumerated_tiny_case():
    """B=1, S=2, ctx=3, one head, D=2, P=2: every term written out with math.exp."""
    q = np.array([[[[1.0, 0.0]], [[0.0, 2.0]]]], dtype=np.float32)          # [1,2,1,2]
    k = [[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]]
    v = [[1.0, 10.0], [2.0, 20.0], [4.0, 40.0]]
    K = [np.array(k, dtype=np.float32)[:, None, :]]
    V = [np.array(v, dtype=np.float32)[:, None, :]]
    kc, vc, table = _paged(K, V, [3], 2, np.random.default_rng(0))
    got = oracle.attention(q, kc, vc, table, [3], 2, Hq=1, Hkv=1, D=2, P=2, scale=0.5)
    # row 0 sits at position 1 -> sees keys 0,1 ; row 1 at position 2 -> sees keys 0,1,2
    s0 = [0.5 * 1.0, 0.5 * 0.0]
    w0 = [math.exp(x) for x in s0]
    e0 = [(w0[0] * v[0][d] + w0[1] * v[1][d]) / sum(w0) for d in range(2)]
    s1 = [0.5 * 0.0, 0.5 * 2.0, 0.5 * 2.0]
    w1 = [math.exp(x) for x in s1]
    e1 = [(w1[0] * v[0][d] + w1[1] * v[1][d] + w1[2] * v[2][d]) / sum(w1) for d in range(2)]
    np.testing.assert_allclose(got[0, 0, 0], e0, rtol=1e-14)
    np.testing.assert_allclose(got[0, 1, 0], e1, rtol=1e-14)


def test_default_scale_is_inverse_sqrt_head_dim():
    rng = np.random.default_rng(1)
    D = 16
    K = [rng.standard_normal((9, 1, D)).astype(np.float32)]
    V = [rng.standard_normal((9, 1, D)).astype(np.float32)]
    q = rng.standard_normal((1, 1, 1, D)).astype(np.float32)
    kc, vc, table = _paged(K, V, [9], 4, rng)
    a = oracle.attention(q, kc, vc, table, [9], 1, Hq=1, Hkv=1, D=D, P=4)
    b = _dense_reference(q, K, V, [9], 1, 1 / math.sqrt(D))
    np.testing.assert_allclose(a, b, rtol=1e-12)


@pytest.mark.parametrize("S", [1, 3, 4])
def test_matches_scipy_softmax_on_unpaged_kv(S):
    """Library-routine pin; S=1 is ordinary decode attention over ctx keys."""
    rng = np.random.default_rng(10 + S)
    B, Hq, Hkv, D, P = 3, 4, 2, 8, 4
    ctx = [S + 0, 13, 22]
    K = [rng.standard_normal((c, Hkv, D)).astype(np.float32) for c in ctx]
    V = [rng.standard_normal((c, Hkv, D)).astype(np.float32) for c in ctx]
    q = rng.standard_normal((B, S, Hq, D)).astype(np.float32)
    kc, vc, table = _paged(K, V, ctx, P, rng)
    got = oracle.attention(q, kc, vc, table, ctx, S, Hq=Hq, Hkv=Hkv, D=D, P=P, scale=0.3)
    want = _dense_reference(q, K, V, ctx, S, 0.3)
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


def test_block_table_permutation_does_not_change_result():
    rng = np.random.default_rng(3)
    B, S, Hq, Hkv, D, P = 2, 2, 2, 1, 4, 4
    ctx = [11, 18]
    K = [rng.standard_normal((c, Hkv, D)).astype(np.float32) for c in ctx]
    V = [rng.standard_normal((c, Hkv, D)).astype(np.float32) for c in ctx]
    q = rng.standard_normal((B, S, Hq, D)).astype(np.float32)
    a = oracle.attention(q, *_paged(K, V, ctx, P, rng, identity=True), ctx, S, Hq=Hq, Hkv=Hkv, D=D, P=P)
    b = oracle.attention(q, *_paged(K, V, ctx, P, rng, identity=False), ctx, S, Hq=Hq, Hkv=Hkv, D=D, P=P)
    np.testing.assert_array_equal(a, b)


def test_row_i_equals_single_row_call_on_prefix():
    """Causal prefix consistency: row i of a stride = a decode call with ctx-S+i+1 keys."""
    rng = np.random.default_rng(4)
    S, Hq, Hkv, D, P = 4, 4, 2, 8, 4
    ctx = [19]
    K = [rng.standard_normal((ctx[0], Hkv, D)).astype(np.float32)]
    V = [rng.standard_normal((ctx[0], Hkv, D)).astype(np.float32)]
    q = rng.standard_normal((1, S, Hq, D)).astype(np.float32)
    kc, vc, table = _paged(K, V, ctx, P, rng)
    full = oracle.attention(q, kc, vc, table, ctx, S, Hq=Hq, Hkv=Hkv, D=D, P=P)
    for i in range(S):
        one = oracle.attention(q[:, i:i + 1], kc, vc, table, [ctx[0] - S + i + 1], 1,
                               Hq=Hq, Hkv=Hkv, D=D, P=P)
        np.testing.assert_array_equal(full[:, i], one[:, 0])


def test_uniform_scores_give_running_mean_of_values():
    """All keys equal -> softmax is uniform -> out = mean of the visible V rows.
    With v_t = t the closed form is (ctx-S+i)/2, which pins the window length."""
    S, P, D = 4, 4, 2
    ctx = [10]
    K = [np.ones((10, 1, D), dtype=np.float32)]
    V = [np.repeat(np.arange(10, dtype=np.float32)[:, None, None], D, axis=2)]
    q = np.random.default_rng(5).standard_normal((1, S, 1, D)).astype(np.float32)
    kc, vc, table = _paged(K, V, ctx, P, np.random.default_rng(5))
    out = oracle.attention(q, kc, vc, table, ctx, S, Hq=1, Hkv=1, D=D, P=P)
    for i in range(S):
        np.testing.assert_allclose(out[0, i, 0], (ctx[0] - S + i) / 2.0, rtol=1e-13)


def test_constant_values_are_reproduced():
    rng = np.random.default_rng(6)
    ctx = [21]
    K = [rng.standard_normal((21, 2, 4)).astype(np.float32)]
    V = [np.full((21, 2, 4), 0.375, dtype=np.float32)]
    q = rng.standard_normal((1, 3, 4, 4)).astype(np.float32)
    kc, vc, table = _paged(K, V, ctx, 8, rng)
    out = oracle.attention(q, kc, vc, table, ctx, 3, Hq=4, Hkv=2, D=4, P=8)
    np.testing.assert_allclose(out, 0.375, rtol=1e-14)


def test_dominant_key_is_seen_only_from_its_own_row_on():
    """A key with an overwhelming score at stride row 2's own position: rows 0,1 must not
    see it (strictly causal), rows 2,3 return its value."""
    S, P, D = 4, 4, 2
    ctx = 9
    K = np.zeros((ctx, 1, D), dtype=np.float32)
    V = np.zeros((ctx, 1, D), dtype=np.float32)
    pos = ctx - S + 2
    K[pos, 0, 0] = 200.0
    V[pos, 0, :] = 7.0
    q = np.zeros((1, S, 1, D), dtype=np.float32)
    q[..., 0] = 1.0
    kc, vc, table = _paged([K], [V], [ctx], P, np.random.default_rng(7))
    out = oracle.attention(q, kc, vc, table, [ctx], S, Hq=1, Hkv=1, D=D, P=P, scale=1.0)
    np.testing.assert_array_equal(out[0, 0, 0], 0.0)
    np.testing.assert_array_equal(out[0, 1, 0], 0.0)
    np.testing.assert_allclose(out[0, 2, 0], 7.0, rtol=1e-12)
    np.testing.assert_allclose(out[0, 3, 0], 7.0, rtol=1e-12)


def test_gqa_heads_of_one_group_share_kv():
    rng = np.random.default_rng(8)
    Hq, Hkv, D, P = 8, 2, 4, 4
    ctx = [14]
    K = [rng.standard_normal((14, Hkv, D)).astype(np.float32)]
    V = [rng.standard_normal((14, Hkv, D)).astype(np.float32)]
    q = np.zeros((1, 2, Hq, D), dtype=np.float32)
    base = rng.standard_normal((2, 2, D)).astype(np.float32)   # one vector per (row, kv head)
    for h in range(Hq):
        q[0, :, h] = base[:, h // 4]
    kc, vc, table = _paged(K, V, ctx, P, rng)
    out = oracle.attention(q, kc, vc, table, ctx, 2, Hq=Hq, Hkv=Hkv, D=D, P=P)
    for h in range(Hq):
        np.testing.assert_array_equal(out[0, :, h], out[0, :, (h // 4) * 4])
    assert not np.allclose(out[0, :, 0], out[0, :, 4])


def test_bf16_inputs_are_decoded_exactly():
    rng = np.random.default_rng(9)
    B, S, Hq, Hkv, D, P = 1, 2, 2, 1, 8, 4
    ctx = [10]
    Kf = [rng.standard_normal((10, Hkv, D)).astype(np.float32)]
    Vf = [rng.standard_normal((10, Hkv, D)).astype(np.float32)]
    qf = rng.standard_normal((B, S, Hq, D)).astype(np.float32)
    kc, vc, table = _paged(Kf, Vf, ctx, P, rng)
    kb, vb, qb = _f32_to_bf16_bits(kc), _f32_to_bf16_bits(vc), _f32_to_bf16_bits(qf)
    assert _f32_to_bf16_bits(np.array([1.0, -2.0, 0.5]))[0] == 0x3F80
    got = oracle.attention(qb, kb, vb, table, ctx, S, Hq=Hq, Hkv=Hkv, D=D, P=P)
    # same computation on the rounded values held as fp32
    k32 = _bf16_bits_to_f64(kb).astype(np.float32)
    v32 = _bf16_bits_to_f64(vb).astype(np.float32)
    q32 = _bf16_bits_to_f64(qb).astype(np.float32)
    want = oracle.attention(q32, k32, v32, table, ctx, S, Hq=Hq, Hkv=Hkv, D=D, P=P)
    np.testing.assert_array_equal(got, want)


def test_token_major_layout_via_strides():
    rng = np.random.default_rng(11)
    S, Hq, Hkv, D, P = 2, 4, 2, 4, 4
    ctx = [13]
    K = [rng.standard_normal((13, Hkv, D)).astype(np.float32)]
    V = [rng.standard_normal((13, Hkv, D)).astype(np.float32)]
    q = rng.standard_normal((1, S, Hq, D)).astype(np.float32)
    kc, vc, table = _paged(K, V, ctx, P, rng)
    a = oracle.attention(q, kc, vc, table, ctx, S, Hq=Hq, Hkv=Hkv, D=D, P=P)
    kt = np.ascontiguousarray(kc.transpose(0, 2, 1, 3))   # [pages,P,Hkv,D]
    vt = np.ascontiguousarray(vc.transpose(0, 2, 1, 3))
    b = oracle.attention(q, kt, vt, table, ctx, S, Hq=Hq, Hkv=Hkv, D=D, P=P,
                         strides=(P * Hkv * D, D, Hkv * D))
    np.testing.assert_array_equal(a, b)


def test_unused_slots_and_table_entries_are_never_read():
    """_paged() leaves NaN in unused slots and -1 in unused table entries."""
    rng = np.random.default_rng(12)
    ctx = [5, 17]
    K = [rng.standard_normal((c, 1, 4)).astype(np.float32) for c in ctx]
    V = [rng.standard_normal((c, 1, 4)).astype(np.float32) for c in ctx]
    q = rng.standard_normal((2, 2, 1, 4)).astype(np.float32)
    kc, vc, table = _paged(K, V, ctx, 4, rng)
    out = oracle.attention(q, kc, vc, table, ctx, 2, Hq=1, Hkv=1, D=4, P=4)
    assert np.isfinite(out).all()
    table[1, 2] = -1                      # a page that *is* needed
    with pytest.raises(ValueError):
        oracle.attention(q, kc, vc, table, ctx, 2, Hq=1, Hkv=1, D=4, P=4)


def test_selection_mask_computes_only_selected_pairs():
    rng = np.random.default_rng(13)
    ctx = [9, 12]
    K = [rng.standard_normal((c, 2, 4)).astype(np.float32) for c in ctx]
    V = [rng.standard_normal((c, 2, 4)).astype(np.float32) for c in ctx]
    q = rng.standard_normal((2, 2, 4, 4)).astype(np.float32)
    kc, vc, table = _paged(K, V, ctx, 4, rng)
    full = oracle.attention(q, kc, vc, table, ctx, 2, Hq=4, Hkv=2, D=4, P=4)
    sel = np.array([[0, 1], [1, 0]], dtype=np.uint8)
    part = oracle.attention(q, kc, vc, table, ctx, 2, Hq=4, Hkv=2, D=4, P=4, sel=sel)
    np.testing.assert_array_equal(part[0, :, 2:4], full[0, :, 2:4])
    np.testing.assert_array_equal(part[1, :, 0:2], full[1, :, 0:2])
    assert np.isnan(part[0, :, 0:2]).all() and np.isnan(part[1, :, 2:4]).all()
