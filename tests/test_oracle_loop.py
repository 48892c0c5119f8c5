"""Pins of the oracle's between-steps functions (KV append, trim-and-commit / next stride).

They are checked against things other than themselves: independent numpy gathers and a
textbook attention on contiguous K/V (append + page walk), the paper's worked example and
closed-form tokens-per-forward (commit), and the lossless property of greedy acceptance: the
token stream of the whole loop must equal plain greedy autoregressive decoding of the same
next-token function, whatever the stride and however bad the proposals are.
"""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.dirname(__file__) + "/golden/isd_commit_worked_example_N3.txt"
MASK = 7_000_000


# ---- KV append -------------------------------------------------------------------------------

def _paged_setup(rng, B, ctx, Hkv, D, P, spare=3):
    pages_per = [(c + P - 1) // P for c in ctx]
    max_pages = max(pages_per) + 1
    num_pages = sum(pages_per) + spare
    perm = rng.permutation(num_pages).astype(np.int32)
    table = np.full((B, max_pages), -1, dtype=np.int32)
    k = 0
    for b in range(B):
        table[b, :pages_per[b]] = perm[k:k + pages_per[b]]
        k += pages_per[b]
    return table, num_pages


def test_append_lands_where_an_independent_gather_finds_it_and_touches_nothing_else():
    rng = np.random.default_rng(1)
    B, S, Hkv, D, P = 5, 4, 2, 8, 16
    ctx = np.array([4, 17, 32, 33, 70], dtype=np.int32)
    table, num_pages = _paged_setup(rng, B, ctx, Hkv, D, P)
    sentinel = np.float32(-777.0)
    kc = np.full((num_pages, Hkv, P, D), sentinel, dtype=np.float32)
    vc = np.full_like(kc, sentinel)
    kn = rng.standard_normal((B, S, Hkv, D)).astype(np.float32)
    vn = rng.standard_normal((B, S, Hkv, D)).astype(np.float32)
    oracle.kv_append(kn, vn, kc, vc, table, ctx, S, Hkv=Hkv, D=D, P=P)
    for b in range(B):
        for i in range(S):
            t = ctx[b] - S + i
            assert (kc[table[b, t // P], :, t % P, :] == kn[b, i]).all()
            assert (vc[table[b, t // P], :, t % P, :] == vn[b, i]).all()
    assert (kc != sentinel).sum() == B * S * Hkv * D and (vc != sentinel).sum() == B * S * Hkv * D


def test_append_into_a_token_major_pool_with_explicit_strides():
    rng = np.random.default_rng(2)
    B, S, Hkv, D, P = 3, 2, 3, 4, 16
    ctx = np.array([2, 16, 40], dtype=np.int32)
    table, num_pages = _paged_setup(rng, B, ctx, Hkv, D, P)
    kc = np.zeros((num_pages, P, Hkv, D), dtype=np.uint16)      # [page, slot, head, d]
    vc = np.zeros_like(kc)
    kn = rng.integers(1, 65535, size=(B, S, Hkv, D)).astype(np.uint16)
    vn = rng.integers(1, 65535, size=(B, S, Hkv, D)).astype(np.uint16)
    oracle.kv_append(kn, vn, kc, vc, table, ctx, S, Hkv=Hkv, D=D, P=P, strides=(P * Hkv * D, D, Hkv * D))
    for b in range(B):
        for i in range(S):
            t = ctx[b] - S + i
            assert (kc[table[b, t // P], t % P] == kn[b, i]).all() and (vc[table[b, t // P], t % P] == vn[b, i]).all()
    assert np.count_nonzero(kc) == B * S * Hkv * D


def test_cache_built_by_appends_gives_textbook_attention_on_the_contiguous_tensors():
    """Token-by-token appends through a shuffled block table, then the paged attention oracle,
    against softmax(QK^T/sqrt(D))V with a causal mask written with numpy on the un-paged K/V."""
    rng = np.random.default_rng(3)
    B, S, Hq, Hkv, D, P = 2, 3, 4, 2, 8, 16
    ctx = np.array([21, 37], dtype=np.int32)
    table, num_pages = _paged_setup(rng, B, ctx, Hkv, D, P)
    kc = np.full((num_pages, Hkv, P, D), np.nan, dtype=np.float32)
    vc = np.full_like(kc, np.nan)
    K = [rng.standard_normal((c, Hkv, D)).astype(np.float32) for c in ctx]
    V = [rng.standard_normal((c, Hkv, D)).astype(np.float32) for c in ctx]
    for t in range(int(ctx.max())):          # one position per call; shorter sequences repeat their last one
        cur = np.minimum(ctx, t + 1).astype(np.int32)
        kn = np.stack([K[b][cur[b] - 1] for b in range(B)])[:, None]
        vn = np.stack([V[b][cur[b] - 1] for b in range(B)])[:, None]
        oracle.kv_append(np.ascontiguousarray(kn), np.ascontiguousarray(vn), kc, vc, table, cur, 1, Hkv=Hkv, D=D, P=P)
    q = rng.standard_normal((B, S, Hq, D)).astype(np.float32)
    got = oracle.attention(q, kc, vc, table, ctx, S, Hq=Hq, Hkv=Hkv, D=D, P=P)
    G = Hq // Hkv
    for b in range(B):
        for i in range(S):
            n = ctx[b] - S + i + 1
            for h in range(Hq):
                s = (K[b][:n, h // G].astype(np.float64) @ q[b, i, h].astype(np.float64)) / np.sqrt(D)
                w = np.exp(s - s.max()); w /= w.sum()
                ref = w @ V[b][:n, h // G].astype(np.float64)
                assert np.allclose(got[b, i, h], ref, rtol=1e-12, atol=1e-12)


def test_append_refuses_broken_preconditions():
    kc = np.zeros((2, 1, 16, 4), dtype=np.float32); vc = np.zeros_like(kc)
    kn = np.zeros((1, 4, 1, 4), dtype=np.float32)
    with pytest.raises(ValueError):      # context shorter than the stride
        oracle.kv_append(kn, kn, kc, vc, np.array([[0, 1]], np.int32), np.array([3], np.int32), 4, Hkv=1, D=4, P=16)
    with pytest.raises(ValueError):      # page id outside the pool
        oracle.kv_append(kn, kn, kc, vc, np.array([[5, 1]], np.int32), np.array([8], np.int32), 4, Hkv=1, D=4, P=16)
    with pytest.raises(ValueError):      # position beyond the block-table row
        oracle.kv_append(kn, kn, kc, vc, np.array([[0, 1]], np.int32), np.array([40], np.int32), 4, Hkv=1, D=4, P=16)


# ---- trim-and-commit -------------------------------------------------------------------------

def make_state(B, S, ctx, n_draft, P=16, max_pages=64, cap=256, free=4096, first_free=1000):
    ctx = np.asarray(ctx, dtype=np.int32)
    pages_used = ((ctx + P - 1) // P).astype(np.int32)
    table = np.full((B, max_pages), -1, dtype=np.int32)
    nxt = 0
    for b in range(B):
        table[b, :pages_used[b]] = np.arange(nxt, nxt + pages_used[b])
        nxt += pages_used[b]
    return dict(n_draft=np.asarray(n_draft, dtype=np.int32).copy(), ctx_lens=ctx.copy(),
                stride_tokens=np.full((B, S), -9, np.int32), draft_tokens=np.full((B, max(S - 1, 1)), -9, np.int32)[:, :S - 1].copy(),
                out_tokens=np.full((B, cap), -9, np.int32), out_lens=np.zeros(B, np.int32), block_table=table,
                pages_used=pages_used, free_list=np.arange(first_free, first_free + free, dtype=np.int32),
                free_top=np.array([free], np.int32))


def test_commit_reproduces_the_worked_example():
    for line in open(GOLD):
        if not line.strip() or line.startswith("#"):
            continue
        case, S, D, r, n_final, kept, nd_next, pattern = line.split()
        S, D, r, n_final, kept, nd_next = map(int, (S, D, r, n_final, kept, nd_next))
        ctx0 = 50
        st = make_state(1, S, [ctx0], [D])
        # accepted drafts 100.., fresh token 200, discarded -1, proposals of the MASK rows 300..
        nt = np.array([[100 + j if j < r else 200 if j == r else -1 if j <= D else 300 + (j - D - 1) for j in range(S)]], np.int32)
        assert oracle.commit(st, [r], nt, n_draft_steady=3, mask_token=MASK, P=16) == 0
        assert st["out_lens"][0] == n_final, case
        assert list(st["out_tokens"][0, :n_final]) == [100 + j for j in range(r)] + [200]
        assert st["ctx_lens"][0] - S == ctx0 - S + kept        # slots of the old stride that stay
        assert st["n_draft"][0] == nd_next
        got = "".join("F" if t == 200 else "M" if t == MASK else "P" for t in st["stride_tokens"][0])
        assert got == pattern, case
        assert list(st["stride_tokens"][0, 1:1 + nd_next]) == [300 + k for k in range(nd_next)]
        assert list(st["draft_tokens"][0]) == [300 + k for k in range(nd_next)] + [-1] * (S - 1 - nd_next)


def tpf(N, p):
    return sum([2.0] + [p ** k for k in range(1, N - 1)]) / (2 - p ** (N - 1))


@pytest.mark.parametrize("N,p", [(2, 0.6), (3, 0.85), (4, 0.83), (5, 0.9)])
def test_loop_driven_by_commit_reaches_the_closed_form_tokens_per_forward(N, p):
    """accept -> commit -> accept ... with every draft accepted with probability p: tokens
    finalised per forward must follow Eq. 3, contexts must grow by exactly the tokens
    finalised, and every position must own a page nobody else owns."""
    S, B, V, P, steps = 2 * N - 1, 3000, 8, 16, 50
    rng = np.random.default_rng(11)
    st = make_state(B, S, np.full(B, S), np.zeros(B), cap=steps * N + 8, max_pages=(S + steps * N) // P + 2, free=B * 40,
                    first_free=1_000_000)
    total = 0
    for step in range(steps):
        drafts = np.where(st["draft_tokens"] >= 0, st["draft_tokens"] % V, 0).astype(np.int32)
        logits = np.full((B, S, V), np.log((1 - p) / (V - 1)), dtype=np.float32)
        bi, ji = np.meshgrid(np.arange(B), np.arange(S - 1), indexing="ij")
        logits[bi, ji, drafts] = np.log(p)
        r = oracle.accept(logits, drafts, 99, n_draft=st["n_draft"], rng_offset=step)
        before_ctx, before_out = st["ctx_lens"].copy(), st["out_lens"].copy()
        assert oracle.commit(st, r["accept_len"], r["new_tokens"], n_draft_steady=N - 1, mask_token=MASK, P=P) == 0
        fin = r["accept_len"] + 1
        total += int(fin.sum())
        assert (st["out_lens"] - before_out == fin).all() and (st["ctx_lens"] - before_ctx == fin).all()
    assert total / (B * steps) == pytest.approx(tpf(N, p), rel=0.02)
    assert (st["pages_used"] == (st["ctx_lens"] + P - 1) // P).all()
    owned = np.concatenate([st["block_table"][b, :st["pages_used"][b]] for b in range(B)])
    assert len(np.unique(owned)) == len(owned)
    new = owned[owned >= 1_000_000]
    assert st["free_top"][0] == B * 40 - len(new)
    assert set(new) == set(st["free_list"][st["free_top"][0]:B * 40])      # popped from the top, nothing else


def test_pages_are_popped_from_the_top_in_sequence_then_position_order():
    S, P = 4, 16
    st = make_state(3, S, [16, 30, 47], [0, 0, 0], P=P, free=10, first_free=500)
    nt = np.zeros((3, S), np.int32)
    assert oracle.commit(st, [0, 0, 0], nt, n_draft_steady=1, mask_token=MASK, P=P) == 0
    # contexts 17, 31, 48: sequence 0 needs page index 1, sequence 1 none, sequence 2 none
    assert list(st["ctx_lens"]) == [17, 31, 48] and list(st["pages_used"]) == [2, 2, 3]
    assert st["block_table"][0, 1] == 509 and st["free_top"][0] == 9
    assert oracle.commit(st, [0, 0, 0], nt, n_draft_steady=1, mask_token=MASK, P=P) == 0
    assert list(st["ctx_lens"]) == [18, 32, 49] and list(st["pages_used"]) == [2, 2, 4]
    assert st["block_table"][2, 3] == 508 and st["free_top"][0] == 8


def test_commit_changes_nothing_when_pages_or_table_rows_run_out():
    S, P = 4, 16
    st = make_state(2, S, [16, 16], [0, 0], P=P, free=1, max_pages=4)
    snap = {k: v.copy() for k, v in st.items()}
    nt = np.zeros((2, S), np.int32)
    assert oracle.commit(st, [0, 0], nt, n_draft_steady=1, mask_token=MASK, P=P) == 1     # two pages needed, one free
    assert all((st[k] == snap[k]).all() for k in st)
    st = make_state(1, S, [64], [0], P=P, free=8, max_pages=4)
    snap = {k: v.copy() for k, v in st.items()}
    assert oracle.commit(st, [0], nt[:1], n_draft_steady=1, mask_token=MASK, P=P) == 2       # row holds 4 pages = 64 positions
    assert all((st[k] == snap[k]).all() for k in st)
    with pytest.raises(ValueError):
        oracle.commit(make_state(1, S, [16], [1]), [2], nt[:1], n_draft_steady=1, mask_token=MASK, P=P)   # accept_len > n_draft


def test_next_drafts_are_the_arg_max_of_the_mask_rows():
    rng = np.random.default_rng(5)
    B, S, V, N = 64, 7, 50, 4
    logits = rng.standard_normal((B, S, V)).astype(np.float32) * 3
    n_draft = rng.integers(0, N, size=B).astype(np.int32)
    drafts = logits[:, :S - 1].argmax(-1).astype(np.int32)          # greedy + arg-max drafts: all accepted
    r = oracle.accept(logits, drafts, 1, n_draft=n_draft, greedy=np.ones(B, np.uint8))
    assert (r["accept_len"] == n_draft).all()
    st = make_state(B, S, np.full(B, 40), n_draft)
    assert oracle.commit(st, r["accept_len"], r["new_tokens"], n_draft_steady=N - 1, mask_token=MASK, P=16) == 0
    for b in range(B):
        D = n_draft[b]
        nd = min(N - 1, S - 1 - D)
        assert st["n_draft"][b] == nd
        assert st["stride_tokens"][b, 0] == logits[b, D].argmax()
        assert list(st["stride_tokens"][b, 1:1 + nd]) == [logits[b, D + 1 + k].argmax() for k in range(nd)]
        assert (st["stride_tokens"][b, 1 + nd:] == MASK).all()


@pytest.mark.parametrize("N,err", [(2, 0.5), (3, 0.3), (4, 0.0), (4, 1.0), (6, 0.4)])
def test_greedy_loop_emits_exactly_plain_greedy_autoregressive_decoding(N, err):
    """A toy model: the next-token logits after a clean token x peak at f(x).  MASK rows guess the
    continuation of the chain and are wrong with probability `err` (a wrong guess poisons the
    guesses after it, as in a real proposer).  Whatever N and err: same tokens as decoding one by
    one (acceptance only keeps drafts equal to the anchor's arg-max, Alg. 1 with T -> 0)."""
    S, B, V, steps = 2 * N - 1, 16, 97, 25
    rng = np.random.default_rng(100 + N)
    f = rng.permutation(V)
    first = rng.integers(0, V, size=B)
    st = make_state(B, S, np.full(B, S), np.zeros(B), cap=steps * N + 4, max_pages=(S + steps * N) // 16 + 2, free=B * 30)
    st["stride_tokens"][:] = MASK
    st["stride_tokens"][:, 0] = first
    for step in range(steps):
        logits = rng.standard_normal((B, S, V)).astype(np.float32)
        for b in range(B):
            chain = None
            for j in range(S):
                tok = st["stride_tokens"][b, j]
                if tok != MASK:
                    chain = f[tok]                                   # anchor: the true next token
                else:
                    chain = f[chain] if rng.random() >= err else (f[chain] + 1 + rng.integers(0, V - 1)) % V
                logits[b, j, chain] = 50.0
        drafts = np.where(st["draft_tokens"] >= 0, st["draft_tokens"], 0).astype(np.int32)
        r = oracle.accept(logits, drafts, 3, n_draft=st["n_draft"], greedy=np.ones(B, np.uint8), rng_offset=step)
        assert oracle.commit(st, r["accept_len"], r["new_tokens"], n_draft_steady=N - 1, mask_token=MASK, P=16) == 0
    for b in range(B):
        n = st["out_lens"][b]
        assert n >= steps
        ref, x = [], first[b]
        for _ in range(n):
            x = f[x]; ref.append(x)
        assert list(st["out_tokens"][b, :n]) == ref
    if err == 0.0 and N > 1:
        assert (st["out_lens"] == 1 + (steps - 1) * N).all()      # propose-only first step, then N per forward
    if err == 1.0:
        assert (st["out_lens"] <= steps).all()
