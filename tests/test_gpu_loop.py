"""GPU parity of the between-steps entry points (KV append, trim-and-commit / next stride) and of
the whole loop append -> attention -> accept -> commit over several steps, through the C ABI,
against the CPU oracle on the same seeded inputs.  Integer and byte work: bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_11035_amd as idlm
from helpers import ATTN_REL_TOL, attention_errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MASK = 7_000_000


def _tables(rng, ctx, P, spare=5, extra_cols=2):
    B = len(ctx)
    pages_per = (np.asarray(ctx) + P - 1) // P
    max_pages = int(pages_per.max()) + extra_cols
    num_pages = int(pages_per.sum()) + spare
    perm = rng.permutation(num_pages).astype(np.int32)
    table = np.full((B, max_pages), -1, dtype=np.int32)
    k = 0
    for b in range(B):
        table[b, :pages_per[b]] = perm[k:k + pages_per[b]]
        k += pages_per[b]
    return table, num_pages


@pytest.mark.parametrize("dtype,B,S,Hkv,D", [("f32", 3, 4, 2, 64), ("bf16", 16, 8, 4, 128), ("bf16", 64, 16, 8, 128),
                                             ("bf16", 5, 1, 8, 128), ("bf16", 7, 32, 1, 128)])
def test_kv_append_matches_the_oracle_bit_for_bit(dtype, B, S, Hkv, D):
    rng = np.random.default_rng(B * 100 + S)
    P = 16
    ctx = rng.integers(S, 400, size=B).astype(np.int32)
    ctx[0] = S                       # a stride that starts the sequence
    ctx[-1] = 16 * 7 + 3             # a stride that crosses a page boundary (for S > 3)
    ctx = np.maximum(ctx, S).astype(np.int32)
    table, num_pages = _tables(rng, ctx, P)
    npdt = np.float32 if dtype == "f32" else np.uint16
    if dtype == "f32":
        kc = rng.standard_normal((num_pages, Hkv, P, D)).astype(np.float32)
        vc = rng.standard_normal((num_pages, Hkv, P, D)).astype(np.float32)
        kn = rng.standard_normal((B, S, Hkv, D)).astype(np.float32)
        vn = rng.standard_normal((B, S, Hkv, D)).astype(np.float32)
        tt = torch.float32
    else:
        kc, vc = (rng.integers(0, 65536, size=(num_pages, Hkv, P, D)).astype(np.uint16) for _ in range(2))
        kn, vn = (rng.integers(0, 65536, size=(B, S, Hkv, D)).astype(np.uint16) for _ in range(2))
        tt = torch.bfloat16
    to_dev = lambda a: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(DEV).view(tt)
    g_kc, g_vc, g_kn, g_vn = map(to_dev, (kc, vc, kn, vn))
    idlm.idlm_isd_kv_append(g_kn, g_vn, g_kc, g_vc, torch.from_numpy(table).to(DEV), torch.from_numpy(ctx).to(DEV), S)
    torch.cuda.synchronize()
    oracle.kv_append(kn, vn, kc, vc, table, ctx, S, Hkv=Hkv, D=D, P=P)
    back = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16) if tt == torch.bfloat16 else t.cpu().numpy()
    assert np.array_equal(back(g_kc).view(np.uint32 if dtype == "f32" else np.uint16), kc.view(np.uint32 if dtype == "f32" else np.uint16))
    assert np.array_equal(back(g_vc).view(np.uint32 if dtype == "f32" else np.uint16), vc.view(np.uint32 if dtype == "f32" else np.uint16))


def test_kv_append_writes_k_pages_in_operand_order():
    """The K pool laid out for the attention kernel's operands: what the kernel writes equals the oracle's
    row-major pool put through the permutation; V is untouched by the option."""
    from isd_inputs import k_pages_in_operand_order
    B, S, Hkv, D, P = 9, 5, 4, 128, 16
    rng = np.random.default_rng(3)
    ctx = (rng.integers(1, 70, size=B) + S).astype(np.int32)
    max_pages = int((ctx.max() + P - 1) // P)
    pages = (ctx + P - 1) // P
    num_pages = int(pages.sum()) + 3
    perm = rng.permutation(num_pages).astype(np.int32)
    table = np.full((B, max_pages), -1, np.int32)
    k = 0
    for b in range(B):
        table[b, :pages[b]] = perm[k:k + pages[b]]; k += pages[b]
    kc = torch.randn(num_pages, Hkv, P, D, device=DEV).to(torch.bfloat16)
    vc = torch.randn(num_pages, Hkv, P, D, device=DEV).to(torch.bfloat16)
    kn = torch.randn(B, S, Hkv, D, device=DEV).to(torch.bfloat16)
    vn = torch.randn(B, S, Hkv, D, device=DEV).to(torch.bfloat16)
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    o_k, o_v = bits(kc).copy(), bits(vc).copy()
    oracle.kv_append(bits(kn), bits(vn), o_k, o_v, table, ctx, S, Hkv=Hkv, D=D, P=P)
    g_k = k_pages_in_operand_order(kc)           # the pool as the option keeps it
    g_v = vc.clone()
    idlm.idlm_isd_kv_append(kn, vn, g_k, g_v, torch.from_numpy(table).to(DEV), torch.from_numpy(ctx).to(DEV), S,
                            k_operand_order=True)
    torch.cuda.synchronize()
    want_k = k_pages_in_operand_order(torch.from_numpy(o_k.view(np.int16)).view(torch.bfloat16).view(num_pages, Hkv, P, D).to(DEV))
    assert torch.equal(g_k.view(torch.int16), want_k.view(torch.int16))
    assert np.array_equal(bits(g_v), o_v)


def test_kv_append_into_a_token_major_pool():
    rng = np.random.default_rng(9)
    B, S, Hkv, D, P = 6, 8, 4, 128, 16
    ctx = rng.integers(S, 200, size=B).astype(np.int32)
    table, num_pages = _tables(rng, ctx, P)
    base_k = rng.integers(0, 65536, size=(num_pages, P, Hkv, D)).astype(np.uint16)     # [page, slot, head, d]
    base_v = rng.integers(0, 65536, size=(num_pages, P, Hkv, D)).astype(np.uint16)
    kn, vn = (rng.integers(0, 65536, size=(B, S, Hkv, D)).astype(np.uint16) for _ in range(2))
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    gk, gv = to_dev(base_k), to_dev(base_v)
    idlm.idlm_isd_kv_append(to_dev(kn), to_dev(vn), gk.permute(0, 2, 1, 3), gv.permute(0, 2, 1, 3),
                            torch.from_numpy(table).to(DEV), torch.from_numpy(ctx).to(DEV), S)
    torch.cuda.synchronize()
    oracle.kv_append(kn, vn, base_k, base_v, table, ctx, S, Hkv=Hkv, D=D, P=P, strides=(P * Hkv * D, D, Hkv * D))
    assert np.array_equal(gk.view(torch.int16).cpu().numpy().view(np.uint16), base_k)
    assert np.array_equal(gv.view(torch.int16).cpu().numpy().view(np.uint16), base_v)


def test_kv_append_skips_rows_it_cannot_place():
    """Positions before the sequence start, beyond the table row, or with a page id outside the
    pool are not written (the oracle refuses such input; here only the placeable rows must land)."""
    B, S, Hkv, D, P = 3, 4, 2, 128, 16
    num_pages = 6
    table = np.array([[0, 1, -1], [2, 99, -1], [3, 4, 5]], dtype=np.int32)
    ctx = np.array([2, 20, 52], dtype=np.int32)        # b0: rows 0,1 negative; b1: rows at 16.. hit page 99; b2: rows 48..51 beyond row (3 pages = 48)
    kc = torch.zeros(num_pages, Hkv, P, D, dtype=torch.bfloat16, device=DEV)
    vc = torch.zeros_like(kc)
    kn = torch.ones(B, S, Hkv, D, dtype=torch.bfloat16, device=DEV)
    idlm.idlm_isd_kv_append(kn, kn, kc, vc, torch.from_numpy(table).to(DEV), torch.from_numpy(ctx).to(DEV), S)
    torch.cuda.synchronize()
    written = (kc != 0).any(-1).any(1).cpu().numpy()      # [page, slot]
    expect = np.zeros((num_pages, P), bool)
    expect[0, 0:2] = True          # b0 rows 2,3 -> positions 0,1
    assert np.array_equal(written, expect) and np.array_equal((vc != 0).any(-1).any(1).cpu().numpy(), expect)


# ---- commit ----------------------------------------------------------------------------------

def random_state(rng, B, S, P, max_pages, cap, free, n_steady):
    ctx = rng.integers(S, (max_pages - 2) * P, size=B).astype(np.int32)
    pages_used = ((ctx + P - 1) // P).astype(np.int32)
    table = np.full((B, max_pages), -1, dtype=np.int32)
    nxt = 0
    for b in range(B):
        table[b, :pages_used[b]] = np.arange(nxt, nxt + pages_used[b]); nxt += pages_used[b]
    n_draft = rng.integers(0, min(n_steady, S - 1) + 1, size=B).astype(np.int32)
    st = dict(n_draft=n_draft, ctx_lens=ctx, stride_tokens=np.full((B, S), -9, np.int32),
              draft_tokens=np.full((B, S - 1), -9, np.int32), out_tokens=np.full((B, cap), -9, np.int32),
              out_lens=rng.integers(0, cap + 1, size=B).astype(np.int32), block_table=table, pages_used=pages_used,
              free_list=(10_000_000 + rng.permutation(free)).astype(np.int32), free_top=np.array([free], np.int32))
    accept_len = (rng.random(B) * (n_draft + 1)).astype(np.int32)
    accept_len = np.where(rng.random(B) < 0.5, n_draft, accept_len).astype(np.int32)
    new_tokens = rng.integers(0, 150000, size=(B, S)).astype(np.int32)
    return st, accept_len, new_tokens


def to_gpu(st):
    g = {k: torch.from_numpy(v.copy()).to(DEV) for k, v in st.items()}
    g["status"] = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    return g


def assert_same(g, st):
    for k, v in st.items():
        assert np.array_equal(g[k].cpu().numpy(), v), k


@pytest.mark.parametrize("B,S,n_steady", [(1, 1, 0), (37, 7, 3), (256, 16, 7), (1024, 8, 3), (2500, 5, 2), (65535, 3, 1)])
def test_commit_matches_the_oracle_bit_for_bit(B, S, n_steady):
    rng = np.random.default_rng(B + S)
    P = 16
    st, r, nt = random_state(rng, B, S, P, max_pages=12, cap=9, free=B + 50, n_steady=n_steady)
    g = to_gpu(st)
    idlm.idlm_isd_commit(torch.from_numpy(r).to(DEV), torch.from_numpy(nt).to(DEV), g, n_draft_steady=n_steady,
                         mask_token=MASK, P=P)
    torch.cuda.synchronize()
    assert oracle.commit(st, r, nt, n_draft_steady=n_steady, mask_token=MASK, P=P) == 0
    assert int(g["status"].item()) == 0
    assert_same(g, st)


def test_commit_refusals_change_nothing():
    rng = np.random.default_rng(77)
    P, S, B = 16, 6, 300
    # 1: free list too short
    st, r, nt = random_state(rng, B, S, P, max_pages=12, cap=9, free=B + 50, n_steady=2)
    st["ctx_lens"][:] = 32; st["pages_used"][:] = 2; st["free_top"][0] = 10      # every sequence needs a page
    g = to_gpu(st); snap = {k: v.copy() for k, v in st.items()}
    idlm.idlm_isd_commit(torch.from_numpy(r).to(DEV), torch.from_numpy(nt).to(DEV), g, n_draft_steady=2, mask_token=MASK, P=P)
    torch.cuda.synchronize()
    assert oracle.commit(st, r, nt, n_draft_steady=2, mask_token=MASK, P=P) == 1 and int(g["status"].item()) == 1
    assert_same(g, snap); assert_same(g, st)
    # 2: a table row too short
    st, r, nt = random_state(rng, B, S, P, max_pages=12, cap=9, free=B + 50, n_steady=2)
    st["ctx_lens"][123] = 12 * P; st["pages_used"][123] = 12
    g = to_gpu(st); snap = {k: v.copy() for k, v in st.items()}
    idlm.idlm_isd_commit(torch.from_numpy(r).to(DEV), torch.from_numpy(nt).to(DEV), g, n_draft_steady=2, mask_token=MASK, P=P)
    torch.cuda.synchronize()
    assert oracle.commit(st, r, nt, n_draft_steady=2, mask_token=MASK, P=P) == 2 and int(g["status"].item()) == 2
    assert_same(g, snap)
    # 3: accept_len beyond n_draft (the oracle raises)
    st, r, nt = random_state(rng, B, S, P, max_pages=12, cap=9, free=B + 50, n_steady=2)
    r[7] = st["n_draft"][7] + 1
    g = to_gpu(st); snap = {k: v.copy() for k, v in st.items()}
    idlm.idlm_isd_commit(torch.from_numpy(r).to(DEV), torch.from_numpy(nt).to(DEV), g, n_draft_steady=2, mask_token=MASK, P=P)
    torch.cuda.synchronize()
    with pytest.raises(ValueError):
        oracle.commit(st, r, nt, n_draft_steady=2, mask_token=MASK, P=P)
    assert int(g["status"].item()) == 3
    assert_same(g, snap)


# ---- the whole loop --------------------------------------------------------------------------

@pytest.mark.parametrize("N,greedy,kop", [(3, False, False), (4, True, False), (3, True, True)])
def test_several_steps_of_the_whole_loop(N, greedy, kop):
    """append -> attention -> accept -> commit, eight steps, state compared after every call.
    There is no model here: K/V rows and Q are seeded noise, logits are seeded noise with a planted
    peak on every draft (so that some drafts pass and some do not).  kop: the K pool lives in the
    attention kernel's operand order from the start (the oracle's pool stays slot-major; the two
    are compared through the permutation)."""
    from isd_inputs import k_pages_in_operand_order
    rng = np.random.default_rng(40 + N)
    B, S, Hq, Hkv, D, P, V = 24, 2 * N - 1, 16, 4, 128, 16, 4096
    steps, max_pages = 8, 16
    prompt = rng.integers(20, 150, size=B).astype(np.int32)
    ctx0 = (prompt + S).astype(np.int32)               # the first stride is already appended to the lengths
    num_pages = int(((ctx0 + P - 1) // P).sum()) + B * 4 + 8
    perm = rng.permutation(num_pages).astype(np.int32)
    pages_used = ((ctx0 + P - 1) // P).astype(np.int32)
    table = np.full((B, max_pages), -1, np.int32)
    k = 0
    for b in range(B):
        table[b, :pages_used[b]] = perm[k:k + pages_used[b]]; k += pages_used[b]
    free = perm[k:].copy()
    st = dict(n_draft=np.zeros(B, np.int32), ctx_lens=ctx0.copy(), stride_tokens=np.full((B, S), MASK, np.int32),
              draft_tokens=np.full((B, S - 1), -1, np.int32), out_tokens=np.full((B, 64), -9, np.int32),
              out_lens=np.zeros(B, np.int32), block_table=table, pages_used=pages_used, free_list=free,
              free_top=np.array([len(free)], np.int32))
    st["stride_tokens"][:, 0] = rng.integers(0, V, size=B)
    g = to_gpu(st)
    bf = lambda a: torch.from_numpy(a).to(DEV).to(torch.bfloat16)
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    kc = bf(rng.standard_normal((num_pages, Hkv, P, D)).astype(np.float32))    # prompts' K/V: anything
    vc = bf(rng.standard_normal((num_pages, Hkv, P, D)).astype(np.float32))
    o_kc, o_vc = bits(kc).copy(), bits(vc).copy()
    if kop:
        kc = k_pages_in_operand_order(kc)
    as_stored = lambda o: bits(k_pages_in_operand_order(torch.from_numpy(o.view(np.int16)).view(torch.bfloat16).to(DEV))) if kop else o
    gflag = np.full(B, 1 if greedy else 0, np.uint8)
    ws_a = torch.empty(max(256, idlm.idlm_isd_attention_workspace(B, S, Hq, Hkv, D, P, max_pages, 1)), dtype=torch.uint8, device=DEV)
    ws_c = torch.empty(max(256, idlm.idlm_isd_accept_workspace(B, S, V)), dtype=torch.uint8, device=DEV)
    finalised = 0
    for step in range(steps):
        kn, vn, q = (bf(rng.standard_normal(shape).astype(np.float32)) for shape in ((B, S, Hkv, D), (B, S, Hkv, D), (B, S, Hq, D)))
        idlm.idlm_isd_kv_append(kn, vn, kc, vc, g["block_table"], g["ctx_lens"], S, k_operand_order=kop)
        oracle.kv_append(bits(kn), bits(vn), o_kc, o_vc, st["block_table"], st["ctx_lens"], S, Hkv=Hkv, D=D, P=P)
        out = torch.empty_like(q)
        idlm.idlm_isd_attention(q, kc, vc, g["block_table"], g["ctx_lens"], S, out, workspace=ws_a, k_operand_order=kop)
        torch.cuda.synchronize()
        assert np.array_equal(bits(kc), as_stored(o_kc)) and np.array_equal(bits(vc), o_vc)
        ref = oracle.attention(bits(q), o_kc, o_vc, st["block_table"], st["ctx_lens"], S, Hq=Hq, Hkv=Hkv, D=D, P=P)
        err, _ = attention_errors(out.float().cpu().numpy().astype(np.float64), ref)
        assert err <= ATTN_REL_TOL
        drafts = np.where(st["draft_tokens"] >= 0, st["draft_tokens"], 0).astype(np.int32)
        logits = (rng.standard_normal((B, S, V)) * 2).astype(np.float32)
        bi, ji = np.meshgrid(np.arange(B), np.arange(S - 1), indexing="ij")
        logits[bi, ji, drafts] += rng.choice([0.0, 12.0], size=(B, S - 1), p=[0.3, 0.7]).astype(np.float32)
        r = oracle.accept(logits, drafts, 555, n_draft=st["n_draft"], greedy=gflag, rng_offset=step)
        assert (np.abs(r["accept_margin"][ji < st["n_draft"][:, None]]) > 1e-5).all() or greedy
        accept_len = torch.empty(B, dtype=torch.int32, device=DEV)
        new_tokens = torch.empty(B, S, dtype=torch.int32, device=DEV)
        idlm.idlm_isd_accept(torch.from_numpy(logits).to(DEV), g["draft_tokens"].clamp(min=0), 555, accept_len, new_tokens,
                             n_draft=g["n_draft"], greedy=torch.from_numpy(gflag).to(DEV), rng_offset=step, workspace=ws_c)
        torch.cuda.synchronize()
        assert np.array_equal(accept_len.cpu().numpy(), r["accept_len"])
        assert np.array_equal(new_tokens.cpu().numpy(), r["new_tokens"])
        idlm.idlm_isd_commit(accept_len, new_tokens, g, n_draft_steady=N - 1, mask_token=MASK, P=P)
        torch.cuda.synchronize()
        assert oracle.commit(st, r["accept_len"], r["new_tokens"], n_draft_steady=N - 1, mask_token=MASK, P=P) == 0
        assert int(g["status"].item()) == 0
        assert_same(g, st)
        finalised += int((r["accept_len"] + 1).sum())
    assert (st["out_lens"] >= steps).all() and st["out_lens"].sum() == finalised
    assert finalised > B * steps                      # some drafts were accepted


def test_the_loop_replays_from_a_captured_graph():
    """The four calls of a step allocate nothing and never synchronise, so a caller can capture
    them in a HIP graph and replay it step after step with the inputs refreshed in place (the
    deployment the paper describes in Sec. 3.3 (1)).  Every replay is checked against the oracle,
    with eager work and synchronisations in between."""
    N, steps = 3, 5
    rng = np.random.default_rng(123)
    B, S, Hq, Hkv, D, P, V = 12, 2 * N - 1, 8, 2, 128, 16, 2048
    max_pages = 12
    ctx0 = (rng.integers(20, 90, size=B) + S).astype(np.int32)
    pages_used = ((ctx0 + P - 1) // P).astype(np.int32)
    num_pages = int(pages_used.sum()) + B * 3 + 4
    perm = rng.permutation(num_pages).astype(np.int32)
    table = np.full((B, max_pages), -1, np.int32)
    k = 0
    for b in range(B):
        table[b, :pages_used[b]] = perm[k:k + pages_used[b]]; k += pages_used[b]
    free = perm[k:].copy()
    st = dict(n_draft=np.zeros(B, np.int32), ctx_lens=ctx0.copy(), stride_tokens=np.full((B, S), MASK, np.int32),
              draft_tokens=np.full((B, S - 1), -1, np.int32), out_tokens=np.full((B, 40), -9, np.int32),
              out_lens=np.zeros(B, np.int32), block_table=table, pages_used=pages_used, free_list=free,
              free_top=np.array([len(free)], np.int32))
    g = to_gpu(st)
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    kc = torch.randn(num_pages, Hkv, P, D, device=DEV).to(torch.bfloat16)
    vc = torch.randn(num_pages, Hkv, P, D, device=DEV).to(torch.bfloat16)
    o_kc, o_vc = bits(kc).copy(), bits(vc).copy()
    # static buffers the graph reads and writes
    kn = torch.zeros(B, S, Hkv, D, dtype=torch.bfloat16, device=DEV); vn = torch.zeros_like(kn)
    q = torch.zeros(B, S, Hq, D, dtype=torch.bfloat16, device=DEV); out = torch.zeros_like(q)
    logits = torch.zeros(B, S, V, dtype=torch.float32, device=DEV)
    drafts_in = torch.zeros(B, S - 1, dtype=torch.int32, device=DEV)
    accept_len = torch.zeros(B, dtype=torch.int32, device=DEV); new_tokens = torch.zeros(B, S, dtype=torch.int32, device=DEV)
    greedy = torch.ones(B, dtype=torch.uint8, device=DEV)
    ws_a = torch.empty(max(256, idlm.idlm_isd_attention_workspace(B, S, Hq, Hkv, D, P, max_pages, 1)), dtype=torch.uint8, device=DEV)
    ws_c = torch.empty(max(256, idlm.idlm_isd_accept_workspace(B, S, V)), dtype=torch.uint8, device=DEV)

    def step_calls(stream):
        idlm.idlm_isd_kv_append(kn, vn, kc, vc, g["block_table"], g["ctx_lens"], S, stream=stream)
        idlm.idlm_isd_attention(q, kc, vc, g["block_table"], g["ctx_lens"], S, out, workspace=ws_a, stream=stream)
        idlm.idlm_isd_accept(logits, drafts_in, 777, accept_len, new_tokens, n_draft=g["n_draft"], greedy=greedy,
                             rng_offset=0, workspace=ws_c, stream=stream)
        idlm.idlm_isd_commit(accept_len, new_tokens, g, n_draft_steady=N - 1, mask_token=MASK, P=P, stream=stream)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    snapshot = {k_: v.clone() for k_, v in g.items()}
    kc_snap, vc_snap = kc.clone(), vc.clone()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        step_calls(side)
    torch.cuda.synchronize()
    for k_, v in snapshot.items():      # capture does not run anything, but start from a known state anyway
        g[k_].copy_(v)
    kc.copy_(kc_snap); vc.copy_(vc_snap)
    for step in range(steps):
        h_kn, h_vn, h_q = (rng.standard_normal(sh).astype(np.float32) for sh in ((B, S, Hkv, D), (B, S, Hkv, D), (B, S, Hq, D)))
        kn.copy_(torch.from_numpy(h_kn)); vn.copy_(torch.from_numpy(h_vn)); q.copy_(torch.from_numpy(h_q))
        h_drafts = np.where(st["draft_tokens"] >= 0, st["draft_tokens"], 0).astype(np.int32)
        h_logits = (rng.standard_normal((B, S, V)) * 2).astype(np.float32)
        bi, ji = np.meshgrid(np.arange(B), np.arange(S - 1), indexing="ij")
        h_logits[bi, ji, h_drafts] += rng.choice([0.0, 14.0], size=(B, S - 1), p=[0.3, 0.7]).astype(np.float32)
        logits.copy_(torch.from_numpy(h_logits)); drafts_in.copy_(torch.from_numpy(h_drafts))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        oracle.kv_append(bits(kn), bits(vn), o_kc, o_vc, st["block_table"], st["ctx_lens"], S, Hkv=Hkv, D=D, P=P)
        assert np.array_equal(bits(kc), o_kc) and np.array_equal(bits(vc), o_vc), step
        ref = oracle.attention(bits(q), o_kc, o_vc, st["block_table"], st["ctx_lens"], S, Hq=Hq, Hkv=Hkv, D=D, P=P)
        err, _ = attention_errors(out.float().cpu().numpy().astype(np.float64), ref)
        assert err <= ATTN_REL_TOL, step
        r = oracle.accept(h_logits, h_drafts, 777, n_draft=st["n_draft"], greedy=np.ones(B, np.uint8), rng_offset=0)
        assert np.array_equal(accept_len.cpu().numpy(), r["accept_len"]), step
        assert np.array_equal(new_tokens.cpu().numpy(), r["new_tokens"]), step
        assert oracle.commit(st, r["accept_len"], r["new_tokens"], n_draft_steady=N - 1, mask_token=MASK, P=P) == 0
        assert int(g["status"].item()) == 0
        assert_same(g, st)
        _ = (torch.randn(1 << 16, device=DEV) * 2).sum().item()      # unrelated eager work between replays
