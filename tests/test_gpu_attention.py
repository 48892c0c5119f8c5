"""GPU parity of idlm_isd_attention against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from isd_inputs import AttentionInputs, get_config, make_attention_inputs  # noqa: E402

DEV = "cuda"


def _helpers():
    import helpers
    return helpers


def _check(inp, num_workgroups=0, sel=None, scale=0.0, tol=None):
    h = _helpers()
    got = h.gpu_attention(inp, num_workgroups=num_workgroups, scale=scale)
    ref = h.oracle_attention(inp, sel=sel, scale=scale)
    rel, nvec = h.attention_errors(got, ref)
    tol = tol or (h.ATTN_REL_TOL if inp.q.dtype == torch.bfloat16 else h.ATTN_REL_TOL_F32)
    assert nvec > 0
    assert rel <= tol, "max relative error %g over %d vectors" % (rel, nvec)
    excess = h.attention_elementwise_excess(got, ref)
    print("max relative error %.3g over %d vectors; element-wise excess %.3g rms" % (rel, nvec, excess))
    # element by element: |err| <= 1e-2 |ref| + c rms(ref); c is set by the rounding of the softmax weights to the MFMA
    # operand type (2^-9 of a few dominant terms, relative to the vector's scale rather than the element's)
    assert excess <= (1.5e-2 if inp.q.dtype == torch.bfloat16 else 1e-4), excess
    if inp.q.dtype == torch.bfloat16 and inp.k_cache.is_contiguous() and inp.q.shape[-1] == 128:
        # The same K pool with its pages in operand order: other addresses, the same arithmetic.  Where the tile list is cut
        # at the same places in both layouts the bits are the same; with eight (or a multiple of eight) KV heads and up to
        # 64 rows per KV head the operand-order launch cuts its slices unequally (longer ones on even XCDs), sequences are
        # then split elsewhere, and the result is held to the oracle's tolerance like the first one.
        alt = h.gpu_attention(inp, num_workgroups=num_workgroups, scale=scale, k_operand_order=True)
        S_, Hq_, Hkv_ = inp.q.shape[1], inp.q.shape[2], inp.k_cache.shape[1]
        if Hkv_ % 8 != 0 or S_ * (Hq_ // Hkv_) > 64:
            assert np.array_equal(alt, got), "the operand-order K layout changed the result"
        else:
            rel_alt, _ = h.attention_errors(alt, ref)
            assert rel_alt <= tol, "operand-order K pages: max relative error %g" % rel_alt
            assert h.attention_elementwise_excess(alt, ref) <= 1.5e-2
    return got, ref


def test_tiny_fp32():
    inp = make_attention_inputs(get_config("tiny"), device=DEV, poison_unused=True)
    _check(inp)


@pytest.mark.parametrize("num_workgroups", [0, 1, 7, 64, 1024])
def test_small_model_bf16(num_workgroups):
    """Different grids cut the tile list at different places: items are whole, split in two,
    or spread over many workgroups (1024 workgroups: about one tile each)."""
    inp = make_attention_inputs(get_config("small"), device=DEV, poison_unused=True)
    _check(inp, num_workgroups=num_workgroups)


def test_8b_class_bf16():
    inp = make_attention_inputs(get_config("8b"), device=DEV, poison_unused=True)
    _check(inp)


def _sample_pairs(B, Hkv, n, seed):
    rng = np.random.default_rng(seed)
    sel = np.zeros((B, Hkv), dtype=np.uint8)
    flat = rng.choice(B * Hkv, size=n, replace=False)
    sel.reshape(-1)[flat] = 1
    return sel


def test_serving_config_full_size_every_pair():
    """B=256, S=16 with fragmented tables, default grid (what the benchmark times).  The slice boundaries of
    the persistent grid fall into sequences that depend on the context lengths, so the oracle computes every
    (sequence, KV head) pair: all 2048 of them, 131 072 output vectors."""
    cfg = get_config("serve256")
    inp = make_attention_inputs(cfg, device=DEV)
    got, ref = _check(inp)
    assert not np.isnan(ref).any() and ref.shape == (cfg.B, cfg.S, cfg.Hq, cfg.D)


def _one_pair_per_sequence(B, Hkv, shift):
    """Every sequence with one KV head each, every KV head used: (b, (3b + shift) mod Hkv)."""
    sel = np.zeros((B, Hkv), dtype=np.uint8)
    sel[np.arange(B), (3 * np.arange(B) + shift) % Hkv] = 1
    return sel


@pytest.mark.parametrize("S", [1, 4, 8, 16, 32])
def test_long_context_stride_sweep_small_batch(S):
    cfg = get_config("long32k", S=S, B=4)
    inp = make_attention_inputs(cfg, device=DEV)
    sel = _sample_pairs(cfg.B, cfg.Hkv, 2 if S >= 16 else 3, S)
    got, ref = _check(inp, sel=sel)
    if S == 1:
        # S = 1 is plain causal decode: one query at the last position sees every key
        assert (inp.ctx_lens == 32768).all()


@pytest.mark.parametrize("S", [1, 4, 8, 16, 32])
def test_long_context_full_batch(S):
    """The long-context workload at its stated size (B=32, 32 768 tokens each, 64 / 8 heads, 4.3 GB of K/V) in
    the launch configuration the benchmark's stride sweep times, for every stride of the sweep.  With 1024
    tiles per sequence and at least 32 slices per KV head every sequence is cut by slice boundaries, so the
    oracle computes one (sequence, KV head) pair of every sequence (32 pairs, every KV head among them).
    S = 1, 4, 8: one row group per KV head; S = 16: 128 rows share a head; S = 32: 256 rows."""
    cfg = get_config("long32k", S=S)
    assert cfg.B == 32 and cfg.Hq == 64 and cfg.Hkv == 8
    inp = make_attention_inputs(cfg, device=DEV)
    sel = _one_pair_per_sequence(cfg.B, cfg.Hkv, S)
    assert sel.sum() == 32 and sel.any(axis=0).all()
    _check(inp, sel=sel)


def _manual(B, S, Hq, Hkv, ctx, dtype=torch.bfloat16, D=128, seed=0, token_major=False, extra_pages=2):
    """Small hand-shaped inputs (ragged contexts, paddings) with NaN-poisoned unused slots."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    P = 16
    pages = [(c + P - 1) // P for c in ctx]
    num_pages = sum(pages) + extra_pages
    perm = torch.randperm(num_pages, generator=g)
    max_pages = max(pages) + 1
    table = torch.full((B, max_pages), -1, dtype=torch.int32)
    k = torch.full((num_pages, Hkv, P, D), float("nan"))
    v = torch.full((num_pages, Hkv, P, D), float("nan"))
    off = 0
    for b in range(B):
        for pi in range(pages[b]):
            pg = int(perm[off]); off += 1
            table[b, pi] = pg
            nvalid = min(P, ctx[b] - pi * P)
            k[pg, :, :nvalid] = torch.randn(Hkv, nvalid, D, generator=g)
            v[pg, :, :nvalid] = torch.randn(Hkv, nvalid, D, generator=g)
    q = torch.randn(B, S, Hq, D, generator=g)
    k, v, q = k.to(dtype).to(DEV), v.to(dtype).to(DEV), q.to(dtype).to(DEV)
    if token_major:
        k = k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)   # memory [pages,P,Hkv,D]
        v = v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    cfg = get_config("tiny")
    return AttentionInputs(cfg, q, k, v, table.to(DEV), torch.tensor(ctx, dtype=torch.int32, device=DEV),
                           num_pages, max_pages)


@pytest.mark.parametrize("S,Hq,Hkv", [(1, 8, 1), (1, 8, 8), (3, 8, 2), (5, 8, 2), (4, 4, 2), (8, 32, 8),
                                      (16, 16, 2), (32, 8, 1), (7, 6, 2), (32, 64, 8)])
def test_row_paddings_and_group_sizes(S, Hq, Hkv):
    ctx = [S, S + 1, 15 + S, 16 + S, 31 + S, 32 + S, 127 + S, 300]
    inp = _manual(len(ctx), S, Hq, Hkv, ctx, seed=S * 100 + Hq)
    for nwg in (0, 3):
        _check(inp, num_workgroups=nwg)


@pytest.mark.parametrize("S,G,Hkv", [(13, 5, 2), (12, 8, 3), (16, 8, 2), (26, 5, 1), (25, 8, 2), (32, 8, 3), (32, 4, 8)])
def test_more_than_64_rows_per_kv_head(S, G, Hkv):
    """S*G = 65 .. 256 query rows per KV head with 128-wide heads run on the kernel whose wavefronts share the K/V
    tiles of a workgroup through LDS: row counts that leave wavefronts partly or wholly without rows, one and two
    row groups per KV head, contexts around tile and page edges, grids smaller than the number of (KV head, row
    group) pairs (one workgroup walks several of them), grids of 16 and more (workgroup numbers are remapped in blocks
    of 16) and the largest grid (about one tile per workgroup); both pool layouts, and K pages in operand order."""
    ctx = [S, S + 1, 31 + S, 32 + S, 33 + S, 95 + S, 300, 1025, 64 + S]
    for token_major in (False, True):
        inp = _manual(len(ctx), S, Hkv * G, Hkv, ctx, seed=S * 10 + G, token_major=token_major)
        for nwg in ((0, 1, 2, 5, 16, 64, 1024) if not token_major else (0, 3, 48)):
            _check(inp, num_workgroups=nwg)


@pytest.mark.parametrize("ctx", [[128], [129], [256], [257], [255], [383, 384, 385], [1024, 1, 513]])
def test_tile_and_slice_boundaries(ctx):
    S = 1 if min(ctx) == 1 else 4
    inp = _manual(len(ctx), S, 8, 2, ctx, seed=sum(ctx))
    for nwg in (0, 1, 2, 5):
        _check(inp, num_workgroups=nwg)


def test_token_major_pool_and_explicit_scale():
    inp = _manual(3, 4, 8, 2, [40, 200, 333], seed=5, token_major=True)
    _check(inp, num_workgroups=4, scale=0.05)
    _check(inp, scale=0.2)


@pytest.mark.parametrize("S,Hq,Hkv,ctx", [(1, 8, 2, [5, 70]), (4, 4, 4, [16, 33, 4]), (7, 6, 2, [100]), (8, 32, 8, [300, 17, 1025]),
                                          (16, 16, 2, [64, 700]), (32, 64, 8, [96, 450])])
def test_bf16_head_dimension_64(S, Hq, Hkv, ctx):
    """bf16 with D = 64 runs on the same matrix-unit kernels as D = 128 (two contraction steps for the scores,
    four sixteen-row blocks of the output): every row tiling, whole and cut sequences, both pool layouts."""
    for token_major in (False, True):
        inp = _manual(len(ctx), S, Hq, Hkv, [c + S for c in ctx], D=64, seed=S, token_major=token_major)
        for nwg in (0, 1, 5, 64):
            _check(inp, num_workgroups=nwg)


def test_bf16_head_dimension_64_at_the_8b_shape():
    """The 8B-class step's shape with 64-wide heads (B=64, S=8, 32 / 8 heads, contexts 1024..4096), default grid."""
    inp = make_attention_inputs(get_config("8b", D=64), device=DEV, poison_unused=True)
    _check(inp)


@pytest.mark.parametrize("S,G,Hkv", [(8, 4, 8), (16, 8, 2)])
def test_wavefront_trace_accounts_for_every_tile(S, G, Hkv):
    """The debug trace of the main kernel (one record per wavefront: start, end, tiles, sequence parts): every 32-token tile
    of every KV head's list is worked on exactly once per group of query rows, whatever the partition (the streaming
    kernel with its slices of unequal length on even and odd XCDs, and the kernel whose four wavefronts share a tile), and
    switching the trace off leaves the records alone."""
    import paper_2604_11035_amd as idlm
    h = _helpers()
    ctx = [S + 5, 100, 333, 1025, 64 + S, 700, 31 + S, 2000]
    inp = _manual(len(ctx), S, Hkv * G, Hkv, ctx, seed=3)
    tiles_per_head = sum((c + 31) // 32 for c in ctx)
    shared = S * G > 64
    rec = torch.zeros(4096, 4, dtype=torch.int64, device=DEV)
    for nwg in (0, 16, 64):
        rec.zero_()
        idlm.idlm_isd_attention_wave_trace(rec)
        try:
            got = h.gpu_attention(inp, num_workgroups=nwg)
        finally:
            idlm.idlm_isd_attention_wave_trace(None)
        r = rec.cpu().numpy()
        act = r[:, 1] > 0
        assert act.any() and (r[act, 1] >= r[act, 0]).all()
        # streaming kernel (up to 64 rows per KV head): one wavefront per slice; shared-tile kernel: the four wavefronts
        # of a workgroup report the same tiles, one or two workgroup-level row groups per KV head
        expect = tiles_per_head * Hkv * ((4 * (1 if S * G <= 128 else 2)) if shared else 1)
        assert int(r[act, 2].sum()) == expect, (nwg, int(r[act, 2].sum()), expect)
        assert (r[act, 3] >= 1).all()
        before = r.copy()
        again = h.gpu_attention(inp, num_workgroups=nwg)      # tracing is off: the records stay as they are
        assert np.array_equal(rec.cpu().numpy(), before) and np.array_equal(again, got)


def test_shared_tile_kernel_replays_from_a_captured_graph():
    """The kernel for more than 64 rows per KV head allocates nothing and never synchronises either: captured in a HIP
    graph, every replay (with Q refreshed in place and eager work in between) gives the bits of the eager call."""
    import paper_2604_11035_amd as idlm
    h = _helpers()
    S, G, Hkv = 16, 8, 2
    ctx = [S + 3, 90, 400, 1025, 64 + S, 700]
    inp = _manual(len(ctx), S, Hkv * G, Hkv, ctx, seed=21)
    B, D, P = len(ctx), 128, 16
    ws = torch.empty(max(256, idlm.idlm_isd_attention_workspace(B, S, Hkv * G, Hkv, D, P, inp.block_table.shape[1], 1)),
                     dtype=torch.uint8, device=DEV)
    out = torch.zeros_like(inp.q)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        idlm.idlm_isd_attention(inp.q, inp.k_cache, inp.v_cache, inp.block_table, inp.ctx_lens, S, out, workspace=ws, stream=side)
    torch.cuda.synchronize()
    g = torch.Generator(device="cpu").manual_seed(5)
    for rep in range(3):
        inp.q.copy_(torch.randn(inp.q.shape, generator=g).to(torch.bfloat16))
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replayed = h.bf16_to_f64(out)
        eager = h.gpu_attention(inp)
        assert np.array_equal(replayed, eager), rep
        if rep == 0:
            rel, _ = h.attention_errors(eager, h.oracle_attention(inp))
            assert rel <= h.ATTN_REL_TOL
        _ = (torch.randn(1 << 16, device=DEV) * 2).sum().item()      # unrelated eager work between replays


def test_fp32_path_shapes():
    for D in (64, 128):
        inp = _manual(3, 4, 4, 2, [4, 37, 120], dtype=torch.float32, D=D, seed=D)
        _check(inp)


def test_large_scores_do_not_overflow():
    """Scores that grow along the context force the running reference exponent to be raised."""
    inp = _manual(2, 4, 8, 2, [600, 333], seed=9)
    ramp = torch.linspace(0.2, 6.0, 16, device=DEV).to(torch.bfloat16)
    inp.k_cache.mul_(ramp[None, None, :, None])          # later slots of every page score higher
    inp.q.mul_(4.0)
    _check(inp, num_workgroups=3)
    _check(inp)


def test_repeatable_and_empty_batch():
    import paper_2604_11035_amd as idlm
    h = _helpers()
    inp = make_attention_inputs(get_config("small"), device=DEV)
    a = h.gpu_attention(inp)
    b = h.gpu_attention(inp)
    assert np.array_equal(a, b)
    q = torch.empty(0, 4, 8, 128, dtype=torch.bfloat16, device=DEV)
    idlm.idlm_isd_attention(q, inp.k_cache, inp.v_cache, torch.empty(0, 4, dtype=torch.int32, device=DEV),
                            torch.empty(0, dtype=torch.int32, device=DEV), 4, torch.empty_like(q))
    torch.cuda.synchronize()


@pytest.mark.parametrize("case", range(24))
def test_random_shapes_grids_and_layouts(case):
    """Seeded random draws over batch size, stride, head grouping (also group sizes that are not
    powers of two), context lengths around tile and page boundaries, grid sizes and pool layout."""
    rng = np.random.default_rng(1000 + case)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 3, 4, 5, 8]))
    S = int(rng.integers(1, min(32, 256 // G) + 1))
    B = int(rng.integers(1, 24))
    hi = int(rng.choice([40, 200, 700]))
    ctx = [int(c) for c in rng.integers(S, S + hi, size=B)]
    for k in range(min(3, B)):                       # a few lengths right at tile / page edges
        ctx[k] = max(S, int(rng.choice([16, 17, 31, 32, 33, 63, 64, 65, 96, 128, 129])))
    inp = _manual(B, S, Hkv * G, Hkv, ctx, seed=5000 + case, token_major=bool(rng.integers(0, 2)),
                  D=128 if case % 3 else 64)
    for nwg in (0, int(rng.choice([1, 2, 3, 7, 17, 64, 300, 1024]))):
        _check(inp, num_workgroups=nwg)
