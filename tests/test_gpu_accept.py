"""GPU parity of idlm_isd_accept against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from isd_inputs import get_config, make_accept_inputs  # noqa: E402

DEV = "cuda"


def _helpers():
    import helpers
    return helpers


def _mk(name, **kw):
    seed = kw.pop("seed", None)
    return make_accept_inputs(get_config(name, **kw), device=DEV, seed=seed)


@pytest.mark.parametrize("nd", [0, 1, 2, 3])
def test_tiny_greedy(nd):
    h = _helpers()
    inp = _mk("tiny")
    # make about half of the drafts the arg-max so that both branches are taken
    am = inp.logits.argmax(-1)[:, :3].to(torch.int32)
    inp.draft_tokens[0] = am[0]
    got, ref = h.gpu_accept(inp, n_draft=nd), h.oracle_accept(inp, n_draft=nd)
    assert h.compare_accept(got, ref, nd) == 0


@pytest.mark.parametrize("mode", ["greedy", "stochastic"])
def test_small_model(mode):
    h = _helpers()
    inp = _mk("small", mode=mode, draft_hit=0.6 if mode == "greedy" else 0.8)
    got, ref = h.gpu_accept(inp), h.oracle_accept(inp)
    assert h.compare_accept(got, ref, inp.cfg.drafts) == 0
    assert 0 < ref["accept_len"].mean() < inp.cfg.drafts      # both outcomes occur


def test_8b_class_stochastic():
    h = _helpers()
    inp = _mk("8b")
    got, ref = h.gpu_accept(inp), h.oracle_accept(inp)
    assert h.compare_accept(got, ref, inp.cfg.drafts) == 0


def test_serving_config_full_size_mixed_modes():
    """B=256, S=16, V=151936 in the launch configuration the benchmark times; the oracle runs
    the whole batch.  Decisions within fp32 error of their threshold may go either way."""
    h = _helpers()
    inp = _mk("serve256")
    got, ref = h.gpu_accept(inp), h.oracle_accept(inp)
    undecided = h.compare_accept(got, ref, inp.cfg.drafts, strict=False)
    assert undecided <= 2
    assert (ref["accept_len"] < inp.cfg.drafts).any() and (ref["accept_len"] == inp.cfg.drafts).any()


@pytest.mark.parametrize("S", [1, 4, 8, 16, 32])
def test_long_context_config_rows(S):
    """The long-context workload's logits at its stated batch (B=32, V=151 936) for every stride of the sweep;
    the oracle runs the whole batch."""
    h = _helpers()
    inp = _mk("long32k", S=S)
    assert inp.logits.shape == (32, S, 151936)
    got, ref = h.gpu_accept(inp), h.oracle_accept(inp)
    assert h.compare_accept(got, ref, inp.cfg.drafts, strict=False) <= 1


def _custom(logits, drafts, n_draft, greedy, seed=11, rng_offset=0):
    from isd_inputs import AcceptInputs, get_config
    B, S, V = logits.shape
    dt = torch.zeros(B, max(S - 1, 1), dtype=torch.int32)
    if S > 1:
        dt[:, :S - 1] = torch.as_tensor(drafts, dtype=torch.int32)
    nd = torch.as_tensor(np.broadcast_to(np.asarray(n_draft, dtype=np.int32), (B,)).copy())
    gr = torch.as_tensor(np.broadcast_to(np.asarray(greedy, dtype=np.uint8), (B,)).copy())
    return AcceptInputs(get_config("tiny"), torch.as_tensor(logits, dtype=torch.float32).to(DEV), dt.to(DEV),
                        nd.to(DEV), gr.to(DEV), seed, rng_offset)


@pytest.mark.parametrize("V", [4, 8, 1028, 4100, 33000])
@pytest.mark.parametrize("S", [1, 2, 5])
def test_ragged_vocabulary_and_small_strides(V, S):
    h = _helpers()
    rng = np.random.default_rng(V * 10 + S)
    B = 7
    logits = (rng.standard_normal((B, S, V)) * 2).astype(np.float32)
    drafts = logits.argmax(-1)[:, :S - 1]
    flip = rng.random(drafts.shape) < 0.4
    drafts = np.where(flip, rng.integers(0, V, drafts.shape), drafts)
    nd = rng.integers(0, S, size=B)
    gr = rng.integers(0, 2, size=B)
    inp = _custom(logits, drafts, nd, gr, seed=1000 + V + S)
    got, ref = h.gpu_accept(inp), h.oracle_accept(inp)
    assert h.compare_accept(got, ref, nd, strict=False) <= 1


def test_ties_minus_infinity_and_point_masses():
    h = _helpers()
    B, S, V = 6, 4, 2048
    logits = np.zeros((B, S, V), dtype=np.float32)
    logits[0, 0, [100, 1500]] = 3.0           # tie: lowest index wins
    logits[0, 1, :] = -1.0                    # whole row tied -> index 0
    logits[1] = -np.inf
    logits[1, :, 77] = 0.0                    # point mass
    logits[2] = -np.inf
    logits[2, :, [5, 2000]] = 1.0             # two-point distribution
    logits[3, :, 1023] = 50.0
    logits[4, :, 1024] = 50.0
    logits[5, :, V - 1] = 50.0
    drafts = np.array([[1500, 0, 0], [77, 77, 77], [6, 5, 5], [1023, 1023, 1], [1024, 7, 1024], [V - 1, V - 1, V - 1]])
    for gr in (1, 0):
        inp = _custom(logits, drafts, 3, gr)
        got, ref = h.gpu_accept(inp), h.oracle_accept(inp)
        # hand-built rows: the only decision without a margin is the draw between the two equal atoms of sequence 2
        assert h.compare_accept(got, ref, 3, strict=False) <= 1
        if gr:
            assert got["accept_len"][0] == 0 and got["new_tokens"][0, 0] == 100
        assert got["accept_len"][1] == 3 and (got["new_tokens"][1] == 77).all()
        assert got["accept_len"][2] == 0 and got["new_tokens"][2, 0] in (5, 2000)


def test_rng_offset_seed_and_repeatability():
    h = _helpers()
    inp = _mk("small", B=8)
    a = h.gpu_accept(inp, rng_offset=0)
    b = h.gpu_accept(inp, rng_offset=0)
    c = h.gpu_accept(inp, rng_offset=5)
    assert np.array_equal(a["new_tokens"], b["new_tokens"]) and np.array_equal(a["accept_len"], b["accept_len"])
    assert np.array_equal(a["draft_probs"], b["draft_probs"])       # reductions are order-deterministic
    assert not np.array_equal(a["new_tokens"], c["new_tokens"])
    ref = h.oracle_accept(inp, rng_offset=5)
    assert h.compare_accept(c, ref, inp.cfg.drafts, strict=False) <= 1


def test_empty_batch_is_a_noop():
    import paper_2604_11035_amd as idlm
    logits = torch.empty(0, 4, 1024, device=DEV)
    al = torch.empty(0, dtype=torch.int32, device=DEV)
    nt = torch.empty(0, 4, dtype=torch.int32, device=DEV)
    idlm.idlm_isd_accept(logits, torch.empty(0, 3, dtype=torch.int32, device=DEV), 1, al, nt, n_draft=1)
    torch.cuda.synchronize()


@pytest.mark.parametrize("S,V,B", [(64, 1024, 5), (64, 50000, 3), (33, 151936, 4)])
def test_largest_strides(S, V, B):
    """S = 64 is the most rows a sequence may have (one lane of the chain's wavefront per row); every
    draft count from 0 to S-1 occurs, greedy and stochastic."""
    h = _helpers()
    rng = np.random.default_rng(S + V)
    logits = (rng.standard_normal((B, S, V)) * 2).astype(np.float32)
    drafts = logits.argmax(-1)[:, :S - 1]
    flip = rng.random(drafts.shape) < 0.05
    drafts = np.where(flip, rng.integers(0, V, drafts.shape), drafts)
    logits[np.arange(B)[:, None], np.arange(S - 1)[None, :], logits.argmax(-1)[:, :S - 1]] += 6.0   # confident rows: long accepted prefixes
    nd = np.array([S - 1, 0, S // 2, 1, S - 2][:B])
    gr = np.array([1, 0, 0, 1, 0][:B])
    inp = _custom(logits, drafts, nd, gr, seed=77)
    got, ref = h.gpu_accept(inp), h.oracle_accept(inp)
    assert h.compare_accept(got, ref, nd, strict=False) <= 1
    assert ref["accept_len"].max() >= 8
