"""GPU parity of idlm_isd_accept_bf16 against the CPU oracle, through the C ABI.  The oracle is
the fp32-logits one, fed the bf16 values widened to fp32 (exact), so the bar is that of
idlm_isd_accept: integer outputs bit-exact wherever the oracle's decision margins exceed the
single-precision evaluation error, draft probabilities within 1e-5."""
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


def _custom(logits, drafts, n_draft, greedy, seed=11, rng_offset=0):
    from isd_inputs import AcceptInputs
    B, S, V = logits.shape
    dt = torch.zeros(B, max(S - 1, 1), dtype=torch.int32)
    if S > 1:
        dt[:, :S - 1] = torch.as_tensor(drafts, dtype=torch.int32)
    nd = torch.as_tensor(np.broadcast_to(np.asarray(n_draft, dtype=np.int32), (B,)).copy())
    gr = torch.as_tensor(np.broadcast_to(np.asarray(greedy, dtype=np.uint8), (B,)).copy())
    return AcceptInputs(get_config("tiny"), torch.as_tensor(logits, dtype=torch.float32).to(DEV), dt.to(DEV),
                        nd.to(DEV), gr.to(DEV), seed, rng_offset)


@pytest.mark.parametrize("mode", ["greedy", "stochastic"])
def test_small_model(mode):
    h = _helpers()
    inp = _mk("small", mode=mode, draft_hit=0.6 if mode == "greedy" else 0.8)
    got, ref = h.gpu_accept(inp, bf16=True), h.oracle_accept(inp, bf16=True)
    assert h.compare_accept(got, ref, inp.cfg.drafts, strict=False) <= 1
    assert 0 < ref["accept_len"].mean() < inp.cfg.drafts


def test_greedy_ties_of_rounded_rows_go_to_the_lowest_index():
    """bf16 keeps 8 significant bits, so the maximum of a 32K row is shared by several entries
    more often than not; the greedy decisions and proposals must still be bit-exact."""
    h = _helpers()
    rng = np.random.default_rng(5)
    B, S, V = 16, 6, 32768
    logits = (rng.standard_normal((B, S, V)) * 0.02 + 3.0).astype(np.float32)   # one binade, grid of 2^-6
    widened = torch.as_tensor(logits).to(torch.bfloat16).float().numpy()
    assert ((widened == widened.max(-1, keepdims=True)).sum(-1) > 1).mean() > 0.5
    drafts = widened.argmax(-1)[:, :S - 1]
    drafts[:, 1] = V - 1 - drafts[:, 1]
    inp = _custom(logits, drafts, S - 1, 1)
    got, ref = h.gpu_accept(inp, bf16=True), h.oracle_accept(inp, bf16=True)
    assert h.compare_accept(got, ref, S - 1) == 0
    assert (got["accept_len"] == 1).all()


def test_serving_config_full_size_mixed_modes():
    """B=256, S=16, V=151936, the benchmark's launch configuration; the oracle runs the batch."""
    h = _helpers()
    inp = _mk("serve256")
    got, ref = h.gpu_accept(inp, bf16=True), h.oracle_accept(inp, bf16=True)
    assert h.compare_accept(got, ref, inp.cfg.drafts, strict=False) <= 2
    assert (ref["accept_len"] < inp.cfg.drafts).any() and (ref["accept_len"] == inp.cfg.drafts).any()


@pytest.mark.parametrize("V", [8, 16, 1032, 4104, 33000])
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
    got, ref = h.gpu_accept(inp, bf16=True), h.oracle_accept(inp, bf16=True)
    assert h.compare_accept(got, ref, nd, strict=False) <= 1


def test_minus_infinity_and_point_masses():
    h = _helpers()
    B, S, V = 4, 4, 2048
    logits = np.zeros((B, S, V), dtype=np.float32)
    logits[0, 0, [100, 1500]] = 3.0
    logits[1] = -np.inf
    logits[1, :, 77] = 0.0
    logits[2] = -np.inf
    logits[2, :, [5, 2000]] = 1.0
    logits[3, :, V - 1] = 50.0
    drafts = np.array([[1500, 0, 0], [77, 77, 77], [6, 5, 5], [V - 1, V - 1, V - 1]])
    for gr in (1, 0):
        inp = _custom(logits, drafts, 3, gr)
        got, ref = h.gpu_accept(inp, bf16=True), h.oracle_accept(inp, bf16=True)
        assert h.compare_accept(got, ref, 3, strict=False) <= 1
        assert got["accept_len"][1] == 3 and (got["new_tokens"][1] == 77).all()
        assert got["accept_len"][2] == 0 and got["new_tokens"][2, 0] in (5, 2000)
        assert got["accept_len"][3] == 3


def test_matches_the_fp32_entry_point_on_the_widened_values():
    """Bit-identical integer outputs AND probabilities: after the load the arithmetic is the same."""
    h = _helpers()
    inp = _mk("small", B=16)
    a = h.gpu_accept(inp, bf16=True)
    inp.logits.copy_(h.as_bf16(inp.logits).float())
    b = h.gpu_accept(inp)
    assert np.array_equal(a["accept_len"], b["accept_len"]) and np.array_equal(a["new_tokens"], b["new_tokens"])
    np.testing.assert_allclose(a["draft_probs"], b["draft_probs"], rtol=0, atol=1e-6)


def test_vocabulary_must_be_a_multiple_of_eight():
    import paper_2604_11035_amd as idlm
    B, S, V = 2, 3, 1028
    logits = torch.zeros(B, S, V, dtype=torch.bfloat16, device=DEV)
    al = torch.empty(B, dtype=torch.int32, device=DEV)
    nt = torch.empty(B, S, dtype=torch.int32, device=DEV)
    ws = torch.empty(1 << 16, dtype=torch.uint8, device=DEV)
    with pytest.raises(idlm.IdlmError):
        idlm.idlm_isd_accept_bf16(logits, torch.zeros(B, S - 1, dtype=torch.int32, device=DEV), 1, al, nt,
                                  n_draft=1, workspace=ws)
