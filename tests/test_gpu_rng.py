"""The HIP path's counter-based generator against the oracle's, number by number (two implementations written
separately from the same specification): a million uniforms bit for bit, and the Gumbel noise within
single-precision evaluation error."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_11035_amd as idlm

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("seed,offset,tag,row0,n_rows,V", [
    (20260411, 0, 1, 0, 8, 131072),                       # 2^20 numbers of the fresh-token stream
    (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFF, 2, 2**31 - 9, 8, 1031),   # all-ones key and offset, the largest rows, ragged V
    (0x0123456789ABCDEF, 7, 0, 4095, 3, 5),               # accept-test stream
])
def test_uniforms_are_bit_identical_and_noise_agrees(seed, offset, tag, row0, n_rows, V):
    u = torch.full((n_rows, V), -1.0, device=DEV)
    g = torch.full((n_rows, V), -1.0, device=DEV)
    idlm.idlm_isd_rng_dump(seed, offset, tag, row0, n_rows, V, uniforms=u, gumbels=g)
    torch.cuda.synchronize()
    ru, rg = oracle.rng_dump(seed, offset, tag, row0, n_rows, V)
    assert np.array_equal(u.cpu().numpy().astype(np.float64), ru)          # 24-bit numerators: exact in fp32
    assert ((ru > 0) & (ru < 1)).all()
    err = np.abs(g.cpu().numpy().astype(np.float64) - rg)
    # -ln u carries a relative error of a few 2^-24; the outer logarithm turns it into an absolute one
    assert err.max() < 4e-6 * np.maximum(1.0, np.abs(rg)).max(), err.max()
    # the accept test of row (b, j) uses element 0 of stream 0
    if tag == 0:
        for r in range(n_rows):
            assert ru[r, 0] == oracle.accept_uniform(seed, offset, row0 + r)


def test_only_one_output_and_argument_checks():
    u = torch.zeros((2, 64), device=DEV)
    idlm.idlm_isd_rng_dump(5, 0, 1, 0, 2, 64, uniforms=u)
    g = torch.zeros((2, 64), device=DEV)
    idlm.idlm_isd_rng_dump(5, 0, 1, 0, 2, 64, gumbels=g)
    torch.cuda.synchronize()
    ru, rg = oracle.rng_dump(5, 0, 1, 0, 2, 64)
    assert np.array_equal(u.cpu().numpy().astype(np.float64), ru) and np.allclose(g.cpu().numpy(), rg, atol=1e-5)
    with pytest.raises(idlm.IdlmError):
        idlm.idlm_isd_rng_dump(5, 0, 1, 0, 2, 64)
    with pytest.raises(idlm.IdlmError):
        idlm.idlm_isd_rng_dump(5, 0, 1, -1, 2, 64, uniforms=u)
    idlm.idlm_isd_rng_dump(5, 0, 1, 0, 0, 64)             # nothing to do
