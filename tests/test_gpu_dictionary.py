"""Atom norms of a dictionary (Section "Sparse representation": unit-norm atoms) against numpy in fp64."""
import numpy as np
import pytest
import torch

import paper_2412_11741_amd as csr
from paper_2412_11741_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,dtype", [((3, 1024, 128), torch.float16), ((2, 4, 256, 32), torch.float16),
                                         ((1, 37, 100), torch.float32), ((5, 1), torch.float16),
                                         ((1030, 4096), torch.float32), ((2, 8192, 128), torch.float16)])
def test_atom_norms_match_numpy(shape, dtype):
    g = torch.Generator().manual_seed(sum(shape))
    D = (torch.randn(shape, generator=g) * torch.rand(shape[:-1], generator=g).unsqueeze(-1) * 3).to(dtype)
    want = (D.double().numpy() ** 2).sum(-1)
    got = csr.csr_atom_norms2(D.cuda())
    torch.cuda.synchronize()
    assert got.shape == shape[:-1] and got.dtype == torch.float32
    np.testing.assert_allclose(got.cpu().numpy(), want, rtol=2e-6 * max(1, shape[-1] / 64), atol=0)


def test_synthetic_dictionaries_have_unit_atoms():
    D = synth.dictionary(3, "dict_k", 4, 1024, 128)
    n2 = csr.csr_atom_norms2(torch.from_numpy(D).cuda()).cpu().numpy()
    assert np.abs(n2 - 1).max() < 2e-3   # fp16 rounding of a unit vector's 128 elements


def test_empty_and_output_checks():
    assert csr.csr_atom_norms2(torch.zeros(0, 64, dtype=torch.float16, device="cuda")).shape == (0,)
    with pytest.raises(ValueError, match="shape"):
        csr.csr_atom_norms2(torch.zeros(2, 8, 64, dtype=torch.float16, device="cuda"),
                            out=torch.zeros(16, dtype=torch.float32, device="cuda"))


def test_check_codes_counts_indices_outside_the_dictionary():
    rng = np.random.default_rng(8)
    for dtype, N in ((np.int32, 1000), (np.int16, 40000), (np.int16, 4096)):
        idx = rng.integers(0, N, size=(3, 7, 1001, 8)).astype(np.int64)
        bad = rng.random(idx.shape) < 0.001
        idx[bad] = N + rng.integers(0, 20000, size=int(bad.sum()))
        if dtype == np.int32:
            idx[0, 0, 0, 0] = -5; bad[0, 0, 0, 0] = True            # a negative index is outside too
        host = idx.astype(np.uint16).view(np.int16) if dtype == np.int16 else idx.astype(np.int32)
        got = csr.csr_check_codes(torch.from_numpy(host).cuda(), N)
        torch.cuda.synchronize()
        assert int(got.item()) == int(bad.sum()) > 0
    clean = torch.zeros(5, 8, dtype=torch.int16, device="cuda")
    assert int(csr.csr_check_codes(clean, 1).item()) == 0
    assert int(csr.csr_check_codes(clean[:0], 7).item()) == 0
