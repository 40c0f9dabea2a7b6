"""GPU parity of the Gram-update encoder (csr_encode with algo = CSR_ENCODE_GRAM) against the oracle."""
import numpy as np
import pytest
import torch

import paper_2412_11741_amd as csr
from paper_2412_11741_amd import synth
from tests.test_gpu_encode import _assert_ok, _compare_chunked

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("H,T,N,d,sn,s,dicts", [
    (4, 1000, 256, 128, 1, 8, 4),      # the paper's 256 atoms per head
    (2, 513, 32, 128, 1, 4, 2),        # two tiles; a second workgroup with a single vector
    (6, 300, 256, 128, 2, 4, 3),       # values in two chunks of 64; blocks sharing dictionaries
    (2, 2000, 96, 64, 1, 6, 2),        # 64-dimensional vectors, six tiles, 12 pieces per row
    (3, 100, 160, 128, 1, 16, 3),      # many iterations
])
def test_gram_encoder_parity(H, T, N, d, sn, s, dicts):
    dc = d // sn
    D = synth.dictionary(72, "dict_k", dicts * sn, N, dc, "f16").reshape(dicts, sn, N, dc)
    X = synth.vectors(72, "keys", H, T, d, "f16", outliers=8)
    Dg = torch.from_numpy(D if sn > 1 else D[:, 0]).cuda()
    print(f"[gram] H{H} T{T} N{N} d{d} sn{sn} s{s}", flush=True)
    idx, coef = csr.csr_encode(torch.from_numpy(X).cuda(), Dg, s, algo=csr.CSR_ENCODE_GRAM)
    torch.cuda.synchronize()
    idx, coef = idx.cpu().numpy().reshape(H, T, sn, s), coef.cpu().numpy().reshape(H, T, sn, s)
    D_blocks = np.stack([D[h % dicts] for h in range(H)])
    _assert_ok(_compare_chunked(X, D_blocks, s, idx.view(np.uint16).astype(np.int32), coef))


def test_gram_encoder_edge_cases_zero_vectors_scaled_atoms_and_residual_norms():
    import oracle
    H, T, N, d, s = 2, 70, 64, 128, 5
    D = synth.dictionary(73, "dict_k", H, N, d, "f16")
    D[1] = (D[1].astype(np.float32) * 1.5).astype(np.float16)          # atoms of norm 1.5: Eq.4 is not a projection
    X = synth.vectors(73, "keys", H, T, d, "f16", outliers=4)
    X[0, 3] = 0                                                        # a zero vector
    X[1, 5] = D[1, 17]                                                 # a vector that is an atom
    X[0, 7] = (X[0, 7].astype(np.float32) * 1e-3).astype(np.float16)   # tiny and huge norms
    X[1, 9] = (X[1, 9].astype(np.float32) * 300).astype(np.float16)
    rn = torch.empty((H, T), dtype=torch.float32, device="cuda")
    idx, coef = csr.csr_encode(torch.from_numpy(X).cuda(), torch.from_numpy(D).cuda(), s, algo=csr.CSR_ENCODE_GRAM,
                               coef_dtype=torch.float32, idx_dtype=torch.int32, res_norm2=rn)
    torch.cuda.synchronize()
    idx, coef, rn = idx.cpu().numpy(), coef.cpu().numpy(), rn.cpu().numpy()
    assert np.all(idx[0, 3] == 0) and np.all(coef[0, 3] == 0) and rn[0, 3] == 0
    assert idx[1, 5, 0] == 17
    _assert_ok(_compare_chunked(X, D[:, None], s, idx.reshape(H, T, 1, s), coef.reshape(H, T, 1, s)))
    for h in range(H):
        rec = oracle.reconstruct(idx[h], coef[h], D[h])
        err = ((X[h].astype(np.float64) - rec) ** 2).sum(axis=1)
        x2 = (X[h].astype(np.float64) ** 2).sum(axis=1)
        assert np.all(np.abs(rn[h] - err) <= 1e-4 * err + 1e-6 * x2)


def test_gram_encoder_is_refused_beyond_256_atoms_and_never_chosen_by_default():
    D = torch.from_numpy(synth.dictionary(74, "dict_k", 1, 512, 128, "f16")).cuda()
    X = torch.from_numpy(synth.vectors(74, "keys", 1, 64, 128, "f16")).cuda()
    with pytest.raises(csr.CsrError, match="at most 256"):
        csr.csr_encode(X, D, 4, algo=csr.CSR_ENCODE_GRAM)
    # the default choice for a dictionary it could take stays the LDS-resident encoder (faster on this chip)
    D = torch.from_numpy(synth.dictionary(74, "dict_k", 1, 256, 128, "f16")).cuda()
    a = csr.csr_encode(X, D, 4)
    b = csr.csr_encode(X, D, 4, algo=csr.CSR_ENCODE_RESIDENT)
    c = csr.csr_encode(X, D, 4, algo=csr.CSR_ENCODE_GRAM)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert torch.equal(a[0], c[0])   # (and the two encoders agree on the atoms)
