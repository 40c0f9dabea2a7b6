"""GPU parity: csr_reconstruct (Eq.12, through the C ABI) against the oracle's dense rebuild."""
import numpy as np
import pytest
import torch

import oracle
import paper_2412_11741_amd as csr
from paper_2412_11741_amd import synth

pytestmark = pytest.mark.gpu


def _ref(D, idx, coef):
    """Per block and chunk: oracle.reconstruct, chunks side by side.  D [H', (sn,) N, dc], codes [H, T, (sn,) s]."""
    if D.ndim == 3:
        D, idx, coef = D[:, None], idx[:, :, None], coef[:, :, None]
    H, T, sn, s = idx.shape
    u = idx.view(np.uint16).astype(np.int32) if idx.dtype == np.int16 else idx
    return np.stack([np.concatenate([oracle.reconstruct(u[h, :, c], coef[h, :, c], D[h % D.shape[0], c])
                                     for c in range(sn)], axis=1) for h in range(H)])


def _check(out, ref, D, coef, storage):
    # fp32 accumulation of s products: a few 2^-24 of sum |c| |d| per element; fp16 output adds one rounding
    mag = np.abs(coef.astype(np.float64)).reshape(coef.shape[0], coef.shape[1], -1).sum(-1)[..., None] * np.abs(D.astype(np.float64)).max()
    tol = 4 * 2.0 ** -24 * mag + (2.0 ** -11 * np.abs(ref) + 6e-8 if storage == "f16" else 0.0)
    err = np.abs(out.astype(np.float64) - ref)
    assert np.all(err <= tol), (err.max(), (err / np.maximum(tol, 1e-300)).max())


@pytest.mark.parametrize("H,T,N,d,sn,s,dicts,dtype,itype", [
    (3, 777, 1024, 128, 1, 8, 3, "f16", "i16"),
    (4, 300, 512, 128, 2, 4, 2, "f16", "i16"),       # values in two chunks, blocks sharing dictionaries
    (2, 65, 96, 64, 1, 5, 2, "f32", "i32"),
    (1, 1, 4096, 128, 1, 32, 1, "f16", "i16"),
    (2, 40, 256, 256, 4, 3, 1, "f16", "i32"),
])
def test_reconstruct_matches_the_dense_rebuild(H, T, N, d, sn, s, dicts, dtype, itype):
    dc = d // sn
    D = synth.dictionary(51, "dict_v", dicts * sn, N, dc, dtype).reshape(dicts, sn, N, dc)
    idx, coef = synth.random_codes(51, 0, 1, H, T, sn * s, N, dtype, itype)
    idx, coef = idx[0].reshape(H, T, sn, s), coef[0].reshape(H, T, sn, s)
    if sn == 1:
        D, idx, coef = D[:, 0], idx[:, :, 0], coef[:, :, 0]
    g = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    out = csr.csr_reconstruct(g(D), g(idx), g(coef))
    out32 = csr.csr_reconstruct(g(D), g(idx), g(coef), out_dtype=torch.float32)
    torch.cuda.synchronize()
    ref = _ref(D, idx, coef)
    _check(out.cpu().numpy(), ref, D, coef, dtype)
    _check(out32.cpu().numpy(), ref, D, coef, "f32")


def test_reconstruct_of_the_encoders_codes_shrinks_the_error_and_reads_codes_in_place():
    # encode into a cache of codes, rebuild from a window of that cache into a strided output
    H, T_max, T, N, d, s = 4, 200, 150, 1024, 128, 8
    D = synth.dictionary(52, "dict_k", H, N, d, "f16")
    X = synth.vectors(52, "keys", H, T, d, "f16", outliers=8)
    Dg, Xg = torch.from_numpy(D).cuda(), torch.from_numpy(X).cuda()
    ci = torch.zeros((H, T_max, s), dtype=torch.int16, device="cuda")
    cc = torch.zeros((H, T_max, s), dtype=torch.float16, device="cuda")
    csr.csr_encode(Xg, Dg, s, idx=ci[:, 10:10 + T], coef=cc[:, 10:10 + T])
    wide = torch.full((H, T, 2 * d), 9.0, dtype=torch.float16, device="cuda")
    csr.csr_reconstruct(Dg, ci[:, 10:10 + T], cc[:, 10:10 + T], out=wide[:, :, d:])
    torch.cuda.synchronize()
    assert (wide[:, :, :d] == 9.0).all()
    rec = wide[:, :, d:].cpu().numpy()
    ref = _ref(D, ci[:, 10:10 + T].cpu().numpy(), cc[:, 10:10 + T].cpu().numpy())
    _check(rec, ref, D, cc[:, 10:10 + T].cpu().numpy(), "f16")
    x = X.astype(np.float64)
    assert np.all(((x - ref) ** 2).sum(-1) < (x ** 2).sum(-1))      # Eq.4 removes energy at every step
