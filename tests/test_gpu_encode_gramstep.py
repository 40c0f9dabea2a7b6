"""GPU parity of the Gram-update encoder for a decoding step (csr_encode with the descriptor's Gram matrices: one sweep
of every dictionary, then one row of G = D D^T per iteration) against the oracle, and of csr_gram_build against numpy."""
import numpy as np
import pytest
import torch

import paper_2412_11741_amd as csr
from paper_2412_11741_amd import synth
from tests.test_gpu_encode import _adversarial_cases, _assert_ok, _compare, _compare_chunked

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dicts,N,d", [(3, 512, 128), (2, 96, 64), (1, 4128, 128)])
def test_gram_build_matches_numpy(dicts, N, d):
    D = synth.dictionary(80, "dict_k", dicts, N, d, "f16")
    D[0, 1::5] = (D[0, 1::5].astype(np.float32) * 1.7).astype(np.float16)
    G = csr.csr_gram_build(torch.from_numpy(D).cuda())
    torch.cuda.synchronize()
    assert G.shape == (dicts, N, N) and G.dtype == torch.float16
    want = np.einsum("hnd,hmd->hnm", D.astype(np.float64), D.astype(np.float64))
    got = G.cpu().numpy().astype(np.float64)
    # fp32 accumulation of exact products, then one rounding to fp16
    assert np.all(np.abs(got - want) <= 2.0 ** -11 * np.abs(want) + 3e-5)
    assert np.array_equal(got, got.transpose(0, 2, 1))


@pytest.mark.parametrize("H,T,N,d,sn,s,dicts", [
    (64, 1, 4096, 128, 1, 8, 64),    # one new token for every head of the benchmark layer (keys and values)
    (8, 1, 1024, 128, 2, 4, 4),      # values in two chunks of 64; two sequences share the dictionaries
    (4, 4, 8192, 128, 1, 16, 1),     # 16 vectors on one dictionary, two rounds of atoms per thread, many iterations
    (2, 3, 16384, 64, 1, 6, 2),      # the largest dictionary, 64-dimensional vectors
    (3, 5, 96, 128, 1, 4, 3),        # fewer atoms than one sweep slice
    (2, 1, 4128, 128, 1, 8, 2),      # a ragged last slice, a partly filled second round
    (64, 1, 4096, 128, 1, 8, 2),     # a decoding step of 32 sequences: the sweep runs on the matrix cores
    (6, 42, 1056, 128, 2, 4, 2),     # 126 vectors per dictionary, three blocks sharing each, two chunks of 64
    (5, 25, 2080, 64, 1, 5, 1),      # 125 vectors of 64 dimensions on one dictionary, ragged vector and atom tiles
])
def test_gram_step_encoder_parity(H, T, N, d, sn, s, dicts):
    dc = d // sn
    D = synth.dictionary(81, "dict_k", dicts * sn, N, dc, "f16").reshape(dicts, sn, N, dc)
    X = synth.vectors(81, "keys", H, T, d, "f16", outliers=8)
    Dg = torch.from_numpy(D if sn > 1 else D[:, 0]).cuda()
    print(f"[gram step] H{H} T{T} N{N} d{d} sn{sn} s{s} dicts{dicts}", flush=True)
    G = csr.csr_gram_build(Dg)
    idx, coef = csr.csr_encode(torch.from_numpy(X).cuda(), Dg, s, algo=csr.CSR_ENCODE_GRAM, gram=G)
    torch.cuda.synchronize()
    idx, coef = idx.cpu().numpy().reshape(H, T, sn, s), coef.cpu().numpy().reshape(H, T, sn, s)
    D_blocks = np.stack([D[h % dicts] for h in range(H)])
    _assert_ok(_compare_chunked(X, D_blocks, s, idx.view(np.uint16).astype(np.int32), coef))


@pytest.mark.parametrize("name", ["atom norms 0.25 .. 2", "duplicated atoms", "dynamic range",
                                  "sparse combinations of atoms", "constant and one-hot vectors"])
def test_gram_step_adversarial_inputs(name):
    D, X = _adversarial_cases()[name]
    D16, X16 = D.astype(np.float16)[None], X.astype(np.float16)[None, :16]
    Dg = torch.from_numpy(D16).cuda()
    idx, coef = csr.csr_encode(torch.from_numpy(X16).cuda(), Dg, 8, gram=csr.csr_gram_build(Dg))
    torch.cuda.synchronize()
    idx, coef = idx.cpu().numpy(), coef.cpu().numpy()
    assert np.all(np.isfinite(coef.astype(np.float32)))
    _assert_ok(_compare(X16, D16, 8, idx, coef))


def test_gram_step_zero_vectors_equal_atoms_and_residual_norms():
    import oracle
    H, T, N, d, s = 3, 4, 320, 128, 5
    D = synth.dictionary(82, "dict_k", H, N, d, "f16")
    D[1] = (D[1].astype(np.float32) * 1.5).astype(np.float16)   # atoms of norm 1.5: Eq.4 is not a projection
    D[2] = D[2, 7]                                              # 320 equal atoms: more candidates than the list holds
    X = synth.vectors(82, "keys", H, T, d, "f16", outliers=4)
    X[0, 1] = 0                                                 # a zero vector
    X[1, 2] = D[1, 17]                                          # a vector that is an atom: the residual collapses
    X[0, 3] = (X[0, 3].astype(np.float32) * 1e-3).astype(np.float16)
    X[1, 0] = (X[1, 0].astype(np.float32) * 300).astype(np.float16)
    Dg = torch.from_numpy(D).cuda()
    rn = torch.empty((H, T), dtype=torch.float32, device="cuda")
    idx, coef = csr.csr_encode(torch.from_numpy(X).cuda(), Dg, s, gram=csr.csr_gram_build(Dg), coef_dtype=torch.float32,
                               idx_dtype=torch.int32, res_norm2=rn)
    torch.cuda.synchronize()
    idx, coef, rn = idx.cpu().numpy(), coef.cpu().numpy(), rn.cpu().numpy()
    assert np.all(idx[0, 1] == 0) and np.all(coef[0, 1] == 0) and rn[0, 1] == 0
    assert idx[1, 2, 0] == 17
    assert np.all(idx[2, :, 0] == 0)                            # lowest atom among equals
    _assert_ok(_compare_chunked(X, D[:, None], s, idx.reshape(H, T, 1, s), coef.reshape(H, T, 1, s)))
    for h in range(H):
        rec = oracle.reconstruct(idx[h], coef[h], D[h])
        err = ((X[h].astype(np.float64) - rec) ** 2).sum(axis=1)
        x2 = (X[h].astype(np.float64) ** 2).sum(axis=1)
        assert np.all(np.abs(rn[h] - err) <= 1e-4 * err + 1e-6 * x2)


def test_gram_step_is_the_default_with_gram_matrices_appends_in_place_and_agrees_with_the_split_encoder():
    B, Hkv, T_max, N, d, s, pos = 3, 4, 50, 1024, 128, 8, 17
    D = synth.dictionary(83, "dict_k", Hkv, N, d, "f16")
    X = synth.vectors(83, "keys", B * Hkv, 1, d, "f16", outliers=8)
    Xg, Dg = torch.from_numpy(X).cuda(), torch.from_numpy(D).cuda()
    G = csr.csr_gram_build(Dg)
    cache_i = torch.full((B * Hkv, T_max, s), -7, dtype=torch.int16, device="cuda")
    cache_c = torch.full((B * Hkv, T_max, s), 123.0, dtype=torch.float16, device="cuda")
    csr.csr_encode(Xg, Dg, s, gram=G, idx=cache_i[:, pos:pos + 1], coef=cache_c[:, pos:pos + 1])
    i_ref, c_ref = csr.csr_encode(Xg, Dg, s, algo=csr.CSR_ENCODE_GRAM, gram=G)
    i_split, c_split = csr.csr_encode(Xg, Dg, s, algo=csr.CSR_ENCODE_SPLIT, gram=G)   # explicit algos ignore G
    torch.cuda.synchronize()
    assert torch.equal(cache_i[:, pos:pos + 1], i_ref) and torch.equal(cache_c[:, pos:pos + 1], c_ref)
    keep = torch.ones(T_max, dtype=torch.bool, device="cuda"); keep[pos] = False
    assert (cache_i[:, keep] == -7).all() and (cache_c[:, keep] == 123.0).all()    # neighbours untouched
    assert torch.equal(i_ref, i_split)
    assert (c_ref.float() - c_split.float()).abs().max() <= 2e-3 * c_split.float().abs().max()
    D_blocks = np.stack([D[h % Hkv] for h in range(B * Hkv)])
    _assert_ok(_compare(X, D_blocks, s, i_ref.cpu().numpy(), c_ref.cpu().numpy()))
    # run to run
    again = csr.csr_encode(Xg, Dg, s, gram=G)
    assert torch.equal(again[0], i_ref) and torch.equal(again[1], c_ref)


def test_both_gram_encoders_with_atoms_long_enough_to_make_residuals_grow():
    # |d|^2 > 2: Eq.4 can lengthen the residual, and the screening bound follows the largest residual norm so far
    H, T, N, d, s = 2, 16, 256, 128, 12
    D = synth.dictionary(85, "dict_k", H, N, d, "f16").astype(np.float32)
    D[:, ::3] *= 3.0
    D[:, 1::3] *= 1.6
    D = D.astype(np.float16)
    X = synth.vectors(85, "keys", H, T, d, "f16", outliers=8)
    Dg, Xg = torch.from_numpy(D).cuda(), torch.from_numpy(X).cuda()
    for kw in (dict(algo=csr.CSR_ENCODE_GRAM), dict(gram=csr.csr_gram_build(Dg))):
        idx, coef = csr.csr_encode(Xg, Dg, s, coef_dtype=torch.float32, idx_dtype=torch.int32, **kw)
        torch.cuda.synchronize()
        _assert_ok(_compare_chunked(X, D[:, None], s, idx.cpu().numpy().reshape(H, T, 1, s), coef.cpu().numpy().reshape(H, T, 1, s)))


def test_gram_step_limits():
    D = torch.from_numpy(synth.dictionary(84, "dict_k", 1, 512, 128, "f16")).cuda()
    X = torch.from_numpy(synth.vectors(84, "keys", 1, 129, 128, "f16")).cuda()
    G = csr.csr_gram_build(D)
    with pytest.raises(csr.CsrError, match="at most 128 vectors"):
        csr.csr_encode(X, D, 4, algo=csr.CSR_ENCODE_GRAM, gram=G)
    # by default more vectors than that simply take the encoder they would take without G
    a = csr.csr_encode(X, D, 4, gram=G)
    b = csr.csr_encode(X, D, 4)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    with pytest.raises(ValueError, match="gram must be"):
        csr.csr_encode(X[:, :4], D, 4, gram=G[:, :100])
    with pytest.raises(csr.CsrError, match="multiple of 32"):
        csr.csr_gram_build(torch.zeros(1, 40, 128, dtype=torch.float16, device="cuda"))
