"""Pins for the oracle's decode attention (Eq.12 + softmax attention) from outside the oracle:
library attention on special cases, closed forms, and equivalences the definition implies."""
import numpy as np
import pytest
import torch

import oracle


def _sdpa(q, K, V, scale):
    """torch's CPU attention as a third opinion: q [d], K/V [T, d] (float64)."""
    qt = torch.from_numpy(q)[None, None, None, :]
    Kt = torch.from_numpy(K)[None, None]
    Vt = torch.from_numpy(V)[None, None]
    return torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=scale)[0, 0, 0].numpy()


def _dense(idx, coef, D):
    """X~ = r D with r scattered densely (independent of oracle.reconstruct's loop)."""
    T, s = idx.shape
    r = np.zeros((T, D.shape[0]))
    np.add.at(r, (np.repeat(np.arange(T), s), idx.ravel()), coef.ravel())
    return r @ D


def _case(rng, B, Hq, Hkv, T, d, N, sK, sV):
    q = rng.standard_normal((B, Hq, d))
    DK = rng.standard_normal((Hkv, N, d)) / np.sqrt(d)
    DV = rng.standard_normal((Hkv, N, d)) / np.sqrt(d)
    idxK = rng.integers(0, N, size=(B, Hkv, T, sK)).astype(np.int32)
    idxV = rng.integers(0, N, size=(B, Hkv, T, sV)).astype(np.int32)
    coefK = rng.standard_normal((B, Hkv, T, sK)) * 2
    coefV = rng.standard_normal((B, Hkv, T, sV))
    return q, DK, idxK, coefK, DV, idxV, coefV


def test_one_pair_unit_coefficient_is_plain_attention_over_atom_rows():
    rng = np.random.default_rng(0)
    B, H, T, d, N = 2, 3, 40, 16, 25
    q, DK, idxK, _, DV, idxV, _ = _case(rng, B, H, H, T, d, N, 1, 1)
    ones = np.ones((B, H, T, 1))
    out = oracle.decode_attn(q, DK, idxK, ones, DV, idxV, ones, scale=0.3)
    for b in range(B):
        for h in range(H):
            ref = _sdpa(q[b, h], DK[h][idxK[b, h, :, 0]], DV[h][idxV[b, h, :, 0]], 0.3)
            np.testing.assert_allclose(out[b, h], ref, rtol=1e-11, atol=1e-13)


def test_general_codes_against_library_attention_on_densely_rebuilt_cache_with_gqa():
    rng = np.random.default_rng(1)
    B, Hq, Hkv, T, d, N, sK, sV = 2, 6, 2, 33, 8, 20, 4, 3
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, B, Hq, Hkv, T, d, N, sK, sV)
    idxK[..., 2] = idxK[..., 0]                              # repeated atoms inside codes
    out = oracle.decode_attn(q, DK, idxK, coefK, DV, idxV, coefV)    # default scale 1/sqrt(d)
    G = Hq // Hkv
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            ref = _sdpa(q[b, hq], _dense(idxK[b, h], coefK[b, h], DK[h]),
                        _dense(idxV[b, h], coefV[b, h], DV[h]), 1.0 / np.sqrt(d))
            np.testing.assert_allclose(out[b, hq], ref, rtol=1e-10, atol=1e-12)


def test_zero_key_coefficients_give_the_mean_of_values():
    rng = np.random.default_rng(2)
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, 1, 2, 2, 17, 8, 12, 3, 2)
    out = oracle.decode_attn(q, DK, idxK, np.zeros_like(coefK), DV, idxV, coefV)
    for h in range(2):
        np.testing.assert_allclose(out[0, h], _dense(idxV[0, h], coefV[0, h], DV[h]).mean(axis=0),
                                   rtol=1e-12, atol=1e-14)


def test_single_token_returns_its_value_whatever_the_query():
    rng = np.random.default_rng(3)
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, 3, 2, 1, 1, 8, 12, 2, 4)
    out = oracle.decode_attn(q * 50, DK, idxK, coefK, DV, idxV, coefV)
    for b in range(3):
        for hq in range(2):
            np.testing.assert_allclose(out[b, hq], _dense(idxV[b, 0], coefV[b, 0], DV[0])[0],
                                       rtol=1e-12, atol=1e-14)


def test_duplicate_index_equals_summed_coefficient():
    rng = np.random.default_rng(4)
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, 1, 1, 1, 20, 8, 12, 2, 2)
    idxK[..., 1] = idxK[..., 0]
    idxV[..., 1] = idxV[..., 0]
    a = oracle.decode_attn(q, DK, idxK, coefK, DV, idxV, coefV)
    b = oracle.decode_attn(q, DK, idxK[..., :1], coefK.sum(-1, keepdims=True), DV, idxV[..., :1],
                           coefV.sum(-1, keepdims=True))
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)


def test_gqa_equals_mha_on_replicated_heads():
    rng = np.random.default_rng(5)
    B, Hq, Hkv, T, d, N = 2, 8, 2, 15, 8, 10
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, B, Hq, Hkv, T, d, N, 3, 3)
    a = oracle.decode_attn(q, DK, idxK, coefK, DV, idxV, coefV)
    rep = lambda x, ax: np.repeat(x, Hq // Hkv, axis=ax)
    b = oracle.decode_attn(q, rep(DK, 0), rep(idxK, 1), rep(coefK, 1), rep(DV, 0), rep(idxV, 1),
                           rep(coefV, 1))
    assert np.array_equal(a, b)


def test_seq_lens_equal_truncation_and_empty_sequence_is_zero():
    rng = np.random.default_rng(6)
    B, T = 3, 12
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, B, 2, 2, T, 8, 10, 2, 2)
    lens = np.array([12, 5, 0], dtype=np.int32)
    out = oracle.decode_attn(q, DK, idxK, coefK, DV, idxV, coefV, seq_lens=lens)
    for b in range(B):
        L = int(lens[b])
        if L == 0:
            assert np.all(out[b] == 0.0)
            continue
        ref = oracle.decode_attn(q[b:b + 1], DK, idxK[b:b + 1, :, :L], coefK[b:b + 1, :, :L], DV,
                                 idxV[b:b + 1, :, :L], coefV[b:b + 1, :, :L])
        assert np.array_equal(out[b], ref[0])
    with pytest.raises(RuntimeError):
        oracle.decode_attn(q, DK, idxK, coefK, DV, idxV, coefV, seq_lens=np.array([13, 0, 0]))


def test_huge_scores_do_not_overflow_and_pick_the_arg_max_token():
    rng = np.random.default_rng(7)
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, 1, 1, 1, 30, 8, 10, 2, 2)
    out = oracle.decode_attn(q, DK, idxK, coefK, DV, idxV, coefV, scale=1e4)
    K = _dense(idxK[0, 0], coefK[0, 0], DK[0])
    t = int(np.argmax(K @ q[0, 0]))
    assert np.all(np.isfinite(out))
    np.testing.assert_allclose(out[0, 0], _dense(idxV[0, 0], coefV[0, 0], DV[0])[t], rtol=1e-9, atol=1e-12)


def test_sixteen_bit_indices_are_read_unsigned():
    rng = np.random.default_rng(8)
    N = 40000
    DK = rng.standard_normal((1, N, 4))
    DV = rng.standard_normal((1, N, 4))
    q = rng.standard_normal((1, 1, 4))
    idx32 = np.array([[[[39999], [123], [32768]]]], dtype=np.int32)
    idx16 = idx32.astype(np.uint16).view(np.int16)
    c = np.ones((1, 1, 3, 1))
    assert np.array_equal(oracle.decode_attn(q, DK, idx32, c, DV, idx32, c),
                          oracle.decode_attn(q, DK, idx16, c, DV, idx16, c))
