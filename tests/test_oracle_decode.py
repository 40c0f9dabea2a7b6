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


def _chunked_case(seed, B, Hq, Hkv, T, N, d, snK, sK, snV, sV):
    rng = np.random.default_rng(seed)
    def dic(sn):
        D = rng.standard_normal((Hkv, sn, N, d // sn)); return D / np.linalg.norm(D, axis=-1, keepdims=True)
    q = rng.standard_normal((B, Hq, d))
    DK, DV = dic(snK), dic(snV)
    idxK = rng.integers(0, N, (B, Hkv, T, snK, sK)).astype(np.int32); coefK = rng.standard_normal((B, Hkv, T, snK, sK))
    idxV = rng.integers(0, N, (B, Hkv, T, snV, sV)).astype(np.int32); coefV = rng.standard_normal((B, Hkv, T, snV, sV))
    return q, DK, idxK, coefK, DV, idxV, coefV


def _block_diagonal(D, idx, coef):
    """Chunked dictionary [Hkv, sn, N, dc] and codes [B, Hkv, T, sn, s] as ONE dictionary of sn*N atoms of full
    length (atom (c, n) lives in the dimensions of chunk c, zero elsewhere) with offset indices."""
    Hkv, sn, N, dc = D.shape
    big = np.zeros((Hkv, sn * N, sn * dc))
    for c in range(sn):
        big[:, c * N:(c + 1) * N, c * dc:(c + 1) * dc] = D[:, c]
    off = (np.arange(sn) * N)[None, None, None, :, None]
    B, _, T, _, s = idx.shape
    return big, (idx + off).reshape(B, Hkv, T, sn * s).astype(np.int32), coef.reshape(B, Hkv, T, sn * s)


def test_chunked_attention_with_one_chunk_is_the_plain_one():
    q, DK, idxK, coefK, DV, idxV, coefV = _chunked_case(40, 2, 4, 2, 37, 50, 16, 1, 3, 1, 2)
    a = oracle.decode_attn_chunked(q, DK, idxK, coefK, DV, idxV, coefV)
    b = oracle.decode_attn(q, DK[:, 0], idxK[:, :, :, 0], coefK[:, :, :, 0], DV[:, 0], idxV[:, :, :, 0], coefV[:, :, :, 0])
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)


def test_chunked_attention_equals_plain_attention_on_block_diagonal_dictionaries():
    # Independent route: cutting a vector into s_n chunks, each on its own dictionary, is the same as ONE dictionary
    # of s_n*N zero-padded atoms; the plain C oracle on that dictionary must agree with the numpy chunked one.
    q, DK, idxK, coefK, DV, idxV, coefV = _chunked_case(41, 2, 6, 2, 61, 40, 32, 1, 4, 2, 3)
    a = oracle.decode_attn_chunked(q, DK, idxK, coefK, DV, idxV, coefV, scale=0.3)
    bk, ik, ck = _block_diagonal(DK, idxK, coefK)
    bv, iv, cv = _block_diagonal(DV, idxV, coefV)
    bk = np.concatenate([bk, np.zeros((bk.shape[0], bv.shape[1] - bk.shape[1], bk.shape[2]))], axis=1)  # same N for both
    b = oracle.decode_attn(q, bk, ik, ck, bv, iv, cv, scale=0.3)
    assert np.allclose(a, b, rtol=1e-11, atol=1e-13)


def test_chunked_attention_value_chunks_only_touch_their_own_dimensions():
    q, DK, idxK, coefK, DV, idxV, coefV = _chunked_case(42, 1, 2, 1, 20, 30, 16, 2, 2, 4, 2)
    base = oracle.decode_attn_chunked(q, DK, idxK, coefK, DV, idxV, coefV)
    coefV2 = coefV.copy(); coefV2[:, :, :, 2] *= -3.0          # change chunk 2 of the values only
    out = oracle.decode_attn_chunked(q, DK, idxK, coefK, DV, idxV, coefV2)
    assert np.allclose(out[..., :8], base[..., :8]) and np.allclose(out[..., 12:], base[..., 12:])
    assert np.allclose(out[..., 8:12], -3.0 * base[..., 8:12])
    lens = np.array([7], dtype=np.int32)
    cut = oracle.decode_attn_chunked(q, DK, idxK[:, :, :7], coefK[:, :, :7], DV, idxV[:, :, :7], coefV[:, :, :7])
    assert np.allclose(oracle.decode_attn_chunked(q, DK, idxK, coefK, DV, idxV, coefV, seq_lens=lens), cut)


# --- keys coded before the rotary embedding (Section "Position embedding makes nonstationary Keys") ------------

def _complex_rotate(X, pos, base, layout):
    """The rotary embedding as multiplication of complex pairs by e^{i p theta_k} (independent of the oracle's
    real-arithmetic form)."""
    T, d = X.shape
    hd = d // 2
    z = X[:, :hd] + 1j * X[:, hd:] if layout == 0 else X[:, 0::2] + 1j * X[:, 1::2]
    k = np.arange(hd)
    w = np.exp(1j * np.outer(np.asarray(pos, dtype=np.float64), np.exp(-2.0 * k / d * np.log(base))))
    z = z * w
    out = np.empty_like(X)
    if layout == 0:
        out[:, :hd], out[:, hd:] = z.real, z.imag
    else:
        out[:, 0::2], out[:, 1::2] = z.real, z.imag
    return out


def test_rotary_single_pair_closed_form():
    # d = 2: one pair, theta_0 = 1; the unit vector e_0 at position p becomes (cos p, sin p)
    pos = np.array([0, 1, 2, 7])
    X = np.tile(np.array([[1.0, 0.0]]), (4, 1))
    for layout in (0, 1):
        out = oracle.rope_rotate(X, pos, 10000.0, layout)
        np.testing.assert_allclose(out, np.stack([np.cos(pos), np.sin(pos)], axis=1), atol=1e-15)
    # d = 4, base 16: theta = (1, 1/4); layout 0 pairs (0,2),(1,3), layout 1 pairs (0,1),(2,3)
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    p = 3.0
    c0, s0, c1, s1 = np.cos(p), np.sin(p), np.cos(p / 4), np.sin(p / 4)
    np.testing.assert_allclose(oracle.rope_rotate(x, [3], 16.0, 0)[0],
                               [1 * c0 - 3 * s0, 2 * c1 - 4 * s1, 3 * c0 + 1 * s0, 4 * c1 + 2 * s1], atol=1e-14)
    np.testing.assert_allclose(oracle.rope_rotate(x, [3], 16.0, 1)[0],
                               [1 * c0 - 2 * s0, 2 * c0 + 1 * s0, 3 * c1 - 4 * s1, 4 * c1 + 3 * s1], atol=1e-14)


@pytest.mark.parametrize("layout", [0, 1])
def test_rotary_matches_complex_multiplication_and_keeps_norms(layout):
    rng = np.random.default_rng(40 + layout)
    X = rng.standard_normal((50, 32))
    pos = rng.integers(0, 100000, size=50)
    out = oracle.rope_rotate(X, pos, 10000.0, layout)
    np.testing.assert_allclose(out, _complex_rotate(X, pos, 10000.0, layout), rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(np.linalg.norm(out, axis=1), np.linalg.norm(X, axis=1), rtol=1e-12)
    # position 0 is the identity; rotations compose additively
    np.testing.assert_array_equal(oracle.rope_rotate(X, np.zeros(50), 10000.0, layout), X)
    twice = oracle.rope_rotate(oracle.rope_rotate(X, pos, 10000.0, layout), 17 - pos, 10000.0, layout)
    np.testing.assert_allclose(twice, oracle.rope_rotate(X, np.full(50, 17), 10000.0, layout), atol=1e-9)


@pytest.mark.parametrize("layout", [0, 1])
def test_rope_attention_against_library_attention_on_rotated_rebuilt_keys(layout):
    rng = np.random.default_rng(42)
    B, Hq, Hkv, T, d, N, sK, sV = 2, 4, 2, 37, 16, 24, 4, 3
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, B, Hq, Hkv, T, d, N, sK, sV)
    out = oracle.decode_attn_rope(q, DK, idxK, coefK, DV, idxV, coefV, 500.0, layout, pos0=11, scale=0.4)
    G = Hq // Hkv
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            K = _complex_rotate(_dense(idxK[b, h], coefK[b, h], DK[h]), 11 + np.arange(T), 500.0, layout)
            ref = _sdpa(q[b, hq], K, _dense(idxV[b, h], coefV[b, h], DV[h]), 0.4)
            np.testing.assert_allclose(out[b, hq], ref, rtol=1e-9, atol=1e-11)


def test_rope_attention_depends_on_relative_positions_only():
    # turning the query by +m and placing the cache m positions later leaves every score unchanged
    rng = np.random.default_rng(43)
    B, H, T, d, N, s = 1, 2, 29, 16, 20, 3
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, B, H, H, T, d, N, s, s)
    base = 10000.0
    q_at = lambda p: np.stack([oracle.rope_rotate(q[0], np.full(H, p), base, 0)])  # noqa: E731
    a = oracle.decode_attn_rope(q_at(T), DK, idxK, coefK, DV, idxV, coefV, base, 0, pos0=0)
    b = oracle.decode_attn_rope(q_at(T + 1000), DK, idxK, coefK, DV, idxV, coefV, base, 0, pos0=1000)
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-11)
    # and it is NOT the position-free attention (the rotation matters)
    plain = oracle.decode_attn(q_at(T), DK, idxK, coefK, DV, idxV, coefV)
    assert np.abs(a - plain).max() > 1e-3


def test_rope_attention_single_token_and_lengths_and_chunked_values():
    rng = np.random.default_rng(44)
    B, H, T, d, N, s = 3, 2, 12, 8, 10, 2
    q, DK, idxK, coefK, DV, idxV, coefV = _case(rng, B, H, H, T, d, N, s, s)
    one = oracle.decode_attn_rope(q, DK, idxK[:, :, :1], coefK[:, :, :1], DV, idxV[:, :, :1], coefV[:, :, :1], 10000.0)
    for b in range(B):
        for h in range(H):
            np.testing.assert_allclose(one[b, h], _dense(idxV[b, h, :1], coefV[b, h, :1], DV[h])[0], atol=1e-13)
    lens = np.array([5, 0, 12], dtype=np.int32)
    out = oracle.decode_attn_rope(q, DK, idxK, coefK, DV, idxV, coefV, 10000.0, seq_lens=lens)
    assert np.all(out[1] == 0.0)
    cut = oracle.decode_attn_rope(q[:1], DK, idxK[:1, :, :5], coefK[:1, :, :5], DV, idxV[:1, :, :5], coefV[:1, :, :5], 10000.0)
    np.testing.assert_allclose(out[0], cut[0], rtol=1e-12)
    # chunked values: two chunks on block-diagonal dictionaries equal whole-vector values
    DVc = rng.standard_normal((H, 2, N, d // 2))
    idxVc = rng.integers(0, N, size=(B, H, T, 2, s)).astype(np.int32)
    coefVc = rng.standard_normal((B, H, T, 2, s))
    DVw = np.zeros((H, 2 * N, d))
    DVw[:, :N, :d // 2], DVw[:, N:, d // 2:] = DVc[:, 0], DVc[:, 1]
    idxVw = np.concatenate([idxVc[:, :, :, 0], idxVc[:, :, :, 1] + N], axis=3)
    coefVw = np.concatenate([coefVc[:, :, :, 0], coefVc[:, :, :, 1]], axis=3)
    DKw = np.concatenate([DK, np.zeros_like(DK)], axis=1)  # same atom count for both whole dictionaries
    a = oracle.decode_attn_rope(q, DK, idxK, coefK, DVc, idxVc, coefVc, 10000.0, 1, pos0=3)
    b = oracle.decode_attn_rope(q, DKw, idxK, coefK, DVw, idxVw, coefVw, 10000.0, 1, pos0=3)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-14)
