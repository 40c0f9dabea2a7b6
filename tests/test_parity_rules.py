"""The comparison rules of tests/parity.py, exercised on the CPU with mistakes planted on purpose."""
import numpy as np
import pytest

import oracle
from tests import parity


def _setup(seed=0, T=40, d=16, N=60, s=5):
    rng = np.random.default_rng(seed)
    D = rng.standard_normal((N, d)); D /= np.linalg.norm(D, axis=1, keepdims=True)
    X = rng.standard_normal((T, d))
    idx, coef, diag = oracle.mp_encode(X, D, s, diagnostics=True)
    return X, D, idx, coef, diag


def test_identical_output_passes():
    X, D, idx, coef, diag = _setup()
    rep = parity.check_encode(X, D, idx, coef.astype(np.float32), idx, coef, diag, 1e-5)
    assert rep.ok and rep.exact_steps == rep.steps and rep.tie_vectors == 0


def test_wrong_index_without_tie_fails():
    X, D, idx, coef, diag = _setup()
    bad = idx.copy(); bad[3, 2] = (bad[3, 2] + 1) % len(D)
    rep = parity.check_encode(X, D, bad, coef, idx, coef, diag, 1e-3)
    assert not rep.ok and "not a tie" in rep.failures[0]


def test_wrong_coefficient_fails_and_sign_flip_fails():
    X, D, idx, coef, diag = _setup()
    bad = coef.copy(); bad[5, 1] *= 1.01
    assert not parity.check_encode(X, D, idx, bad, idx, coef, diag, 1e-3).ok
    bad = coef.copy(); bad[7, 0] = -bad[7, 0]
    assert not parity.check_encode(X, D, idx, bad, idx, coef, diag, 1e-3).ok


def test_exact_tie_accepts_either_atom_and_then_checks_greedy_validity():
    X, D, idx, coef, diag = _setup(seed=1)
    t = 4
    a = int(idx[t, 0])
    D2 = np.vstack([D, D[a:a + 1]])                       # a duplicate atom at the end: exact tie
    idx_o, coef_o, diag_o = oracle.mp_encode(X, D2, idx.shape[1], diagnostics=True)
    assert idx_o[t, 0] == a                               # oracle keeps the lower index
    cand = idx_o.copy(); cand[t, 0] = len(D)              # a candidate that took the twin instead
    rep = parity.check_encode(X, D2, cand, coef_o, idx_o, coef_o, diag_o, 1e-6)
    assert rep.ok and rep.tie_vectors == 1
    # ... but a non-greedy pick after the tie is still caught
    cand[t, 2] = (cand[t, 2] + 7) % len(D)
    rep = parity.check_encode(X, D2, cand, coef_o, idx_o, coef_o, diag_o, 1e-6)
    assert not rep.ok and "not a greedy pick" in rep.failures[0]


def test_decode_errors():
    a = np.ones((2, 3, 4)); b = a.copy(); b[1, 2, 0] += 0.02
    rel, mx = parity.decode_errors(b, a)
    assert rel.shape == (2, 3) and abs(rel[1, 2] - 0.01) < 1e-12 and abs(mx - 0.02) < 1e-12
    parity.assert_decode_close(b, a, 0.021)
    # one element off by 2 % of its vector's peak fails the element rule although the L2 error is 1 %
    with pytest.raises(AssertionError, match="largest element error"):
        parity.assert_decode_close(b, a, 0.015)
    with pytest.raises(AssertionError, match="relative L2"):
        parity.assert_decode_close(b, a, 0.005)
    # the element rule is relative to the vector's own peak, not to the whole output's
    c = a.copy(); c[0] *= 1e-3; e = c.copy(); e[0, 0, 0] += 1e-4
    assert parity.decode_errors(e, c)[1] > 0.09


def test_collapsed_residual_floor_accepts_only_what_fp32_cannot_resolve():
    # x is exactly one atom: after the first pick the fp64 residual is ~1e-16 |x|.  A candidate working in
    # fp32 cannot know which atom "wins" there, so any index with a coefficient below one fp32 ulp of |x|
    # passes; a coefficient error above that floor, or a wrong first pick, still fails.
    rng = np.random.default_rng(3)
    D = rng.standard_normal((40, 16)); D /= np.linalg.norm(D, axis=1, keepdims=True)
    X = 2.0 * D[7:8]
    idx, coef, diag = oracle.mp_encode(X, D, 3, diagnostics=True)
    assert idx[0, 0] == 7 and abs(coef[0, 1]) < 1e-12
    cand_i, cand_c = idx.copy(), coef.copy()
    cand_i[0, 1] = (idx[0, 1] + 5) % 40; cand_c[0, 1] = 3e-8          # noise-level pick, as fp32 would give
    cand_c[0, 2] = 0.0
    assert parity.check_encode(X, D, cand_i, cand_c, idx, coef, diag, 1e-3).ok
    cand_c[0, 1] = 1e-5                                                # well above one fp32 ulp of |x| = 2.4e-7
    assert not parity.check_encode(X, D, cand_i, cand_c, idx, coef, diag, 1e-3).ok
    cand_i, cand_c = idx.copy(), coef.copy(); cand_i[0, 0] = 8
    assert not parity.check_encode(X, D, cand_i, cand_c, idx, coef, diag, 1e-3).ok


def test_fp16_storage_allows_one_storage_ulp_and_no_more():
    X, D, idx, coef, diag = _setup(seed=2)
    coef = coef * 1e-5                                  # stored values fall into the fp16 subnormals
    X = X * 1e-5
    c16 = coef.astype(np.float16).astype(np.float64)
    one_ulp = c16 + np.spacing(np.abs(c16).astype(np.float16)).astype(np.float64)
    assert parity.check_encode(X, D, idx, one_ulp, idx, c16, diag, 1e-3, coef_storage="f16").ok
    three_ulp = c16 + 3 * np.spacing(np.abs(c16).astype(np.float16)).astype(np.float64)
    assert not parity.check_encode(X, D, idx, three_ulp, idx, c16, diag, 1e-3, coef_storage="f16").ok
    assert not parity.check_encode(X, D, idx, one_ulp, idx, c16, diag, 1e-3, coef_storage="f32").ok
