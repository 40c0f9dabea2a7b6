"""The comparison rules of tests/parity.py, exercised on the CPU with mistakes planted on purpose."""
import numpy as np

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
