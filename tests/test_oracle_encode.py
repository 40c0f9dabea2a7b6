"""Pins for the oracle's Matching Pursuit (Eq.2-4) that do not come from the oracle itself:
brute force, orthonormal dictionaries (top-|s| selection), energy identities, structure."""
import itertools

import numpy as np
import pytest

import oracle


def _unit_rows(rng, n, d):
    a = rng.standard_normal((n, d))
    return a / np.linalg.norm(a, axis=1, keepdims=True)


def _brute_best_atom(x, D):
    """Exhaustive solution of Eq.1 for s = 1: least-squares coefficient per atom, smallest error."""
    best = None
    for n in range(D.shape[0]):
        c = np.linalg.lstsq(D[n][:, None], x, rcond=None)[0][0]
        err = float(np.sum((x - c * D[n]) ** 2))
        if best is None or err < best[0] - 1e-13 * max(1.0, best[0]):
            best = (err, n, c)
    return best[1], best[2]


@pytest.mark.parametrize("seed", range(8))
def test_single_step_is_exact_optimum_of_eq1(seed):
    rng = np.random.default_rng(seed)
    d, N = int(rng.integers(2, 9)), int(rng.integers(2, 17))
    D = _unit_rows(rng, N, d)
    D *= rng.choice([-1.0, 1.0], size=(N, 1))            # adversarial signs
    X = rng.standard_normal((20, d))
    idx, coef = oracle.mp_encode(X, D, 1)
    for t in range(len(X)):
        n, c = _brute_best_atom(X[t], D)
        assert idx[t, 0] == n
        assert coef[t, 0] == pytest.approx(c, rel=1e-12, abs=1e-14)


@pytest.mark.parametrize("seed", range(4))
def test_every_greedy_step_matches_exhaustive_search_on_the_residual(seed):
    rng = np.random.default_rng(100 + seed)
    d, N, s = 6, 13, 5
    D = _unit_rows(rng, N, d)
    X = rng.standard_normal((10, d))
    idx, coef = oracle.mp_encode(X, D, s)
    for t in range(len(X)):
        R = X[t].copy()
        for g in range(s):
            n, c = _brute_best_atom(R, D)
            assert idx[t, g] == n
            assert coef[t, g] == pytest.approx(c, rel=1e-10, abs=1e-13)
            R = R - c * D[n]


def test_identity_dictionary_returns_top_s_coordinates():
    rng = np.random.default_rng(1)
    d, s = 16, 5
    X = rng.standard_normal((50, d))
    idx, coef = oracle.mp_encode(X, np.eye(d), s)
    order = np.argsort(-np.abs(X), axis=1, kind="stable")[:, :s]
    assert np.array_equal(idx, order)
    assert np.array_equal(coef, np.take_along_axis(X, order, axis=1))     # exact: products by 1.0


@pytest.mark.parametrize("seed", range(3))
def test_orthonormal_dictionary_is_partial_sort_and_exact_at_s_equals_d(seed):
    rng = np.random.default_rng(10 + seed)
    d = 24
    Q, _ = np.linalg.qr(rng.standard_normal((d, d)))      # rows of Q.T are an orthonormal basis
    D = Q.T.copy()
    X = rng.standard_normal((30, d))
    proj = X @ D.T
    s = 7
    idx, coef = oracle.mp_encode(X, D, s)
    order = np.argsort(-np.abs(proj), axis=1, kind="stable")[:, :s]
    assert np.array_equal(idx, order)
    np.testing.assert_allclose(coef, np.take_along_axis(proj, order, axis=1), rtol=1e-12, atol=1e-13)
    # s = d: every basis vector is used once and reconstruction is exact
    idx, coef, diag = oracle.mp_encode(X, D, d, diagnostics=True)
    assert all(sorted(row) == list(range(d)) for row in idx.tolist())
    rec = oracle.reconstruct(idx, coef, D)
    assert np.max(np.linalg.norm(rec - X, axis=1) / np.linalg.norm(X, axis=1)) < 1e-12
    assert np.all(diag["res_norm2"][:, -1] <= 1e-24 * diag["res_norm2"][:, 0])


def test_energy_identity_orthogonality_and_decomposition():
    rng = np.random.default_rng(3)
    d, N, s = 32, 200, 9
    D = _unit_rows(rng, N, d)
    X = rng.standard_normal((40, d)) * 3.0
    idx, coef, diag = oracle.mp_encode(X, D, s, diagnostics=True)
    rn = diag["res_norm2"]
    # |R_{g+1}|^2 = |R_g|^2 - c_g^2 for unit atoms, hence non-increasing
    np.testing.assert_allclose(rn[:, 1:], rn[:, :-1] - coef ** 2, rtol=1e-11, atol=1e-12)
    assert np.all(rn[:, 1:] <= rn[:, :-1] + 1e-12)
    np.testing.assert_allclose(rn[:, 0], np.sum(X ** 2, axis=1), rtol=1e-13)
    # |x|^2 = sum c^2 + |R_{s+1}|^2 ;  x = sum c d + R_{s+1}
    np.testing.assert_allclose(np.sum(X ** 2, axis=1), np.sum(coef ** 2, axis=1) + rn[:, -1], rtol=1e-11)
    rec = oracle.reconstruct(idx, coef, D)
    np.testing.assert_allclose(np.sum((X - rec) ** 2, axis=1), rn[:, -1], rtol=1e-9, atol=1e-12)
    # R_{g+1} is orthogonal to the atom just removed; best_abs is |c_g| and dominates the runner-up
    for t in range(5):
        R = X[t].copy()
        for g in range(s):
            R = R - coef[t, g] * D[idx[t, g]]
            assert abs(R @ D[idx[t, g]]) < 1e-12 * np.linalg.norm(X[t])
    np.testing.assert_allclose(diag["best_abs"], np.abs(coef), rtol=0, atol=0)
    assert np.all(diag["second_abs"] <= diag["best_abs"])
    # never the same atom twice in a row
    assert np.all(idx[:, 1:] != idx[:, :-1])


def test_non_unit_atoms_follow_the_generalised_energy_identity():
    # No division by |d|^2 happens: |R'|^2 = |R|^2 - c^2 (2 - |d|^2) for the picked atom.
    rng = np.random.default_rng(4)
    d, N, s = 16, 60, 4
    D = _unit_rows(rng, N, d).astype(np.float16).astype(np.float64)      # unit only to ~1e-3
    X = rng.standard_normal((25, d))
    idx, coef, diag = oracle.mp_encode(X, D, s, diagnostics=True)
    n2 = np.sum(D ** 2, axis=1)[idx]
    rn = diag["res_norm2"]
    np.testing.assert_allclose(rn[:, 1:], rn[:, :-1] - coef ** 2 * (2.0 - n2), rtol=1e-11, atol=1e-12)


def test_negative_projection_keeps_its_sign():
    # x = -3 d_2 : the coefficient must be -3 (not +3) and the residual must vanish.
    D = np.eye(4)
    idx, coef, diag = oracle.mp_encode(np.array([[0.0, 0.0, -3.0, 0.0]]), D, 2, diagnostics=True)
    assert idx[0, 0] == 2 and coef[0, 0] == -3.0
    assert diag["res_norm2"][0, 1] == 0.0
    # zero residual afterwards: (0, 0)
    assert idx[0, 1] == 0 and coef[0, 1] == 0.0


def test_scaled_atom_input_gives_that_atom_first():
    rng = np.random.default_rng(5)
    D = _unit_rows(rng, 50, 12)
    for k, alpha in [(0, 2.5), (17, -0.75), (49, 1e-3)]:
        idx, coef = oracle.mp_encode((alpha * D[k])[None], D, 4)
        assert idx[0, 0] == k
        assert coef[0, 0] == pytest.approx(alpha, rel=1e-13)
        assert np.all(np.abs(coef[0, 1:]) < 1e-12 * abs(alpha))


def test_zero_vector_and_lowest_index_tie_break():
    rng = np.random.default_rng(6)
    D = _unit_rows(rng, 9, 5)
    idx, coef = oracle.mp_encode(np.zeros((2, 5)), D, 3)
    assert np.all(idx == 0) and np.all(coef == 0.0) and not np.any(np.isnan(coef))
    D[7] = D[3]                                            # exact duplicate: 3 must win over 7
    D[5] = -D[3]                                           # equal magnitude, opposite sign
    idx, coef = oracle.mp_encode((2.0 * D[3])[None], D, 1)
    assert idx[0, 0] == 3 and coef[0, 0] == pytest.approx(2.0)
    D[1] = -D[3]                                           # now the earlier atom wins, negative coef
    idx, coef = oracle.mp_encode((2.0 * D[3])[None], D, 1)
    assert idx[0, 0] == 1 and coef[0, 0] == pytest.approx(-2.0)


def test_symmetries_negation_power_of_two_scaling_atom_permutation():
    rng = np.random.default_rng(7)
    d, N, s = 16, 80, 6
    D = _unit_rows(rng, N, d)
    X = rng.standard_normal((30, d))
    idx, coef = oracle.mp_encode(X, D, s)
    idx_n, coef_n = oracle.mp_encode(-X, D, s)
    assert np.array_equal(idx, idx_n) and np.array_equal(coef, -coef_n)
    idx_s, coef_s = oracle.mp_encode(X * 2.0 ** -7, D, s)
    assert np.array_equal(idx, idx_s) and np.array_equal(coef * 2.0 ** -7, coef_s)
    perm = rng.permutation(N)
    idx_p, coef_p = oracle.mp_encode(X, D[perm], s)
    assert np.array_equal(perm[idx_p], idx) and np.array_equal(coef_p, coef)


def test_repeated_atoms_are_allowed_and_sum_in_reconstruction():
    # Two non-orthogonal atoms in the plane: MP must alternate between them, re-using each.
    D = np.array([[1.0, 0.0], [np.cos(0.7), np.sin(0.7)]])
    x = np.array([[0.9, 1.3]])
    idx, coef, diag = oracle.mp_encode(x, D, 12, diagnostics=True)
    assert set(idx[0].tolist()) == {0, 1} and np.all(idx[0, 1:] != idx[0, :-1])
    rec = oracle.reconstruct(idx, coef, D)
    np.testing.assert_allclose(np.sum((x - rec) ** 2), diag["res_norm2"][0, -1], rtol=1e-9, atol=1e-15)
    # After the first step the residual is orthogonal to the atom just used, so projecting on the
    # other atom (angle 0.7 away) leaves the fraction cos^2(0.7) of its energy, every step.
    ratios = diag["res_norm2"][0, 2:] / diag["res_norm2"][0, 1:-1]
    np.testing.assert_allclose(ratios, np.cos(0.7) ** 2, rtol=1e-9)


def test_greedy_is_never_better_than_best_support_least_squares():
    rng = np.random.default_rng(8)
    d, N, s = 5, 8, 3
    D = _unit_rows(rng, N, d)
    X = rng.standard_normal((12, d))
    idx, coef, diag = oracle.mp_encode(X, D, s, diagnostics=True)
    for t in range(len(X)):
        best = np.inf
        for sup in itertools.combinations(range(N), s):
            A = D[list(sup)].T
            r = X[t] - A @ np.linalg.lstsq(A, X[t], rcond=None)[0]
            best = min(best, float(r @ r))
        assert diag["res_norm2"][t, -1] >= best - 1e-12


def test_reconstruct_equals_dense_r_times_dictionary():
    # Eq.12 through a different route: scatter the pairs into a dense r (T x N), then r @ D.
    rng = np.random.default_rng(9)
    T, N, d, s = 37, 50, 11, 6
    D = rng.standard_normal((N, d))
    idx = rng.integers(0, N, size=(T, s)).astype(np.int32)
    idx[:, 3] = idx[:, 1]                                   # repeated atoms inside a code
    coef = rng.standard_normal((T, s))
    r = np.zeros((T, N))
    np.add.at(r, (np.repeat(np.arange(T), s), idx.ravel()), coef.ravel())
    np.testing.assert_allclose(oracle.reconstruct(idx, coef, D), r @ D, rtol=1e-12, atol=1e-13)
    with pytest.raises(RuntimeError):
        bad = idx.copy(); bad[0, 0] = N
        oracle.reconstruct(bad, coef, D)


def test_more_iterations_and_more_atoms_reduce_error_on_average():
    # Soft trend behind the paper's MSE tables (they need trained dictionaries; only the trend holds here).
    rng = np.random.default_rng(11)
    d = 32
    X = rng.standard_normal((200, d))
    D_big = _unit_rows(rng, 512, d)
    mse = {}
    for N in (128, 512):
        for s in (2, 4, 8):
            _, _, diag = oracle.mp_encode(X, D_big[:N], s, diagnostics=True)
            mse[(N, s)] = diag["res_norm2"][:, -1].mean()
    assert mse[(128, 2)] > mse[(128, 4)] > mse[(128, 8)]
    assert mse[(512, 2)] > mse[(512, 4)] > mse[(512, 8)]
    assert all(mse[(512, s)] < mse[(128, s)] for s in (2, 4, 8))


def test_thread_count_does_not_change_results():
    rng = np.random.default_rng(12)
    D = _unit_rows(rng, 300, 64)
    X = rng.standard_normal((100, 64))
    a = oracle.mp_encode(X, D, 5, nthreads=1)
    b = oracle.mp_encode(X, D, 5, nthreads=4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


# --- chunked vectors (the s_n of Section "NeuralDict") ---------------------------------------------------

def test_chunked_identity_dictionaries_give_each_chunks_top_coordinates_in_local_numbering():
    rng = np.random.default_rng(11)
    T, sn, dc, s = 40, 4, 8, 3
    X = rng.standard_normal((T, sn * dc))
    # chunk c's dictionary: the unit vectors in an order of its own, so that mixing up dictionaries shows
    perms = [rng.permutation(dc) for _ in range(sn)]
    D = np.stack([np.eye(dc)[perms[c]] for c in range(sn)])          # atom n of chunk c = e_{perm_c[n]}
    idx, coef = oracle.mp_encode_chunked(X, D, s)
    assert idx.shape == coef.shape == (T, sn, s)
    for c in range(sn):
        Xc = X[:, c * dc:(c + 1) * dc]
        top = np.argsort(-np.abs(Xc), axis=1, kind="stable")[:, :s]     # coordinates, largest magnitude first
        inv = np.argsort(perms[c])                                      # coordinate -> atom number
        assert np.array_equal(idx[:, c], inv[top])
        assert np.array_equal(coef[:, c], np.take_along_axis(Xc, top, axis=1))


def test_chunks_are_independent_and_one_chunk_is_the_plain_encoder():
    rng = np.random.default_rng(12)
    T, sn, dc, N, s = 30, 2, 16, 64, 4
    X = rng.standard_normal((T, sn * dc))
    D = np.stack([_unit_rows(rng, N, dc) for _ in range(sn)])
    idx, coef = oracle.mp_encode_chunked(X, D, s)
    X2 = X.copy()
    X2[:, dc:] = rng.standard_normal((T, dc))                           # other values in chunk 1 only
    idx2, coef2 = oracle.mp_encode_chunked(X2, D, s)
    assert np.array_equal(idx[:, 0], idx2[:, 0]) and np.array_equal(coef[:, 0], coef2[:, 0])
    assert not np.array_equal(idx[:, 1], idx2[:, 1])
    # one chunk: the plain encoder with a leading axis of length one
    Dw = _unit_rows(rng, N, sn * dc)
    i1, c1 = oracle.mp_encode_chunked(X, Dw[None], s)
    i0, c0 = oracle.mp_encode(X, Dw, s)
    assert np.array_equal(i1[:, 0], i0) and np.array_equal(c1[:, 0], c0)


def test_chunked_energy_identity_per_chunk_and_error_of_the_concatenation():
    rng = np.random.default_rng(13)
    T, sn, dc, N, s = 25, 2, 32, 128, 6
    X = rng.standard_normal((T, sn * dc))
    D = np.stack([_unit_rows(rng, N, dc) for _ in range(sn)])
    idx, coef = oracle.mp_encode_chunked(X, D, s)
    rec = np.concatenate([oracle.reconstruct(idx[:, c], coef[:, c], D[c]) for c in range(sn)], axis=1)
    # unit atoms: every step removes c^2 from the chunk's squared residual, so the whole vector's error is
    # |x|^2 minus the sum of all squared coefficients
    err = ((X - rec) ** 2).sum(axis=1)
    assert np.allclose(err, (X ** 2).sum(axis=1) - (coef ** 2).sum(axis=(1, 2)), rtol=1e-10, atol=1e-12)
    for c in range(sn):
        Xc = X[:, c * dc:(c + 1) * dc]
        errc = ((Xc - rec[:, c * dc:(c + 1) * dc]) ** 2).sum(axis=1)
        assert np.allclose(errc, (Xc ** 2).sum(axis=1) - (coef[:, c] ** 2).sum(axis=1), rtol=1e-10, atol=1e-12)


# --- Eq.4 with the coefficient as it is stored ("closed loop": Section "Analysis for CSR" stores fp16) -------------

def test_closed_loop_on_the_identity_dictionary_has_a_closed_form():
    # Orthonormal atoms: the residual's coordinates are independent.  x = (1000.3, 0.1, 0, ...): fp16 values near
    # 1000 are 0.5 apart, so the stored first coefficient is 1000.5 and leaves -0.2 on coordinate 0 - more than the
    # 0.1 on coordinate 1.  Closed loop therefore picks atom 0 AGAIN (coefficient fp16(-0.2) = -0.199951171875),
    # then atom 1 (fp16(0.1) = 0.0999755859375); open loop picks atom 1 second and then has nothing left.
    d = 8
    D = np.eye(d)
    x = np.zeros((1, d)); x[0, 0] = 1000.3; x[0, 1] = 0.1
    io, co = oracle.mp_encode(x, D, 3)
    assert io[0].tolist() == [0, 1, 0] and co[0, 0] == pytest.approx(1000.3) and co[0, 1] == pytest.approx(0.1)
    assert abs(co[0, 2]) < 1e-12
    ic, cc = oracle.mp_encode(x, D, 3, closed_loop="f16")
    assert ic[0].tolist() == [0, 0, 1]
    assert cc[0].tolist() == [1000.5, -0.199951171875, 0.0999755859375]
    # fp32 storage: 1000.3 is not an fp32 value either, but the remainder (3e-5) stays below 0.1
    i32, c32 = oracle.mp_encode(x, D, 3, closed_loop="f32")
    assert i32[0].tolist() == [0, 1, 0] and c32[0, 0] == float(np.float32(1000.3)) and c32[0, 1] == float(np.float32(0.1))
    assert c32[0, 2] == float(np.float32(1000.3 - float(np.float32(1000.3))))


@pytest.mark.parametrize("storage,np_t", [("f16", np.float16), ("f32", np.float32)])
def test_closed_loop_residual_is_the_error_of_the_stored_code(storage, np_t):
    # What closed loop is for: x - sum_g c_g d_{i_g}, with the coefficients exactly as returned (= as stored), equals
    # the residual the iterations worked on; every returned coefficient is a value of the storage type; and each
    # step is still the greedy pick (largest |R . d_n|) on that residual.  Open loop with rounding applied
    # afterwards does not have the first property.
    rng = np.random.default_rng(5)
    N, d, s, T = 48, 12, 5, 30
    D = _unit_rows(rng, N, d)
    X = rng.standard_normal((T, d)) * 37.0
    idx, coef, diag = oracle.mp_encode(X, D, s, diagnostics=True, closed_loop=storage)
    assert np.array_equal(coef, coef.astype(np_t).astype(np.float64))
    R = X.copy()
    for g in range(s):
        C = R @ D.T
        n = np.argmax(np.abs(C), axis=1)
        assert np.array_equal(n, idx[:, g])
        c = C[np.arange(T), n]
        assert np.array_equal(coef[:, g], c.astype(np_t).astype(np.float64))       # the projection, rounded
        assert np.allclose((R ** 2).sum(axis=1), diag["res_norm2"][:, g], rtol=1e-12)
        R = R - coef[:, g:g + 1] * D[n]
    assert np.allclose((R ** 2).sum(axis=1), diag["res_norm2"][:, s], rtol=1e-12)
    io, co = oracle.mp_encode(X, D, s)
    stored_open = co.astype(np_t).astype(np.float64)
    R_open = X - np.einsum("tg,tgk->tk", stored_open, D[io])
    if storage == "f16":   # rounding after the fact leaves an error the open-loop residual does not know about
        _, _, dopen = oracle.mp_encode(X, D, s, diagnostics=True)
        assert np.abs((R_open ** 2).sum(axis=1) - dopen["res_norm2"][:, s]).max() > 1e-6


def test_closed_loop_equals_open_loop_when_every_coefficient_is_a_storage_value():
    # identity dictionary and fp16 inputs: every coefficient is a coordinate of x, already an fp16 value
    rng = np.random.default_rng(6)
    X = rng.standard_normal((50, 16)).astype(np.float16).astype(np.float64)
    D = np.eye(16)
    io, co = oracle.mp_encode(X, D, 6)
    ic, cc = oracle.mp_encode(X, D, 6, closed_loop="f16")
    assert np.array_equal(io, ic) and np.array_equal(co, cc)


def test_fp16_rounding_of_the_oracle_matches_the_formats_definition():
    # round_to_half is only reachable through closed loop: one atom, one step, c = x . d = x
    vals = np.array([1.0, 1.00048828125, 1.000732421875, 2049.0, 2051.0, 65519.0, 65520.0, 6.1e-5, 5.9e-8, 2.9e-8, 3.1e-8,
                     -0.1, 1e-9, 0.333333333])
    _, c = oracle.mp_encode(vals[:, None], np.ones((1, 1)), 1, closed_loop="f16")
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).astype(np.float64)          # numpy's own binary16 conversion (ties to even)
    assert np.array_equal(c[:, 0], want)
    assert want[1] == 1.0 and want[3] == 2048.0 and want[4] == 2052.0 and np.isinf(want[6]) and want[5] == 65504.0
