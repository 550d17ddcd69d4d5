"""Pins for the oracle's Hessian, damped inverse and salience (Eq. 3, Def. 1, Alg. 1 lines 1-2,
Theorem 1 and its proof).  None of these tests re-types the oracle's own formula: they use
closed forms, brute force, a different library route, or invariants."""
import numpy as np
import pytest

from oracle import slim_oracle as orc


def _rand_x(m, t, seed, outlier=None):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((m, t))
    if outlier is not None:
        X[outlier] *= 30.0
    return X


def test_gram_brute_force_and_chunking():
    m, t = 7, 23
    X = _rand_x(m, t, 0).astype(np.float16)
    G = np.zeros((m, m))
    orc.gram_accumulate(G, X[:, :10])
    orc.gram_accumulate(G, X[:, 10:])
    ref = np.zeros((m, m))
    for i in range(m):
        for j in range(m):
            for s in range(t):
                ref[i, j] += float(X[i, s]) * float(X[j, s])
    assert np.allclose(G, ref, rtol=1e-13, atol=1e-13)
    H = orc.hessian_from_gram(G, t)
    assert np.allclose(H * t / 2.0, ref, rtol=1e-13)


def test_inverse_defining_identities():
    m, t = 48, 400
    X = _rand_x(m, t, 1, outlier=5)
    G = X @ X.T
    U, d, lam = orc.hessian_inverse(G, t, 0.01)
    H = 2.0 / t * G
    assert lam == pytest.approx(0.01 * np.trace(H) / m, rel=1e-14)
    Hd = H + lam * np.eye(m)
    # U upper triangular with positive diagonal, and U^T U (H + lam I) = I
    assert np.all(np.tril(U, -1) == 0.0)
    assert np.all(np.diag(U) > 0)
    assert np.max(np.abs(U.T @ U @ Hd - np.eye(m))) < 1e-10
    # different library route: explicit inverse, then numpy's (lower) Cholesky transposed
    Hinv = np.linalg.inv(Hd)
    assert np.allclose(d, np.diag(Hinv), rtol=1e-10)
    U2 = np.linalg.cholesky(Hinv).T      # Hinv = L L^T  =>  U = L^T
    assert np.allclose(U, U2, rtol=1e-9, atol=1e-12)
    # a transposed / lower-factor mistake would break this: the LAST row of U is
    # e_m^T * sqrt(Hinv_mm), the first row is generally dense
    assert np.count_nonzero(U[-1]) == 1 and np.count_nonzero(U[0]) == m


def test_inverse_diagonal_closed_form():
    m, t = 16, 64
    rng = np.random.default_rng(2)
    diagG = rng.uniform(1.0, 50.0, m)
    G = np.diag(diagG)
    U, d, lam = orc.hessian_inverse(G, t, 0.01)
    h = 2.0 / t * diagG
    lam_ref = 0.01 * h.mean()
    assert np.allclose(np.diag(U), (h + lam_ref) ** -0.5, rtol=1e-13)
    assert np.allclose(d, 1.0 / (h + lam_ref), rtol=1e-13)
    assert np.allclose(U, np.diag(np.diag(U)))


def test_inverse_scale_of_h_only_rescales_u():
    # H -> c H (c a power of two) gives U -> U / sqrt(c): damping is relative, nothing else moves
    m, t = 24, 200
    X = _rand_x(m, t, 3)
    G = X @ X.T
    U1, d1, _ = orc.hessian_inverse(G, t, 0.01)
    U4, d4, _ = orc.hessian_inverse(4.0 * G, t, 0.01)
    assert np.allclose(U4, U1 / 2.0, rtol=1e-12, atol=0)
    assert np.allclose(d4, d1 / 4.0, rtol=1e-12)


def test_inverse_rejects_indefinite():
    m = 6
    G = np.eye(m)
    G[2, 2] = -1.0
    with pytest.raises(np.linalg.LinAlgError):
        orc.hessian_inverse(G, 10, 0.0)
    # a dead channel without damping is singular
    G = np.eye(m)
    G[3, 3] = 0.0
    with pytest.raises(np.linalg.LinAlgError):
        orc.hessian_inverse(G, 10, 0.0)


def test_salience_diagonal_closed_form_and_group_mean():
    # Def. 1 with a diagonal H: delta_ij = w_ij^2 (H_jj + lam)^2
    n, m, beta, t = 5, 12, 4, 10
    rng = np.random.default_rng(4)
    W = rng.standard_normal((n, m))
    diagG = rng.uniform(1.0, 9.0, m)
    U, d, lam = orc.hessian_inverse(np.diag(diagG), t, 0.01)
    col, grp, elem = orc.salience(W, d, beta)
    h = 2.0 / t * diagG + lam
    ref = np.empty((n, m))
    for i in range(n):
        for j in range(m):
            ref[i, j] = W[i, j] ** 2 * h[j] ** 2
    assert np.allclose(elem, ref, rtol=1e-12)
    for j in range(m):
        assert col[j] == pytest.approx(sum(ref[i, j] for i in range(n)), rel=1e-12)
    for g in range(m // beta):
        vals = [ref[i, j] for i in range(n) for j in range(g * beta, (g + 1) * beta)]
        assert grp[g] == pytest.approx(sum(vals) / len(vals), rel=1e-12)
    # the mode that reads Alg. 2's [H^in]_diag literally divides by U_jj^2 = 1/(H_jj+lam)
    col2, grp2, elem2 = orc.salience(W, d, beta, U=U, sal_mode=orc.SAL_CHOL_DIAG)
    assert np.allclose(elem2, W ** 2 * h[None, :], rtol=1e-12)


def test_salience_appendix_approximation():
    # Proof of Theorem 1: for small damping and nearly diagonal x^T x,
    # delta_ij ~ (w_ij * ||x_j||^2)^2 up to the constant scale of H (here (2/T)^2).
    n, m, beta, t = 4, 8, 4, 200000
    rng = np.random.default_rng(5)
    X = rng.standard_normal((m, t)) * rng.uniform(0.5, 3.0, m)[:, None]
    W = rng.standard_normal((n, m))
    G = X @ X.T
    U, d, lam = orc.hessian_inverse(G, t, 1e-9)
    _, _, elem = orc.salience(W, d, beta)
    approx = (W * (2.0 / t) * np.sum(X * X, axis=1)[None, :]) ** 2
    assert np.allclose(elem, approx, rtol=0.05)


def test_theorem1_outlier_channel_is_most_salient():
    n, m, beta, t = 32, 64, 8, 4096
    p = 37
    X = _rand_x(m, t, 6, outlier=p)
    rng = np.random.default_rng(7)
    W = rng.standard_normal((n, m)) * 0.02
    G = X @ X.T
    assert np.argmax(np.diag(G)) == p
    U, d, lam = orc.hessian_inverse(G, t, 0.01)
    col, grp, _ = orc.salience(W, d, beta)
    assert np.argmax(col) == p
    assert np.argmax(grp) == p // beta
