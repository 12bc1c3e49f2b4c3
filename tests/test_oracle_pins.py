"""Pins for the CPU oracle: every part of it is checked against something other than itself --
closed forms, brute force, library routines, invariants (Sections 1 eq. (1), 3.1, 3.2)."""
import math

import numpy as np
import pytest
import scipy.optimize
import scipy.sparse as sp

import oracle
from oracle import Matrix

pytestmark = pytest.mark.usefixtures("oracle_lib")
rng = np.random.default_rng(12345)


def dense_to_csc(X):
    S = sp.csc_matrix(X)
    S.sort_indices()
    return Matrix("csc", X.shape[0], X.shape[1], S.indptr.astype(np.int64), S.indices.astype(np.int32),
                  S.data.astype(np.float32))


def dense_to_csr(X):
    S = sp.csr_matrix(X)
    S.sort_indices()
    return Matrix("csr", X.shape[0], X.shape[1], S.indptr.astype(np.int64), S.indices.astype(np.int32),
                  S.data.astype(np.float32))


def dense_colmajor(X):
    return Matrix("dense_colmajor", X.shape[0], X.shape[1], None, None,
                  np.ascontiguousarray(X.T, dtype=np.float32).reshape(-1))


def sparse_random(n, d, density, r):
    X = r.standard_normal((n, d)) * (r.random((n, d)) < density)
    return X.astype(np.float32).astype(np.float64)


# independent numpy definitions of the objectives (written from eq. (1) with the 1/n scaling)
def P_ridge(X, y, w, lam):
    return 0.5 * np.mean((X @ w - y) ** 2) + 0.5 * lam * w @ w


def P_logistic(X, y, w, lam):
    return np.mean(np.logaddexp(0.0, -y * (X @ w))) + 0.5 * lam * w @ w


def P_hinge(X, y, w, lam):
    return np.mean(np.maximum(0.0, 1 - y * (X @ w))) + 0.5 * lam * w @ w


def ridge_closed_form(X, y, lam):
    n, d = X.shape
    return np.linalg.solve(X.T @ X / n + lam * np.eye(d), X.T @ y / n)


# ---------------------------------------------------------------------------------------------
# ridge
@pytest.mark.parametrize("layout", ["csc", "dense"])
def test_ridge_converges_to_normal_equations(layout):
    n, d, lam = 60, 7, 0.05
    X = sparse_random(n, d, 0.6, rng)
    y = rng.standard_normal(n).astype(np.float32)
    A = dense_to_csc(X) if layout == "csc" else dense_colmajor(X)
    s = oracle.solve(A, y, "ridge", lam, epochs=400)
    wstar = ridge_closed_form(X, y.astype(np.float64), lam)
    np.testing.assert_allclose(s.weights(), wstar, rtol=0, atol=1e-10)
    assert abs(s.primal() - P_ridge(X, y, wstar, lam)) < 1e-13
    np.testing.assert_allclose(s.v, X @ s.x, atol=1e-12)


def test_ridge_single_feature_one_update_is_exact():
    a = np.array([[1.5], [-2.0], [0.5], [3.0]], dtype=np.float32)
    y = np.array([1.0, 0.5, -1.0, 2.0], dtype=np.float32)
    lam, n = 0.3, 4
    s = oracle.solve(dense_to_csc(a.astype(np.float64)), y, "ridge", lam, epochs=1)
    expect = (a[:, 0].astype(np.float64) @ y / n) / (a[:, 0].astype(np.float64) @ a[:, 0] / n + lam)
    assert s.x[0] == pytest.approx(expect, rel=1e-15)


def test_ridge_objective_never_increases_per_update():
    n, d, lam = 40, 12, 0.01
    X = sparse_random(n, d, 0.5, rng)
    y = rng.standard_normal(n).astype(np.float32)
    A = dense_to_csc(X)
    s = oracle.Solver(A, y, "ridge", lam)
    lib = oracle.lib()
    import ctypes as C
    prev = P_ridge(X, y, s.x, lam)
    for e in range(3):
        perm = oracle.permutation(e, d)
        for k in range(d):
            one = perm[k:k + 1].copy()
            lib.oracle_epoch_primal_sparse(C.c_int(0), C.c_int64(n), oracle._p(A.ptr), oracle._p(A.idx),
                                           oracle._p(A.val), oracle._p(s.y), C.c_double(lam), C.c_double(0.0),
                                           oracle._p(one),
                                           C.c_int64(0), C.c_int64(1), oracle._p(s.x), oracle._p(s.v))
            cur = P_ridge(X, y, s.x, lam)
            assert cur <= prev + 1e-15
            # exact coordinate minimiser: the partial derivative along that coordinate vanishes
            j = int(one[0])
            gj = X[:, j] @ (X @ s.x - y) / n + lam * s.x[j]
            assert abs(gj) < 1e-14
            prev = cur


@pytest.mark.parametrize("seed", [0, 1, 7])
def test_ridge_orthogonal_columns_converge_in_one_epoch(seed):
    n, d, lam = 30, 10, 0.2
    X = np.zeros((n, d))
    X[np.arange(n), np.arange(n) % d] = rng.standard_normal(n).astype(np.float32)  # one nonzero per row
    y = rng.standard_normal(n).astype(np.float32)
    s = oracle.solve(dense_to_csc(X), y, "ridge", lam, epochs=1, seed0=seed)
    np.testing.assert_allclose(s.x, ridge_closed_form(X, y.astype(np.float64), lam), atol=1e-14)


def test_ridge_config2_slice_against_normal_equations():
    import datagen
    p = datagen.dense_ridge(n=2000, d=200)
    A = Matrix.from_problem(p)
    y = p.y.numpy()
    s = oracle.solve(A, y, "ridge", p.lam, epochs=3000, tol=1e-14)
    X = A.to_dense()
    wstar = ridge_closed_form(X, y.astype(np.float64), p.lam)
    assert abs(s.primal() - P_ridge(X, y, wstar, p.lam)) <= 1e-9 * P_ridge(X, y, wstar, p.lam)
    assert np.linalg.norm(s.x - wstar) <= 1e-3 * np.linalg.norm(wstar)


# ---------------------------------------------------------------------------------------------
# logistic
def test_logistic_single_feature_newton_vs_bisection():
    a = np.array([0.5, -1.0, 2.0, 1.0, -0.7], dtype=np.float32).astype(np.float64)
    y = np.array([1, 1, -1, 1, -1], dtype=np.float32)
    lam, n = 0.1, 5
    dP = lambda w: np.mean(-y * a / (1 + np.exp(y * a * w))) + lam * w
    root = scipy.optimize.brentq(dP, -50, 50, xtol=1e-15, rtol=1e-15)
    A = dense_to_csc(a.reshape(-1, 1))
    s = oracle.Solver(A, y, "logistic", lam)
    errs = []
    for e in range(8):
        s.epoch(e)
        errs.append(abs(s.x[0] - root))
    assert errs[-1] < 1e-14
    # Newton's quadratic convergence: error_{k+1} <= C error_k^2 once close
    k = next(i for i, e in enumerate(errs) if e < 1e-2)
    assert errs[k + 1] < 10 * errs[k] ** 2 + 1e-15
    # the first step from w = 0 is -g/h with p = 1/2 everywhere
    s1 = oracle.solve(A, y, "logistic", lam, epochs=1)
    assert s1.x[0] == pytest.approx(-(np.mean(-y * a * 0.5) / (np.mean(a * a * 0.25) + lam)), rel=1e-14)


def test_logistic_two_features_brute_force():
    n, lam = 25, 0.05
    X = rng.standard_normal((n, 2)).astype(np.float32).astype(np.float64)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    s = oracle.solve(dense_to_csc(X), y, "logistic", lam, epochs=200)
    g = np.linspace(-3, 3, 601)
    W0, W1 = np.meshgrid(g, g, indexing="ij")
    Z = X[:, 0][:, None, None] * W0 + X[:, 1][:, None, None] * W1
    Pgrid = np.mean(np.logaddexp(0, -y[:, None, None] * Z), axis=0) + 0.5 * lam * (W0 ** 2 + W1 ** 2)
    i, j = np.unravel_index(np.argmin(Pgrid), Pgrid.shape)
    assert abs(s.x[0] - g[i]) <= 0.011 and abs(s.x[1] - g[j]) <= 0.011
    assert s.primal() <= Pgrid.min() + 1e-12
    assert s.primal() == pytest.approx(P_logistic(X, y, s.x, lam), rel=1e-13)


@pytest.mark.parametrize("layout", ["csc", "dense"])
def test_logistic_against_quasi_newton(layout):
    n, d, lam = 200, 15, 0.01
    X = sparse_random(n, d, 0.4, rng)
    y = np.where(X @ rng.standard_normal(d) + 0.3 * rng.standard_normal(n) > 0, 1.0, -1.0).astype(np.float32)
    A = dense_to_csc(X) if layout == "csc" else dense_colmajor(X)
    s = oracle.solve(A, y, "logistic", lam, epochs=500, tol=1e-15)
    f = lambda w: P_logistic(X, y, w, lam)
    gr = lambda w: X.T @ (-y / (1 + np.exp(y * (X @ w)))) / n + lam * w
    r = scipy.optimize.minimize(f, np.zeros(d), jac=gr, method="L-BFGS-B", options={"ftol": 1e-16, "gtol": 1e-12,
                                                                                      "maxiter": 5000})
    assert np.max(np.abs(gr(s.x))) < 1e-8          # gradient computed independently vanishes
    assert abs(s.primal() - r.fun) < 1e-10
    np.testing.assert_allclose(s.x, r.x, atol=2e-5)
    np.testing.assert_allclose(s.v, X @ s.x, atol=1e-11)


def test_logistic_extreme_margins_are_finite():
    X = np.array([[800.0], [-800.0]])
    y = np.array([1.0, -1.0], dtype=np.float32)
    s = oracle.Solver(dense_to_csc(X), y, "logistic", 1e-3)
    s.x[:] = 5.0
    s.v[:] = X[:, 0] * 5.0
    assert np.isfinite(s.primal()) and np.isfinite(s.gap()) and np.isfinite(s.gap("fenchel"))
    s.x[:] = -5.0
    s.v[:] = X[:, 0] * -5.0
    assert s.primal() == pytest.approx(4000.0 + 0.5e-3 * 25, rel=1e-12)
    s.epoch(0)
    assert np.all(np.isfinite(s.x))


# ---------------------------------------------------------------------------------------------
# hinge (dual)
def test_hinge_single_example_closed_form():
    for scale, lam in [(1.0, 0.5), (3.0, 0.5), (0.2, 2.0)]:
        x = np.array([[0.6 * scale, -0.8 * scale]], dtype=np.float32)
        s = oracle.solve(dense_to_csr(x.astype(np.float64)), np.array([1.0], dtype=np.float32), "hinge", lam, epochs=1)
        nrm = float(x.astype(np.float64)[0] @ x.astype(np.float64)[0])
        assert s.x[0] == pytest.approx(min(1.0, max(0.0, lam * 1 / nrm)), rel=1e-12)


def test_hinge_box_monotone_and_weak_duality():
    n, d, lam = 50, 6, 0.02
    X = sparse_random(n, d, 0.7, rng)
    X[3, :] = 0.0   # an empty row
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    A = dense_to_csr(X)
    s = oracle.Solver(A, y, "hinge", lam)
    import ctypes as C
    lib = oracle.lib()
    prevD = s.dual()
    assert prevD == 0.0
    for e in range(4):
        perm = oracle.permutation(e, n)
        for k in range(n):
            one = perm[k:k + 1].copy()
            lib.oracle_epoch_dual_hinge(C.c_int64(n), oracle._p(A.ptr), oracle._p(A.idx), oracle._p(A.val),
                                        oracle._p(s.y), C.c_double(lam), oracle._p(one), C.c_int64(0),
                                        C.c_int64(1), oracle._p(s.x), oracle._p(s.v))
            assert s.x.min() >= 0.0 and s.x.max() <= 1.0
            D = s.dual()
            assert D >= prevD - 1e-15
            prevD = D
        P, D = s.primal_dual()
        w = s.weights()
        assert P == pytest.approx(P_hinge(X, y, w, lam), rel=1e-13)
        assert D == pytest.approx(np.mean(s.x) - 0.5 * lam * w @ w, rel=1e-13, abs=1e-15)
        assert P >= D - 1e-15
        np.testing.assert_allclose(s.v, X.T @ (y * s.x), atol=1e-12)
    assert s.x[3] == 1.0


def test_hinge_two_features_brute_force():
    n, lam = 30, 0.1
    X = rng.standard_normal((n, 2)).astype(np.float32).astype(np.float64)
    y = np.where(X @ np.array([1.0, -0.5]) + 0.5 * rng.standard_normal(n) > 0, 1.0, -1.0).astype(np.float32)
    s = oracle.solve(dense_to_csr(X), y, "hinge", lam, epochs=3000, tol=1e-13)
    g = np.linspace(-4, 4, 801)
    W0, W1 = np.meshgrid(g, g, indexing="ij")
    Z = X[:, 0][:, None, None] * W0 + X[:, 1][:, None, None] * W1
    Pgrid = np.mean(np.maximum(0, 1 - y[:, None, None] * Z), axis=0) + 0.5 * lam * (W0 ** 2 + W1 ** 2)
    i, j = np.unravel_index(np.argmin(Pgrid), Pgrid.shape)
    P, D = s.primal_dual()
    assert P - D < 1e-10
    assert P <= Pgrid.min() + 1e-12 and P >= Pgrid.min() - 1e-3
    w = s.weights()
    assert abs(w[0] - g[i]) <= 0.02 and abs(w[1] - g[j]) <= 0.02


# ---------------------------------------------------------------------------------------------
# duality gap
@pytest.mark.parametrize("loss", ["ridge", "logistic"])
def test_gap_forms_agree_closed_form_at_zero_and_bounds(loss):
    n, d, lam = 80, 9, 0.03
    X = sparse_random(n, d, 0.5, rng)
    y = (rng.standard_normal(n) if loss == "ridge" else np.where(rng.random(n) < 0.4, 1.0, -1.0)).astype(np.float32)
    A = dense_to_csc(X)
    s = oracle.Solver(A, y, loss, lam)
    g0 = np.linalg.norm(X.T @ y) ** 2 / (2 * lam * n * n) / (1.0 if loss == "ridge" else 4.0)
    assert s.gap() == pytest.approx(g0, rel=1e-12)
    assert s.gap("fenchel") == pytest.approx(g0, rel=1e-10)
    if loss == "ridge":
        Pstar = P_ridge(X, y, ridge_closed_form(X, y.astype(np.float64), lam), lam)
    else:
        Pstar = oracle.solve(A, y, loss, lam, epochs=2000, tol=1e-15).primal()
    last = None
    for e in range(30):
        s.epoch(e)
        G, Gf = s.gap(), s.gap("fenchel")
        assert G >= 0 and abs(G - Gf) <= 1e-9 * max(1.0, G)
        assert G >= s.primal() - Pstar - 1e-12
        last = G
    assert last < 1e-8 * g0


def test_gap_hinge_goes_to_zero_and_bounds_suboptimality():
    n, d, lam = 60, 5, 0.05
    X = sparse_random(n, d, 0.8, rng)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    A = dense_to_csr(X)
    ref = oracle.solve(A, y, "hinge", lam, epochs=5000, tol=1e-14)
    Dstar = ref.dual()
    s = oracle.Solver(A, y, "hinge", lam)
    assert s.gap() == pytest.approx(1.0, rel=1e-15)      # alpha = 0: P = 1, D = 0
    for e in range(200):
        s.epoch(e)
        assert s.gap() >= Dstar - s.dual() - 1e-12
    assert s.gap() < 1e-6


# ---------------------------------------------------------------------------------------------
# products
@pytest.mark.parametrize("layout", ["csr", "csc", "dense"])
def test_products_against_dense_and_scipy(layout):
    n, d = 37, 23
    X = sparse_random(n, d, 0.3, rng)
    A = {"csr": dense_to_csr, "csc": dense_to_csc, "dense": dense_colmajor}[layout](X)
    x, u = rng.standard_normal(d), rng.standard_normal(n)
    np.testing.assert_allclose(A.matvec(x), X @ x, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(A.rmatvec(u), X.T @ u, rtol=1e-13, atol=1e-13)
    assert u @ A.matvec(x) == pytest.approx(x @ A.rmatvec(u), rel=1e-12)
    np.testing.assert_allclose(A.to_dense(), X)


def test_products_medium_against_scipy():
    S = sp.random(3000, 800, density=0.01, format="csr", random_state=3, dtype=np.float32)
    S.sort_indices()
    A = Matrix("csr", 3000, 800, S.indptr.astype(np.int64), S.indices.astype(np.int32), S.data)
    x = rng.standard_normal(800)
    np.testing.assert_allclose(A.matvec(x), S.astype(np.float64) @ x, rtol=1e-12, atol=1e-12)
    Sc = S.tocsc()
    Sc.sort_indices()
    Ac = Matrix("csc", 3000, 800, Sc.indptr.astype(np.int64), Sc.indices.astype(np.int32), Sc.data)
    np.testing.assert_allclose(Ac.matvec(x), S.astype(np.float64) @ x, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------------------------------------
# streaming order: chunks in sequence, permutation inside each chunk (Section 3.2)
def test_chunked_epoch_visits_every_coordinate_once_in_chunk_order():
    n, d, lam = 50, 20, 0.05
    X = sparse_random(n, d, 0.5, rng)
    y = rng.standard_normal(n).astype(np.float32)
    bounds = [0, 7, 12, 20]
    s = oracle.Solver(dense_to_csc(X), y, "ridge", lam, chunk_bounds=bounds)
    s.epoch(3)
    assert sorted(s.last_perm.tolist()) == list(range(d))
    for ch in range(3):
        seg = s.last_perm[bounds[ch]:bounds[ch + 1]]
        assert seg.min() >= bounds[ch] and seg.max() < bounds[ch + 1]
    for e in range(400):
        s.epoch(e)
    np.testing.assert_allclose(s.x, ridge_closed_form(X, y.astype(np.float64), lam), atol=1e-10)


def test_pass_in_a_given_order_is_the_epoch_of_that_order():
    """Solver.visit takes the order from the caller: with the seeded permutation it is Solver.epoch bit
    for bit (every form), and with one coordinate it is that coordinate's exact ridge update."""
    n, d = 60, 25
    X = sparse_random(n, d, 0.4, rng)
    y = np.sign(rng.standard_normal(n)).astype(np.float32)
    for A, loss in [(dense_to_csc(X), "ridge"), (dense_to_csc(X), "logistic"), (dense_colmajor(X), "ridge"),
                    (dense_to_csr(X), "hinge"), (dense_to_csr(X), "logistic")]:
        a, b = oracle.Solver(A, y, loss, 0.1), oracle.Solver(A, y, loss, 0.1)
        for e in range(3):
            a.epoch(e)
            b.visit(oracle.permutation(e, a.m))
            assert np.array_equal(a.x, b.x) and np.array_equal(a.v, b.v)
            assert np.array_equal(a.last_perm, b.last_perm)
    s = oracle.Solver(dense_to_csc(X), y, "ridge", 0.1)
    s.visit([7])
    a7 = X[:, 7]
    want = (a7 @ y.astype(np.float64) / n) / (a7 @ a7 / n + 0.1)
    assert abs(s.x[7] - want) <= 1e-14 and np.count_nonzero(s.x) == 1
    np.testing.assert_allclose(s.v, a7 * want, atol=1e-15)


def test_shuffled_chunks_visit_every_coordinate_once_and_converge():
    n, d, lam = 50, 20, 0.05
    X = sparse_random(n, d, 0.5, rng)
    y = rng.standard_normal(n).astype(np.float32)
    bounds = [0, 3, 7, 12, 16, 20]
    s = oracle.Solver(dense_to_csc(X), y, "ridge", lam, chunk_bounds=bounds, shuffle_chunks=True)
    orders = set()
    for e in range(12):
        s.epoch(e)
        assert sorted(s.last_perm.tolist()) == list(range(d))
        # chunks stay contiguous in the visiting order, and their order is the sorted-key order
        first = [int(np.searchsorted(bounds, c, side="right") - 1) for c in s.last_perm]
        seq = [k for i, k in enumerate(first) if i == 0 or first[i - 1] != k]
        assert sorted(seq) == list(range(5))
        assert seq == oracle.permutation(e, 5, chunk=0xFFFFFFFF).tolist()
        orders.add(tuple(seq))
    assert len(orders) > 3
    for e in range(400):
        s.epoch(e)
    np.testing.assert_allclose(s.x, ridge_closed_form(X, y.astype(np.float64), lam), atol=1e-10)


# ---------------------------------------------------------------------------------------------
# l1 / elastic-net term of the primal forms:  P(w) = (1/n) sum loss + (lam/2)||w||^2 + lam1 ||w||_1
def kkt_violation(gf, w, lam, lam1):
    """Distance of 0 from the subdifferential of P at w; gf = gradient of the loss term."""
    r = gf + lam * w
    nz = w != 0
    out = np.zeros_like(w)
    out[nz] = np.abs(r[nz] + lam1 * np.sign(w[nz]))
    out[~nz] = np.maximum(np.abs(r[~nz]) - lam1, 0.0)
    return float(out.max())


@pytest.mark.parametrize("layout", ["csc", "dense"])
def test_elastic_net_ridge_loss_against_sklearn(layout):
    from sklearn.linear_model import ElasticNet
    n, d, lam, lam1 = 120, 15, 0.02, 0.05
    X = sparse_random(n, d, 0.5, rng)
    wtrue = rng.standard_normal(d) * (rng.random(d) < 0.4)
    y = (X @ wtrue + 0.1 * rng.standard_normal(n)).astype(np.float32)
    A = dense_to_csc(X) if layout == "csc" else dense_colmajor(X)
    s = oracle.solve(A, y, "ridge", lam, epochs=600, lam1=lam1)
    # sklearn: 1/(2n)||y - Xw||^2 + alpha*l1_ratio*||w||_1 + alpha*(1-l1_ratio)/2*||w||^2
    alpha = lam + lam1
    ref = ElasticNet(alpha=alpha, l1_ratio=lam1 / alpha, fit_intercept=False, tol=1e-14, max_iter=100000)
    ref.fit(X, y.astype(np.float64))
    np.testing.assert_allclose(s.weights(), ref.coef_, atol=1e-9)
    assert np.sum(s.weights() == 0.0) == np.sum(ref.coef_ == 0.0) > 0        # exact zeros, same support
    P = P_ridge(X, y, s.weights(), lam) + lam1 * np.abs(s.weights()).sum()
    assert s.primal() == pytest.approx(P, rel=1e-13)


def test_elastic_net_one_update_minimises_the_coordinate_problem():
    # ridge loss: the step is the exact minimiser along the coordinate -- check against a fine scan
    n, d, lam, lam1 = 30, 4, 0.1, 0.08
    X = sparse_random(n, d, 0.9, rng)
    y = rng.standard_normal(n).astype(np.float32)
    s = oracle.Solver(dense_to_csc(X), y, "ridge", lam, lam1=lam1)
    s.x[:] = rng.standard_normal(d)
    s.v[:] = X @ s.x
    w0 = s.x.copy()
    s.epoch(3)
    j0 = int(s.last_perm[0])

    def P(w):
        return P_ridge(X, y, w, lam) + lam1 * np.abs(w).sum()
    # replay the epoch coordinate by coordinate with a golden-section search on the 1-D problem
    w = w0.copy()
    for j in s.last_perm:
        f = lambda t: P(np.concatenate([w[:j], [t], w[j + 1:]]))
        t = scipy.optimize.minimize_scalar(f, bracket=(-3, 3), tol=1e-14).x
        cand = [t, 0.0]                                     # the kink at 0 may be the minimiser
        w[j] = min(cand, key=f)
    np.testing.assert_allclose(s.x, w, atol=2e-7)
    assert j0 in range(d)


def test_l1_large_enough_gives_the_zero_model():
    n, d, lam = 50, 6, 0.01
    X = sparse_random(n, d, 0.7, rng)
    y = rng.standard_normal(n).astype(np.float32)
    lam1 = 1.0001 * np.abs(X.T @ y).max() / n               # ridge loss: gradient at 0 is -X^T y / n
    s = oracle.solve(dense_to_csc(X), y, "ridge", lam, epochs=3, lam1=lam1)
    assert np.all(s.weights() == 0.0) and np.all(s.v == 0.0)
    yl = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    lam1 = 1.0001 * np.abs(X.T @ yl).max() / (2 * n)         # logistic: gradient at 0 is -X^T y / (2n)
    s = oracle.solve(dense_to_csc(X), yl, "logistic", lam, epochs=3, lam1=lam1)
    assert np.all(s.weights() == 0.0)
    s = oracle.solve(dense_to_csc(X), yl, "logistic", lam, epochs=3, lam1=0.5 * lam1)
    assert np.any(s.weights() != 0.0)


@pytest.mark.parametrize("loss", ["ridge", "logistic"])
def test_elastic_net_kkt_and_gap(loss):
    n, d, lam, lam1 = 90, 12, 0.02, 0.03
    X = sparse_random(n, d, 0.5, rng)
    y = (rng.standard_normal(n) if loss == "ridge" else np.where(rng.random(n) < 0.45, 1.0, -1.0)).astype(np.float32)
    A = dense_to_csc(X)
    s = oracle.Solver(A, y, loss, lam, lam1=lam1)
    # gap at w = 0: u = grad f(0), P + f*(u) = 0 for both losses, so the gap is sum_j g*(x_j.u)
    gf0 = -X.T @ y / n / (1.0 if loss == "ridge" else 2.0)
    g0 = np.sum(np.maximum(np.abs(gf0) - lam1, 0.0) ** 2) / (2 * lam)
    assert s.gap() == pytest.approx(g0, rel=1e-10)
    ref = oracle.solve(A, y, loss, lam, epochs=3000, tol=1e-16, lam1=lam1)
    w = ref.weights()
    z = X @ w
    gf = X.T @ ((z - y) if loss == "ridge" else (-y / (1 + np.exp(y * z)))) / n
    assert kkt_violation(gf, w, lam, lam1) < 1e-9          # entries of gf are ~3e-2
    assert 0 < np.sum(w == 0.0) < d
    Pfun = P_ridge if loss == "ridge" else P_logistic
    Pstar = Pfun(X, y, w, lam) + lam1 * np.abs(w).sum()
    assert ref.primal() == pytest.approx(Pstar, rel=1e-13)
    # a perturbed model has a larger objective (w is the minimiser, not just a stationary point)
    for _ in range(20):
        wp = w + 1e-3 * rng.standard_normal(d)
        assert Pfun(X, y, wp, lam) + lam1 * np.abs(wp).sum() > Pstar
    last = None
    for e in range(40):
        s.epoch(e)
        G = s.gap()
        assert G >= s.primal() - Pstar - 1e-12
        last = G
    assert -1e-14 <= last < 1e-8 * g0                      # P + D* cancels to rounding at the optimum


def test_l1_zero_reproduces_the_plain_step_and_dual_form_rejects_it():
    n, d, lam = 40, 5, 0.05
    X = sparse_random(n, d, 0.6, rng)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    a = oracle.solve(dense_to_csc(X), y, "logistic", lam, epochs=5)
    b = oracle.solve(dense_to_csc(X), y, "logistic", lam, epochs=5, lam1=1e-300)   # takes the thresholded branch
    np.testing.assert_allclose(a.x, b.x, rtol=0, atol=1e-15)
    with pytest.raises(ValueError):
        oracle.Solver(dense_to_csr(X), y, "hinge", lam, lam1=0.1)


# ---------------------------------------------------------------------------------------------
# logistic regression in the dual form (examples as coordinates)
def D_logistic(X, y, alpha, lam):
    """Independent numpy definition of the logistic dual (conjugate of log(1+exp(-z)) is the entropy)."""
    n = X.shape[0]
    w = X.T @ (y * alpha) / (lam * n)
    ent = np.sum(alpha * np.log(alpha) + (1 - alpha) * np.log1p(-alpha))
    return -ent / n - 0.5 * lam * w @ w


def test_dual_logistic_start_and_one_newton_step():
    n, d, lam = 12, 4, 0.1
    X = sparse_random(n, d, 0.8, rng)
    y = np.where(rng.random(n) < 0.5, 1.0, -1.0).astype(np.float32)
    s = oracle.Solver(dense_to_csr(X), y, "logistic", lam)
    assert s.form == "dual" and np.all(s.x == 0.5)
    np.testing.assert_allclose(s.v, X.T @ (0.5 * y), atol=1e-14)
    assert s.dual() == pytest.approx(D_logistic(X, y, s.x, lam), rel=1e-13)
    a0 = s.x.copy()
    s.epoch(0)
    # replay with derivatives of D taken numerically (central differences), coordinate by coordinate
    a = a0.copy()
    for i in s.last_perm:
        f = lambda t: -n * D_logistic(X, y, np.concatenate([a[:i], [t], a[i + 1:]]), lam)
        e = 1e-5
        g = (f(a[i] + e) - f(a[i] - e)) / (2 * e)
        h = (f(a[i] + e) - 2 * f(a[i]) + f(a[i] - e)) / (e * e)
        a[i] = min(max(a[i] - g / h, 2.0 ** -20), 1 - 2.0 ** -20)
    np.testing.assert_allclose(s.x, a, atol=2e-5)
    np.testing.assert_allclose(s.v, X.T @ (y * s.x), atol=1e-12)


def test_dual_logistic_reaches_the_primal_solution():
    n, d, lam = 80, 6, 0.05
    X = sparse_random(n, d, 0.7, rng)
    wtrue = rng.standard_normal(d)
    y = np.where(X @ wtrue + 0.5 * rng.standard_normal(n) > 0, 1.0, -1.0).astype(np.float32)
    # independent primal solution (quasi-Newton on the numpy objective)
    res = scipy.optimize.minimize(lambda w: P_logistic(X, y, w, lam), np.zeros(d), method="L-BFGS-B",
                                  jac=lambda w: X.T @ (-y / (1 + np.exp(y * (X @ w)))) / n + lam * w,
                                  options={"ftol": 1e-16, "gtol": 1e-12, "maxiter": 5000})
    wstar, Pstar = res.x, res.fun
    s = oracle.Solver(dense_to_csr(X), y, "logistic", lam)
    prev_gap = None
    for e in range(300):
        s.epoch(e)
        P, D = s.primal_dual()
        assert P >= D - 1e-13                                            # weak duality at every iterate
        assert D <= Pstar + 1e-12 and P >= Pstar - 1e-12
        assert s.x.min() >= 2.0 ** -20 and s.x.max() <= 1 - 2.0 ** -20    # stays inside the box
        prev_gap = P - D
    assert prev_gap < 1e-10
    np.testing.assert_allclose(s.weights(), wstar, atol=1e-6)
    assert s.dual() == pytest.approx(Pstar, abs=1e-10)                    # strong duality
    np.testing.assert_allclose(s.x, 1 / (1 + np.exp(y * (X @ wstar))), atol=1e-6)   # alpha* = sigmoid(-y x.w*)
    assert s.dual() == pytest.approx(D_logistic(X, y, s.x, lam), rel=1e-12)
    assert s.primal() == pytest.approx(P_logistic(X, y, s.weights(), lam), rel=1e-12)


def test_dual_logistic_two_examples_brute_force():
    X = np.array([[1.0, 0.5], [-0.75, 1.25]], dtype=np.float32).astype(np.float64)
    y = np.array([1.0, -1.0], dtype=np.float32)
    lam = 0.3
    s = oracle.solve(dense_to_csr(X), y, "logistic", lam, epochs=200)
    g = np.linspace(0.001, 0.999, 999)
    A1, A2 = np.meshgrid(g, g, indexing="ij")
    W = (np.outer(A1.ravel() * y[0], X[0]) + np.outer(A2.ravel() * y[1], X[1])) / (lam * 2)
    ent = A1 * np.log(A1) + (1 - A1) * np.log(1 - A1) + A2 * np.log(A2) + (1 - A2) * np.log(1 - A2)
    Dg = -ent.ravel() / 2 - 0.5 * lam * np.sum(W * W, axis=1)
    k = int(np.argmax(Dg))
    assert abs(s.x[0] - A1.ravel()[k]) <= 0.002 and abs(s.x[1] - A2.ravel()[k]) <= 0.002
    assert s.dual() >= Dg[k] - 1e-12


def test_dual_logistic_well_separated_examples_leave_the_boundary():
    # margins large enough that the first Newton step from 1/2 overshoots and is clipped; the iterates
    # then have to grow back from the clip value to alpha* = sigmoid(-margin)
    n, d, lam = 6, 2, 0.02
    X = np.array([[3.0, 0.0], [2.5, 0.5], [-3.0, 0.2], [0.1, 2.0], [-0.2, -2.5], [2.0, 2.0]])
    y = np.sign(X @ np.array([1.0, 1.0])).astype(np.float32)
    s = oracle.Solver(dense_to_csr(X), y, "logistic", lam)
    s.epoch(0)
    assert np.any(s.x == 2.0 ** -20)
    for e in range(1, 400):
        s.epoch(e)
    w = s.weights()
    np.testing.assert_allclose(s.x, 1 / (1 + np.exp(y * (X @ w))), rtol=1e-6)
    assert s.gap() < 1e-10


# ---------------------------------------------------------------------------------------------
# gap shares of the coordinates / chunks and passes over part of the chunks (Section 3.2: choosing
# the data to process by its share in the duality gap)
@pytest.mark.parametrize("loss,lam1", [("ridge", 0.0), ("logistic", 0.0), ("ridge", 3e-3), ("logistic", 2e-3)])
def test_gap_shares_add_up_to_the_gap_and_are_nonnegative(loss, lam1):
    r = np.random.default_rng(77)
    X = sparse_random(300, 40, 0.3, r)
    y = (np.sign(r.standard_normal(300)) if loss == "logistic" else r.standard_normal(300)).astype(np.float32)
    s = oracle.Solver(dense_to_csc(X), y, loss, 1e-2, chunk_bounds=[0, 7, 19, 40], lam1=lam1)
    for e in range(3):
        s.epoch(e)
        share = oracle.primal_gap_shares(s.A, s.loss, s.v, s.y, s.x, s.lam, s.lam1)
        assert share.min() >= -1e-15
        assert abs(share.sum() - s.gap("fenchel")) <= 1e-12 * max(1.0, abs(s.primal()))
        if lam1 == 0.0:
            assert abs(share.sum() - s.gap("gradient")) <= 1e-12
            # written out for the l2 regulariser alone: (z_j + lam w_j)^2 / (2 lam) with z = X^T grad f
            u = np.array([(v - yy) if loss == "ridge" else -yy / (1.0 + math.exp(yy * v))
                          for v, yy in zip(s.v.tolist(), y.astype(np.float64).tolist())]) / 300
            z = X.T @ u
            np.testing.assert_allclose(share, (z + 1e-2 * s.x) ** 2 / (2 * 1e-2), rtol=1e-9, atol=1e-18)
        cg = s.chunk_gaps()
        assert cg.shape == (3,)
        np.testing.assert_allclose(cg, [share[0:7].sum(), share[7:19].sum(), share[19:40].sum()], rtol=1e-13)


@pytest.mark.parametrize("lam1", [0.0, 5e-3])
def test_gap_share_of_a_coordinate_is_zero_right_after_its_exact_update(lam1):
    """For the ridge loss the update is the exact minimiser along the coordinate, so with the dual
    candidate of the state right after it the coordinate's own share vanishes; the others' do not."""
    r = np.random.default_rng(5)
    X = sparse_random(200, 12, 0.5, r)
    y = r.standard_normal(200).astype(np.float32)
    A = dense_to_csc(X)
    s = oracle.Solver(A, y, "ridge", 1e-2, chunk_bounds=list(range(13)), lam1=lam1)   # one coordinate per chunk
    s.epoch(0)
    for j in (3, 0, 11):
        s.epoch(1, chunks=[j])
        share = oracle.primal_gap_shares(A, s.loss, s.v, s.y, s.x, s.lam, s.lam1)
        assert abs(share[j]) <= 1e-16 + 1e-12 * share.max()
        assert share.max() > 1e-8


def test_pass_over_selected_chunks_touches_only_them_and_all_chunks_is_an_epoch():
    r = np.random.default_rng(6)
    X = sparse_random(150, 30, 0.4, r)
    y = np.sign(r.standard_normal(150)).astype(np.float32)
    A = dense_to_csc(X)
    bounds = [0, 10, 18, 30]
    a = oracle.Solver(A, y, "logistic", 1e-2, chunk_bounds=bounds)
    b = oracle.Solver(A, y, "logistic", 1e-2, chunk_bounds=bounds)
    a.epoch(4)
    b.epoch(4, chunks=[0, 1, 2])
    assert np.array_equal(a.x, b.x) and np.array_equal(a.v, b.v)
    before = b.x.copy()
    b.epoch(5, chunks=[2, 0])
    assert np.array_equal(b.x[10:18], before[10:18])                   # chunk 1 untouched
    assert not np.array_equal(b.x[0:10], before[0:10]) and not np.array_equal(b.x[18:30], before[18:30])
    assert sorted(b.last_perm.tolist()) == list(range(0, 10)) + list(range(18, 30))
    assert b.last_perm[0] >= 18                                        # chunk 2 first, as asked
    np.testing.assert_allclose(b.v, A.matvec(b.x), rtol=0, atol=1e-12)


def test_selection_picks_the_largest_shares_and_the_selected_solve_reaches_the_optimum():
    assert oracle.select_chunks([0.1, 0.5, 0.5, 0.0, 0.7], 3) == [4, 1, 2]
    assert oracle.select_chunks([0.0, 0.0], 5) == [0, 1]
    r = np.random.default_rng(8)
    # block structure: the columns of the last chunk carry ten times the signal of the others
    X = sparse_random(400, 24, 0.3, r)
    w = r.standard_normal(24)
    w[18:] *= 10.0
    y = (X @ w + 0.01 * r.standard_normal(400)).astype(np.float32)
    A = dense_to_csc(X)
    bounds = [0, 6, 12, 18, 24]
    ref = oracle.solve(A, y, "ridge", 1e-3, 400, tol=1e-10)
    s = oracle.Solver(A, y, "ridge", 1e-3, chunk_bounds=bounds)
    assert oracle.select_chunks(s.chunk_gaps(), 1) == [3]              # at the zero model the strong block has the largest share
    passes, visits, gap = oracle.solve_selected(s, 0, 2000, 1e-10, refresh_every=3, keep=2)
    assert gap <= 1e-10
    assert visits < passes * 4                                          # part of the passes visited part of the chunks
    assert abs(s.primal() - ref.primal()) <= 1e-9 * abs(ref.primal())


@pytest.mark.parametrize("loss", ["hinge", "logistic"])
def test_dual_gap_shares_add_up_to_the_gap_and_are_nonnegative(loss):
    r = np.random.default_rng(21)
    X = sparse_random(120, 30, 0.4, r)
    y = np.sign(r.standard_normal(120)).astype(np.float32)
    s = oracle.Solver(dense_to_csr(X), y, loss, 5e-2, chunk_bounds=[0, 50, 120])
    for e in range(4):
        share = oracle.dual_gap_shares(s.A, s.loss, s.x, s.v, s.y, s.lam)
        assert share.min() >= -1e-15
        assert abs(share.sum() - s.gap()) <= 1e-12 * max(1.0, abs(s.primal()))
        np.testing.assert_allclose(s.chunk_gaps(), [share[:50].sum(), share[50:].sum()], rtol=1e-13)
        s.epoch(e)
    # hinge: right after the exact update of example i (alone in its chunk) its own share vanishes
    if loss == "hinge":
        t = oracle.Solver(dense_to_csr(X), y, loss, 5e-2, chunk_bounds=list(range(121)))
        t.epoch(0)
        for i in (7, 0, 119):
            t.epoch(1, chunks=[i])
            share = oracle.dual_gap_shares(t.A, t.loss, t.x, t.v, t.y, t.lam)
            assert abs(share[i]) <= 1e-15 and share.max() > 1e-6
