"""Pins for the oracle's Sparse GGT path (Appendix "Sparse GGT", Algorithm
"Detailed Sparse GGT Implementation"): the Jacobi eigensolver against LAPACK,
the direction against the dense definition ((G G^T)^{1/2} + eps I)^-1 x built
with numpy on small d, and closed forms."""
import numpy as np
import pytest


def _dense_rows(o):
    C = np.zeros((o.m, o.d))
    for r in range(o.m):
        i, v = o.row(r)
        if i is not None:
            C[r, i] = v
    return C


def _dense_ggt(C, eps, x):
    """((G G^T)^{1/2} + eps I)^-1 x with G = C^T (d x m), the square root taken from LAPACK's
    SVD of G (G = U S V^T gives (G G^T)^{1/2} = U S U^T) so that the null space of G G^T is
    not polluted by square roots of rounding-size eigenvalues."""
    U, sv, _ = np.linalg.svd(C.T, full_matrices=False)
    root = (U * sv) @ U.T
    return np.linalg.solve(root + eps * np.eye(C.shape[1]), x.astype(np.float64))


def _rel(a, b):
    return np.linalg.norm(a - b) / np.linalg.norm(b)


@pytest.mark.parametrize("n", [1, 2, 7, 40, 100])
def test_jacobi_matches_lapack(oracle_mod, n):
    rng = np.random.default_rng(n)
    B = rng.standard_normal((n, max(n // 2, 1)))          # rank deficient Gram matrix: zero eigenvalues
    A = B @ B.T + 1e-3 * np.diag(rng.random(n) < 0.3)
    lam, V = oracle_mod.jacobi_eigh(A)
    ref = np.linalg.eigvalsh(A)
    assert np.allclose(np.sort(lam), ref, rtol=1e-12, atol=1e-12 * max(abs(ref).max(), 1.0))
    assert np.allclose(V.T @ V, np.eye(n), atol=1e-12)
    assert np.allclose((V * lam) @ V.T, A, atol=1e-11 * max(abs(A).max(), 1.0))


def test_jacobi_diagonal_and_2x2_closed_form(oracle_mod):
    lam, V = oracle_mod.jacobi_eigh(np.diag([3.0, -1.0, 0.0]))
    assert np.array_equal(lam, [3.0, -1.0, 0.0]) and np.array_equal(V, np.eye(3))
    lam, V = oracle_mod.jacobi_eigh(np.array([[2.0, 1.0], [1.0, 2.0]]))
    assert np.allclose(np.sort(lam), [1.0, 3.0], atol=1e-15)
    assert np.allclose(np.abs(V), np.full((2, 2), np.sqrt(0.5)), atol=1e-15)


@pytest.mark.parametrize("d,m,k,eps,T", [(120, 4, 9, 1e-2, 10), (200, 6, 200, 1e-1, 9), (90, 8, 5, 1e-3, 20)])
def test_ggt_step_matches_dense_definition(oracle_mod, d, m, k, eps, T):
    """Partly filled, full and evicting windows; x = g, x = c_t (the paper's) and apply."""
    o = oracle_mod.Oracle(d, m, k, eps, ggt=True)
    p = oracle_mod.Oracle(d, m, k, eps, ggt=True)
    rng = np.random.default_rng(d)
    for t in range(T):
        g = (rng.standard_normal(d) * np.exp(rng.standard_normal(d) * 0.5)).astype(np.float32)
        y = o.step(g)
        C = _dense_rows(o)
        assert _rel(y, _dense_ggt(C, eps, g)) < 1e-9
        yc = p.step_compressed(g)
        assert np.array_equal(_dense_rows(p), C)
        assert _rel(yc, _dense_ggt(C, eps, C[p.newest_slot])) < 1e-9
        x = rng.standard_normal(d).astype(np.float32)
        assert _rel(o.apply(x), _dense_ggt(C, eps, x)) < 1e-9
        # u is x/eps minus a combination of the stored vectors
        assert _rel(o.apply(x), x.astype(np.float64) / eps - o.coef @ C) < 1e-9


def test_ggt_closed_forms(oracle_mod):
    d, eps = 64, 0.5
    o = oracle_mod.Oracle(d, 3, 4, eps, ggt=True)
    x0 = np.arange(d, dtype=np.float32)
    assert np.array_equal(o.apply(x0), x0.astype(np.float64) / eps)         # empty window
    g = np.zeros(d, np.float32)
    g[[3, 10, 20, 33]] = [3.0, -4.0, 12.0, 0.5]
    g[40:] = 0.01
    o.step(g)
    c = _dense_rows(o)[0]
    nc = np.linalg.norm(c)
    x = np.random.default_rng(0).standard_normal(d).astype(np.float32)
    # one stored vector: (G G^T)^{1/2} = c c^T / |c|
    expect = x / eps + c * (c @ x) / nc ** 2 * (1.0 / (nc + eps) - 1.0 / eps)
    assert _rel(o.apply(x), expect) < 1e-13
    # x orthogonal to the window: only the eps term acts
    xo = x.astype(np.float64) - c * (c @ x) / nc ** 2
    xo32 = xo.astype(np.float32)
    xo32[c != 0] = 0.0
    assert np.allclose(o.apply(xo32), xo32.astype(np.float64) / eps, rtol=0, atol=1e-12)
    # x = c itself: u = c / (|c| + eps)
    assert _rel(o.apply(c.astype(np.float32)), c / (nc + eps)) < 1e-13


def test_ggt_unfilled_slots_and_duplicate_rows_use_the_pseudo_inverse(oracle_mod):
    """Two identical stored vectors make G^T G singular; the direction must still be the
    dense definition's."""
    d, eps = 50, 1e-2
    o = oracle_mod.Oracle(d, 5, d, eps, ggt=True)           # k = d: e stays 0, rows are the gradients
    rng = np.random.default_rng(3)
    g = rng.standard_normal(d).astype(np.float32)
    o.step(g)
    o.step(g)                                               # same vector again
    o.step(rng.standard_normal(d).astype(np.float32))
    C = _dense_rows(o)
    assert np.linalg.matrix_rank(C) == 2
    x = rng.standard_normal(d).astype(np.float32)
    assert _rel(o.apply(x), _dense_ggt(C, eps, x)) < 1e-9
