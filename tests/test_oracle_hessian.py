"""Pins for the oracle's Hessian regulariser (Sec. 3.5, App. C): closed forms the
finite-difference formulas must reproduce, the uniform-grid special case the paper prints,
and finite differences of the value for the gradient."""
import numpy as np
import pytest


def _sigma_grid(oracle, G):
    return oracle.grid(G)


@pytest.mark.parametrize("G", [3, 4, 8, 13, 16])
def test_linear_tables_cost_nothing(oracle, G):
    # the Hessian of a function is zero iff the function is linear (Sec. 3.5)
    E = _sigma_grid(oracle, G)
    p = 0.3 + 1.7 * E[:, None] - 2.2 * E[None, :]
    v, g = oracle.hessian_reg_2d(G, E, p, want_grad=True)
    assert abs(v) < 1e-20
    assert np.abs(g).max() < 1e-10


@pytest.mark.parametrize("G", [3, 5, 8, 16])
def test_quadratic_forms_on_the_nonuniform_grid(oracle, G):
    # p = A11 x1^2 + 2 A12 x1 x2 + A22 x2^2 + linear part: the three-point formulas are exact for
    # quadratics on any spacing, so D11 = 2 A11, D12 = 2 A12, D22 = 2 A22 at every centre and the
    # mean of H is the squared Frobenius norm of the Hessian, 4 A11^2 + 8 A12^2 + 4 A22^2
    E = _sigma_grid(oracle, G)
    x1, x2 = E[:, None], E[None, :]
    for A11, A12, A22 in [(1.0, 0.0, 0.0), (0.0, 1.0, 0.0), (0.0, 0.0, 1.0), (0.7, -0.4, 1.3)]:
        p = A11 * x1 ** 2 + 2 * A12 * x1 * x2 + A22 * x2 ** 2 + 0.5 * x1 - 0.25 * x2 + 3.0
        v = oracle.hessian_reg_2d(G, E, p)
        assert v == pytest.approx(4 * A11 ** 2 + 8 * A12 ** 2 + 4 * A22 ** 2, rel=1e-9)


def test_bilinear_table_counts_the_mixed_term_twice(oracle):
    G = 6
    E = _sigma_grid(oracle, G)
    v = oracle.hessian_reg_2d(G, E, E[:, None] * E[None, :])
    assert v == pytest.approx(2.0, rel=1e-12)      # D12 = 1 everywhere, H = 2 D12^2


def test_uniform_grid_reduces_to_the_printed_second_difference(oracle):
    # Sec. 3.5: on a uniform grid the second-derivative penalty is sum (p_i - 2 p_{i+1} + p_{i+2})^2
    # (up to the 1/h^4 of the spacing); a table constant along the second axis has only D11
    G, h = 9, 0.25
    E = h * np.arange(G + 1)
    rng = np.random.default_rng(3)
    q = rng.normal(size=G + 1)
    p = np.repeat(q[:, None], G + 1, axis=1)
    v = oracle.hessian_reg_2d(G, E, p)
    second = (q[2:] - 2 * q[1:-1] + q[:-2]) / h ** 2           # centres 1 .. G-1
    assert v == pytest.approx(np.mean(second ** 2), rel=1e-12)
    # and along the other axis
    v2 = oracle.hessian_reg_2d(G, E, p.T.copy())
    assert v2 == pytest.approx(v, rel=1e-12)


def test_axes_enter_symmetrically(oracle):
    G = 7
    E = _sigma_grid(oracle, G)
    rng = np.random.default_rng(5)
    p = rng.normal(size=(G + 1, G + 1))
    assert oracle.hessian_reg_2d(G, E, p) == pytest.approx(oracle.hessian_reg_2d(G, E, p.T.copy()), rel=1e-12)


@pytest.mark.parametrize("G", [3, 4, 9])
def test_gradient_matches_finite_differences(oracle, G):
    E = _sigma_grid(oracle, G)
    rng = np.random.default_rng(G)
    p = rng.normal(size=(G + 1, G + 1))
    v, g = oracle.hessian_reg_2d(G, E, p, want_grad=True)
    eps = 1e-6
    for a in range(G + 1):
        for b in range(G + 1):
            pp, pm = p.copy(), p.copy()
            pp[a, b] += eps
            pm[a, b] -= eps
            fd = (oracle.hessian_reg_2d(G, E, pp) - oracle.hessian_reg_2d(G, E, pm)) / (2 * eps)
            assert g[a, b] == pytest.approx(fd, rel=1e-6, abs=1e-6 * np.abs(g).max())
    # the value is a quadratic form in p: <grad, p> = 2 value (Euler)
    assert float((g * p).sum()) == pytest.approx(2 * v, rel=1e-10)


def test_corner_ghost_nodes_only_enter_the_mixed_term(oracle):
    # p[0][0] is a neighbour of centre (1,1) only through D12
    G = 5
    E = _sigma_grid(oracle, G)
    p = np.zeros((G + 1, G + 1))
    p[0, 0] = 1.0
    v = oracle.hessian_reg_2d(G, E, p)
    d12 = 1.0 / ((E[2] - E[0]) * (E[2] - E[0]))
    assert v == pytest.approx(2 * d12 ** 2 / (G - 1) ** 2, rel=1e-12)


def test_layer_value_is_the_sum_over_functions(oracle):
    G, K, n_out = 4, 3, 5
    rng = np.random.default_rng(11)
    P = rng.normal(size=(G + 1, G + 1, K, n_out)).astype(np.float32)
    value, grad = oracle.hessian_reg(P, G)
    E = oracle.grid_f32(G).astype(np.float64)
    want = 0.0
    for k in range(K):
        for j in range(n_out):
            v, g = oracle.hessian_reg_2d(G, E, P[:, :, k, j].astype(np.float64), want_grad=True)
            want += v
            np.testing.assert_allclose(grad[:, :, k, j], g, rtol=0, atol=1e-12 * max(1.0, np.abs(g).max()))
    assert value == pytest.approx(want, rel=1e-12)
