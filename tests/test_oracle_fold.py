"""Pins for the oracle's inference-time folds (App. E Eq. 4b, App. F.1): the folded table must
evaluate to  scale * (gamma lmKAN(x) + Linear(ReLU(x))) + shift  at every point, inside the grid,
on grid points and far beyond the ghost points, for even G; for odd G the ReLU part cannot be
absorbed (0 is not a grid point), which the last test shows."""
import numpy as np
import pytest


def _layer(oracle, P64, G, x):
    """y[j] = sum_k f_kj(x_2k, x_2k+1) with double tables, through the oracle's 2-D evaluator."""
    E32 = oracle.grid_f32(G)
    K, n_out = P64.shape[2], P64.shape[3]
    y = np.zeros(n_out)
    for k in range(K):
        for j in range(n_out):
            y[j] += oracle.eval2d(G, E32, np.ascontiguousarray(P64[:, :, k, j]), float(x[2 * k]), float(x[2 * k + 1]))
    return y


def _points(G, n_in, oracle, rng):
    E = oracle.grid_f32(G).astype(np.float64)
    pts = [rng.normal(size=n_in) for _ in range(12)]
    pts += [rng.normal(size=n_in) * 8.0 for _ in range(6)]             # beyond the ghost points
    pts += [rng.choice(E, size=n_in) for _ in range(6)]                 # on grid points
    pts += [np.zeros(n_in), np.full(n_in, -1e-3), np.full(n_in, 1e-3)]  # around the kink
    return [p.astype(np.float32) for p in pts]


@pytest.mark.parametrize("G", [4, 8, 16])
def test_folded_table_equals_the_unfolded_layer(oracle, G):
    rng = np.random.default_rng(G)
    n_in, n_out = 6, 3
    P = rng.normal(size=(G + 1, G + 1, n_in // 2, n_out)).astype(np.float32)
    gamma = 0.3
    lin_w, lin_b = rng.normal(size=(n_out, n_in)), rng.normal(size=n_out)
    scale, shift = rng.uniform(0.5, 2.0, size=n_out), rng.normal(size=n_out)
    folded = oracle.fold(P, G, gamma, lin_w, lin_b, scale, shift)
    P64 = P.astype(np.float64)
    for x in _points(G, n_in, oracle, rng):
        xd = x.astype(np.float64)
        want = scale * (gamma * _layer(oracle, P64, G, x) + lin_w @ np.maximum(xd, 0.0) + lin_b) + shift
        got = _layer(oracle, folded, G, x)
        np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-11 * max(1.0, np.abs(want).max()))


def test_each_term_alone(oracle):
    G, n_in, n_out = 6, 4, 2
    rng = np.random.default_rng(1)
    P = rng.normal(size=(G + 1, G + 1, n_in // 2, n_out)).astype(np.float32)
    np.testing.assert_array_equal(oracle.fold(P, G), P.astype(np.float64))            # nothing to fold
    np.testing.assert_allclose(oracle.fold(P, G, gamma=0.25), 0.25 * P.astype(np.float64), rtol=1e-15)
    shift = np.array([1.5, -2.0])
    only_shift = oracle.fold(P, G, shift=shift) - P
    assert np.all(only_shift[:, :, 1:, :] == 0)                                       # one pair carries it
    np.testing.assert_allclose(only_shift[:, :, 0, :], np.broadcast_to(shift, (G + 1, G + 1, 2)), atol=1e-6)


def test_odd_grids_cannot_absorb_relu(oracle):
    # App. E / F.1: exact whenever the origin is a grid point, i.e. G even; with G odd the kink of
    # ReLU falls inside a cell and the table can only interpolate across it
    G, n_in, n_out = 5, 2, 1
    P = np.zeros((G + 1, G + 1, 1, 1), dtype=np.float32)
    folded = oracle.fold(P, G, gamma=1.0, lin_w=np.array([[1.0, 0.0]]))
    x = np.array([0.0, 0.3], dtype=np.float32)
    got = _layer(oracle, folded, G, x)[0]
    assert abs(got - 0.0) > 1e-2        # ReLU(0) = 0 is missed by the chord across the kink
    x = np.array([1.0, 0.3], dtype=np.float32)   # away from the kink's cell it is still exact
    assert _layer(oracle, folded, G, x)[0] == pytest.approx(1.0, rel=1e-12)
