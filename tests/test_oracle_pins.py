"""CPU pins for the oracle: every check compares it with something the paper or
the mathematics fixes, never with itself."""
import math
import os

import numpy as np
import pytest
from scipy.stats import laplace

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
GRIDS = [3, 4, 5, 8, 12, 16, 20, 32, 40, 64]


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


# --------------------------------------------------------------------------
# sigma (App. B, Eq. 5 / Alg. 2)
# --------------------------------------------------------------------------

def test_sigma_is_the_two_branch_function_of_eq5(oracle):
    xs = np.concatenate([np.linspace(-30, 30, 601), [0.0, -0.0, 1e-300, -1e-300, 700.0, -700.0]])
    for x in xs:
        # Eq. 5 branch by branch (Alg. 2 folds both into one exp(-|x|)); this is also the
        # CDF of the unit Laplace distribution, which scipy evaluates independently.
        want = 0.5 * math.exp(x) if x <= 0 else 1.0 - 0.5 * math.exp(-x)
        got = oracle.sigma(x)
        assert got == pytest.approx(want, rel=1e-15, abs=1e-300)
        assert got == pytest.approx(laplace.cdf(x), rel=1e-13, abs=1e-300)
    assert oracle.sigma(0.0) == 0.5
    for x in [0.1, 1.0, 3.7, 25.0]:
        assert oracle.sigma(-x) == pytest.approx(1.0 - oracle.sigma(x), abs=1e-16)
    vals = [oracle.sigma(x) for x in np.linspace(-20, 20, 2001)]
    assert all(b > a for a, b in zip(vals, vals[1:]))


# --------------------------------------------------------------------------
# grid (Sec. 3.1 "Sigma grid", App. B "Edge cases")
# --------------------------------------------------------------------------

@pytest.mark.parametrize("G", GRIDS)
def test_real_grid_points_sit_on_the_percentile_levels(oracle, G):
    E = oracle.grid(G)
    assert E.shape == (G + 1,)
    k = np.arange(1, G)
    # the defining property: sigma(E[k]) = k / G, checked with scipy's Laplace CDF
    np.testing.assert_allclose(laplace.cdf(E[1:G]) * G, k, rtol=0, atol=1e-13 * G)
    assert np.all(np.diff(E) > 0)
    # mirror symmetry of sigma carries over to the grid; origin is a node iff G is even
    np.testing.assert_array_equal(E, -E[::-1])
    if G % 2 == 0:
        assert E[G // 2] == 0.0
    else:
        assert not np.any(E == 0.0)
    # ghosts: first - (second - first), and the mirror image on the right
    assert E[1] - E[0] == pytest.approx(E[2] - E[1], rel=1e-15)
    assert E[G] - E[G - 1] == pytest.approx(E[G - 1] - E[G - 2], rel=1e-15)
    # finest resolution at the origin, coarser outwards
    h = np.diff(E[1:G])
    mid = len(h) // 2
    assert np.all(np.diff(h[mid:]) >= -1e-15) and np.all(np.diff(h[: mid + 1]) <= 1e-15)


def test_grid_matches_hand_worked_values(oracle):
    rows = _golden_rows("grid_closed_form.txt")
    assert len(rows) == 15
    for G, idx, val in rows:
        E = oracle.grid(int(G))
        assert E[int(idx)] == pytest.approx(float(val), rel=1e-15, abs=1e-16)


@pytest.mark.parametrize("G", GRIDS)
def test_float_grid_is_the_rounded_double_grid(oracle, G):
    E, E32 = oracle.grid(G), oracle.grid_f32(G)
    assert E32.dtype == np.float32
    np.testing.assert_array_equal(E32, E.astype(np.float32))
    assert np.all(np.diff(E32) > 0)


def test_grid_rejects_too_few_intervals(oracle):
    for G in [-1, 0, 1, 2]:
        with pytest.raises(ValueError):
            oracle.grid(G)


# --------------------------------------------------------------------------
# locate (Sec. 3.1: i = floor(sigma(x) G))
# --------------------------------------------------------------------------

@pytest.mark.parametrize("G", GRIDS)
def test_locate_equals_floor_sigma_times_G(oracle, G):
    rng = np.random.default_rng(100 + G)
    E32 = oracle.grid_f32(G)
    xs = np.concatenate([rng.standard_normal(3000), rng.standard_t(3, 1000) * 3,
                         rng.uniform(-12, 12, 1000)]).astype(np.float32)
    checked = 0
    for x in xs:
        s = laplace.cdf(float(x)) * G
        if abs(s - round(s)) < 1e-5:      # too close to a node for the float grid to agree
            continue
        want = min(max(int(math.floor(s)), 0), G - 1)
        assert oracle.locate(G, E32, x) == want
        assert oracle.locate_sigma(G, float(x)) == want
        checked += 1
    assert checked > 4500


@pytest.mark.parametrize("G", [3, 4, 8, 16, 33])
def test_locate_on_and_around_grid_points(oracle, G):
    E32 = oracle.grid_f32(G)
    for k in range(1, G):
        node = E32[k]
        below = np.nextafter(node, np.float32(-np.inf))
        above = np.nextafter(node, np.float32(np.inf))
        assert oracle.locate(G, E32, node) == k          # a node belongs to the cell on its right
        assert oracle.locate(G, E32, below) == k - 1
        assert oracle.locate(G, E32, above) == k
    # ghosts are not cell boundaries: the edge cells run to infinity
    assert oracle.locate(G, E32, E32[0]) == 0
    assert oracle.locate(G, E32, E32[0] - 5) == 0
    assert oracle.locate(G, E32, E32[G]) == G - 1
    assert oracle.locate(G, E32, E32[G] + 5) == G - 1
    assert oracle.locate(G, E32, -np.inf) == 0
    assert oracle.locate(G, E32, np.inf) == G - 1
    assert oracle.locate(G, E32, np.nan) == 0
    assert oracle.locate(G, E32, 3e38) == G - 1
    assert oracle.locate(G, E32, -3e38) == 0


# --------------------------------------------------------------------------
# the four weights of the preamble (Alg. 1)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("G", [3, 4, 8, 16, 32])
def test_weights_sum_to_one_and_stay_in_range(oracle, G):
    rng = np.random.default_rng(200 + G)
    E32 = oracle.grid_f32(G)
    lo, hi = float(E32[0]), float(E32[G])
    for _ in range(2000):
        x1, x2 = (rng.standard_t(3, 2) * 2).astype(np.float32)
        cell, w = oracle.preamble(G, E32, x1, x2)
        assert 0 <= cell < G * G
        assert w.sum() == pytest.approx(1.0, abs=1e-14 * max(1.0, np.abs(w).max() ** 2))
        if lo <= x1 <= hi and lo <= x2 <= hi:
            assert np.all(w >= 0) and np.all(w <= 1)
    # beyond a ghost the inner weight goes negative and the outer one exceeds one
    cell, w = oracle.preamble(G, E32, np.float32(lo - 1.0), np.float32(0.25))
    assert cell // G == 0 and w[1] + w[3] < 0 and w[0] + w[2] > 1
    assert w.sum() == pytest.approx(1.0, abs=1e-13)


@pytest.mark.parametrize("G", [3, 4, 7, 16])
def test_exactly_one_nonzero_weight_on_a_grid_point(oracle, G):
    E32 = oracle.grid_f32(G)
    for a in range(0, G + 1):
        for b in range(0, G + 1):
            cell, w = oracle.preamble(G, E32, E32[a], E32[b])
            # (h1 h2) * (1 / (h1 h2)) may round one ulp below one
            assert np.count_nonzero(w) == 1 and w.max() == pytest.approx(1.0, abs=3e-16)
            i1, i2 = divmod(cell, G)
            # which of the four corners carries the weight tells which node was hit
            hit = int(np.argmax(w))          # order: (i1,i2), (i1+1,i2), (i1,i2+1), (i1+1,i2+1)
            assert (i1 + (hit & 1), i2 + (hit >> 1)) == (a, b)


# --------------------------------------------------------------------------
# values of one 2-D function (Eq. 3, Alg. 3)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("G", [3, 4, 8, 13])
def test_coefficients_are_the_function_values_on_the_nodes(oracle, G):
    rng = np.random.default_rng(300 + G)
    E32 = oracle.grid_f32(G)
    P2 = rng.standard_normal((G + 1, G + 1))
    for a in range(G + 1):
        for b in range(G + 1):
            assert oracle.eval2d(G, E32, P2, E32[a], E32[b]) == pytest.approx(
                P2[a, b], rel=3e-16, abs=0)


def test_hand_worked_evaluations(oracle):
    G = 4
    E32 = oracle.grid_f32(G)
    rows = _golden_rows("eval2d_worked.txt")
    cases = {r[0]: r for r in rows if r[0] != "coef"}
    assert set(cases) == {"A", "B"}
    for name, (_, u1, u2, want) in cases.items():
        P2 = np.full((G + 1, G + 1), 100.0)
        for r in rows:
            if r[0] == "coef" and r[1] == name:
                P2[int(r[2]), int(r[3])] = float(r[4])
        x1, x2 = float(u1) * math.log(2.0), float(u2) * math.log(2.0)
        got = oracle.eval2d(G, E32, P2, x1, x2)
        assert got == pytest.approx(float(want), abs=5e-5)   # float32 rounding of x and grid
        # and straight from the definition in double on the exact grid
        got_def = oracle.eval2d_def(G, oracle.grid(G), P2, x1, x2)
        assert got_def == pytest.approx(float(want), abs=1e-12)


@pytest.mark.parametrize("G", [3, 4, 8, 16, 32])
def test_bilinear_tables_are_reproduced_everywhere(oracle, G):
    """A table sampled from alpha + beta x1 + gamma x2 + delta x1 x2 gives back exactly that
    function, also on the infinite edge intervals (each function is bilinear per cell and
    linear out to infinity)."""
    rng = np.random.default_rng(400 + G)
    E32 = oracle.grid_f32(G)
    E = E32.astype(np.float64)
    al, be, ga, de = 0.3, -1.7, 0.9, 0.45
    P2 = al + be * E[:, None] + ga * E[None, :] + de * E[:, None] * E[None, :]
    pts = np.concatenate([rng.standard_normal((400, 2)), rng.standard_t(2, (200, 2)) * 4,
                          [[-40.0, 35.0], [50.0, -0.01], [E32[0], E32[G]]]]).astype(np.float32)
    for x1, x2 in pts:
        want = al + be * float(x1) + ga * float(x2) + de * float(x1) * float(x2)
        got = oracle.eval2d(G, E32, P2, x1, x2)
        assert got == pytest.approx(want, rel=1e-12, abs=1e-11)


@pytest.mark.parametrize("G", [4, 8, 16])
def test_relu_terms_are_absorbed_exactly_for_even_G(oracle, oracle_clip, G):
    """App. F.1: w1 ReLU(x1) + w2 ReLU(x2) can be folded into a table exactly when the
    origin is a grid point."""
    rng = np.random.default_rng(500 + G)
    E32 = oracle.grid_f32(G)
    E = E32.astype(np.float64)
    w1, w2 = 0.8, -1.3
    P2 = w1 * np.maximum(E[:, None], 0) + w2 * np.maximum(E[None, :], 0)
    pts = np.concatenate([rng.standard_normal((300, 2)), rng.uniform(-9, 9, (300, 2))])
    pts = pts.astype(np.float32)
    worst_clip = 0.0
    for x1, x2 in pts:
        want = w1 * max(float(x1), 0.0) + w2 * max(float(x2), 0.0)
        assert oracle.eval2d(G, E32, P2, x1, x2) == pytest.approx(want, rel=1e-12, abs=1e-12)
        worst_clip = max(worst_clip, abs(oracle_clip.eval2d(G, E32, P2, x1, x2) - want))
    # the reading that cuts the edge hats at the ghosts cannot satisfy the statement
    assert worst_clip > 0.1


def test_odd_G_cannot_absorb_relu(oracle):
    G = 5
    E32 = oracle.grid_f32(G)
    E = E32.astype(np.float64)
    P2 = np.maximum(E[:, None], 0) + 0 * E[None, :]
    x1 = np.float32(0.05)      # inside the cell that straddles the origin
    assert abs(oracle.eval2d(G, E32, P2, x1, 0.3) - 0.05) > 1e-3


@pytest.mark.parametrize("G", [3, 5, 8])
def test_functions_are_continuous_across_cell_boundaries(oracle, G):
    rng = np.random.default_rng(600 + G)
    E32 = oracle.grid_f32(G)
    P2 = rng.standard_normal((G + 1, G + 1))
    for k in range(1, G):
        node = E32[k]
        below = np.nextafter(node, np.float32(-np.inf))
        for other in rng.standard_normal(5).astype(np.float32):
            assert oracle.eval2d(G, E32, P2, below, other) == pytest.approx(
                oracle.eval2d(G, E32, P2, node, other), abs=1e-5)
            assert oracle.eval2d(G, E32, P2, other, below) == pytest.approx(
                oracle.eval2d(G, E32, P2, other, node), abs=1e-5)


# --------------------------------------------------------------------------
# basis functions from their description, and the definition of the layer
# --------------------------------------------------------------------------

@pytest.mark.parametrize("G", [3, 4, 9])
def test_basis_functions_match_their_description(oracle, G):
    E = oracle.grid(G)
    for a in range(1, G):
        assert oracle.basis(G, E, a, E[a]) == 1.0
        assert oracle.basis(G, E, a, E[a - 1]) == 0.0
        assert oracle.basis(G, E, a, E[a + 1]) == 0.0
        assert oracle.basis(G, E, a, 0.5 * (E[a - 1] + E[a])) == pytest.approx(0.5)
        assert oracle.basis(G, E, a, 0.5 * (E[a] + E[a + 1])) == pytest.approx(0.5)
        if 2 <= a <= G - 2:
            assert oracle.basis(G, E, a, E[a - 1] - 0.1) == 0.0
            assert oracle.basis(G, E, a, E[a + 1] + 0.1) == 0.0
    # edge functions: zero on the outermost real point, one on the ghost, same slope beyond
    assert oracle.basis(G, E, 0, E[1]) == 0.0 and oracle.basis(G, E, 0, E[0]) == 1.0
    assert oracle.basis(G, E, G, E[G - 1]) == 0.0 and oracle.basis(G, E, G, E[G]) == 1.0
    h0 = E[1] - E[0]
    assert oracle.basis(G, E, 0, E[0] - 3 * h0) == pytest.approx(4.0)
    assert oracle.basis(G, E, G, E[G] + 2 * h0) == pytest.approx(3.0)
    assert oracle.basis(G, E, 0, E[1] + 0.2) == 0.0 and oracle.basis(G, E, G, E[G - 1] - 0.2) == 0.0
    # at most two non-zero functions at any point, and they sum to one
    for x in np.linspace(E[0] - 2, E[G] + 2, 173):
        vals = np.array([oracle.basis(G, E, a, x) for a in range(G + 1)])
        assert np.count_nonzero(vals) <= 2
        assert vals.sum() == pytest.approx(1.0, abs=1e-14)


@pytest.mark.parametrize("shape", [(2, 1, 3), (4, 3, 4), (6, 4, 5), (8, 2, 8)])
def test_fast_layer_equals_the_full_double_sum(oracle, shape):
    """Alg. 1 (one cell, four terms) against Eq. 2 + Eq. 3 with all (G+1)^2 terms."""
    N_in, N_out, G = shape
    rng = np.random.default_rng(700 + G)
    E32 = oracle.grid_f32(G)
    x = np.concatenate([rng.standard_normal((20, N_in)), rng.standard_t(2, (10, N_in)) * 3])
    x = x.astype(np.float32)
    x[0, :] = E32[rng.integers(0, G + 1, N_in)]          # exactly on nodes and ghosts
    x[1, :] = 25.0
    x[2, :] = -25.0
    P = rng.standard_normal((G + 1, G + 1, N_in // 2, N_out)).astype(np.float32)
    y_fast = oracle.forward(x, P, G)
    y_def = oracle.forward_def(x, P, G)
    np.testing.assert_allclose(y_fast, y_def, rtol=1e-12, atol=1e-12)


def test_layer_is_a_sum_of_pair_functions(oracle):
    """The 4-input / 3-output example of Sec. 3 (Fig. 2): y_q = f_q0(x0,x1) + f_q1(x2,x3)."""
    G, N_in, N_out = 6, 4, 3
    rng = np.random.default_rng(800)
    E32 = oracle.grid_f32(G)
    x = rng.standard_normal((7, N_in)).astype(np.float32)
    P = rng.standard_normal((G + 1, G + 1, 2, N_out)).astype(np.float32)
    y = oracle.forward(x, P, G)
    for n in range(7):
        for q in range(N_out):
            want = (oracle.eval2d(G, E32, P[:, :, 0, q].astype(np.float64), x[n, 0], x[n, 1]) +
                    oracle.eval2d(G, E32, P[:, :, 1, q].astype(np.float64), x[n, 2], x[n, 3]))
            assert y[n, q] == pytest.approx(want, rel=1e-14, abs=1e-14)
    # pair 1's inputs do not reach pair 0's functions
    x2 = x.copy()
    x2[:, 2:] += 0.37
    P0 = P.copy()
    P0[:, :, 1, :] = 0
    np.testing.assert_array_equal(oracle.forward(x, P0, G), oracle.forward(x2, P0, G))


def test_layer_reproduces_a_dense_linear_map(oracle):
    """Tables sampled from a x1 + b x2 turn the layer into an ordinary matrix product
    (Sec. 3.5: fully linearised lmKAN is an MLP layer of the same shape)."""
    G, N_in, N_out, B = 8, 10, 6, 40
    rng = np.random.default_rng(900)
    E = oracle.grid_f32(G).astype(np.float64)
    Wm = rng.standard_normal((N_in, N_out))
    P = np.empty((G + 1, G + 1, N_in // 2, N_out))
    for k in range(N_in // 2):
        P[:, :, k, :] = (E[:, None, None] * Wm[2 * k][None, None, :] +
                         E[None, :, None] * Wm[2 * k + 1][None, None, :])
    P32 = P.astype(np.float32)
    x = (rng.standard_t(3, (B, N_in)) * 2).astype(np.float32)
    y = oracle.forward(x, P32, G)
    # compare against the matrix product with the same rounded tables: rebuild W from P32
    want = np.zeros((B, N_out))
    for k in range(N_in // 2):
        # a linear table is reproduced exactly, so the pair function is its own bilinear fit
        a = (P32[G, 0, k, :].astype(np.float64) - P32[0, 0, k, :]) / (E[G] - E[0])
        b = (P32[0, G, k, :].astype(np.float64) - P32[0, 0, k, :]) / (E[G] - E[0])
        c = P32[0, 0, k, :].astype(np.float64) - a * E[0] - b * E[0]
        want += x[:, [2 * k]].astype(np.float64) * a + x[:, [2 * k + 1]].astype(np.float64) * b + c
    np.testing.assert_allclose(y, want, rtol=0, atol=2e-5)
    np.testing.assert_allclose(y, x.astype(np.float64) @ Wm, rtol=0, atol=2e-5 * np.abs(x).max())


# --------------------------------------------------------------------------
# stored formats
# --------------------------------------------------------------------------

def test_half_and_bfloat_decoding_against_numpy_and_torch(oracle):
    import torch
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want16 = bits.view(np.float16).astype(np.float64)
    want_bf = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    for b in range(0, 65536, 7):
        g16 = oracle.half_bits_to_double(b)
        gbf = oracle.bf16_bits_to_double(b)
        for got, want in ((g16, want16[b]), (gbf, want_bf[b])):
            if math.isnan(want):
                assert math.isnan(got)
            else:
                assert got == want and math.copysign(1, got) == math.copysign(1, want)


def test_forward_reads_stored_half_and_bfloat_bits(oracle):
    import torch
    G, N_in, N_out = 5, 6, 4
    rng = np.random.default_rng(1000)
    x = rng.standard_normal((9, N_in)).astype(np.float32)
    P = (rng.standard_normal((G + 1, G + 1, N_in // 2, N_out)) * 0.1).astype(np.float32)
    P16 = P.astype(np.float16)
    Pbf = torch.from_numpy(P).to(torch.bfloat16)
    y16 = oracle.forward(x, P16.view(np.uint16), G, dtype=1)
    ybf = oracle.forward(x, Pbf.view(torch.int16).numpy().view(np.uint16), G, dtype=2)
    np.testing.assert_array_equal(y16, oracle.forward(x, P16.astype(np.float32), G))
    np.testing.assert_array_equal(ybf, oracle.forward(x, Pbf.float().numpy(), G))


# --------------------------------------------------------------------------
# backward (derivatives of Alg. 1's four-term sum)
# --------------------------------------------------------------------------

def _loss_def(oracle, G, E, x64, P, gy):
    """sum_{n,q} gy[n,q] y[n,q] from the full double sum, at double-precision inputs."""
    B, N_in = x64.shape
    tot = 0.0
    for n in range(B):
        for q in range(P.shape[-1]):
            for k in range(N_in // 2):
                tot += float(gy[n, q]) * oracle.eval2d_def(G, E, P[:, :, k, q].astype(np.float64),
                                                    x64[n, 2 * k], x64[n, 2 * k + 1])
    return tot


@pytest.mark.parametrize("G", [3, 4, 8])
def test_input_gradient_against_central_differences(oracle, G):
    rng = np.random.default_rng(1100 + G)
    N_in, N_out, B = 6, 3, 6
    E32 = oracle.grid_f32(G)
    E = E32.astype(np.float64)
    x = (rng.standard_t(3, (B, N_in)) * 1.5).astype(np.float32)
    P = rng.standard_normal((G + 1, G + 1, N_in // 2, N_out)).astype(np.float32)
    gy = rng.standard_normal((B, N_out)).astype(np.float32)
    gx = oracle.backward_input(x, P, gy, G)
    h = 1e-6
    x64 = x.astype(np.float64)
    for n in range(B):
        for c in range(N_in):
            if np.min(np.abs(E[1:G] - x64[n, c])) < 1e-4:
                continue
            xp, xm = x64[[n]].copy(), x64[[n]].copy()
            xp[0, c] += h
            xm[0, c] -= h
            fd = (_loss_def(oracle, G, E, xp, P, gy[[n]]) -
                  _loss_def(oracle, G, E, xm, P, gy[[n]])) / (2 * h)
            assert gx[n, c] == pytest.approx(fd, rel=1e-7, abs=1e-7)


def test_input_gradient_of_a_linear_layer_is_the_transposed_matrix(oracle):
    G, N_in, N_out, B = 8, 8, 5, 12
    rng = np.random.default_rng(1200)
    E = oracle.grid_f32(G).astype(np.float64)
    Wm = rng.standard_normal((N_in, N_out))
    P = np.empty((G + 1, G + 1, N_in // 2, N_out))
    for k in range(N_in // 2):
        P[:, :, k, :] = (E[:, None, None] * Wm[2 * k][None, None, :] +
                         E[None, :, None] * Wm[2 * k + 1][None, None, :])
    x = (rng.standard_t(3, (B, N_in)) * 2).astype(np.float32)
    gy = rng.standard_normal((B, N_out)).astype(np.float32)
    gx = oracle.backward_input(x, P.astype(np.float32), gy, G)
    np.testing.assert_allclose(gx, gy.astype(np.float64) @ Wm.T, rtol=0, atol=3e-5)


@pytest.mark.parametrize("G", [3, 5, 8])
def test_coefficient_gradient_properties(oracle, G):
    rng = np.random.default_rng(1300 + G)
    N_in, N_out, B = 6, 4, 15
    K = N_in // 2
    x = (rng.standard_t(3, (B, N_in)) * 1.5).astype(np.float32)
    gy = rng.standard_normal((B, N_out)).astype(np.float32)
    gP = oracle.backward_coef(x, gy, G)
    assert gP.shape == (G + 1, G + 1, K, N_out)
    # y is linear in P:  sum gy*y(P) == <gP, P>  for any P, and y(P + dP) - y(P) == y(dP)
    for seed in range(3):
        P = np.random.default_rng(seed).standard_normal(gP.shape).astype(np.float32)
        lhs = float((gy.astype(np.float64) * oracle.forward(x, P, G)).sum())
        assert lhs == pytest.approx(float((gP * P).sum()), rel=1e-12, abs=1e-12)
    # single-coefficient probes: dL/dP[a,b,k,j] is the response to a unit table entry
    for _ in range(20):
        a, b = rng.integers(0, G + 1, 2)
        k, j = rng.integers(0, K), rng.integers(0, N_out)
        Pu = np.zeros(gP.shape, dtype=np.float32)
        Pu[a, b, k, j] = 1.0
        want = float((gy.astype(np.float64) * oracle.forward(x, Pu, G)).sum())
        assert gP[a, b, k, j] == pytest.approx(want, rel=1e-13, abs=1e-14)
    # weights sum to one, so the table gradient of pair k sums to sum_n gy
    np.testing.assert_allclose(gP.sum(axis=(0, 1)), np.broadcast_to(
        gy.astype(np.float64).sum(axis=0), (K, N_out)), rtol=1e-12, atol=1e-12)
    # nodes that no row touches get exactly zero (Sec. 3.5)
    cell = oracle.locate_batch(x, G)
    touched = np.zeros((G + 1, G + 1, K), dtype=bool)
    for n in range(B):
        for k in range(K):
            i1, i2 = divmod(int(cell[n, k]), G)
            touched[i1:i1 + 2, i2:i2 + 2, k] = True
    assert np.all(gP[~touched] == 0.0)
    assert touched.sum() < touched.size or G == 3


def test_locate_batch_matches_scalar_locate(oracle):
    G = 7
    rng = np.random.default_rng(1400)
    E32 = oracle.grid_f32(G)
    x = rng.standard_normal((11, 6)).astype(np.float32)
    cell = oracle.locate_batch(x, G)
    for n in range(11):
        for k in range(3):
            i1 = oracle.locate(G, E32, x[n, 2 * k])
            i2 = oracle.locate(G, E32, x[n, 2 * k + 1])
            assert cell[n, k] == i1 * G + i2
