"""Pins of the CPU oracle against things other than itself: hand-derived exact
rational examples, closed forms, invariants, textbook identities, central
finite differences, and the agreement of its independent routes."""
import math

import numpy as np
import pytest

from conftest import read_golden


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- worked examples

@pytest.mark.parametrize("name", ["apply_rational_3x2.txt", "apply_rational_ties_3x3.txt"])
@pytest.mark.parametrize("route", ["brute", "scan"])
def test_golden_apply(oracle, name, route):
    gd = read_golden(name)
    a = np.log(np.array(gd["exp_a"])); b = np.log(np.array(gd["exp_b"]))
    x = np.array(gd["x"]).reshape(-1, 1); g = np.array(gd["g"]).reshape(-1, 1)
    if route == "brute":
        y, _ = oracle.apply_brute(a, b, x)
        (gx, ga, gb), _ = oracle.apply_backward_brute(a, b, x, g)
    else:
        y, _ = oracle.apply_scan(a, b, x)
        (gx, ga, gb), _ = oracle.apply_backward_scan(a, b, x, g)
    np.testing.assert_allclose(y[:, 0], gd["y"], rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(gx[:, 0], gd["gx"], rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(ga, gd["ga"], rtol=1e-14, atol=1e-13)
    np.testing.assert_allclose(gb, gd["gb"], rtol=1e-14, atol=1e-13)
    perm = oracle.merged_permutation(a.astype(np.float32), b.astype(np.float32))
    assert perm.tolist() == [int(v) for v in gd["perm"]]


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_golden_gram(oracle, route):
    gd = read_golden("gram_rational_3.txt")
    a = np.log(np.array(gd["exp_a"]))
    x = np.array(gd["x"]).reshape(-1, 1); g = np.array(gd["g"]).reshape(-1, 1)
    if route == "brute":
        y, _ = oracle.gram_brute(a, x)
        (gx, ga), _ = oracle.gram_backward_brute(a, x, g)
    else:
        y, _ = oracle.gram_scan(a, x)
        (gx, ga), _ = oracle.gram_backward_scan(a, x, g)
    np.testing.assert_allclose(y[:, 0], gd["y"], rtol=1e-14)
    np.testing.assert_allclose(gx[:, 0], gd["gx"], rtol=1e-14)
    np.testing.assert_allclose(ga, gd["ga"], rtol=1e-14, atol=1e-13)
    assert oracle.merged_permutation(a.astype(np.float32)).tolist() == [int(v) for v in gd["perm"]]


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("n", [1, 2, 9, 257])
@pytest.mark.parametrize("route", ["brute", "scan"])
def test_uniform_grid_geometric_closed_form(oracle, n, route):
    """a_i = b_i = i*delta, x = 1: rows of the Toeplitz matrix rho^|i-j| sum to
    (1 + rho - rho^(i+1) - rho^(n-i)) / (1 - rho)  (two geometric series)."""
    delta = 1.0 / n
    rho = math.exp(-delta)
    a = np.arange(n) * delta
    x = np.ones((n, 1))
    y = (oracle.apply_brute if route == "brute" else oracle.apply_scan)(a, a, x)[0][:, 0]
    i = np.arange(n)
    want = (1 + rho - rho ** (i + 1) - rho ** (n - i)) / (1 - rho)
    np.testing.assert_allclose(y, want, rtol=1e-12)
    yg = (oracle.gram_brute if route == "brute" else oracle.gram_scan)(a, x)[0][:, 0]
    np.testing.assert_allclose(yg, want, rtol=1e-12)


def tridiagonal_inverse_apply(a_sorted, y):
    """K^{-1} y for K_ij = exp(-|a_i-a_j|), a strictly increasing: the
    Ornstein-Uhlenbeck / AR(1) precision matrix, tridiagonal with
    rho_i = exp(-(a_{i+1}-a_i)), off-diagonals -rho_i/(1-rho_i^2), diagonal
    1 + rho_{i-1}^2/(1-rho_{i-1}^2) + rho_i^2/(1-rho_i^2) (absent neighbours dropped)."""
    n = a_sorted.size
    rho = np.exp(-np.diff(a_sorted))
    r2 = rho ** 2 / (1 - rho ** 2)
    off = -rho / (1 - rho ** 2)
    diag = np.ones(n)
    diag[:-1] += r2
    diag[1:] += r2
    out = diag[:, None] * y
    out[:-1] += off[:, None] * y[1:]
    out[1:] += off[:, None] * y[:-1]
    return out


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_gram_tridiagonal_inverse_recovers_x(oracle, route):
    r = rng(3)
    n, batch = 200, 3
    a_sorted = np.cumsum(r.uniform(0.05, 1.5, n))
    p = r.permutation(n)
    a = a_sorted[p]                              # oracle sees unsorted anchors
    x = r.normal(size=(n, batch))
    y = (oracle.gram_brute if route == "brute" else oracle.gram_scan)(a, x)[0]
    inv = np.empty(n, dtype=int); inv[p] = np.arange(n)
    x_back = tridiagonal_inverse_apply(a_sorted, y[inv])     # rows back in sorted order
    np.testing.assert_allclose(x_back, x[inv], rtol=1e-9, atol=1e-9)


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_countsketch_limit_is_exact_bucket_sum(oracle, route):
    """App. A (Lemma 1 / Prop. 1): with anchors equal to well separated labels,
    L(a,b) becomes the indicator of a_i == b_j, so y is a bucket sum."""
    r = rng(4)
    k, n, batch = 7, 60, 2
    labels = 800.0 * np.arange(k)          # exp(-800) == 0 in fp64
    h = r.integers(0, k, n)
    x = r.normal(size=(n, batch))
    f = oracle.apply_brute if route == "brute" else oracle.apply_scan
    y = f(labels, labels[h], x)[0]
    want = np.zeros((k, batch))
    np.add.at(want, h, x)
    np.testing.assert_allclose(y, want, rtol=1e-14, atol=1e-14)


def test_one_hot_reads_matrix_entry(oracle):
    r = rng(5)
    a = r.uniform(-3, 3, 6); b = r.uniform(-3, 3, 5)
    for j in range(5):
        x = np.zeros((5, 1)); x[j] = 1.0
        y = oracle.apply_scan(a, b, x)[0][:, 0]
        for i in range(6):
            assert y[i] == pytest.approx(math.exp(-abs(a[i] - b[j])), rel=1e-13)


# ---------------------------------------------------------------- invariants

def test_gram_symmetry_unit_diagonal_positive(oracle):
    r = rng(6)
    n = 40
    a = r.normal(size=n) * 2
    e = np.eye(n)
    K = oracle.gram_scan(a, e)[0]                # columns of K
    np.testing.assert_allclose(np.diag(K), 1.0, rtol=0, atol=1e-15)
    np.testing.assert_allclose(K, K.T, rtol=1e-13)
    assert np.linalg.eigvalsh((K + K.T) / 2).min() > 0
    u = r.normal(size=(n, 1)); v = r.normal(size=(n, 1))
    assert (u.T @ oracle.gram_brute(a, v)[0]).item() == pytest.approx(
        (v.T @ oracle.gram_brute(a, u)[0]).item(), rel=1e-12)


def test_permuting_anchors_permutes_result(oracle):
    r = rng(7)
    n = 33
    a = np.round(r.normal(size=n) * 2, 1)        # duplicates
    x = r.normal(size=(n, 2))
    p = r.permutation(n)
    y = oracle.gram_scan(a, x)[0]
    np.testing.assert_allclose(oracle.gram_scan(a[p], x[p])[0], y[p], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_translation_and_reflection(oracle, route):
    r = rng(8)
    a = r.uniform(0, 8, 11); b = r.uniform(0, 8, 17)
    x = r.normal(size=(17, 2)); g = r.normal(size=(11, 2))
    f = oracle.apply_brute if route == "brute" else oracle.apply_scan
    fb = oracle.apply_backward_brute if route == "brute" else oracle.apply_backward_scan
    y = f(a, b, x)[0]
    np.testing.assert_allclose(f(a + 4.0, b + 4.0, x)[0], y, rtol=1e-12)
    np.testing.assert_allclose(f(-a, -b, x)[0], y, rtol=1e-12)
    (gx, ga, gb), _ = fb(a, b, x, g)
    assert abs(ga.sum() + gb.sum()) < 1e-11 * (np.abs(ga).sum() + np.abs(gb).sum())
    (gx2, ga2, gb2), _ = fb(-a, -b, x, g)        # reflection flips anchor gradients
    np.testing.assert_allclose(gx2, gx, rtol=1e-12)
    np.testing.assert_allclose(ga2, -ga, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(gb2, -gb, rtol=1e-11, atol=1e-12)


def test_transpose_identity(oracle):
    """L(a,b)^T = L(b,a): the input gradient is the apply with roles swapped."""
    r = rng(9)
    a = r.uniform(0, 5, 9); b = r.uniform(0, 5, 14)
    x = r.normal(size=(14, 1)); g = r.normal(size=(9, 3))
    (gx, _, _), _ = oracle.apply_backward_scan(a, b, np.repeat(x, 3, 1), g)
    np.testing.assert_allclose(gx, oracle.apply_brute(b, a, g)[0], rtol=1e-12)


# ---------------------------------------------------------------- dense library route

def test_against_numpy_dense_matmul(oracle):
    r = rng(10)
    a = r.uniform(0, 20, 50); b = r.uniform(0, 20, 70)
    x = r.normal(size=(70, 4))
    dense = np.exp(-np.abs(a[:, None] - b[None, :]))
    for f in (oracle.apply_brute, oracle.apply_scan):
        y, tol = f(a, b, x)
        np.testing.assert_allclose(y, dense @ x, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(tol, dense @ np.abs(x), rtol=1e-12)


# ---------------------------------------------------------------- finite differences

def _loss(oracle, a, b, x, g):
    return float(np.sum(g * oracle.apply_brute(a, b, x)[0]))


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_apply_gradients_central_differences(oracle, route):
    r = rng(11)
    k, n, batch = 6, 8, 2
    a = r.uniform(0, 4, k); b = r.uniform(0, 4, n)
    x = r.normal(size=(n, batch)); g = r.normal(size=(k, batch))
    fb = oracle.apply_backward_brute if route == "brute" else oracle.apply_backward_scan
    (gx, ga, gb), _ = fb(a, b, x, g)
    h = 1e-6
    for i in range(k):
        d = np.zeros(k); d[i] = h
        fd = (_loss(oracle, a + d, b, x, g) - _loss(oracle, a - d, b, x, g)) / (2 * h)
        assert ga[i] == pytest.approx(fd, rel=1e-6, abs=1e-8)
    for j in range(n):
        d = np.zeros(n); d[j] = h
        fd = (_loss(oracle, a, b + d, x, g) - _loss(oracle, a, b - d, x, g)) / (2 * h)
        assert gb[j] == pytest.approx(fd, rel=1e-6, abs=1e-8)
        for t in range(batch):
            dx = np.zeros_like(x); dx[j, t] = 1.0
            assert gx[j, t] == pytest.approx(
                _loss(oracle, a, b, x + dx, g) - _loss(oracle, a, b, x, g), rel=1e-9, abs=1e-10)


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_anchor_gradient_at_exact_ties_is_central_difference(oracle, route):
    """sgn(0) = 0: at a_i == b_j the two one-sided slopes cancel in the central
    difference, and so they do in the analytic gradient."""
    a = np.array([1.0, 2.0, 2.0, 3.5]); b = np.array([2.0, 1.0, 3.5, 2.0, 0.25])
    r = rng(12)
    x = r.normal(size=(5, 2)); g = r.normal(size=(4, 2))
    fb = oracle.apply_backward_brute if route == "brute" else oracle.apply_backward_scan
    (_, ga, gb), _ = fb(a, b, x, g)
    h = 1e-6
    for i in range(4):
        d = np.zeros(4); d[i] = h
        fd = (_loss(oracle, a + d, b, x, g) - _loss(oracle, a - d, b, x, g)) / (2 * h)
        assert ga[i] == pytest.approx(fd, rel=1e-6, abs=1e-8)
    for j in range(5):
        d = np.zeros(5); d[j] = h
        fd = (_loss(oracle, a, b + d, x, g) - _loss(oracle, a, b - d, x, g)) / (2 * h)
        assert gb[j] == pytest.approx(fd, rel=1e-6, abs=1e-8)


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_gram_gradients_central_differences(oracle, route):
    r = rng(13)
    n, batch = 7, 2
    a = r.uniform(0, 3, n); a[4] = a[1]          # one duplicated anchor
    x = r.normal(size=(n, batch)); g = r.normal(size=(n, batch))
    fb = oracle.gram_backward_brute if route == "brute" else oracle.gram_backward_scan
    (gx, ga), _ = fb(a, x, g)
    np.testing.assert_allclose(gx, oracle.gram_brute(a, g)[0], rtol=1e-12)
    h = 1e-6
    loss = lambda aa: float(np.sum(g * oracle.gram_brute(aa, x)[0]))
    for m in range(n):
        d = np.zeros(n); d[m] = h
        assert ga[m] == pytest.approx((loss(a + d) - loss(a - d)) / (2 * h), rel=1e-6, abs=1e-8)
    assert abs(ga.sum()) < 1e-10 * np.abs(ga).sum()


# ---------------------------------------------------------------- route against route

CASES = {
    "uniform": lambda r, k, n: (r.uniform(0, 30, k), r.uniform(0, 30, n)),
    "ties": lambda r, k, n: (np.round(r.uniform(0, 8, k) * 4) / 4, np.round(r.uniform(0, 8, n) * 4) / 4),
    "all_equal": lambda r, k, n: (np.full(k, 1.5), np.full(n, 1.5)),
    "huge_gaps": lambda r, k, n: (r.integers(0, 6, k) * 900.0, r.integers(0, 6, n) * 900.0 + 0.5),
    "negative": lambda r, k, n: (-r.uniform(0, 10, k), r.normal(size=n) * 3),
    "outside": lambda r, k, n: (np.concatenate([[-50.0], r.uniform(0, 5, k - 2), [60.0]]), r.uniform(1, 4, n)),
}


@pytest.mark.parametrize("case", sorted(CASES))
@pytest.mark.parametrize("k,n,batch", [(1, 1, 1), (5, 1, 2), (1, 6, 1), (37, 53, 3)])
def test_scan_route_matches_brute_force(oracle, case, k, n, batch):
    if case == "outside" and k < 3:
        pytest.skip("needs k >= 3")
    r = rng(100 + k + n)
    a, b = CASES[case](r, k, n)
    a = a.astype(np.float32); b = b.astype(np.float32)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    y0, t0 = oracle.apply_brute(a, b, x); y1, t1 = oracle.apply_scan(a, b, x)
    assert np.all(np.abs(y0 - y1) <= 1e-12 * t0 + 1e-300)
    np.testing.assert_allclose(t1, t0, rtol=1e-12)
    (gx0, ga0, gb0), (tx0, ta0, tb0) = oracle.apply_backward_brute(a, b, x, g)
    (gx1, ga1, gb1), (tx1, ta1, tb1) = oracle.apply_backward_scan(a, b, x, g)
    assert np.all(np.abs(gx0 - gx1) <= 1e-12 * tx0 + 1e-300)
    assert np.all(np.abs(ga0 - ga1) <= 1e-12 * ta0 + 1e-300)
    assert np.all(np.abs(gb0 - gb1) <= 1e-12 * tb0 + 1e-300)
    for u, v in ((tx0, tx1), (ta0, ta1), (tb0, tb1)):
        np.testing.assert_allclose(v, u, rtol=1e-12, atol=1e-300)


@pytest.mark.parametrize("case", ["uniform", "ties", "all_equal", "huge_gaps"])
def test_gram_scan_route_matches_brute_force(oracle, case):
    r = rng(200)
    a, _ = CASES[case](r, 41, 1)
    a = a.astype(np.float32)
    x = r.normal(size=(41, 2)); g = r.normal(size=(41, 2))
    y0, t0 = oracle.gram_brute(a, x); y1, t1 = oracle.gram_scan(a, x)
    assert np.all(np.abs(y0 - y1) <= 1e-12 * t0)
    (gx0, ga0), (tx0, ta0) = oracle.gram_backward_brute(a, x, g)
    (gx1, ga1), (tx1, ta1) = oracle.gram_backward_scan(a, x, g)
    assert np.all(np.abs(gx0 - gx1) <= 1e-12 * tx0)
    assert np.all(np.abs(ga0 - ga1) <= 1e-12 * ta0 + 1e-300)
    np.testing.assert_allclose(ta1, ta0, rtol=1e-12)


def test_window_route_matches_brute_force(oracle):
    r = rng(300)
    b = r.uniform(0, 400, 3000).astype(np.float32); a = r.uniform(-10, 410, 200).astype(np.float32)
    x = r.normal(size=(3000, 1)).astype(np.float32)
    y0, t0 = oracle.apply_brute(a, b, x)
    y1, t1 = oracle.apply_window(a, b, x, window=64.0)
    bound = math.exp(-64.0) * np.abs(x).sum()
    assert np.all(np.abs(y0[:, 0] - y1) <= 1e-13 * t0[:, 0] + bound)
    assert np.all(np.abs(t0[:, 0] - t1) <= 1e-13 * t0[:, 0] + bound)


def test_empty_input_side(oracle):
    y, tol = oracle.apply_scan(np.array([1.0, 2.0]), np.zeros(0), np.zeros((0, 2)))
    assert y.shape == (2, 2) and not y.any() and not tol.any()


# ---------------------------------------------------------------- merged order

def test_merged_permutation_is_stable_with_outputs_first(oracle):
    a = np.array([2.0, -0.0, 1.0, 2.0], dtype=np.float32)
    b = np.array([0.0, 2.0, -3.0, 1.0], dtype=np.float32)
    # keys: -3(b2) | 0(a1), 0(b0) | 1(a2), 1(b3) | 2(a0), 2(a3), 2(b1); signed zeros tie
    assert oracle.merged_permutation(a, b).tolist() == [6, 1, 4, 2, 7, 0, 3, 5]


def test_merged_permutation_brute_force_rank(oracle):
    r = rng(14)
    m = np.round(r.normal(size=300) * 3).astype(np.float32)
    perm = oracle.merged_permutation(m[:120], m[120:])
    # rank of id i = #{j : m_j < m_i} + #{j < i : m_j == m_i}
    rank = np.array([(m < m[i]).sum() + (m[:i] == m[i]).sum() for i in range(300)])
    want = np.empty(300, dtype=np.int64); want[rank] = np.arange(300)
    assert perm.tolist() == want.tolist()


# ---------------------------------------------------------------- phased kernel

def _phased_routes(oracle, route):
    if route == "brute":
        return oracle.phased_apply_brute, oracle.phased_backward_brute
    return oracle.phased_apply_scan, oracle.phased_backward_scan


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_golden_phased(oracle, route):
    gd = read_golden("phased_rational_3x2.txt")
    a = np.log(np.array(gd["exp_a"])); b = np.log(np.array(gd["exp_b"]))
    phi = np.array(gd["phi_thirds"]) * math.pi / 3; psi = np.array(gd["psi_thirds"]) * math.pi / 3
    x = np.array(gd["x"]).reshape(-1, 1); g = np.array(gd["g"]).reshape(-1, 1)
    fwd, bwd = _phased_routes(oracle, route)
    y, _ = fwd(a, phi, b, psi, x)
    (gx, ga, gb, gphi, gpsi), _ = bwd(a, phi, b, psi, x, g)
    np.testing.assert_allclose(y[:, 0], gd["y"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(gx[:, 0], gd["gx"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(ga, gd["ga"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(gb, gd["gb"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(gphi / math.sqrt(3), gd["gphi_over_sqrt3"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(gpsi / math.sqrt(3), gd["gpsi_over_sqrt3"], rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_phased_with_zero_phases_is_the_plain_kernel(oracle, route):
    r = rng(41)
    k, n, batch = 9, 14, 3
    a = np.round(r.uniform(0, 3, k) * 2) / 2; b = np.round(r.uniform(0, 3, n) * 2) / 2      # with ties
    x = r.normal(size=(n, batch)); g = r.normal(size=(k, batch))
    fwd, bwd = _phased_routes(oracle, route)
    y, tol = fwd(a, np.zeros(k), b, np.zeros(n), x)
    (gx, ga, gb, gphi, gpsi), _ = bwd(a, np.zeros(k), b, np.zeros(n), x, g)
    y0, tol0 = oracle.apply_brute(a, b, x)
    (gx0, ga0, gb0), _ = oracle.apply_backward_brute(a, b, x, g)
    np.testing.assert_allclose(y, y0, atol=1e-13); np.testing.assert_allclose(tol, tol0, atol=1e-13)
    np.testing.assert_allclose(gx, gx0, atol=1e-13)
    np.testing.assert_allclose(ga, ga0, atol=1e-12); np.testing.assert_allclose(gb, gb0, atol=1e-12)
    assert np.all(gphi == 0) and np.all(gpsi == 0)


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_phased_closed_forms_and_invariances(oracle, route):
    fwd, bwd = _phased_routes(oracle, route)
    # one anchor each: the matrix entry itself
    y, _ = fwd([0.3], [1.1], [1.0], [0.4], [[2.0]])
    assert y[0, 0] == pytest.approx(2.0 * math.exp(-0.7) * math.cos(0.7), rel=1e-14)
    r = rng(42)
    k, n, batch = 8, 12, 2
    a = r.uniform(0, 3, k); b = r.uniform(0, 3, n); phi = r.uniform(-3, 3, k); psi = r.uniform(-3, 3, n)
    x = r.normal(size=(n, batch)); g = r.normal(size=(k, batch))
    y, _ = fwd(a, phi, b, psi, x)
    # quadrature: every phase difference pi/2 -> nothing passes
    yq, tq = fwd(a, np.full(k, 0.25 + math.pi / 2), b, np.full(n, 0.25), x)
    assert np.all(np.abs(yq) <= 1e-15 * tq + 1e-300)
    # opposite phase: the plain product with the sign flipped
    yo, _ = fwd(a, np.full(k, math.pi), b, np.zeros(n), x)
    np.testing.assert_allclose(yo, -oracle.apply_brute(a, b, x)[0], atol=1e-13)
    # a common shift of all phases changes nothing; the phase gradients sum to zero, the anchor gradients too
    ys, _ = fwd(a, phi + 0.9, b, psi + 0.9, x)
    np.testing.assert_allclose(ys, y, atol=1e-13)
    (gx, ga, gb, gphi, gpsi), _ = bwd(a, phi, b, psi, x, g)
    assert gphi.sum() + gpsi.sum() == pytest.approx(0.0, abs=1e-12)
    assert ga.sum() + gb.sum() == pytest.approx(0.0, abs=1e-12)
    # transposition: sum(g * P x) = sum(x * P^T g)
    assert float(np.sum(g * y)) == pytest.approx(float(np.sum(x * gx)), rel=1e-12)


@pytest.mark.parametrize("route", ["brute", "scan"])
def test_phased_gradients_central_differences(oracle, route):
    r = rng(43)
    k, n, batch = 5, 7, 2
    a = r.uniform(0, 4, k); b = r.uniform(0, 4, n); phi = r.uniform(-3, 3, k); psi = r.uniform(-3, 3, n)
    x = r.normal(size=(n, batch)); g = r.normal(size=(k, batch))
    _, bwd = _phased_routes(oracle, route)
    (gx, ga, gb, gphi, gpsi), _ = bwd(a, phi, b, psi, x, g)

    def loss(a_, phi_, b_, psi_, x_):
        return float(np.sum(g * oracle.phased_apply_brute(a_, phi_, b_, psi_, x_)[0]))

    h = 1e-6
    for name, grad, idx in (("a", ga, 0), ("phi", gphi, 1), ("b", gb, 2), ("psi", gpsi, 3)):
        args = [a, phi, b, psi, x]
        for i in range(grad.size):
            d = np.zeros(grad.size); d[i] = h
            up = list(args); up[idx] = args[idx] + d
            dn = list(args); dn[idx] = args[idx] - d
            fd = (loss(*up) - loss(*dn)) / (2 * h)
            assert grad[i] == pytest.approx(fd, rel=1e-6, abs=1e-8), name
    for j in range(n):
        for t in range(batch):
            dx = np.zeros_like(x); dx[j, t] = 1.0
            assert gx[j, t] == pytest.approx(loss(a, phi, b, psi, x + dx) - loss(a, phi, b, psi, x), rel=1e-9, abs=1e-10)


def test_phased_scan_route_matches_brute_force(oracle):
    r = rng(44)
    k, n, batch = 300, 700, 3
    a = np.round(r.uniform(0, 12, k) * 8) / 8; b = np.round(r.uniform(0, 12, n) * 8) / 8       # many exact ties
    phi = r.uniform(-6, 6, k); psi = r.uniform(-6, 6, n)
    x = r.normal(size=(n, batch)); g = r.normal(size=(k, batch))
    y, tol = oracle.phased_apply_brute(a, phi, b, psi, x)
    ys, tols = oracle.phased_apply_scan(a, phi, b, psi, x)
    assert np.all(np.abs(y - ys) <= 1e-12 * tol + 1e-300)
    np.testing.assert_allclose(tols, tol, rtol=1e-12)
    G, T = oracle.phased_backward_brute(a, phi, b, psi, x, g)
    Gs, Ts = oracle.phased_backward_scan(a, phi, b, psi, x, g)
    for u, v, t, ts in zip(G, Gs, T, Ts):
        assert np.all(np.abs(u - v) <= 1e-11 * t + 1e-300)
        np.testing.assert_allclose(ts, t, rtol=1e-11)


# ---------------------------------------------------------------- temperature

def test_temperature_is_scaling_of_the_anchors(oracle):
    r = rng(51)
    k, n, batch = 7, 9, 2
    a = r.uniform(0, 3, k); b = r.uniform(0, 3, n); x = r.normal(size=(n, batch))
    for tau in (0.25, 1.0, 3.5):
        y, tol = oracle.tau_apply_dense(a, b, tau, x)
        ys, tols = oracle.tau_apply(a, b, tau, x, fp32=False)
        np.testing.assert_allclose(ys, y, atol=1e-13); np.testing.assert_allclose(tols, tol, atol=1e-13)


def test_zero_temperature_limit_is_equality_routing(oracle):
    """App. A, Lemma "Zero-temperature limit": as t -> 0 the matrix tends to 1{a_i == b_j}."""
    r = rng(52)
    labels = np.arange(6, dtype=np.float64)
    b = labels[r.integers(0, 6, 40)]; x = r.normal(size=(40, 3))
    y, _ = oracle.tau_apply(labels, b, 800.0, x)
    want = np.stack([x[b == c].sum(axis=0) for c in labels])
    np.testing.assert_allclose(y, want, atol=1e-300, rtol=1e-15)


@pytest.mark.parametrize("brute", [True, False])
def test_temperature_gradients_central_differences(oracle, brute):
    r = rng(53)
    k, n, batch, tau = 5, 8, 2, 1.7
    a = r.uniform(0, 3, k); b = r.uniform(0, 3, n)
    x = r.normal(size=(n, batch)); g = r.normal(size=(k, batch))
    (gx, ga, gb, gtau), _ = oracle.tau_backward(a, b, tau, x, g, fp32=False, brute=brute)

    def loss(a_, b_, t_):
        return float(np.sum(g * oracle.tau_apply_dense(a_, b_, t_, x)[0]))

    h = 1e-6
    assert gtau == pytest.approx((loss(a, b, tau + h) - loss(a, b, tau - h)) / (2 * h), rel=1e-6, abs=1e-8)
    for i in range(k):
        d = np.zeros(k); d[i] = h
        assert ga[i] == pytest.approx((loss(a + d, b, tau) - loss(a - d, b, tau)) / (2 * h), rel=1e-6, abs=1e-8)
    for j in range(n):
        d = np.zeros(n); d[j] = h
        assert gb[j] == pytest.approx((loss(a, b + d, tau) - loss(a, b - d, tau)) / (2 * h), rel=1e-6, abs=1e-8)
    np.testing.assert_allclose(gx, oracle.tau_apply_dense(b, a, tau, g)[0], atol=1e-13)     # the transposed operator
    # Euler: the kernel depends on tau * (a, b) only
    assert gtau * tau == pytest.approx(float(np.dot(a, ga) + np.dot(b, gb)), rel=1e-12)


def test_temperature_gram_gradient_central_difference(oracle):
    r = rng(54)
    n, batch, tau = 7, 2, 0.6
    a = r.uniform(0, 5, n); x = r.normal(size=(n, batch)); g = r.normal(size=(n, batch))
    (gx, ga, gtau), _ = oracle.tau_gram_backward(a, tau, x, g, fp32=False)

    def loss(a_, t_):
        return float(np.sum(g * oracle.tau_apply_dense(a_, a_, t_, x)[0]))

    h = 1e-6
    assert gtau == pytest.approx((loss(a, tau + h) - loss(a, tau - h)) / (2 * h), rel=1e-6, abs=1e-8)
    for i in range(n):
        d = np.zeros(n); d[i] = h
        assert ga[i] == pytest.approx((loss(a + d, tau) - loss(a - d, tau)) / (2 * h), rel=1e-6, abs=1e-8)


def test_scaled_anchors_fp32_is_the_correctly_rounded_product(oracle):
    """scaled_anchors(fp32=True) is fl32(fl32(tau) * a_i): pinned against the product formed exactly (two 24-bit
    significands multiply exactly in fp64) and rounded to fp32 once; it is monotone, so equal anchors stay equal
    and the order of distinct ones is never reversed."""
    r = rng(55)
    a = np.concatenate([r.uniform(0, 2.0 ** 14, 4000), -r.uniform(0, 3, 500), [0.0, -0.0, 2.0 ** 14, 1e-30]]).astype(np.float32)
    for tau in (0.37, 1.0, 5.0, 1.0 / 3.0):
        got = oracle.scaled_anchors(a, tau)
        assert got.dtype == np.float32
        exact = np.float64(np.float32(tau)) * a.astype(np.float64)          # exact: 48 significant bits at most
        np.testing.assert_array_equal(got, exact.astype(np.float32))
        order = np.argsort(a, kind="stable")
        assert np.all(np.diff(got[order].astype(np.float64)) >= 0)
        np.testing.assert_array_equal(oracle.scaled_anchors(a, tau, fp32=False), float(tau) * a.astype(np.float64))


def test_temperature_fp32_route_is_within_the_input_rounding_of_the_definition(oracle):
    """How far the route on fp32-rounded products tau*a, tau*b (the one the GPU parity tests use) can be from
    the definition exp(-tau |a_i - b_j|) (App. A): each rounded product is off by at most 2^-24 of itself, so an
    exponent moves by at most delta = 2^-24 tau (|a_i| + |b_j|) and the sum by at most (e^delta - 1) T."""
    r = rng(56)
    k, n, batch = 60, 900, 3
    for top, tau in ((2.0 ** 14, 5.0), (2.0 ** 14, 0.37), (64.0, 5.0)):
        a = r.uniform(0, top, k).astype(np.float32); b = r.uniform(0, top, n).astype(np.float32)
        b[:50] = a[r.integers(0, k, 50)] + np.float32(0.001)               # near neighbours: terms of order one
        x = r.normal(size=(n, batch))
        y_def, t_def = oracle.tau_apply_dense(a, b, tau, x)
        y_32, _ = oracle.tau_apply(a, b, tau, x, fp32=True)
        delta = 2.0 ** -24 * tau * 2 * top
        assert np.all(np.abs(y_32 - y_def) <= np.expm1(delta) * t_def + 1e-300)
        assert np.abs(y_32 - y_def).max() > 0                                  # and the routes do differ


def test_gram_gradient_denominators_against_numpy(oracle):
    """tgx, tga of both Gram backward routes are the sums over absolute values of the summands of gx, ga
    (the dense kernel matrix formed with numpy, duplicates included)."""
    r = rng(57)
    n, batch = 40, 3
    a = r.uniform(0, 6, n); a[7] = a[3]; a[20] = a[21]
    x = r.normal(size=(n, batch)); g = r.normal(size=(n, batch))
    K = np.exp(-np.abs(a[:, None] - a[None, :]))
    want_tgx = K @ np.abs(g)
    want_tga = np.sum(np.abs(g) * (K @ np.abs(x)) + np.abs(x) * (K @ np.abs(g)), axis=1)
    S = -np.sign(a[:, None] - a[None, :])
    want_ga = np.sum(g * ((S * K) @ x) + x * ((S * K) @ g), axis=1)
    for f in (oracle.gram_backward_brute, oracle.gram_backward_scan):
        (gx, ga), (tgx, tga) = f(a, x, g)
        np.testing.assert_allclose(tgx, want_tgx, rtol=1e-12)
        np.testing.assert_allclose(tga, want_tga, rtol=1e-12)
        np.testing.assert_allclose(gx, K @ g, rtol=1e-11, atol=1e-13)
        assert np.all(np.abs(ga - want_ga) <= 1e-12 * want_tga)


# ---------------------------------------------------------------- weighted Gram matrix

@pytest.mark.parametrize("route", ["dense", "scan"])
def test_golden_weighted_gram(oracle, route):
    gd = read_golden("wgram_rational_2x3.txt")
    a = np.log(np.array(gd["exp_a"])); b = np.log(np.array(gd["exp_b"])); d = np.array(gd["d"])
    M, T = (oracle.wgram_dense if route == "dense" else oracle.wgram_scan)(a, b, d)
    np.testing.assert_allclose(M, [gd["m_row0"], gd["m_row1"]], rtol=1e-14)
    np.testing.assert_allclose(T, M, rtol=1e-14)                  # positive weights


@pytest.mark.parametrize("route", ["dense", "scan"])
def test_weighted_gram_is_the_composition_of_two_applies(oracle, route):
    """M z = A (d * (A^T z)), with A z' and A^T z from the pinned apply (L(a,b)^T = L(b,a))."""
    r = rng(61)
    k, n = 9, 23
    a = r.uniform(0, 4, k); b = r.uniform(-1, 5, n); d = r.normal(size=n); z = r.normal(size=(k, 2))
    b[3] = a[2]; b[7] = a[2]; a[5] = a[2]                        # ties between and inside the two sets
    M, _ = (oracle.wgram_dense if route == "dense" else oracle.wgram_scan)(a, b, d)
    atz, _ = oracle.apply_brute(b, a, z)
    want, _ = oracle.apply_brute(a, b, d[:, None] * atz)
    np.testing.assert_allclose(M @ z, want, atol=1e-12)
    np.testing.assert_allclose(M, M.T, atol=1e-14)


@pytest.mark.parametrize("route", ["dense", "scan"])
def test_weighted_gram_special_cases(oracle, route):
    f = oracle.wgram_dense if route == "dense" else oracle.wgram_scan
    r = rng(62)
    k, n = 7, 15
    a = r.uniform(0, 3, k); b = r.uniform(0, 3, n)
    # one unit weight: the outer product of a column of A with itself
    for t in (0, 6, n - 1):
        d = np.zeros(n); d[t] = 1.0
        col = np.exp(-np.abs(a - b[t]))
        np.testing.assert_allclose(f(a, b, d)[0], np.outer(col, col), atol=1e-15)
    # every middle anchor at one point c left of all a: M_ij = e^{-(a_i - c)} e^{-(a_j - c)} sum(d)
    d = r.normal(size=n); c = -2.5
    e = np.exp(-(a - c))
    np.testing.assert_allclose(f(a, np.full(n, c), d)[0], np.outer(e, e) * d.sum(), atol=1e-14)
    # one Gram anchor: the scalar sum_t d_t exp(-2 |a - b_t|), a plain apply on the doubled anchors
    y, _ = oracle.apply_brute(2 * a[:1], 2 * b, d[:, None])
    np.testing.assert_allclose(f(a[:1], b, d)[0], y, atol=1e-14)
    # non-negative weights: positive semi-definite
    M, T = f(a, b, np.abs(d))
    assert np.linalg.eigvalsh(M).min() > -1e-12
    np.testing.assert_allclose(T, M, rtol=1e-13)
    # depends on differences only; reflection swaps left and right
    M0 = f(a, b, d)[0]
    np.testing.assert_allclose(f(a + 7.0, b + 7.0, d)[0], M0, atol=1e-13)
    np.testing.assert_allclose(f(-a, -b, d)[0], M0, atol=1e-13)
    # permuting the Gram anchors permutes rows and columns
    p = r.permutation(k)
    np.testing.assert_allclose(f(a[p], b, d)[0], M0[np.ix_(p, p)], atol=1e-14)


@pytest.mark.parametrize("kind", ["uniform", "ties", "all_equal", "huge_gaps", "outside"])
def test_weighted_gram_routes_agree(oracle, kind):
    r = rng(63)
    k, n = 40, 500
    if kind == "uniform":
        a, b = r.uniform(0, 8, k), r.uniform(0, 8, n)
    elif kind == "ties":
        a, b = np.round(r.uniform(0, 6, k) * 2) / 2, np.round(r.uniform(0, 6, n) * 2) / 2
    elif kind == "all_equal":
        a, b = np.full(k, 1.5), np.full(n, 1.5)
    elif kind == "huge_gaps":      # intervals 600 wide: e^{2 * 600} would overflow, the decays underflow to 0
        a, b = r.integers(0, 5, k) * 600.0, r.integers(0, 5, n) * 600.0 + r.integers(0, 3, n) * 0.25
    else:                          # every middle anchor outside the range of a, on both sides
        a, b = r.uniform(10, 12, k), np.concatenate([r.uniform(5, 9, n // 2), r.uniform(13, 20, n - n // 2)])
    d = r.normal(size=n)
    M, T = oracle.wgram_dense(a, b, d)
    Ms, Ts = oracle.wgram_scan(a, b, d)
    assert np.all(np.isfinite(Ms))
    assert np.all(np.abs(M - Ms) <= 1e-12 * T + 1e-300)
    np.testing.assert_allclose(Ts, T, rtol=1e-12, atol=1e-300)


# ---------------------------------------------------------------- LAPLEX^(r): weighted sums of operators

def _mix_case(seed, r=3, k=5, n=7, batch=2):
    q = rng(seed)
    a = q.uniform(0, 3, (r, k)); b = q.uniform(0, 3, (r, n)); w = q.normal(size=r)
    x = q.normal(size=(n, batch)); g = q.normal(size=(k, batch))
    return a, b, w, x, g


def test_mix_is_the_dense_weighted_sum(oracle):
    a, b, w, x, g = _mix_case(71)
    dense = sum(w[q] * np.exp(-np.abs(a[q][:, None] - b[q][None, :])) for q in range(w.size))
    for brute in (True, False):
        y, tol = oracle.mix_apply(a, b, w, x, brute=brute)
        np.testing.assert_allclose(y, dense @ x, atol=1e-13)
        (gx, ga, gb, gw), _ = oracle.mix_backward(a, b, w, x, g, brute=brute)
        np.testing.assert_allclose(gx, dense.T @ g, atol=1e-13)
    # one operator with weight 1 is the plain apply; the golden example, doubled and negated, cancels
    y1, _ = oracle.mix_apply(a[:1], b[:1], [1.0], x)
    np.testing.assert_array_equal(y1, oracle.apply_brute(a[0], b[0], x)[0])
    gd = read_golden("apply_rational_3x2.txt")
    ea = np.log(np.array(gd["exp_a"])); eb = np.log(np.array(gd["exp_b"])); ex = np.array(gd["x"]).reshape(-1, 1)
    y2, _ = oracle.mix_apply(np.stack([ea, ea]), np.stack([eb, eb]), [2.0, -0.5], ex)
    np.testing.assert_allclose(y2[:, 0], 1.5 * np.array(gd["y"]), rtol=1e-14)


def test_mix_gradients_central_differences(oracle):
    a, b, w, x, g = _mix_case(72)
    (gx, ga, gb, gw), _ = oracle.mix_backward(a, b, w, x, g)

    def loss(a_, b_, w_):
        dense = sum(w_[q] * np.exp(-np.abs(a_[q][:, None] - b_[q][None, :])) for q in range(w_.size))
        return float(np.sum(g * (dense @ x)))

    h = 1e-6
    for q in range(w.size):
        d = np.zeros_like(w); d[q] = h
        assert gw[q] == pytest.approx((loss(a, b, w + d) - loss(a, b, w - d)) / (2 * h), rel=1e-7, abs=1e-9)
        for i in range(a.shape[1]):
            d = np.zeros_like(a); d[q, i] = h
            assert ga[q, i] == pytest.approx((loss(a + d, b, w) - loss(a - d, b, w)) / (2 * h), rel=1e-6, abs=1e-8)
        for j in range(b.shape[1]):
            d = np.zeros_like(b); d[q, j] = h
            assert gb[q, j] == pytest.approx((loss(a, b + d, w) - loss(a, b - d, w)) / (2 * h), rel=1e-6, abs=1e-8)
    (gxs, gas, gbs, gws), _ = oracle.mix_backward(a, b, w, x, g, brute=False)
    for u, v in ((gx, gxs), (ga, gas), (gb, gbs), (gw, gws)):
        np.testing.assert_allclose(u, v, atol=1e-12)
