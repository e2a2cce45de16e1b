"""Pins of the linear-module oracle (oracle/linear.py): element-by-element sums written as loops, closed
forms (selection and all-ones weights), the adjoint identities that tie the two backward products to the
forward one, and central finite differences of L = <y, dy> in float64."""
import numpy as np

from oracle import linear as lin


def rnd(*shape, seed=0):
    return np.random.default_rng(seed).standard_normal(shape)


def test_every_element_by_loops():
    M, N, K = 5, 4, 7
    x, w, dy = rnd(M, K, seed=1), rnd(N, K, seed=2), rnd(M, N, seed=3)
    y, dx, dw = lin.linear_fwd(x, w), lin.linear_bwd_input(dy, w), lin.linear_bwd_weight(dy, x)
    for m in range(M):
        for n in range(N):
            assert abs(y[m, n] - sum(x[m, k] * w[n, k] for k in range(K))) < 1e-12
    for m in range(M):
        for k in range(K):
            assert abs(dx[m, k] - sum(dy[m, n] * w[n, k] for n in range(N))) < 1e-12
    for n in range(N):
        for k in range(K):
            assert abs(dw[n, k] - sum(dy[m, n] * x[m, k] for m in range(M))) < 1e-12


def test_selection_and_all_ones_weights():
    M, K = 6, 9
    x = rnd(M, K, seed=4)
    sel = np.zeros((3, K))
    sel[0, 2] = sel[1, 7] = sel[2, 0] = 1.0            # output n copies input column (2, 7, 0)
    np.testing.assert_array_equal(lin.linear_fwd(x, sel), x[:, [2, 7, 0]])
    np.testing.assert_allclose(lin.linear_fwd(x, np.ones((2, K)))[:, 0], x.sum(axis=1), rtol=1e-13)
    dy = rnd(M, 3, seed=5)
    dx = lin.linear_bwd_input(dy, sel)                 # gradient flows back to the selected columns only
    want = np.zeros((M, K))
    want[:, [2, 7, 0]] = dy
    np.testing.assert_array_equal(dx, want)


def test_backward_products_are_the_adjoints_of_the_forward():
    M, N, K = 11, 6, 13
    x, w, dy = rnd(M, K, seed=6), rnd(N, K, seed=7), rnd(M, N, seed=8)
    inner = np.sum(lin.linear_fwd(x, w) * dy)
    assert abs(inner - np.sum(lin.linear_bwd_input(dy, w) * x)) < 1e-10 * abs(inner) + 1e-10
    assert abs(inner - np.sum(lin.linear_bwd_weight(dy, x) * w)) < 1e-10 * abs(inner) + 1e-10


def test_gradients_by_central_differences():
    M, N, K = 4, 3, 5
    x, w, dy = rnd(M, K, seed=9), rnd(N, K, seed=10), rnd(M, N, seed=11)
    loss = lambda x_, w_: np.sum(lin.linear_fwd(x_, w_) * dy)
    dx, dw = lin.linear_bwd_input(dy, w), lin.linear_bwd_weight(dy, x)
    h = 1e-6
    for m in range(M):
        for k in range(K):
            e = np.zeros_like(x)
            e[m, k] = h
            assert abs((loss(x + e, w) - loss(x - e, w)) / (2 * h) - dx[m, k]) < 1e-7
    for n in range(N):
        for k in range(K):
            e = np.zeros_like(w)
            e[n, k] = h
            assert abs((loss(x, w + e) - loss(x, w - e)) / (2 * h) - dw[n, k]) < 1e-7


def test_shapes_and_transposition_are_not_interchangeable():
    """Rectangular shapes with M, N, K all different: a transposed operand cannot give the right shape."""
    M, N, K = 3, 4, 5
    x, w, dy = rnd(M, K), rnd(N, K), rnd(M, N)
    assert lin.linear_fwd(x, w).shape == (M, N)
    assert lin.linear_bwd_input(dy, w).shape == (M, K)
    assert lin.linear_bwd_weight(dy, x).shape == (N, K)
