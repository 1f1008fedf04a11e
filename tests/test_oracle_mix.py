"""Pins for the oracle's mix+step, mean and consensus distance (Algorithm 1 steps 4, 5, 7;
global form of Section 3; recursions in the proof of Theorem 1; Lemma 5)."""
import numpy as np
import pytest

import oracle


def ring_power_apply(n, k, X0):
    """W^k X0 for the ring through the circulant's Fourier diagonalisation (independent of the
    oracle's builder): DFT along the worker axis, scale mode m by lambda_m^k."""
    lam = (1.0 + 2.0 * np.cos(2.0 * np.pi * np.arange(n) / n)) / 3.0
    return np.real(np.fft.ifft((lam ** k)[:, None] * np.fft.fft(X0, axis=0), axis=0))


def ring_dense(n):
    W = np.zeros((n, n))
    for i in range(n):
        for j in (i - 1, i, i + 1):
            W[i, j % n] += 1.0 / 3.0
    return W


@pytest.mark.parametrize("n,d", [(8, 5), (16, 7), (33, 3)])
def test_mix_only_equals_fourier_power(n, d):
    rng = np.random.default_rng(n * 100 + d)
    X0 = rng.standard_normal((n, d))
    t = oracle.ring(n)
    X = X0.copy()
    for k in range(1, 13):
        X = oracle.mix_step(t, X, np.zeros_like(X), 0.3)
        np.testing.assert_allclose(X, ring_power_apply(n, k, X0), atol=1e-13)


def test_single_fourier_mode_is_scaled_by_its_eigenvalue():
    n, m = 16, 3
    mode = np.cos(2 * np.pi * m * np.arange(n) / n)[:, None] * np.array([[1.0, -2.0]])
    out = oracle.mix_step(oracle.ring(n), mode, np.zeros_like(mode), 1.0)
    lam = (1 + 2 * np.cos(2 * np.pi * m / n)) / 3
    np.testing.assert_allclose(out, lam * mode, atol=1e-14)


@pytest.mark.parametrize("topo", ["ring12", "torus4x5"])
def test_lemma5_bound_and_consensus_decay(topo):
    t = oracle.ring(12) if topo == "ring12" else oracle.torus(4, 5)
    n = t.n
    lam = np.sort(np.abs(np.linalg.eigvalsh(t.dense())))
    rho = lam[-2] ** 2
    X = np.eye(n)               # column i of W^k is W^k e_i; W symmetric
    prev = oracle.consensus(X)
    for k in range(1, 40):
        X = oracle.mix_step(t, X, np.zeros_like(X), 0.0)
        dist = np.sum((1.0 / n - X) ** 2, axis=0)     # ||1/n - W^k e_i||^2 for every i
        assert np.all(dist <= rho ** k + 1e-15)
        cur = oracle.consensus(X)
        assert cur <= prev + 1e-18
        prev = cur


@pytest.mark.parametrize("builder", [lambda: oracle.ring(9), lambda: oracle.torus(3, 4), lambda: oracle.complete(6)])
def test_node_average_recursion(builder):
    """Proof of Theorem 1: X_{k+1} 1/n = X_k 1/n - gamma dF(X_k) 1/n, for any doubly stochastic W."""
    t = builder()
    rng = np.random.default_rng(5)
    X = rng.standard_normal((t.n, 11))
    gamma = 0.07
    for _ in range(20):
        G = rng.standard_normal(X.shape)
        Xn = oracle.mix_step(t, X, G, gamma)
        np.testing.assert_allclose(oracle.mean(Xn), X.mean(0) - gamma * G.mean(0), atol=1e-14)
        X = Xn


def test_unrolled_recursion_with_dense_powers():
    """Proof of Theorem 1: X_K = W^K X_0 - gamma sum_j W^(K-1-j) G_j (rows = workers)."""
    n, d, K, gamma = 10, 6, 15, 0.05
    rng = np.random.default_rng(11)
    X0 = rng.standard_normal((n, d))
    Gs = [rng.standard_normal((n, d)) for _ in range(K)]
    t = oracle.ring(n)
    X = X0.copy()
    for k in range(K):
        X = oracle.mix_step(t, X, Gs[k], gamma)
    W = ring_dense(n)
    ref = np.linalg.matrix_power(W, K) @ X0
    for j in range(K):
        ref -= gamma * np.linalg.matrix_power(W, K - 1 - j) @ Gs[j]
    np.testing.assert_allclose(X, ref, atol=1e-13)


def test_general_csr_matches_dense_product():
    rng = np.random.default_rng(3)
    n, d = 7, 9
    # a symmetric doubly stochastic W: average of permutation matrices and their transposes
    W = np.zeros((n, n))
    for _ in range(3):
        P = np.eye(n)[rng.permutation(n)]
        W += (P + P.T) / 6.0
    rowptr, col, val = [0], [], []
    for i in range(n):
        for j in range(n):
            if W[i, j] != 0:
                col.append(j)
                val.append(W[i, j])
        rowptr.append(len(col))
    t = oracle.Topology(n, rowptr, col, val)
    assert t.check(1e-12) == 0
    X = rng.standard_normal((n, d))
    G = rng.standard_normal((n, d))
    np.testing.assert_allclose(oracle.mix_step(t, X, G, 0.2), W @ X - 0.2 * G, atol=1e-14)
    np.testing.assert_allclose(oracle.mix_step(t, X, G, 0.2, swapped=True), W @ (X - 0.2 * G), atol=1e-14)


def test_mean_and_consensus_brute_force():
    rng = np.random.default_rng(8)
    X = rng.standard_normal((13, 17)) * 3 + 1
    np.testing.assert_allclose(oracle.mean(X), X.sum(0) / 13, atol=1e-15)
    xbar = X.mean(0)
    brute = sum(np.sum((xbar - X[i]) ** 2) for i in range(13)) / 13
    assert oracle.consensus(X) == pytest.approx(brute, rel=1e-14)
    assert oracle.consensus(np.tile(xbar, (13, 1))) < 1e-28


# ------------------------------------------------------------------ momentum variant (Section 5.3: momentum 0.9)
def test_momentum_zero_is_the_plain_step():
    rng = np.random.default_rng(21)
    topo = oracle.ring(7)
    X, G, V = rng.standard_normal((3, 7, 13))
    Xn, Vn = oracle.mix_step_momentum(topo, X, G, V, 0.1, 0.0)
    assert np.array_equal(Xn, oracle.mix_step(topo, X, G, 0.1))
    assert np.array_equal(Vn, G)


def test_momentum_heavy_ball_identity_over_three_steps():
    """Eliminating V: X_{k+1} - W X_k = mu (X_k - W X_{k-1}) - gamma G_k, checked with a dense W product."""
    rng = np.random.default_rng(22)
    topo = oracle.torus(3, 4)
    W = topo.dense()
    gamma, mu = 0.05, 0.9
    X = [rng.standard_normal((12, 9))]
    V = np.zeros((12, 9))
    Gs = [rng.standard_normal((12, 9)) for _ in range(4)]
    for k in range(4):
        Xn, V = oracle.mix_step_momentum(topo, X[-1], Gs[k], V, gamma, mu)
        X.append(Xn)
    np.testing.assert_allclose(X[1], W @ X[0] - gamma * Gs[0], atol=1e-14)          # V_0 = 0
    for k in range(1, 4):
        lhs = X[k + 1] - W @ X[k]
        rhs = mu * (X[k] - W @ X[k - 1]) - gamma * Gs[k]
        np.testing.assert_allclose(lhs, rhs, atol=1e-13)


def test_momentum_node_average_follows_textbook_heavy_ball():
    """1^T W = 1^T, so the node average obeys vbar' = mu vbar + gbar, xbar' = xbar - gamma vbar'."""
    rng = np.random.default_rng(23)
    topo = oracle.ring_chord(8)
    X, G, V = rng.standard_normal((3, 8, 11))
    Xn, Vn = oracle.mix_step_momentum(topo, X, G, V, 0.07, 0.8)
    vbar = 0.8 * V.mean(0) + G.mean(0)
    np.testing.assert_allclose(Vn.mean(0), vbar, atol=1e-14)
    np.testing.assert_allclose(Xn.mean(0), X.mean(0) - 0.07 * vbar, atol=1e-14)


def test_momentum_on_a_quadratic_matches_the_mode_recurrence():
    """Complete graph, identical workers, f(x) = lambda x^2 / 2 per coordinate: each coordinate follows the 2 x 2
    linear recurrence (x, v) -> (x - gamma (mu v + lambda x), mu v + lambda x), evaluated here by a matrix power."""
    n, K = 5, 25
    lam = np.array([0.3, 1.0, 2.5, 7.0])
    gamma, mu = 0.1, 0.9
    topo = oracle.complete(n)
    X = np.tile(np.array([1.0, -2.0, 0.5, 3.0]), (n, 1))
    V = np.zeros_like(X)
    for _ in range(K):
        X, V = oracle.mix_step_momentum(topo, X, lam * X, V, gamma, mu)
    for c, l in enumerate(lam):
        M = np.array([[1.0 - gamma * l, -gamma * mu], [l, mu]])
        x0 = np.array([[1.0, -2.0, 0.5, 3.0][c], 0.0])
        want = np.linalg.matrix_power(M, K) @ x0
        np.testing.assert_allclose(X[:, c], want[0], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(V[:, c], want[1], rtol=1e-12, atol=1e-14)
