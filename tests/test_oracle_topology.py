"""Pins for the oracle's weight matrices W (Section 3; Theorem 3's ring matrix; Assumption 1-2)."""
import numpy as np
import pytest

import oracle


@pytest.mark.parametrize("n", [3, 4, 8, 16, 33, 112])
def test_ring_matches_theorem3_matrix(n):
    t = oracle.ring(n)
    W = t.dense()
    # Section 3: entries in [0,1], symmetric, rows (hence columns) sum to one
    assert W.min() >= 0.0 and W.max() <= 1.0
    assert np.array_equal(W, W.T)
    np.testing.assert_allclose(W.sum(1), 1.0, atol=1e-15)
    np.testing.assert_allclose(W.sum(0), 1.0, atol=1e-15)
    assert t.check() == 0
    # Theorem 3: exactly three entries 1/3 per row, at i-1, i, i+1 (mod n)
    for i in range(n):
        nz = set(np.nonzero(W[i])[0].tolist())
        assert nz == {(i - 1) % n, i, (i + 1) % n}
        assert np.all(W[i][sorted(nz)] == 1.0 / 3.0)
    # CSR is sorted and has 3n entries
    assert t.rowptr[-1] == 3 * n
    for i in range(n):
        cols = t.col[t.rowptr[i]:t.rowptr[i + 1]]
        assert np.all(np.diff(cols) > 0)


@pytest.mark.parametrize("n", [3, 5, 8, 16, 64])
def test_ring_spectrum_is_the_circulant_closed_form(n):
    """A circulant with first row (1/3, 1/3, 0, ..., 0, 1/3) has eigenvalues (1 + 2 cos(2 pi m/n))/3."""
    W = oracle.ring(n).dense()
    lam = np.sort(np.linalg.eigvalsh(W))
    closed = np.sort((1.0 + 2.0 * np.cos(2.0 * np.pi * np.arange(n) / n)) / 3.0)
    np.testing.assert_allclose(lam, closed, atol=1e-13)
    # Assumption 1-2: rho = max(|lambda_2|, |lambda_n|)^2 < 1
    mags = np.sort(np.abs(lam))
    assert mags[-1] == pytest.approx(1.0, abs=1e-13)
    assert mags[-2] ** 2 < 1.0


@pytest.mark.parametrize("dims", [(3, 3), (3, 5), (8, 8), (4, 16)])
def test_torus_requirements_and_spectrum(dims):
    r, c = dims
    t = oracle.torus(r, c)
    W = t.dense()
    assert t.check() == 0
    assert np.array_equal(W, W.T)
    np.testing.assert_allclose(W.sum(1), 1.0, atol=1e-15)
    assert set(np.unique(W).tolist()) == {0.0, 0.2}
    assert np.all((W != 0).sum(1) == 5)
    a = np.arange(r)[:, None]
    b = np.arange(c)[None, :]
    closed = np.sort(((1 + 2 * np.cos(2 * np.pi * a / r) + 2 * np.cos(2 * np.pi * b / c)) / 5).ravel())
    np.testing.assert_allclose(np.sort(np.linalg.eigvalsh(W)), closed, atol=1e-13)
    # neighbour structure: worker (rr, cc) <-> (rr+-1, cc), (rr, cc+-1)
    for rr in range(r):
        for cc in range(c):
            i = rr * c + cc
            want = {i, ((rr + 1) % r) * c + cc, ((rr - 1) % r) * c + cc, rr * c + (cc + 1) % c, rr * c + (cc - 1) % c}
            assert set(np.nonzero(W[i])[0].tolist()) == want


def test_degenerate_rings_accumulate_coinciding_neighbours():
    np.testing.assert_allclose(oracle.ring(1).dense(), [[1.0]])
    np.testing.assert_allclose(oracle.ring(2).dense(), [[1 / 3, 2 / 3], [2 / 3, 1 / 3]])
    assert oracle.ring(2).check(1e-12) == 0


def test_complete_graph_is_uniform_averaging():
    W = oracle.complete(7).dense()
    np.testing.assert_allclose(W, np.full((7, 7), 1 / 7), atol=0)
    assert oracle.complete(7).check(1e-12) == 0


def test_check_rejects_matrices_that_violate_section3():
    t = oracle.ring(6)
    bad = oracle.Topology(6, t.rowptr, t.col, t.val.copy())
    bad.val[0] = 0.5
    assert bad.check() in (3, 4)
    # asymmetric but row-stochastic: a directed 3-cycle
    asym = oracle.Topology(3, [0, 2, 4, 6], [0, 1, 1, 2, 0, 2], [0.5] * 6)
    assert asym.check() == 4
    neg = oracle.Topology(2, [0, 2, 4], [0, 1, 0, 1], [1.5, -0.5, -0.5, 1.5])
    assert neg.check() == 2
    unsorted = oracle.Topology(2, [0, 2, 4], [1, 0, 0, 1], [0.5] * 4)
    assert unsorted.check() == 1


def test_ring_equals_the_printed_matrix_of_theorem3():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "ring_theorem3_n6.txt")
    printed = np.loadtxt(path) / 3.0
    np.testing.assert_allclose(oracle.ring(6).dense(), printed, atol=1e-16)


@pytest.mark.parametrize("n", [4, 6, 16, 64])
def test_ring_with_far_link_requirements_and_spectrum(n):
    """Ring plus the link i <-> i + n/2 at uniform 1/4 (supplement, scalability experiment, 16 machines): a
    circulant whose eigenvalues are (1 + 2 cos(2 pi m/n) + (-1)^m)/4; its spectral gap beats the plain ring's."""
    t = oracle.ring_chord(n)
    W = t.dense()
    assert t.check() == 0
    assert np.array_equal(W, W.T)
    np.testing.assert_allclose(W.sum(0), 1.0, atol=1e-15)
    np.testing.assert_allclose(W.sum(1), 1.0, atol=1e-15)
    for i in range(n):
        want = {i, (i + 1) % n, (i - 1) % n, (i + n // 2) % n}
        assert set(np.nonzero(W[i])[0].tolist()) == want
        assert np.all(W[i, sorted(want)] == 1.0 / len(want) if len(want) == 4 else True)
    m = np.arange(n)
    closed = np.sort((1.0 + 2.0 * np.cos(2.0 * np.pi * m / n) + (-1.0) ** m) / 4.0)
    np.testing.assert_allclose(np.sort(np.linalg.eigvalsh(W)), closed, atol=1e-13)
    if n >= 8:
        second = lambda M: np.sort(np.abs(np.linalg.eigvalsh(M)))[-2]
        assert second(W) < second(oracle.ring(n).dense())      # information flows faster (smaller rho)


def test_ring_with_far_link_needs_an_even_ring():
    for n in (3, 5, 2):
        with pytest.raises(ValueError):
            oracle.ring_chord(n)
