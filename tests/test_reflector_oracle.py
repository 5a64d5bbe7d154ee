"""Pins of the oracle's orthogonal A built as a product of directly drawn reflectors (no GPU): closed forms,
a dense brute-force product, and the moments of the Haar measure that a wrong construction misses."""
import math

import numpy as np
import pytest

from oracle import gelo_oracle as o


def _gauss(seed, n):
    return o.gaussian_matrix(seed, 7, o.STREAM_MIXING, 0, n, n)


@pytest.mark.parametrize("n", [1, 2, 3, 17, 64, 130])
def test_orthogonal_and_first_column(n):
    G = _gauss(11 + n, n)
    A = o.orthogonal_from_reflectors(G)
    assert np.abs(A @ A.T - np.eye(n)).max() < 1e-12
    assert np.abs(A.T @ A - np.eye(n)).max() < 1e-12
    # H_0 maps G[:, 0] to beta_0 e_0 and the later reflectors leave e_0 alone: column 0 of A is G[:, 0] normalised
    assert np.abs(A[:, 0] - G[:, 0] / np.linalg.norm(G[:, 0])).max() < 1e-13


def test_two_by_two_closed_form():
    """n = 2: H_0 = [[a, c], [c, -a]] / beta with beta = -sign(a) r, r = |(a, c)|; x_1 = (d) gives H_1 = diag(1, -1)
    and beta_1 = -d, so A = [ (a, c)/r , sign(d) (c, -a)/beta ]."""
    for a, b, c, d in ((0.3, -1.2, 0.7, 0.4), (-0.9, 0.1, 0.2, -2.0), (1.5, 0.0, -0.5, 0.25)):
        G = np.array([[a, b], [c, d]])
        r = math.hypot(a, c)
        beta = -math.copysign(r, a)
        want = np.array([[a / r, math.copysign(1.0, d) * c / beta], [c / r, -math.copysign(1.0, d) * a / beta]])
        assert np.abs(o.orthogonal_from_reflectors(G) - want).max() < 1e-14


@pytest.mark.parametrize("n", [4, 7])
def test_equals_the_dense_product_of_reflection_matrices(n):
    """Every H_k written out as a full n x n matrix from the definition, multiplied with matmul; the signs taken from
    what the dense H_k does to its own column."""
    G = _gauss(5, n)
    Hs, signs = [], []
    for k in range(n):
        x = G[k:, k]
        v = x.copy()
        v[0] += math.copysign(np.linalg.norm(x), x[0])
        Hk = np.eye(n)
        Hk[k:, k:] -= 2.0 * np.outer(v, v) / (v @ v)
        image = Hk[k:, k:] @ x
        assert np.abs(image[1:]).max() < 1e-13 if n - k > 1 else True      # H_k x_k = beta_k e_0
        assert abs(abs(image[0]) - np.linalg.norm(x)) < 1e-13
        Hs.append(Hk)
        signs.append(-1.0 if image[0] < 0 else 1.0)
    want = np.linalg.multi_dot(Hs) @ np.diag(signs) if n > 1 else Hs[0] @ np.diag(signs)
    assert np.abs(o.orthogonal_from_reflectors(G) - want).max() < 1e-13


def test_zero_column_contributes_the_identity():
    G = _gauss(3, 5)
    G[2:, 2] = 0.0
    A = o.orthogonal_from_reflectors(G)
    assert np.abs(A @ A.T - np.eye(5)).max() < 1e-13
    G2 = G.copy()
    G2[:2, 2] = 9.0                                     # entries above the diagonal are never read
    assert np.array_equal(o.orthogonal_from_reflectors(G2), A)


def test_entries_above_the_diagonal_are_not_used():
    G = _gauss(8, 9)
    L = np.tril(G)
    assert np.array_equal(o.orthogonal_from_reflectors(L), o.orthogonal_from_reflectors(G))


def test_selected_columns_are_the_full_matrix_columns():
    G = _gauss(21, 37)
    A = o.orthogonal_from_reflectors(G)
    cols = [0, 1, 15, 16, 17, 36]
    assert np.abs(o.orthogonal_from_reflectors(G, columns=cols) - A[:, cols]).max() < 1e-14      # same sums, the library's own blocking


def test_haar_moments():
    """For Haar-distributed A in O(n), n >= 2: E tr A = 0, E (tr A)^2 = 1, E tr(A^2) = 1, E det A = 0, and every entry
    has variance 1/n (Diaconis and Shahshahani, J. Appl. Probab. 31A, 1994).  A product without the sign matrix has
    a fixed determinant, one with the reflectors in the wrong order or built from the wrong rows fails the traces."""
    n, N = 3, 4000
    tr = np.empty(N); tr2 = np.empty(N); det = np.empty(N); sq = np.zeros((n, n))
    for i in range(N):
        A = o.orthogonal_from_reflectors(o.gaussian_matrix(1000 + i, 0, o.STREAM_MIXING, 0, n, n))
        tr[i] = np.trace(A); tr2[i] = np.trace(A @ A); det[i] = np.linalg.det(A); sq += A * A
    tol = 4.5 / math.sqrt(N)
    assert abs(tr.mean()) < tol                          # variance 1
    assert abs((tr ** 2).mean() - 1.0) < tol * math.sqrt(2.0) * 1.2
    assert abs(tr2.mean() - 1.0) < tol * 1.5
    assert abs(det.mean()) < tol
    assert np.abs(sq / N - 1.0 / n).max() < tol


def test_same_law_as_the_qr_kind_on_a_statistic_of_the_second_column():
    """The second column is where the two constructions differ; its first entry must have the same distribution
    (mean 0, variance 1/n, and the same fourth moment 3 / (n (n + 2)) as any entry of a Haar matrix)."""
    n, N = 4, 4000
    a = np.empty(N); q = np.empty(N)
    for i in range(N):
        G = o.gaussian_matrix(5000 + i, 0, o.STREAM_MIXING, 0, n, n)
        a[i] = o.orthogonal_from_reflectors(G)[0, 1]
        q[i] = o.orthogonal_from_gaussian(G)[0, 1]
    for x in (a, q):
        assert abs(x.mean()) < 4.5 * math.sqrt(1.0 / n / N)
        assert abs((x ** 2).mean() - 1.0 / n) < 4.5 * math.sqrt(2.0) / n / math.sqrt(N) * 1.2
        assert abs((x ** 4).mean() - 3.0 / (n * (n + 2))) < 0.02


def test_sample_reflector_product_and_the_chain():
    A, A_inv = o.sample_reflector_product(1234, 9, 40)
    assert np.abs(A @ A_inv - np.eye(40)).max() < 1e-12
    rng = np.random.default_rng(0)
    H = rng.standard_normal((36, 24)); W = rng.standard_normal((24, 16)) * 0.1
    r = o.qkv_forward(o.KIND_REFLECTOR_PRODUCT, 1234, 9, H, W, k_shield=4)
    assert np.array_equal(r["A"], A)
    assert o.rel_frobenius(r["Z"], H @ W) < 1e-12                       # eq. 4
    assert np.abs(r["U"].T @ r["U"] - np.vstack([H, r["S"]]).T @ np.vstack([H, r["S"]])).max() < 1e-9   # eq. 9
