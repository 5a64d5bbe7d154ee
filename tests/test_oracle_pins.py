"""Pins for the CPU oracle: every check here rests on something other than the
oracle's own formulas (published known-answer vectors, closed forms, LAPACK
routines used as independent checkers, brute force, the paper's identities)."""
import math
import os

import numpy as np
import pytest
import scipy.stats

from oracle import gelo_oracle as o
from paper_2603_05035_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Philox --
def _kat_lines():
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield [int(tok, 16) for tok in line.split()]


def test_philox_known_answer_vectors():
    lines = list(_kat_lines())
    assert len(lines) == 3
    for words in lines:
        ctr, key, want = words[0:4], words[4:6], words[6:10]
        got = o.philox4x32_10([np.array([c]) for c in ctr], key)
        assert [int(g[0]) for g in got] == want


def test_philox_vectorised_equals_scalar_calls():
    rng = np.random.default_rng(1)
    ctr = rng.integers(0, 2**32, size=(4, 64), dtype=np.uint64)
    key = (0x12345678, 0x9ABCDEF0)
    vec = o.philox4x32_10(list(ctr), key)
    for i in (0, 17, 63):
        one = o.philox4x32_10([np.array([int(ctr[j, i])]) for j in range(4)], key)
        assert [int(v[i]) for v in vec] == [int(w[0]) for w in one]


def test_uniform_is_exact_in_float32_and_open():
    w = np.array([0, 0x1FF, 0x200, 0xFFFFFFFF, 0x80000000], dtype=np.uint32)
    u = o.uniform_open01(w)
    assert np.all(u > 0.0) and np.all(u < 1.0)
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)
    assert u[0] == 2.0 ** -24 and u[1] == 2.0 ** -24 and u[2] == 3.0 * 2.0 ** -24
    assert u[3] == 1.0 - 2.0 ** -24 and u[4] == 0.5 + 2.0 ** -24


def test_box_muller_closed_forms():
    # u2 = 1/4 + 2^-24 (word 0x40000000): angle ~ pi/2 -> (cos, sin) ~ (0, 1)
    # u1 = 1/2 + 2^-24 (word 0x80000000): radius = sqrt(2 ln 2) to 1e-7
    z0, z1 = o.box_muller(np.array([0x80000000], dtype=np.uint32), np.array([0x40000000], dtype=np.uint32))
    r = math.sqrt(2.0 * math.log(2.0))
    assert abs(z1[0] - r) < 1e-6 and abs(z0[0]) < 1e-6
    # u2 = 1/2 + 2^-24: angle ~ pi -> (-r, 0)
    z0, z1 = o.box_muller(np.array([0x80000000], dtype=np.uint32), np.array([0x80000000], dtype=np.uint32))
    assert abs(z0[0] + r) < 1e-6 and abs(z1[0]) < 1e-6
    # smallest uniform 2^-24: radius = sqrt(2 * 24 ln 2)
    z0, z1 = o.box_muller(np.array([0], dtype=np.uint32), np.array([0], dtype=np.uint32))
    assert abs(math.hypot(z0[0], z1[0]) - math.sqrt(48.0 * math.log(2.0))) < 1e-9


def test_gaussian_matrix_is_standard_normal():
    G = o.gaussian_matrix(seed=7, batch_id=3, stream=0, attempt=0, rows=1000, cols=1000)
    x = G.reshape(-1)
    n = x.size
    assert abs(x.mean()) < 5.0 / math.sqrt(n)
    assert abs(x.var() - 1.0) < 5.0 * math.sqrt(2.0 / n)
    assert abs(scipy.stats.kurtosis(x)) < 5.0 * math.sqrt(24.0 / n)
    assert abs(scipy.stats.skew(x)) < 5.0 * math.sqrt(6.0 / n)
    assert scipy.stats.kstest(x[:200000], "norm").pvalue > 1e-4
    # the four outputs of a block are mutually uncorrelated
    q = x.reshape(-1, 4)
    c = np.corrcoef(q.T)
    assert np.abs(c - np.eye(4)).max() < 5.0 / math.sqrt(q.shape[0])
    # neighbouring rows are uncorrelated
    assert abs(np.corrcoef(G[0], G[1])[0, 1]) < 0.2


def test_gaussian_matrix_layout_and_stream_separation():
    a = o.gaussian_matrix(5, 9, 0, 0, 6, 10)
    # row-major element order: a reshaped draw of the same element count is the same sequence
    b = o.gaussian_matrix(5, 9, 0, 0, 10, 6)
    assert np.array_equal(a.reshape(-1), b.reshape(-1))
    # a non-multiple-of-4 element count is a prefix of the longer draw
    c = o.gaussian_matrix(5, 9, 0, 0, 1, 7)
    assert np.array_equal(c.reshape(-1), a.reshape(-1)[:7])
    # every field of the counter and the key changes the draw
    for kw in (dict(seed=6), dict(batch_id=10), dict(stream=1), dict(attempt=1),
               dict(batch_id=9 + 2**32), dict(seed=5 + 2**32)):
        args = dict(seed=5, batch_id=9, stream=0, attempt=0, rows=6, cols=10)
        args.update(kw)
        assert not np.allclose(o.gaussian_matrix(**args), a)


# ---------------------------------------------------------------------- QR --
def test_householder_qr_invariants_and_lapack():
    rng = np.random.default_rng(2)
    for n in (1, 2, 5, 33, 130):
        G = rng.standard_normal((n, n))
        Q, R = o.householder_qr(G)
        assert np.abs(Q.T @ Q - np.eye(n)).max() < 1e-13
        assert np.abs(np.tril(R, -1)).max() == 0.0
        assert np.abs(Q @ R - G).max() < 1e-12
        A = o.orthogonal_from_gaussian(G)
        Rpos = A.T @ G
        assert np.all(np.diag(Rpos) > 0.0)
        assert np.abs(np.tril(Rpos, -1)).max() < 1e-12
        # LAPACK's QR, sign-normalised the same way, is the same matrix
        Ql, Rl = np.linalg.qr(G)
        Ql = Ql * np.sign(np.diag(Rl))[None, :]
        assert np.abs(A - Ql).max() < 1e-11
        if n <= 5:
            assert abs(abs(np.linalg.det(A)) - 1.0) < 1e-12


def test_qr_two_by_two_closed_form():
    a, b, c, d = 3.0, 1.0, -4.0, 2.0
    A = o.orthogonal_from_gaussian(np.array([[a, b], [c, d]]))
    r = math.hypot(a, c)
    q1 = np.array([a / r, c / r])
    # second column: unit vector orthogonal to q1 with positive r_22 = q2 . (b, d)
    q2 = np.array([-c / r, a / r])
    if q2 @ np.array([b, d]) < 0:
        q2 = -q2
    assert np.allclose(A[:, 0], q1, atol=1e-15) and np.allclose(A[:, 1], q2, atol=1e-15)


def test_orthogonal_sampler_matches_constructed_pieces():
    A, A_inv = o.sample_orthogonal(seed=11, batch_id=4, n=40)
    assert np.array_equal(A_inv, A.T)
    assert np.abs(A @ A_inv - np.eye(40)).max() < 1e-13
    assert abs(o.cond2(A) - 1.0) < 1e-12
    # fresh per batch: another batch id gives an unrelated matrix
    B, _ = o.sample_orthogonal(seed=11, batch_id=5, n=40)
    assert np.abs(A - B).max() > 0.1


# ------------------------------------------------------------- LU, inverse --
def test_lu_hand_case_with_forced_pivoting():
    # rows must be swapped at step 0 (|4| > |1|) and at step 1
    A = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0], [7.0, 8.0, 10.0]])
    perm, L, U = o.lu_partial_pivot(A)
    assert list(perm) == [2, 0, 1]
    assert np.allclose(L, [[1, 0, 0], [1 / 7, 1, 0], [4 / 7, 0.5, 1]], atol=1e-15)
    assert np.allclose(U, [[7, 8, 10], [0, 6 / 7, 11 / 7], [0, 0, -0.5]], atol=1e-14)
    # exact inverse of this matrix (det = -3)
    want = np.array([[-2.0, -4.0, 3.0], [-2.0, 11.0, -6.0], [3.0, -6.0, 3.0]]) / 3.0
    assert np.allclose(o.inverse(A), want, atol=1e-13)


def test_lu_inverse_against_lapack_and_identity_bound():
    rng = np.random.default_rng(3)
    for n in (1, 4, 57, 200):
        A = rng.standard_normal((n, n))
        perm, L, U = o.lu_partial_pivot(A)
        assert np.abs(A[perm] - L @ U).max() < 1e-12
        assert np.abs(L).max() <= 1.0 + 1e-15          # partial pivoting bounds the multipliers
        X = o.inverse(A)
        assert np.abs(X - np.linalg.inv(A)).max() / np.abs(X).max() < 1e-9
    with pytest.raises(ZeroDivisionError):
        o.lu_partial_pivot(np.zeros((3, 3)))


def test_cond2_closed_forms():
    assert abs(o.cond2(np.diag([4.0, -2.0, 0.5])) - 8.0) < 1e-13
    rot = np.array([[0.6, -0.8], [0.8, 0.6]])
    assert abs(o.cond2(rot) - 1.0) < 1e-14
    assert abs(o.cond2(rot @ np.diag([10.0, 0.1]) @ rot.T) - 100.0) < 1e-10
    assert o.cond2(np.array([[1.0, 2.0], [2.0, 4.0]])) > 1e15


def test_gaussian_sampler_rule_at_paper_shape():
    # n = 512, entries N(0, 1/512), redraw while kappa_2 > 1e3
    A, A_inv, attempt, kappa, kappas = o.sample_gaussian(seed=0xC1, batch_id=0, n=512,
                                                         cond_max=1e3, max_attempts=64)
    assert kappa <= 1e3 and len(kappas) == attempt + 1
    assert all(k > 1e3 for k in kappas[:-1])
    assert abs(kappa - np.linalg.cond(A, 2)) / kappa < 1e-9
    assert abs(A.var() * 512 - 1.0) < 0.02
    assert np.linalg.norm(A @ A_inv - np.eye(512)) <= 1e-10       # Frobenius
    assert np.linalg.norm(A_inv @ A - np.eye(512)) <= 1e-10
    # Gram matrices are masked: A^T A is far from I
    assert np.linalg.norm(A.T @ A - np.eye(512)) / math.sqrt(512) > 0.5


def test_gaussian_acceptance_rate_follows_edelman_law():
    # P(kappa_2/n < x) -> exp(-2/x - 2/x^2) for an n x n real Gaussian matrix
    n, cond_max, trials = 64, 300.0, 300
    x = cond_max / n
    p = math.exp(-2.0 / x - 2.0 / x ** 2)
    acc = 0
    for t in range(trials):
        G = o.gaussian_matrix(seed=99, batch_id=t, stream=0, attempt=0, rows=n, cols=n)
        acc += o.cond2(G / math.sqrt(n)) <= cond_max
    sigma = math.sqrt(trials * p * (1 - p))
    assert abs(acc - trials * p) < 4.5 * sigma + 0.03 * trials   # asymptotic law: allow a finite-n bias


def test_conditioned_sampler_is_dense_nonorthogonal_and_well_conditioned():
    A, A_inv, kappa = o.sample_conditioned(seed=5, batch_id=1, n=96)
    assert kappa < 100.0 and kappa < 6.0
    assert np.linalg.norm(A @ A_inv - np.eye(96)) < 1e-12
    assert np.linalg.norm(A.T @ A - np.eye(96)) / math.sqrt(96) > 0.2
    Q, _ = o.sample_orthogonal(seed=5, batch_id=1, n=96)
    P = (A - Q) * math.sqrt(96) / o.CONDITIONED_BETA
    assert abs(P.var() - 1.0) < 0.1 and abs(np.corrcoef(P.reshape(-1), (Q * math.sqrt(96)).reshape(-1))[0, 1]) < 0.05


# ------------------------------------------------------------------ shields --
def test_shield_rows_norm_and_statistic():
    rng = np.random.default_rng(4)
    H = rng.standard_normal((16, 64)) * rng.uniform(0.5, 3.0, size=(16, 1))
    D = rng.standard_normal((3, 64))
    norms = sorted(math.sqrt(sum(v * v for v in row)) for row in H.tolist())
    median = 0.5 * (norms[7] + norms[8])
    mean = sum(norms) / 16
    assert abs(o.row_norm_statistic(H, o.NORM_MEDIAN) - median) < 1e-13
    assert abs(o.row_norm_statistic(H, o.NORM_MEAN) - mean) < 1e-13
    assert abs(o.row_norm_statistic(H[:15], o.NORM_MEDIAN) - sorted(
        math.sqrt(sum(v * v for v in row)) for row in H[:15].tolist())[7]) < 1e-13
    S = o.shield_rows(H, D, 10.0, o.NORM_MEDIAN)
    assert np.allclose(np.linalg.norm(S, axis=1), 10.0 * median, rtol=1e-13)
    # direction preserved
    cos = np.sum(S * D, axis=1) / (np.linalg.norm(S, axis=1) * np.linalg.norm(D, axis=1))
    assert np.allclose(cos, 1.0, atol=1e-14)
    S_mean = o.shield_rows(H, D, 4.0, o.NORM_MEAN)
    assert np.allclose(np.linalg.norm(S_mean, axis=1), 4.0 * mean, rtol=1e-13)
    assert o.shield_rows(H, np.zeros((0, 64)), 10.0).shape == (0, 64)


# -------------------------------------------------------------------- chain --
def _brute_matmul(X, Y):
    X, Y = X.tolist(), Y.tolist()
    rows, inner, cols = len(X), len(Y), len(Y[0])
    return np.array([[math.fsum(X[i][c] * Y[c][j] for c in range(inner)) for j in range(cols)]
                     for i in range(rows)])


def test_tiny_config_chain_against_brute_force():
    w = wl.WORKLOADS["tiny_f32"]
    H, W = wl.make_inputs(w)
    out = o.qkv_forward(w.kind, w.seed, 0, H, W, k_shield=w.k_shield, shield_scale=10.0)
    Z_brute = _brute_matmul(H.astype(np.float64), W.astype(np.float64))
    assert out["A"].shape == (18, 18) and out["U"].shape == (18, 64)
    assert out["Y"].shape == (18, 192) and out["Z"].shape == (16, 192)
    assert o.rel_frobenius(o.plain_projection(H, W), Z_brute) < 1e-15
    assert o.rel_frobenius(out["Z"], Z_brute) < 1e-13                      # eq. 4
    # each step against brute force
    H_full = np.vstack([H.astype(np.float64), out["S"]])
    assert o.rel_frobenius(out["U"], _brute_matmul(out["A"], H_full)) < 1e-14
    assert o.rel_frobenius(out["Y"][:4], _brute_matmul(out["U"][:4], W.astype(np.float64))) < 1e-14
    assert o.rel_frobenius(out["Z"][:3], _brute_matmul(out["A_inv"][:3], out["Y"])) < 1e-14
    # shields really are 10x the median row norm and sit in the last rows
    med = np.median(np.linalg.norm(H.astype(np.float64), axis=1))
    assert np.allclose(np.linalg.norm(out["S"], axis=1), 10.0 * med, rtol=1e-13)


def test_transposed_operand_would_be_caught():
    # the pins above must notice a transposed A in the unmix step
    w = wl.WORKLOADS["tiny_f32"]
    H, W = wl.make_inputs(w)
    out = o.qkv_forward(w.kind, w.seed, 0, H, W, k_shield=2)
    wrong = o.unmix(out["A"], out["Y"], 16)          # A instead of A^T
    assert o.rel_frobenius(wrong, o.plain_projection(H, W)) > 0.5


@pytest.mark.parametrize("kind", [o.KIND_ORTHOGONAL, o.KIND_GAUSSIAN, o.KIND_CONDITIONED])
def test_identity_holds_for_every_kind(kind):
    rng = np.random.default_rng(6)
    H = rng.standard_normal((48, 96))
    W = rng.standard_normal((96, 40)) * 0.02
    k = 3 if kind == o.KIND_ORTHOGONAL else 0
    out = o.qkv_forward(kind, seed=21, batch_id=8, H=H, W=W, k_shield=k, cond_max=1e4)
    assert o.rel_frobenius(out["Z"], H @ W) < 1e-11
    assert np.linalg.norm(out["A"] @ out["A_inv"] - np.eye(48 + k)) < 1e-10
    # associativity: (A H) W == A (H W) on the mixed rows
    H_full = np.vstack([H, out["S"]]) if k else H
    assert o.rel_frobenius(out["Y"], out["A"] @ (H_full @ W)) < 1e-12


def test_gram_identities_orthogonal():
    rng = np.random.default_rng(7)
    H = rng.standard_normal((30, 50))
    A, _ = o.sample_orthogonal(seed=3, batch_id=0, n=30)
    U = o.mix(A, H)
    assert o.rel_frobenius(U.T @ U, H.T @ H) < 1e-13                       # eq. 5
    ev_u = np.sort(np.linalg.eigvalsh(U @ U.T))
    ev_h = np.sort(np.linalg.eigvalsh(H @ H.T))
    assert np.allclose(ev_u, ev_h, rtol=1e-10, atol=1e-10)                  # eq. 6: similar matrices
    assert o.rel_frobenius(U @ U.T, A @ (H @ H.T) @ A.T) < 1e-13
    # with shields: U^T U = H^T H + S^T S (eq. 9)
    A2, _ = o.sample_orthogonal(seed=3, batch_id=1, n=34)
    S = o.shield_rows(H, o.sample_shield_directions(3, 1, 4, 50), 10.0)
    U2 = o.mix(A2, H, S)
    assert o.rel_frobenius(U2.T @ U2, H.T @ H + S.T @ S) < 1e-13
    assert o.rel_frobenius(U2.T @ U2, H.T @ H) > 1.0                        # the data Gram is buried


def test_gram_is_masked_by_nonorthogonal_mixing():
    rng = np.random.default_rng(8)
    H = rng.standard_normal((64, 80))
    for kind, floor in ((o.KIND_GAUSSIAN, 0.3), (o.KIND_CONDITIONED, 0.05)):
        A, _, _ = o.sample_mixing(kind, seed=13, batch_id=2, n=64, cond_max=1e4)
        U = o.mix(A, H)
        assert o.rel_frobenius(U.T @ U, H.T @ H) > floor


def test_full_knowledge_recovers_mixing_matrix():
    # with H known and of full row rank, A = U H^+ (Section 5.3)
    rng = np.random.default_rng(9)
    H = rng.standard_normal((12, 40))
    A, _ = o.sample_orthogonal(seed=1, batch_id=1, n=12)
    U = o.mix(A, H)
    assert np.abs(U @ np.linalg.pinv(H) - A).max() < 1e-12


def test_workload_shapes_follow_the_configs():
    w = wl.WORKLOADS
    assert (w["tiny_f32"].n, w["llama7b_f32_gaussian"].n, w["llama7b_bf16_prefill"].n) == (18, 512, 2150)
    assert (w["sweep_bf16_orth"].n, w["sweep_bf16_cond"].n, w["decode_bf16"].n) == (4301, 4096, 68)
    assert w["llama7b_bf16_prefill"].k_shield == round(0.05 * 2048)
    assert w["sweep_bf16_orth"].k_shield == round(0.05 * 4096)
    H = wl.make_hidden(256, 4096, 1)
    col_scale = np.sqrt((H.astype(np.float64) ** 2).mean(axis=0))
    assert int((col_scale > 10).sum()) == 8 and abs(np.median(col_scale) - 1.0) < 0.15
    Wt = wl.make_weight(512, 256, 1)
    assert abs(float(Wt.std()) - 0.02) < 1e-3
    assert np.array_equal(H, wl.make_hidden(256, 4096, 1))
