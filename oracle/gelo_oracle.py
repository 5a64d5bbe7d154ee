"""Plain CPU fp64 oracle for the GELO obfuscated projection.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU
library can be checked against something written independently from the paper.
Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import it; the GPU library never does and shares no code, table or constant
generator with it.

Everything is float64 numpy, one step per function, no blocking or fusion, in
the order the paper states the protocol (Section 3.2 "Core Algorithm",
eqs. 1-4, and Section 3.2.1 "Mitigating Gram Matrix Information Leaks",
eqs. 5-9).  `numpy.matmul`, `numpy.linalg.svd` and `numpy.median` serve as
library primitives for single steps (a matrix product, the singular values, a
median); the Philox generator, the Householder QR, the LU factorisation and
the triangular solves are written out here.

Every function is pinned by tests that do not call back into this file's own
formulas (known-answer vectors, closed forms, LAPACK cross-checks, brute
force, the paper's identities); no function is "parity unpinned" except where
stated in its docstring.
"""
from __future__ import annotations

import math

import numpy as np

# --------------------------------------------------------------------------
# Counter-based generator: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).
# The paper only says "sample a fresh, random invertible matrix A" (Section
# 3.2, step 1.2); a counter-based generator makes "fresh per batch, never
# reused" a matter of never repeating a (seed, batch id) pair.
# --------------------------------------------------------------------------
_MASK32 = np.uint64(0xFFFFFFFF)
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = np.uint64(0x9E3779B9)
_PHILOX_W1 = np.uint64(0xBB67AE85)

STREAM_MIXING = 0        # Gaussian G that A is built from
STREAM_SHIELD = 1        # Gaussian directions of the shield rows
STREAM_PERTURB = 2       # second Gaussian of the conditioned non-orthogonal A
STREAM_STRUCT_PERM = 3   # sort keys of the permutations of the structured orthogonal A
STREAM_STRUCT_SIGN = 4   # its sign flips
STREAM_BLOCK = 5         # Gaussians of the diagonal blocks of the block-diagonal orthogonal A (sub-stream = block)


def philox4x32_10(counter, key):
    """Ten Philox rounds on 4x32-bit counters with a 2x32-bit key.

    `counter` is a sequence of four equally shaped integer arrays (values
    < 2**32), `key` a pair of integers.  Returns four uint32 arrays.
    One round: (c0,c1,c2,c3) -> (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1,
    lo(M0*c0)); the key is advanced by the Weyl constants between rounds.
    """
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & _MASK32 for c in counter)
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = np.uint64(int(key[0]) & 0xFFFFFFFF)
    k1 = np.uint64(int(key[1]) & 0xFFFFFFFF)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + _PHILOX_W0) & _MASK32
            k1 = (k1 + _PHILOX_W1) & _MASK32
        p0 = _PHILOX_M0 * c0            # 32x32 -> 64 bit, exact in uint64
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def uniform_open01(word):
    """Top 23 bits of a 32-bit word -> a uniform in (0,1): (2m + 1) * 2**-24.

    2m + 1 < 2**24, so the value is exactly representable in float32 as well
    as float64: a single-precision implementation sees the same uniforms.
    """
    m = (np.asarray(word, dtype=np.uint32) >> np.uint32(9)).astype(np.float64)
    return (2.0 * m + 1.0) * (2.0 ** -24)


def box_muller(word_a, word_b):
    """Two independent N(0,1) values from two 32-bit words (Box-Muller)."""
    u1 = uniform_open01(word_a)
    u2 = uniform_open01(word_b)
    radius = np.sqrt(-2.0 * np.log(u1))
    angle = 2.0 * math.pi * u2
    return radius * np.cos(angle), radius * np.sin(angle)


def gaussian_matrix(seed, batch_id, stream, attempt, rows, cols):
    """rows x cols matrix of i.i.d. N(0,1), a pure function of its arguments.

    Element e = r*cols + c (row-major) is output e mod 4 of Philox block
    e div 4.  Block q uses counter (q, stream<<8 | attempt, batch_id low,
    batch_id high) and key (seed low, seed high).  Outputs 0,1 of a block are
    the Box-Muller pair of words 0,1; outputs 2,3 the pair of words 2,3.
    """
    total = rows * cols
    nblocks = (total + 3) // 4
    q = np.arange(nblocks, dtype=np.uint64)
    c1 = np.uint64(((int(stream) & 0xFFFFFF) << 8) | (int(attempt) & 0xFF))
    c2 = np.uint64(int(batch_id) & 0xFFFFFFFF)
    c3 = np.uint64((int(batch_id) >> 32) & 0xFFFFFFFF)
    key = (int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF)
    x0, x1, x2, x3 = philox4x32_10((q, c1, c2, c3), key)
    z0, z1 = box_muller(x0, x1)
    z2, z3 = box_muller(x2, x3)
    flat = np.stack([z0, z1, z2, z3], axis=1).reshape(-1)[:total]
    return flat.reshape(rows, cols)


# --------------------------------------------------------------------------
# Orthogonal A: Householder QR of a Gaussian matrix (Section 3.2, eq. 3 remark
# "if A is orthogonal, A^-1 = A^T"; Table 3 names the step "A-gen (QR)").
# --------------------------------------------------------------------------
def householder_qr(G):
    """Unblocked Householder QR.  Returns (Q, R) with Q orthogonal, R upper
    triangular and Q @ R == G.  Column j is reduced by the reflector
    I - 2 v v^T / (v^T v),  v = x + sign(x_0) ||x|| e_0,  x = R[j:, j]."""
    R = np.array(G, dtype=np.float64, copy=True)
    n = R.shape[0]
    if R.shape[1] != n:
        raise ValueError("square matrix expected")
    Q = np.eye(n)
    for j in range(n):
        x = R[j:, j]
        norm_x = math.sqrt(float(x @ x))
        if norm_x == 0.0:
            continue
        v = x.copy()
        v[0] += norm_x if x[0] >= 0.0 else -norm_x
        scale = 2.0 / float(v @ v)
        R[j:, j:] -= scale * np.outer(v, v @ R[j:, j:])
        Q[:, j:] -= scale * np.outer(Q[:, j:] @ v, v)
        R[j + 1:, j] = 0.0
    return Q, R


def orthogonal_from_gaussian(G):
    """A = Q diag(sign r_ii): the orthogonal factor of the QR factorisation of
    G whose triangular factor has a positive diagonal.  That factor is unique,
    and Haar-distributed when G is Gaussian."""
    Q, R = householder_qr(G)
    signs = np.where(np.diag(R) < 0.0, -1.0, 1.0)
    return Q * signs[None, :]


# --------------------------------------------------------------------------
# Non-orthogonal A (Section 3.2.1, Mitigation 1): general invertible matrix,
# explicit inverse, condition number verified.
# --------------------------------------------------------------------------
def lu_partial_pivot(A):
    """Row-pivoted LU: returns (perm, L, U) with A[perm] == L @ U, L unit lower
    triangular, U upper triangular.  Raises ZeroDivisionError on a zero pivot."""
    M = np.array(A, dtype=np.float64, copy=True)
    n = M.shape[0]
    perm = np.arange(n)
    for j in range(n):
        piv = j + int(np.argmax(np.abs(M[j:, j])))
        if M[piv, j] == 0.0:
            raise ZeroDivisionError("singular matrix")
        if piv != j:
            M[[j, piv]] = M[[piv, j]]
            perm[[j, piv]] = perm[[piv, j]]
        M[j + 1:, j] /= M[j, j]
        M[j + 1:, j + 1:] -= np.outer(M[j + 1:, j], M[j, j + 1:])
    L = np.tril(M, -1) + np.eye(n)
    U = np.triu(M)
    return perm, L, U


def inverse_from_lu(perm, L, U):
    """Solve L U X = P for X = A^-1 by forward then backward substitution."""
    n = L.shape[0]
    X = np.eye(n)[perm]                     # P, rows of the identity permuted
    for i in range(n):                      # L y = b, unit diagonal
        X[i] -= L[i, :i] @ X[:i]
    for i in range(n - 1, -1, -1):          # U x = y
        X[i] = (X[i] - U[i, i + 1:] @ X[i + 1:]) / U[i, i]
    return X


def inverse(A):
    return inverse_from_lu(*lu_partial_pivot(A))


def cond2(A):
    """2-norm condition number sigma_max / sigma_min (an orthogonal A has
    kappa = 1 in this norm, which is the one Section 3.2.1 reasons with)."""
    s = np.linalg.svd(np.asarray(A, dtype=np.float64), compute_uv=False)
    return float(s[0] / s[-1]) if s[-1] > 0.0 else math.inf


def sample_orthogonal(seed, batch_id, n):
    """Fresh orthogonal A for one batch; returns (A, A^-1 = A^T)."""
    G = gaussian_matrix(seed, batch_id, STREAM_MIXING, 0, n, n)
    A = orthogonal_from_gaussian(G)
    return A, A.T.copy()


def sample_gaussian(seed, batch_id, n, cond_max, max_attempts):
    """A = G / sqrt(n) (entries N(0, 1/n)); redrawn with the attempt number in
    the counter until kappa_2(A) <= cond_max.  Returns (A, A^-1, attempt,
    kappa, kappas_of_all_attempts)."""
    kappas = []
    for attempt in range(max_attempts):
        A = gaussian_matrix(seed, batch_id, STREAM_MIXING, attempt, n, n) / math.sqrt(n)
        kappa = cond2(A)
        kappas.append(kappa)
        if kappa <= cond_max:
            return A, inverse(A), attempt, kappa, kappas
    raise RuntimeError("no well-conditioned draw within max_attempts")


CONDITIONED_BETA = 0.25


def sample_conditioned(seed, batch_id, n, beta=CONDITIONED_BETA):
    """Well-conditioned dense non-orthogonal A = Q + beta * G2 / sqrt(n), Q the
    orthogonal matrix of `sample_orthogonal`, G2 an independent Gaussian.
    ||G2/sqrt(n)||_2 ~ 2, so the singular values stay within about
    [1-2 beta, 1+2 beta]: kappa of a few, inside the paper's "kappa < 100"
    advice, while A^T A != I.  (The construction is a reading of this
    implementation; the paper asks for a well-conditioned general A without saying
    how to get one.)
    Returns (A, A^-1, kappa)."""
    Q, _ = sample_orthogonal(seed, batch_id, n)
    G2 = gaussian_matrix(seed, batch_id, STREAM_PERTURB, 0, n, n)
    A = Q + (beta / math.sqrt(n)) * G2
    return A, inverse(A), cond2(A)


# --------------------------------------------------------------------------
# Structured orthogonal A.  The paper's Conclusion lists "faster constructions
# for fresh, well-conditioned mixing (e.g. structured orthogonal transforms)" as
# future work and gives no construction; the one below is this implementation's:
#   A = P_R (B D_{R-1} P_{R-1}) ... (B D_1 P_1) (B D_0 P_0)
# with P_r random row permutations, D_r random sign flips and B the normalised
# Walsh-Hadamard transform on blocks of rows.  Every factor is orthogonal, so
# A^-1 = A^T; applying A costs O(n log n) per column instead of O(n^2).
# --------------------------------------------------------------------------
STRUCTURED_ROUNDS = 3


def philox_words(seed, batch_id, stream, sub, count):
    """`count` raw 32-bit words: word i is output i mod 4 of Philox block i div 4, block q drawn with
    counter (q, stream<<8 | sub, batch_id low, batch_id high) and key (seed low, seed high)."""
    q = np.arange((count + 3) // 4, dtype=np.uint64)
    c1 = np.uint64(((int(stream) & 0xFFFFFF) << 8) | (int(sub) & 0xFF))
    c2 = np.uint64(int(batch_id) & 0xFFFFFFFF)
    c3 = np.uint64((int(batch_id) >> 32) & 0xFFFFFFFF)
    key = (int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF)
    return np.stack(philox4x32_10((q, c1, c2, c3), key), axis=1).reshape(-1)[:count]


def walsh_hadamard(m):
    """Sylvester's m x m matrix of +-1 (m a power of two): H_1 = [1], H_2m = [[H_m, H_m], [H_m, -H_m]]."""
    if m < 1 or m & (m - 1):
        raise ValueError("power of two expected")
    Hm = np.ones((1, 1))
    while Hm.shape[0] < m:
        Hm = np.block([[Hm, Hm], [Hm, -Hm]])
    return Hm


def hadamard_blocks(n):
    """The powers of two of the binary expansion of n, largest first: the row blocks of B.
    (n = 2150 -> 2048, 64, 32, 4, 2.)"""
    return [1 << b for b in range(int(n).bit_length() - 1, -1, -1) if (n >> b) & 1]


def block_hadamard(n):
    """B: block-diagonal n x n matrix, one block H_m / sqrt(m) per entry of hadamard_blocks(n), in that order."""
    B = np.zeros((n, n))
    at = 0
    for m in hadamard_blocks(n):
        B[at:at + m, at:at + m] = walsh_hadamard(m) / math.sqrt(m)
        at += m
    return B


def permutation_from_keys(keys):
    """The permutation that sorts (key, index) pairs in ascending order: entry j is the index of the
    j-th smallest key, equal keys in index order."""
    return np.argsort(np.asarray(keys, dtype=np.uint32), kind="stable")


def structured_tables(seed, batch_id, n, rounds=STRUCTURED_ROUNDS):
    """The random draws behind one structured A: `rounds + 1` permutations (each from n Philox words
    used as sort keys, stream STREAM_STRUCT_PERM, sub-stream = its number) and `rounds` sign vectors
    (top bit of the words of stream STREAM_STRUCT_SIGN set -> -1)."""
    perms = np.stack([permutation_from_keys(philox_words(seed, batch_id, STREAM_STRUCT_PERM, r, n))
                      for r in range(rounds + 1)])
    signs = np.stack([np.where(philox_words(seed, batch_id, STREAM_STRUCT_SIGN, r, n) >> np.uint32(31), -1.0, 1.0)
                      for r in range(rounds)]) if rounds > 0 else np.zeros((0, n))
    return perms, signs


def structured_matrix(perms, signs):
    """Dense A = P_R (B D_{R-1} P_{R-1}) ... (B D_0 P_0) from its factors, each written out as a matrix:
    (P_r x)[j] = x[perms[r][j]], D_r = diag(signs[r])."""
    perms = np.asarray(perms)
    n = perms.shape[1]
    rounds = perms.shape[0] - 1
    B = block_hadamard(n)
    eye = np.eye(n)
    A = eye
    for r in range(rounds):
        P = eye[perms[r]]                       # row j of P picks x[perms[r][j]]
        D = np.diag(np.asarray(signs[r], dtype=np.float64))
        A = B @ (D @ (P @ A))
    return eye[perms[rounds]] @ A


def structured_apply(perms, signs, X, transposed=False):
    """A X (or A^T X) for an n x m matrix X, factor by factor in the order of the definition, without
    forming A: A^T = P_0^T D_0 B P_1^T D_1 B ... B P_R^T  (B is symmetric, (P^T x)[perm[j]] = x[j])."""
    perms = np.asarray(perms)
    X = np.array(X, dtype=np.float64, copy=True)
    n = perms.shape[1]
    rounds = perms.shape[0] - 1
    B = block_hadamard(n)
    if not transposed:
        for r in range(rounds):
            X = B @ (np.asarray(signs[r], dtype=np.float64)[:, None] * X[perms[r]])
        return X[perms[rounds]]
    out = np.empty_like(X)
    out[perms[rounds]] = X
    X = out
    for r in range(rounds - 1, -1, -1):
        X = np.asarray(signs[r], dtype=np.float64)[:, None] * (B @ X)
        out = np.empty_like(X)
        out[perms[r]] = X
        X = out
    return X


def sample_structured(seed, batch_id, n, rounds=STRUCTURED_ROUNDS):
    """Fresh structured orthogonal A for one batch; returns (A, A^-1 = A^T)."""
    A = structured_matrix(*structured_tables(seed, batch_id, n, rounds))
    return A, A.T.copy()


# --------------------------------------------------------------------------
# Block-diagonal orthogonal A: the mixed rows are cut into blocks of at most
# BLOCK_ROWS rows and each block is mixed by a dense orthogonal matrix of its
# own (a Householder QR of its own Gaussian, as in the paper's A-gen step).
# The paper does not describe it; it is the cheaper-fresh-A direction of its
# Conclusion taken the other way from the structured transform: mixing cost
# O(n b (d + p)) instead of O(n^2 (d + p)), at the price that rows only mix
# inside their block.  Every block takes its share of the shield rows.
# --------------------------------------------------------------------------
BLOCK_ROWS = 256


def block_layout(n_data, k, block=BLOCK_ROWS):
    """How the n = n_data + k mixed rows are cut: a list of (row0, rows, data0, data_rows, shield0, shield_rows).
    Block i owns mixed rows [row0, row0 + rows), rows = min(block, n - row0); of the rows up to a cut r, floor(k r / n)
    are shield rows and the rest data rows, so every block gets shield rows in proportion to its size."""
    n = n_data + k
    cuts = list(range(0, n, block)) + [n]
    out = []
    for i in range(len(cuts) - 1):
        r0, r1 = cuts[i], cuts[i + 1]
        s0, s1 = (k * r0) // n, (k * r1) // n
        out.append((r0, r1 - r0, r0 - s0, (r1 - s1) - (r0 - s0), s0, s1 - s0))
    return out


def sample_block_orthogonal(seed, batch_id, n_data, k, block=BLOCK_ROWS):
    """The dense n x n matrix that acts on the stacked rows [H; S] (data rows first, shield rows last): mixed rows
    [row0, row0 + rows) = A_i [H[data0 : data0 + data_rows]; S[shield0 : shield0 + shield_rows]] with A_i the
    orthogonal factor (positive-diagonal R) of the block's own Gaussian.  Returns (A, A^-1 = A^T)."""
    n = n_data + k
    A = np.zeros((n, n), dtype=np.float64)
    for i, (r0, rows, d0, dn, s0, sn) in enumerate(block_layout(n_data, k, block)):
        Ai = orthogonal_from_gaussian(gaussian_matrix(seed, batch_id, STREAM_BLOCK, i, rows, rows))
        A[r0:r0 + rows, d0:d0 + dn] = Ai[:, :dn]
        A[r0:r0 + rows, n_data + s0:n_data + s0 + sn] = Ai[:, dn:]
    return A, A.T.copy()


# --------------------------------------------------------------------------
# Orthogonal A as a product of reflectors drawn directly (Section 3.2 step 1.2 asks for a fresh random orthogonal
# A; Section 4.2 and Table 3 name its generation as what grows like n^3; the Conclusion asks for faster
# orthogonal transforms).  In the Householder QR of a Gaussian G the k-th reflector is built from column k of
# the UPDATED matrix, rows k onward - which, given the earlier reflectors, is again a vector of independent
# standard Gaussians.  So the reflectors have the same joint law when each is built from the raw entries
# G[k:, k] instead, and  A = H_0 H_1 ... H_{n-1} diag(sign beta_k)  (H_k x_k = beta_k e_0) is Haar-distributed
# like the QR factor - without factorising anything (Stewart, SIAM J. Numer. Anal. 17, 1980).
# --------------------------------------------------------------------------
def orthogonal_from_reflectors(G, columns=None):
    """A = H_0 H_1 ... H_{n-1} diag(sign beta_k), H_k = diag(I_k, I - 2 v v^T / (v^T v)) with
    v = x + sign(x_0) ||x|| e_0 and x = G[k:, k] (raw entries), so that H_k maps x to beta_k e_0,
    beta_k = -sign(x_0) ||x||.  A column of zeros contributes the identity and the sign +1.
    `columns`: only these columns of A (the product applied to those unit vectors: O(n^2) per column)."""
    G = np.asarray(G, dtype=np.float64)
    n = G.shape[0]
    if G.shape[1] != n:
        raise ValueError("square matrix expected")
    Q = np.eye(n) if columns is None else np.eye(n)[:, list(columns)]
    beta = np.zeros(n)
    for k in range(n - 1, -1, -1):                     # Q <- H_k Q: H_{n-1} first, H_0 last
        x = G[k:, k]
        norm_x = math.sqrt(float(x @ x))
        if norm_x == 0.0:
            continue
        v = x.copy()
        v[0] += norm_x if x[0] >= 0.0 else -norm_x
        beta[k] = -norm_x if x[0] >= 0.0 else norm_x
        Q[k:, :] -= (2.0 / float(v @ v)) * np.outer(v, v @ Q[k:, :])
    signs = np.where(beta < 0.0, -1.0, 1.0)
    if columns is not None:
        signs = signs[list(columns)]
    return Q * signs[None, :]


def sample_reflector_product(seed, batch_id, n):
    """Fresh orthogonal A for one batch from the same Gaussian draw as sample_orthogonal; returns (A, A^T)."""
    G = gaussian_matrix(seed, batch_id, STREAM_MIXING, 0, n, n)
    A = orthogonal_from_reflectors(G)
    return A, A.T.copy()


# --------------------------------------------------------------------------
# Shield rows (Section 3.2.1, Mitigation 2, eqs. 7-9).
# --------------------------------------------------------------------------
NORM_MEDIAN = 0
NORM_MEAN = 1


def row_norm_statistic(H, stat=NORM_MEDIAN):
    norms = np.sqrt(np.sum(np.asarray(H, dtype=np.float64) ** 2, axis=1))
    if stat == NORM_MEDIAN:
        return float(np.median(norms))      # even count: mean of the two middle values
    if stat == NORM_MEAN:
        return float(np.mean(norms))
    raise ValueError("unknown statistic")


def shield_rows(H, directions, scale, stat=NORM_MEDIAN):
    """S_i = directions_i * scale * m(H) / ||directions_i||: k secret rows,
    each of norm exactly `scale` times the row-norm statistic of H."""
    directions = np.asarray(directions, dtype=np.float64)
    if directions.shape[0] == 0:
        return directions.reshape(0, np.asarray(H).shape[1])
    m = row_norm_statistic(H, stat)
    norms = np.sqrt(np.sum(directions ** 2, axis=1))
    return directions * (scale * m / norms)[:, None]


def sample_shield_directions(seed, batch_id, k, d):
    return gaussian_matrix(seed, batch_id, STREAM_SHIELD, 0, k, d)


# --------------------------------------------------------------------------
# The protocol (Section 3.2, eqs. 1-3; eq. 8 with shields).
# --------------------------------------------------------------------------
def mix(A, H, S=None):
    """U = A [H; S]  (eq. 1; eq. 8 when shield rows are stacked under H)."""
    H = np.asarray(H, dtype=np.float64)
    H_full = H if S is None or len(S) == 0 else np.vstack([H, np.asarray(S, dtype=np.float64)])
    return np.asarray(A, dtype=np.float64) @ H_full


def project(U, W):
    """Y = U W  (eq. 2), the accelerator's only job."""
    return np.asarray(U, dtype=np.float64) @ np.asarray(W, dtype=np.float64)


def unmix(A_inv, Y, n_data):
    """Z = (A^-1 Y)[0:n_data]  (eq. 3, then the shield rows are dropped)."""
    Z_full = np.asarray(A_inv, dtype=np.float64) @ np.asarray(Y, dtype=np.float64)
    return Z_full[:n_data]


def plain_projection(H, W):
    """What the protocol must reproduce (eq. 4): Z* = H W."""
    return np.asarray(H, dtype=np.float64) @ np.asarray(W, dtype=np.float64)


KIND_ORTHOGONAL = 0
KIND_GAUSSIAN = 1
KIND_CONDITIONED = 2
KIND_STRUCTURED = 3
KIND_BLOCK_ORTHOGONAL = 4
KIND_REFLECTOR_PRODUCT = 5


def sample_mixing(kind, seed, batch_id, n, cond_max=1e3, max_attempts=64):
    """Returns (A, A^-1, info) for one batch."""
    if kind == KIND_ORTHOGONAL:
        A, A_inv = sample_orthogonal(seed, batch_id, n)
        return A, A_inv, {"attempt": 0, "kappa": 1.0}
    if kind == KIND_GAUSSIAN:
        A, A_inv, attempt, kappa, kappas = sample_gaussian(seed, batch_id, n, cond_max, max_attempts)
        return A, A_inv, {"attempt": attempt, "kappa": kappa, "kappas": kappas}
    if kind == KIND_CONDITIONED:
        A, A_inv, kappa = sample_conditioned(seed, batch_id, n)
        return A, A_inv, {"attempt": 0, "kappa": kappa}
    if kind == KIND_STRUCTURED:
        A, A_inv = sample_structured(seed, batch_id, n)
        return A, A_inv, {"attempt": 0, "kappa": 1.0}
    if kind == KIND_REFLECTOR_PRODUCT:
        A, A_inv = sample_reflector_product(seed, batch_id, n)
        return A, A_inv, {"attempt": 0, "kappa": 1.0}
    raise ValueError("unknown kind")


def qkv_forward(kind, seed, batch_id, H, W, k_shield=0, shield_scale=10.0,
                stat=NORM_MEDIAN, cond_max=1e3, max_attempts=64):
    """The whole chain for one batch, every intermediate returned."""
    H = np.asarray(H, dtype=np.float64)
    n_data, d = H.shape
    n = n_data + k_shield
    if kind == KIND_BLOCK_ORTHOGONAL:                      # its blocks depend on how n splits into data and shield rows
        A, A_inv = sample_block_orthogonal(seed, batch_id, n_data, k_shield)
        info = {"attempt": 0, "kappa": 1.0}
    else:
        A, A_inv, info = sample_mixing(kind, seed, batch_id, n, cond_max, max_attempts)
    S = shield_rows(H, sample_shield_directions(seed, batch_id, k_shield, d), shield_scale, stat)
    U = mix(A, H, S)
    Y = project(U, W)
    Z = unmix(A_inv, Y, n_data)
    return {"A": A, "A_inv": A_inv, "S": S, "U": U, "Y": Y, "Z": Z, "info": info}


def rel_frobenius(X, X_ref):
    """||X - X_ref||_F / ||X_ref||_F over the whole matrix."""
    X_ref = np.asarray(X_ref, dtype=np.float64)
    return float(np.linalg.norm(np.asarray(X, dtype=np.float64) - X_ref) / np.linalg.norm(X_ref))
