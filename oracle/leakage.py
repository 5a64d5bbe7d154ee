"""What the accelerator can learn from U = A [H; S]: the leakage measures of the paper and a
blind-source-separation attack to try them with.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see gelo_oracle.py): plain float64 numpy, used by
tests only.  The measures follow Section 3.2.1 "Mitigating Gram Matrix Information Leaks"
(eqs. 5, 6, 9) and the matched-subset Gram error of Section 4.3 "Results: Geometric Recovery";
the attack is the FastICA fixed-point iteration the paper's Section 4.3 / 4.4 attacks run
(Hyvarinen 1999; Hyvarinen & Oja 2000), written from the published algorithm.

The closed-form measures are pinned by the paper's identities in tests/test_leakage.py.  The
attack has no pin in the paper that can be reproduced here (its numbers are measured on LLM
hidden states): what the tests assert about it is what it does on synthetic independent
sources -- parity unpinned against the paper's figures.
"""
from __future__ import annotations

import numpy as np
from scipy.optimize import linear_sum_assignment


def covariance_leak(U, H):
    """||U^T U - H^T H||_F / ||H^T H||_F: zero when the d x d feature covariance of the hidden
    states can be read off the mixed batch (eq. 5, orthogonal A without shields)."""
    G = H.T @ H
    return float(np.linalg.norm(U.T @ U - G) / np.linalg.norm(G))


def similarity_spectrum(X):
    """Eigenvalues of X X^T in descending order: the spectrum of token-token similarities, which an
    orthogonal A leaves unchanged (eq. 6: U U^T = A (H H^T) A^T is similar to H H^T)."""
    return np.sort(np.linalg.eigvalsh(X @ X.T))[::-1]


def spectrum_leak(U, H):
    """Relative distance between the similarity spectra of U and of H (zero: eq. 6 leaks it).
    U may have more rows than H (shields): H's spectrum is padded with zeros."""
    su, sh = similarity_spectrum(U), similarity_spectrum(H)
    sh = np.concatenate([sh, np.zeros(len(su) - len(sh))])
    return float(np.linalg.norm(su - sh) / np.linalg.norm(sh))


def match_rows(estimates, truth):
    """One-to-one pairing of true rows with estimated rows that maximises the total absolute cosine
    similarity (Hungarian algorithm, Section 4.3 "Matching").  Returns (index into estimates for
    every true row, the absolute cosines of the pairs)."""
    e = estimates / np.maximum(np.linalg.norm(estimates, axis=1, keepdims=True), 1e-300)
    t = truth / np.maximum(np.linalg.norm(truth, axis=1, keepdims=True), 1e-300)
    c = np.abs(t @ e.T)
    rows, cols = linear_sum_assignment(-c)
    order = np.empty(len(truth), dtype=int)
    order[rows] = cols
    return order, c[np.arange(len(truth)), order]


def matched_gram_error(estimates, truth):
    """Matched-subset Gram error of Section 4.3: pair the rows, then
    ||G_est - G_true||_F / ||G_true||_F with G = X X^T over the matched rows.  The paper does not say
    how the rows are scaled; a blind attack recovers them only up to scale and sign, so both subsets
    are brought to unit row norm here and every estimate to the sign of its partner (a reading)."""
    order, _ = match_rows(estimates, truth)
    est = estimates[order]
    est = est / np.maximum(np.linalg.norm(est, axis=1, keepdims=True), 1e-300)
    tru = truth / np.maximum(np.linalg.norm(truth, axis=1, keepdims=True), 1e-300)
    sign = np.sign(np.sum(est * tru, axis=1))
    est = est * np.where(sign == 0, 1.0, sign)[:, None]
    g_true, g_est = tru @ tru.T, est @ est.T
    return float(np.linalg.norm(g_est - g_true) / np.linalg.norm(g_true))


def fastica(U, n_sources=None, iterations=200, tol=1e-8, seed=0):
    """Symmetric FastICA with the tanh contrast.  Model: the rows of U (n x d) are unknown
    mixtures of independent source rows, the d columns are the samples.  Steps: centre every row;
    whiten with the leading n_sources eigenvectors of the row covariance; iterate
    W <- E[g(W Z) Z^T] - diag(E[g'(W Z)]) W followed by the symmetric decorrelation
    W <- (W W^T)^(-1/2) W until the rows of W stop turning.  Returns the estimated sources
    (n_sources x d), in arbitrary order, sign and scale."""
    X = U - U.mean(axis=1, keepdims=True)
    n, d = X.shape
    r = n if n_sources is None else n_sources
    evals, evecs = np.linalg.eigh(X @ X.T / d)
    keep = np.argsort(evals)[::-1][:r]
    white = (evecs[:, keep] / np.sqrt(np.maximum(evals[keep], 1e-300))).T      # r x n
    Z = white @ X
    rng = np.random.default_rng(seed)

    def decorrelate(W):
        s, u = np.linalg.eigh(W @ W.T)
        return (u / np.sqrt(np.maximum(s, 1e-300))) @ u.T @ W

    W = decorrelate(rng.standard_normal((r, r)))
    for _ in range(iterations):
        Y = W @ Z
        g = np.tanh(Y)
        W_new = decorrelate(g @ Z.T / d - np.diag((1.0 - g * g).mean(axis=1)) @ W)
        turn = np.max(np.abs(np.abs(np.sum(W_new * W, axis=1)) - 1.0))
        W = W_new
        if turn < tol:
            break
    return W @ Z
