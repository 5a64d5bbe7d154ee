"""Pins for the structured orthogonal mixing matrix of the oracle (the paper's Conclusion names
"structured orthogonal transforms" as the way to cheaper fresh mixing and gives no construction;
the one pinned here is this implementation's).  Nothing below re-uses the oracle's own formulas:
hand-computed cases, the closed form of Sylvester's matrix, a library routine as a checker,
brute force, and the invariants every orthogonal A has (Section 3.2 eq. 4, Section 3.2.1 eq. 5)."""
import math

import numpy as np
import pytest
import scipy.linalg

from oracle import gelo_oracle as o


def test_walsh_hadamard_closed_form_and_library():
    # Sylvester's matrix has entry (a, b) = (-1)^popcount(a & b)
    for m in (1, 2, 8, 64):
        closed = np.array([[(-1.0) ** bin(a & b).count("1") for b in range(m)] for a in range(m)])
        assert np.array_equal(o.walsh_hadamard(m), closed)
        assert np.array_equal(o.walsh_hadamard(m), scipy.linalg.hadamard(m))
    with pytest.raises(ValueError):
        o.walsh_hadamard(12)


def test_blocks_follow_the_binary_expansion():
    assert o.hadamard_blocks(2150) == [2048, 64, 32, 4, 2]
    assert o.hadamard_blocks(4301) == [4096, 128, 64, 8, 4, 1]
    assert o.hadamard_blocks(4096) == [4096] and o.hadamard_blocks(1) == [1]
    for n in range(1, 300):
        blocks = o.hadamard_blocks(n)
        assert sum(blocks) == n and blocks == sorted(set(blocks), reverse=True)
        assert all(b & (b - 1) == 0 for b in blocks)


def test_block_hadamard_hand_case():
    h = 0.5
    r = 1.0 / math.sqrt(2.0)
    want = np.array([[h, h, h, h, 0, 0],
                     [h, -h, h, -h, 0, 0],
                     [h, h, -h, -h, 0, 0],
                     [h, -h, -h, h, 0, 0],
                     [0, 0, 0, 0, r, r],
                     [0, 0, 0, 0, r, -r]])
    assert np.allclose(o.block_hadamard(6), want, atol=1e-15)
    for n in (1, 7, 70, 300):
        B = o.block_hadamard(n)
        assert np.abs(B @ B.T - np.eye(n)).max() < 1e-13 and np.array_equal(B, B.T)


def test_permutation_from_keys_against_tuple_sort():
    keys = np.array([7, 3, 7, 0, 3, 0xFFFFFFFF, 3], dtype=np.uint32)       # ties keep index order
    want = [i for _, i in sorted((int(k), i) for i, k in enumerate(keys))]
    assert list(o.permutation_from_keys(keys)) == want == [3, 1, 4, 6, 0, 2, 5]
    rng = np.random.default_rng(0)
    keys = rng.integers(0, 50, size=400).astype(np.uint32)
    assert list(o.permutation_from_keys(keys)) == [i for _, i in sorted((int(k), i) for i, k in enumerate(keys))]


def test_philox_words_layout():
    # word i = output i % 4 of block i // 4, counter (block, stream << 8 | sub, batch low, batch high)
    seed, batch = 0x1122334455667788, 0x0A0B0C0D01020304
    words = o.philox_words(seed, batch, stream=3, sub=2, count=11)
    for i in (0, 1, 6, 10):
        blk = o.philox4x32_10([np.array([i // 4]), np.array([(3 << 8) | 2]), np.array([0x01020304]), np.array([0x0A0B0C0D])],
                              (0x55667788, 0x11223344))
        assert int(words[i]) == int(blk[i % 4][0])
    assert words.dtype == np.uint32 and len(words) == 11


def test_structured_matrix_hand_case():
    # n = 3 (blocks 2 + 1), one round.  x = (a, b, c): P_0 -> (c, a, b); D_0 -> (c, -a, b);
    # B -> ((c - a)/s, (c + a)/s, b) with s = sqrt 2; P_1 -> ((c + a)/s, b, (c - a)/s)
    r = 1.0 / math.sqrt(2.0)
    A = o.structured_matrix(perms=[[2, 0, 1], [1, 2, 0]], signs=[[1.0, -1.0, 1.0]])
    want = np.array([[r, 0, r], [0, 1, 0], [-r, 0, r]])
    assert np.allclose(A, want, atol=1e-15)
    # no rounds: a bare permutation matrix
    assert np.array_equal(o.structured_matrix(perms=[[1, 2, 0]], signs=np.zeros((0, 3))), np.eye(3)[[1, 2, 0]])


def test_structured_matrix_against_a_loop_over_rows():
    """the same transform applied to vectors step by step with explicit butterflies (brute force)"""
    n = 22                                           # 16 + 4 + 2
    perms, signs = o.structured_tables(seed=5, batch_id=9, n=n, rounds=2)
    def apply(x):
        x = list(x)
        for r in range(2):
            x = [signs[r][j] * x[perms[r][j]] for j in range(n)]
            at = 0
            for m in (16, 4, 2):
                blk = x[at:at + m]
                h = 1
                while h < m:                         # in-place fast Walsh-Hadamard transform
                    for i in range(0, m, 2 * h):
                        for j in range(i, i + h):
                            blk[j], blk[j + h] = blk[j] + blk[j + h], blk[j] - blk[j + h]
                    h *= 2
                x[at:at + m] = [v / math.sqrt(m) for v in blk]
                at += m
        return [x[perms[2][j]] for j in range(n)]
    A = o.structured_matrix(perms, signs)
    cols = np.array([apply(np.eye(n)[:, c]) for c in range(n)]).T
    assert np.abs(A - cols).max() < 1e-14


def test_structured_tables_are_permutations_and_fair_signs():
    perms, signs = o.structured_tables(seed=77, batch_id=3, n=2150)
    assert perms.shape == (4, 2150) and signs.shape == (3, 2150)
    for p in perms:
        assert np.array_equal(np.sort(p), np.arange(2150))
    assert len({tuple(p) for p in perms}) == 4                      # four different permutations
    assert set(np.unique(signs)) == {-1.0, 1.0}
    assert abs(signs.mean()) < 4.0 / math.sqrt(signs.size)          # fair coin within 4 sigma
    other, _ = o.structured_tables(seed=77, batch_id=4, n=2150)     # fresh per batch
    assert not np.array_equal(other[0], perms[0])


@pytest.mark.parametrize("n", [1, 2, 18, 70, 300, 1100])
def test_structured_a_is_orthogonal(n):
    A, A_inv = o.sample_structured(seed=11, batch_id=n, n=n)
    assert np.abs(A @ A.T - np.eye(n)).max() < 1e-12
    assert np.array_equal(A_inv, A.T)
    if n <= 70:
        assert abs(abs(np.linalg.det(A)) - 1.0) < 1e-9


def test_three_rounds_spread_every_row_over_the_batch():
    """With unequal blocks one round leaves rows of A with two non-zero entries (n = 70 = 64 + 4 + 2:
    the last block mixes two rows).  After three rounds the entries look like those of a random
    orthogonal matrix: nearly all non-zero (sums of +-1 products do cancel exactly now and then), none
    much larger than 1 / sqrt(n)."""
    for batch in range(5):
        A = o.structured_matrix(*o.structured_tables(seed=1, batch_id=batch, n=70, rounds=3))
        support = np.abs(A) > 1e-9
        assert support.mean() > 0.97 and support.sum(axis=1).min() >= 45
        assert np.abs(A).max() * math.sqrt(70) < 6.0
    A1 = o.structured_matrix(*o.structured_tables(seed=1, batch_id=0, n=70, rounds=1))
    assert (np.abs(A1) > 1e-9).sum(axis=1).min() == 2


def test_chain_identity_and_gram_leak_with_structured_a():
    rng = np.random.default_rng(4)
    H = rng.standard_normal((48, 96))
    W = rng.standard_normal((96, 40)) * 0.02
    out = o.qkv_forward(o.KIND_STRUCTURED, seed=21, batch_id=8, H=H, W=W, k_shield=3)
    assert o.rel_frobenius(out["Z"], H @ W) < 1e-12                                   # eq. 4
    assert np.linalg.norm(out["A"] @ out["A_inv"] - np.eye(51)) < 1e-12
    S = out["S"]
    assert o.rel_frobenius(out["U"].T @ out["U"], H.T @ H + S.T @ S) < 1e-13          # eq. 9: orthogonal A
    U0 = o.mix(o.sample_structured(3, 0, 48)[0], H)
    assert o.rel_frobenius(U0.T @ U0, H.T @ H) < 1e-13                                # eq. 5: the Gram leak stays


def test_structured_apply_equals_the_dense_matrix():
    rng = np.random.default_rng(12)
    for n in (3, 22, 150):
        perms, signs = o.structured_tables(seed=9, batch_id=n, n=n)
        A = o.structured_matrix(perms, signs)
        X = rng.standard_normal((n, 7))
        assert np.abs(o.structured_apply(perms, signs, X) - A @ X).max() < 1e-13
        assert np.abs(o.structured_apply(perms, signs, X, transposed=True) - A.T @ X).max() < 1e-13


def test_bench_counts_the_butterflies_of_the_blocks():
    """bench.py prices a structured step by its additions: m log2 m per block of the binary expansion"""
    import bench
    assert bench.butterfly_adds(2150) == 2048 * 11 + 64 * 6 + 32 * 5 + 4 * 2 + 2 * 1
    assert bench.butterfly_adds(4096) == 4096 * 12 and bench.butterfly_adds(1) == 0
    for n in (3, 70, 2150):
        assert bench.butterfly_adds(n) == sum(m * int(math.log2(m)) for m in o.hadamard_blocks(n))
