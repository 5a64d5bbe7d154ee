"""Pins of the oracle's block-diagonal orthogonal A (the cheaper-fresh-A variant that keeps dense orthogonal
mixing inside row blocks).  The paper gives no construction, so the pins are what the construction itself fixes:
a layout worked out by hand, orthogonality, the zero pattern, LAPACK's QR of each block's Gaussian with the
positive-diagonal sign rule, and the protocol's identities (eq. 4, eq. 9) through the chain."""
import numpy as np

from oracle import gelo_oracle as o


def test_layout_worked_out_by_hand():
    # n = 45 rows in blocks of 16: cuts 0, 16, 32, 45; shield rows up to a cut r: floor(5 r / 45) = 0, 1, 3, 5
    assert o.block_layout(40, 5, block=16) == [(0, 16, 0, 15, 0, 1), (16, 16, 15, 14, 1, 2), (32, 13, 29, 11, 3, 2)]
    # no shields: plain row blocks; one block when everything fits
    assert o.block_layout(40, 0, block=16) == [(0, 16, 0, 16, 0, 0), (16, 16, 16, 16, 0, 0), (32, 8, 32, 8, 0, 0)]
    assert o.block_layout(10, 3, block=16) == [(0, 13, 0, 10, 0, 3)]


def test_layout_partitions_rows_and_spreads_the_shields():
    for n_data, k, block in ((2048, 102, 256), (4096, 205, 256), (300, 15, 64), (17, 1, 4), (5, 9, 4)):
        lay = o.block_layout(n_data, k, block)
        n = n_data + k
        assert [b[0] for b in lay] == list(range(0, n, block))
        assert sum(b[1] for b in lay) == n and all(0 < b[1] <= block for b in lay)
        d_next = s_next = 0
        for r0, rows, d0, dn, s0, sn in lay:
            assert (d0, s0) == (d_next, s_next) and dn + sn == rows and dn >= 0 and sn >= 0
            d_next, s_next = d0 + dn, s0 + sn
            assert abs(sn - k * rows / n) < 1.0 + 1e-12          # a block's share of the shield rows, to within one
        assert (d_next, s_next) == (n_data, k)


def test_blocks_are_the_qr_factors_of_their_own_gaussians():
    seed, bid, n_data, k, block = 11, 5, 40, 5, 16
    A, A_inv = o.sample_block_orthogonal(seed, bid, n_data, k, block)
    n = n_data + k
    assert np.abs(A.T @ A - np.eye(n)).max() < 1e-13 and np.array_equal(A_inv, A.T)
    covered = np.zeros((n, n), dtype=bool)
    for i, (r0, rows, d0, dn, s0, sn) in enumerate(o.block_layout(n_data, k, block)):
        cols = list(range(d0, d0 + dn)) + list(range(n_data + s0, n_data + s0 + sn))
        covered[np.ix_(range(r0, r0 + rows), cols)] = True
        Ai = A[np.ix_(range(r0, r0 + rows), cols)]
        G = o.gaussian_matrix(seed, bid, o.STREAM_BLOCK, i, rows, rows)
        Q, R = np.linalg.qr(G)                                   # LAPACK; made unique by the positive-diagonal rule
        Q = Q * np.sign(np.diag(R))
        assert np.abs(Ai - Q).max() < 1e-12
    assert np.all(A[~covered] == 0.0)                            # nothing outside the blocks
    B, _ = o.sample_block_orthogonal(seed, bid + 1, n_data, k, block)
    assert np.abs(A - B).max() > 0.05                            # fresh per batch id


def test_single_block_when_everything_fits():
    A, _ = o.sample_block_orthogonal(3, 9, 12, 2, block=16)
    G = o.gaussian_matrix(3, 9, o.STREAM_BLOCK, 0, 14, 14)
    assert np.array_equal(A, o.orthogonal_from_gaussian(G))


def test_chain_identities():
    rng = np.random.default_rng(7)
    H, W = rng.standard_normal((300, 24)), rng.standard_normal((24, 40))
    out = o.qkv_forward(o.KIND_BLOCK_ORTHOGONAL, 21, 4, H, W, k_shield=15, shield_scale=10.0)
    assert o.rel_frobenius(out["Z"], H @ W) < 1e-12              # eq. 4
    U, S = out["U"], out["S"]
    G_u, G_ref = U.T @ U, H.T @ H + S.T @ S                      # eq. 9: an orthogonal A keeps the Gram matrix of [H; S]
    assert np.linalg.norm(G_u - G_ref) / np.linalg.norm(G_ref) < 1e-12
    # rows only mix inside their block: a data row outside block 0 leaves the block's mixed rows unchanged
    r0, rows, d0, dn, s0, sn = o.block_layout(300, 15)[0]
    H2 = H.copy(); H2[d0 + dn + 3] += 1.0
    S_fixed = out["S"]
    assert np.array_equal(o.mix(out["A"], H, S_fixed)[:rows], o.mix(out["A"], H2, S_fixed)[:rows])


def test_bench_restates_the_same_layout():
    """bench.py counts the operations of the block kind from its own statement of the cut (it may not import the
    oracle outside its CPU-baseline leg): both must describe the same blocks."""
    import importlib.util
    import os
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    for n_data, k in ((2048, 102), (4096, 205), (300, 15), (100, 0), (1, 0), (513, 7)):
        assert bench.block_rows(n_data, k) == [(rows, dn) for _, rows, _, dn, _, _ in o.block_layout(n_data, k)]
