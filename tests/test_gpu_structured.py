"""GPU parity of the structured orthogonal kind (GELO_STRUCTURED): its random tables (integer work:
the dense A the library builds for export must be the oracle's matrix), the transform applied
forward (mix) and transposed (unmix, shield rows dropped), and the chain end to end.  Same bars
as for the dense kinds: 1e-4 (f32) / 2e-2 (bf16) end to end, tighter per stage."""
import math

import numpy as np
import pytest
import torch

from oracle import gelo_oracle as o
from paper_2603_05035_amd import binding as g
from paper_2603_05035_amd import workloads as wl

pytestmark = pytest.mark.gpu

SEED = 0x57C7
TOL_END = {"f32": 1e-4, "bf16": 2e-2}
TOL_STAGE = {"f32": 1e-5, "bf16": 4e-3}       # float butterflies + one rounding of the output
TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}
CODE = {"f32": g.GELO_F32, "bf16": g.GELO_BF16}


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(TORCH_DTYPE[dtype]).cuda()


def f64(t):
    return t.detach().to(torch.float64).cpu().numpy()


@pytest.fixture()
def ctx():
    """a context per test: batch ids need not rise from one test to the next (a context refuses ids that
    fall more than GELO_BATCH_WINDOW below the highest one it has seen)"""
    c = g.gelo_create(0, SEED, allow_batch_reuse=False)
    yield c
    g.gelo_destroy(c)


@pytest.mark.parametrize("n_data,k", [(1, 0), (2, 0), (3, 0), (16, 2), (67, 3), (255, 0), (256, 0), (300, 21),
                                      (1000, 24), (2048, 102)])
def test_dense_matrix_of_the_tables_matches_oracle(ctx, n_data, k):
    """Permutations and signs are integer work: a single wrong rank or sign bit changes entries of A by
    about 1 / sqrt(n), far above the float rounding of the butterflies allowed here."""
    n = n_data + k
    bid = 100 + 3 * n
    m = g.gelo_sample_mixing(ctx, g.GELO_STRUCTURED, n_data, k, 64, g.GELO_F32, 0.0, 1, batch_id=bid)
    A, A_inv, _, attempt, kappa = g.gelo_mixing_export(ctx, m, n, k, 64, want_shields=False)
    g.gelo_mixing_free(ctx, m)
    assert attempt == 0 and kappa == 1.0
    A_ref, _ = o.sample_structured(SEED, bid, n)
    assert np.abs(f64(A) - A_ref).max() < 2e-6
    assert np.abs(f64(A_inv) - A_ref.T).max() < 2e-6
    assert np.linalg.norm(f64(A) @ f64(A_inv) - np.eye(n)) / math.sqrt(n) < 1e-5


@pytest.mark.parametrize("n_data,k", [(1, 0), (2, 1), (63, 0), (64, 0), (65, 0), (300, 21), (2048, 102), (4096, 205),
                                      (5000, 120)])
def test_table_words_are_bit_exact(ctx, n_data, k):
    """The tables are pure integer work (ranks of Philox keys, sign bits) and are held bit for bit: every
    word of the library's table against the oracle's permutations (low 31 bits) and signs (top bit; the
    last permutation carries none)."""
    n = n_data + k
    bid = 900000 + n
    m = g.gelo_sample_mixing(ctx, g.GELO_STRUCTURED, n_data, k, 64, g.GELO_F32, 0.0, 1, batch_id=bid)
    table = g.gelo_mixing_export_table(ctx, m, n).cpu().numpy().view(np.uint32)
    g.gelo_mixing_free(ctx, m)
    perms, signs = o.structured_tables(SEED, bid, n)
    assert table.shape == (4, n)
    assert np.array_equal(table & np.uint32(0x7FFFFFFF), perms.astype(np.uint32))
    sign_bits = (table >> np.uint32(31)).astype(np.int64)
    assert np.array_equal(sign_bits[:3], (signs < 0).astype(np.int64))
    assert not sign_bits[3].any()


@pytest.mark.parametrize("n_data,k", [(2272, 0), (2273, 0), (4096, 205), (4304, 0), (4305, 0), (5000, 120)])
def test_tables_at_the_narrow_strip_widths(ctx, n_data, k):
    """A workgroup keeps 16 columns of the strip (and one table) in LDS up to 2272 rows (all 160 KB of it then),
    8 up to 4304, 4 beyond, up to n = GELO_MAX_N: both sides of each boundary.  The dense oracle matrix would cost minutes
    here: sampled columns of A and A^T through the oracle's factor-by-factor transform, and orthogonality of
    the exported pair."""
    n = n_data + k
    bid = 51 + n
    m = g.gelo_sample_mixing(ctx, g.GELO_STRUCTURED, n_data, k, 64, g.GELO_F32, 0.0, 1, batch_id=bid)
    A, A_inv, _, _, _ = g.gelo_mixing_export(ctx, m, n, k, 64, want_shields=False)
    g.gelo_mixing_free(ctx, m)
    perms, signs = o.structured_tables(SEED, bid, n)
    cols = np.random.default_rng(n).choice(n, size=6, replace=False)
    E = np.zeros((n, 6))
    E[cols, np.arange(6)] = 1.0
    assert np.abs(f64(A)[:, cols] - o.structured_apply(perms, signs, E)).max() < 2e-6
    assert np.abs(f64(A_inv)[:, cols] - o.structured_apply(perms, signs, E, transposed=True)).max() < 2e-6
    assert torch.linalg.matrix_norm(A @ A_inv - torch.eye(n, device="cuda")).item() / math.sqrt(n) < 1e-5


def run_chain(ctx, dtype, H32, W32, k, batch_id, scale=10.0):
    H, W = dev(H32, dtype), dev(W32, dtype)
    nd, d = H.shape
    p = W.shape[1]
    n = nd + k
    m = g.gelo_sample_mixing(ctx, g.GELO_STRUCTURED, nd, k, d, CODE[dtype], 0.0, 1, batch_id)
    U = torch.empty((n, d), dtype=H.dtype, device="cuda")
    Y = torch.empty((n, p), dtype=H.dtype, device="cuda")
    Z = torch.full((nd, p), float("nan"), dtype=H.dtype, device="cuda")
    g.gelo_mix(ctx, m, H, U, scale)
    g.gelo_project(ctx, U, W, Y)
    _, _, S, _, _ = g.gelo_mixing_export(ctx, m, n, k, d, want_matrices=False) if k else (None, None, None, 0, 1.0)
    g.gelo_unmix(ctx, m, Y, Z)
    torch.cuda.synchronize()
    g.gelo_mixing_free(ctx, m)
    return dict(H=H, W=W, U=U, Y=Y, Z=Z, S=S)


CASES = [("f32", 16, 2, 64, 192), ("bf16", 16, 2, 64, 192), ("f32", 1, 0, 8, 8), ("bf16", 2, 1, 8, 16),
         ("f32", 300, 15, 256, 520), ("bf16", 300, 15, 264, 520), ("f32", 1031, 0, 72, 40),
         ("bf16", 2048, 102, 512, 776), ("bf16", 4096, 205, 256, 264), ("f32", 5000, 120, 64, 72),
         ("bf16", 200, 10, 2056, 2072), ("f32", 500, 12, 2048, 2056)]      # short strips: 64 columns per workgroup


@pytest.mark.parametrize("dtype,nd,k,d,p", CASES)
def test_chain_stagewise_and_end_to_end(ctx, dtype, nd, k, d, p):
    """Ragged strips (widths that are not multiples of the strip width), all strip widths (64, 16 and 8
    columns per workgroup), blocks of every size in the binary expansion of n, with and without shield rows."""
    H32 = wl.make_hidden(nd, d, 77 + nd, min(4, d))
    W32 = wl.make_weight(d, p, 78 + nd)
    bid = 5000 + nd * 3 + (dtype == "bf16")
    r = run_chain(ctx, dtype, H32, W32, k, bid)
    H, W = f64(r["H"]), f64(r["W"])
    S = f64(r["S"]) if k else np.zeros((0, d))
    perms, signs = o.structured_tables(SEED, bid, nd + k)
    tol = TOL_STAGE[dtype]
    assert o.rel_frobenius(f64(r["U"]), o.structured_apply(perms, signs, np.vstack([H, S]))) < tol        # eq. 1 / eq. 8
    assert o.rel_frobenius(f64(r["Y"]), o.project(f64(r["U"]), W)) < tol                                 # eq. 2
    assert o.rel_frobenius(f64(r["Z"]), o.structured_apply(perms, signs, f64(r["Y"]), transposed=True)[:nd]) < tol   # eq. 3
    assert o.rel_frobenius(f64(r["Z"]), o.plain_projection(H, W)) < TOL_END[dtype]                       # eq. 4
    if k:   # eq. 9: the Gram matrix the accelerator can form is the data's plus the shields'
        U = f64(r["U"])
        assert o.rel_frobenius(U.T @ U, H.T @ H + S.T @ S) < 10 * tol


@pytest.mark.parametrize("name", ["llama7b_bf16_prefill_structured", "sweep_bf16_structured", "decode_bf16_structured",
                                  "llama7b_bf16_mlp_gate_up", "llama7b_bf16_mlp_down"])
def test_full_size_structured_workloads(ctx, name):
    """The benchmark's structured workloads at full size (d = 4096, p = 12288 with 2048 + 102, 4096 + 205 and
    64 + 4 rows; the two MLP projections 4096 -> 22016 and 11008 -> 4096) in the launch configuration it times: every stage against the oracle on sampled columns
    (the transform acts on columns independently), the whole result by a random projection."""
    w = wl.WORKLOADS[name]
    H32, W32 = wl.make_inputs(w)
    bid = 4242 + w.seed * 10000
    r = run_chain(ctx, "bf16", H32, W32, w.k_shield, bid)
    H, W, S = f64(r["H"]), f64(r["W"]), f64(r["S"])
    U, Y, Z = f64(r["U"]), f64(r["Y"]), f64(r["Z"])
    perms, signs = o.structured_tables(SEED, bid, w.n)
    rng = np.random.default_rng(3)
    cd = rng.choice(w.d, size=48, replace=False)
    cp = rng.choice(w.p, size=48, replace=False)
    assert o.rel_frobenius(U[:, cd], o.structured_apply(perms, signs, np.vstack([H, S])[:, cd])) < TOL_STAGE["bf16"]
    assert o.rel_frobenius(Y[:, cp], U @ W[:, cp]) < TOL_STAGE["bf16"]
    assert o.rel_frobenius(Z[:, cp], o.structured_apply(perms, signs, Y[:, cp], transposed=True)[:w.n_data]) < TOL_STAGE["bf16"]
    assert o.rel_frobenius(Z[:, cp], H @ W[:, cp]) < TOL_END["bf16"]
    rvec = rng.standard_normal(w.p)
    assert np.linalg.norm(Z @ rvec - H @ (W @ rvec)) / np.linalg.norm(H @ (W @ rvec)) < TOL_END["bf16"]
    assert not np.isnan(Z).any()


def test_qkv_forward_and_fresh_tables(ctx):
    w = wl.WORKLOADS["tiny_f32"]
    H32, W32 = wl.make_inputs(w)
    H, W = dev(H32, "f32"), dev(W32, "f32")
    Z = torch.empty((w.n_data, w.p), dtype=torch.float32, device="cuda")
    g.gelo_qkv_forward(ctx, g.GELO_STRUCTURED, H, W, Z, k_shield=2, batch_id=31)
    torch.cuda.synchronize()
    assert o.rel_frobenius(f64(Z), o.plain_projection(f64(H), f64(W))) < TOL_END["f32"]
    mats = []
    for bid in (32, 33):
        m = g.gelo_sample_mixing(ctx, g.GELO_STRUCTURED, 16, 2, 64, g.GELO_F32, 0.0, 1, batch_id=bid)
        mats.append(g.gelo_mixing_export(ctx, m, 18, 2, 64, want_shields=False)[0])
        g.gelo_mixing_free(ctx, m)
    assert (mats[0] - mats[1]).abs().max() > 0.05              # a fresh A per batch id


def test_structured_kind_rejects_what_it_cannot_hold(ctx):
    with pytest.raises(g.GeloError) as e:
        g.gelo_sample_mixing(ctx, g.GELO_STRUCTURED, 5120, 1, 64, g.GELO_F32, 0.0, 1, batch_id=1)
    assert g.STATUS_NAMES[e.value.status] == "GELO_ESHAPE"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_strided_operands(ctx, dtype):
    """Leading dimensions larger than the width (views into bigger buffers): the transform must keep to
    its columns on the way in and on the way out, and the rows the unmix drops must stay unwritten."""
    nd, k, d, p = 70, 4, 72, 136
    td = TORCH_DTYPE[dtype]
    big_h = torch.zeros((nd, d + 24), dtype=td, device="cuda")
    H = big_h[:, :d]
    H.copy_(torch.from_numpy(wl.make_hidden(nd, d, 9, 0)).to(td))
    W = dev(wl.make_weight(d, p, 9), dtype)
    U = torch.full((nd + k, d + 8), 7.0, dtype=td, device="cuda")[:, :d]
    Y = torch.full((nd + k, p + 16), 7.0, dtype=td, device="cuda")[:, :p]
    Zbuf = torch.full((nd + k, p + 8), 7.0, dtype=td, device="cuda")        # k rows more than the unmix writes
    Z = Zbuf[:nd, :p]
    m = g.gelo_sample_mixing(ctx, g.GELO_STRUCTURED, nd, k, d, CODE[dtype], 0.0, 1, batch_id=8001 + (dtype == "bf16"))
    g.gelo_mix(ctx, m, H, U)
    g.gelo_project(ctx, U, W, Y)
    g.gelo_unmix(ctx, m, Y, Z)
    torch.cuda.synchronize()
    g.gelo_mixing_free(ctx, m)
    assert o.rel_frobenius(f64(Z), o.plain_projection(f64(H), f64(W))) < TOL_END[dtype]
    assert torch.all(U._base[:, d:] == 7.0) and torch.all(Y._base[:, p:] == 7.0)
    assert torch.all(Zbuf[:, p:] == 7.0) and torch.all(Zbuf[nd:, :] == 7.0)      # shield rows are never stored
