"""The 8-bit (OCP FP8 E4M3) projection against the oracle's rounding functions (oracle/precision.py).

Bars: the quantised codes of U and W are integer work and are held bit for bit - the decision which code a value
gets is taken in float32 on both sides (scale = max / 448 and x * (448 / max) in float32, then the oracle's
round-to-nearest-even onto the E4M3 grid); Y against the float64 product of the decoded operands at the bound
float accumulation plus one bf16 rounding gives; the chain's Z against H W at the bound the storage-format study
predicts for E4M3 with shields (3.7e-2 without, 6.5e-2 with 5% shields at 10x; bound 8e-2), far looser than the bf16 contract."""
import numpy as np
import pytest
import torch

from oracle import gelo_oracle as o
from oracle import precision as prec
from paper_2603_05035_amd import binding as g
from paper_2603_05035_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL_Y = 4e-3            # float accumulation + one bf16 rounding of Y (the bf16 stage bound)
TOL_Z_FP8 = 8e-2        # E4M3 operands: 3.7e-2 without shields, 6.5e-2 with 5 % shields at 10 x (storage-format study)


def f64(t):
    return t.detach().to(torch.float64).cpu().numpy()


def decode_e4m3(codes: np.ndarray) -> np.ndarray:
    """Values of E4M3 codes from the format's definition: 1 sign bit, 4 exponent bits (bias 7), 3 fraction bits,
    exponent field 0 = subnormal (no implicit one)."""
    c = codes.astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e, m = (c >> 3) & 0xF, c & 7
    return sign * np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e - 7.0))


def expected_quantisation(X: np.ndarray, axis: int):
    """(scale, values on the E4M3 grid) as the kernels decide them: max / 448 and x * (448 / max) in float32, then the
    oracle's rounding of that float32 number."""
    X32 = X.astype(np.float32)
    amax = np.max(np.abs(X32), axis=axis, keepdims=True)
    inv = np.where(amax > 0, np.float32(448.0) / amax, np.float32(1.0)).astype(np.float32)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    t = (X32 * inv).astype(np.float32)
    return scale, prec.round_to_e4m3(t.astype(np.float64))


@pytest.fixture()
def ctx():
    c = g.gelo_create(0, 0xF8, allow_batch_reuse=False)
    yield c
    g.gelo_destroy(c)


def test_rounding_of_every_float_between_grid_points(ctx):
    """The float -> E4M3 rounding itself, away from any scaling: rows whose maximum is exactly 448 leave values
    untouched (scale 1), so codes can be compared with the oracle's rounding of the very same numbers - all E4M3
    grid points, their midpoints (ties), neighbours of the midpoints, subnormals, and random values."""
    grid = decode_e4m3(np.arange(0, 0x7F, dtype=np.uint8))                     # 0 .. 448
    mids = (grid[1:] + grid[:-1]) / 2
    vals = np.concatenate([grid, mids, np.nextafter(mids.astype(np.float32), np.float32(0)).astype(np.float64),
                           np.nextafter(mids.astype(np.float32), np.float32(1e9)).astype(np.float64),
                           np.random.default_rng(0).uniform(0, 448, 3000), np.random.default_rng(1).uniform(0, 0.05, 500)])
    vals = torch.tensor(vals, dtype=torch.float32).to(torch.bfloat16).double().numpy()   # what bf16 can carry
    vals = np.concatenate([vals, -vals])
    d = 4096
    rows = -(-len(vals) // (d - 1))
    X = np.zeros((rows, d))
    X[:, 0] = 448.0                                                            # the row maximum: scale exactly 1
    X[:, 1:].reshape(-1)[:len(vals)] = vals
    U = torch.from_numpy(X).to(torch.bfloat16).cuda()
    codes, scales = g.gelo_debug_quantize_rows_fp8(ctx, U)
    torch.cuda.synchronize()
    assert np.all(scales.cpu().numpy() == 1.0)
    assert np.array_equal(decode_e4m3(codes.cpu().numpy()), prec.round_to_e4m3(f64(U)))


@pytest.mark.parametrize("n,d", [(1, 128), (70, 256), (300, 4096)])
def test_row_codes_are_bit_exact(ctx, n, d):
    H = wl.make_hidden(n, d, 3 + n, 8 if d >= 256 else 0)
    H[n // 2] = 0.0                                                            # an all-zero row: scale 1, codes 0
    U = torch.from_numpy(H).to(torch.bfloat16).cuda()
    codes, scales = g.gelo_debug_quantize_rows_fp8(ctx, U)
    torch.cuda.synchronize()
    scale_ref, val_ref = expected_quantisation(f64(U), axis=1)
    assert np.array_equal(scales.cpu().numpy(), scale_ref[:, 0])
    assert np.array_equal(decode_e4m3(codes.cpu().numpy()), val_ref)


@pytest.mark.parametrize("d,p", [(128, 8), (256, 200), (4096, 1544)])
def test_weight_codes_are_bit_exact(ctx, d, p):
    W = torch.from_numpy(wl.make_weight(d, p, d + p)).to(torch.bfloat16).cuda()
    Wq = g.gelo_prepare_weight_fp8(ctx, W)
    torch.cuda.synchronize()
    raw = Wq.cpu().numpy()
    codes = raw[:p * d].reshape(p, d)                                          # the transpose: row j = column j of W
    off = (p * d + 255) // 256 * 256
    scales = raw[off:off + 4 * p].view(np.float32)
    scale_ref, val_ref = expected_quantisation(f64(W), axis=0)
    assert np.array_equal(scales, scale_ref[0])
    assert np.array_equal(decode_e4m3(codes), val_ref.T)


@pytest.mark.parametrize("n,d,p", [(1, 128, 8), (130, 256, 264), (700, 1024, 776), (2150, 4096, 12288)])
def test_projection_against_the_decoded_operands(ctx, n, d, p):
    """Y = (decoded U codes * row scales) (decoded W codes * column scales) in float64, several tiles with ragged
    tails in both directions, and the full-size projection of the prefill workload."""
    rng = np.random.default_rng(n + p)
    U = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32) * 3).to(torch.bfloat16).cuda()
    W = torch.from_numpy(wl.make_weight(d, p, 9)).to(torch.bfloat16).cuda()
    Wq = g.gelo_prepare_weight_fp8(ctx, W)
    parent = torch.full((n, p + 8), 3.0, dtype=torch.bfloat16, device="cuda")
    Y = parent[:, :p]
    g.gelo_project_fp8(ctx, U, Wq, p, Y)
    torch.cuda.synchronize()
    su, vu = expected_quantisation(f64(U), axis=1)
    sw, vw = expected_quantisation(f64(W), axis=0)
    if n * d * p <= 2e10:
        ref = (vu * su.astype(np.float64)) @ (vw * sw.astype(np.float64))
        assert o.rel_frobenius(f64(Y), ref) < TOL_Y
    else:       # full size: the float64 product on the GPU, operands as decoded above
        ref = torch.from_numpy(vu * su.astype(np.float64)).cuda() @ torch.from_numpy(vw * sw.astype(np.float64)).cuda()
        assert ((Y.double() - ref).norm() / ref.norm()).item() < TOL_Y
    assert torch.all(parent[:, p:] == 3.0)
    # and against the unquantised product: the format's own error, per-row / per-column scaled E4M3
    plain = (U.double() @ W.double())
    err = ((Y.double() - plain).norm() / plain.norm()).item()
    if n * p >= 1000:
        assert 1e-2 < err < 6e-2, err


def test_chain_with_the_8_bit_projection(ctx):
    """mix (bf16) -> project in FP8 -> unmix (bf16) on the prefill workload, orthogonal A with 5 % shields at 10 x:
    Z against H W inside the bound of the storage-format study, and the error the oracle's own model of the
    format gives (exact accumulation, operands rounded) within a third of what the GPU shows."""
    w = wl.WORKLOADS["llama7b_bf16_prefill"]
    H32, W32 = wl.make_inputs(w)
    H = torch.from_numpy(H32).to(torch.bfloat16).cuda()
    W = torch.from_numpy(W32).to(torch.bfloat16).cuda()
    Wq = g.gelo_prepare_weight_fp8(ctx, W)
    m = g.gelo_sample_mixing(ctx, w.kind, w.n_data, w.k_shield, w.d, g.GELO_BF16, 0.0, 1, batch_id=1)
    U = torch.empty((w.n, w.d), dtype=torch.bfloat16, device="cuda")
    Y = torch.empty((w.n, w.p), dtype=torch.bfloat16, device="cuda")
    Z = torch.empty((w.n_data, w.p), dtype=torch.bfloat16, device="cuda")
    g.gelo_mix(ctx, m, H, U)
    g.gelo_project_fp8(ctx, U, Wq, w.p, Y)
    g.gelo_unmix(ctx, m, Y, Z)
    torch.cuda.synchronize()
    g.gelo_mixing_free(ctx, m)
    plain = H.double() @ W.double()
    err = ((Z.double() - plain).norm() / plain.norm()).item()
    print("FP8 projection inside the chain: rel Frobenius error of Z", err)
    assert err < TOL_Z_FP8
    # the model: per-operand E4M3 error e; Z sees e from W and e * ||[H;S]|| / ||H|| * sqrt(n_data / n) from U
    assert err > 2e-2


def test_argument_checks(ctx):
    U = torch.zeros((16, 192), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((192, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(g.GeloError) as e:
        g.gelo_prepare_weight_fp8(ctx, W)                                      # d = 192 is not a multiple of 128
    assert g.STATUS_NAMES[e.value.status] == "GELO_ESHAPE"
    W2 = torch.zeros((256, 64), dtype=torch.bfloat16, device="cuda")
    Wq = g.gelo_prepare_weight_fp8(ctx, W2)
    with pytest.raises(g.GeloError):
        g.gelo_project_fp8(ctx, U, Wq, 64, torch.zeros((16, 64), dtype=torch.bfloat16, device="cuda"))   # U has d = 192
