"""Error behaviour of the C ABI: argument errors come back synchronously as status codes with
a message, nothing is enqueued, and no kernel ever sees an invalid shape.  (A context needs a
device, so these need a GPU; none of them launches a kernel that could fault.)"""
import pytest
import torch

from paper_2603_05035_amd import binding as g

pytestmark = pytest.mark.gpu


@pytest.fixture()
def ctx():
    c = g.gelo_create(0, 1, allow_batch_reuse=False)
    yield c
    g.gelo_destroy(c)


def status_of(fn, *a, **kw):
    with pytest.raises(g.GeloError) as e:
        fn(*a, **kw)
    return g.STATUS_NAMES[e.value.status]


def test_create_rejects_bad_device():
    with pytest.raises(g.GeloError):
        g.gelo_create(99, 0)


def test_sample_argument_checks(ctx):
    S = g.gelo_sample_mixing
    assert status_of(S, ctx, 7, 16, 0, 64, g.GELO_F32) == "GELO_EINVAL"
    assert status_of(S, ctx, g.GELO_ORTHOGONAL, 0, 0, 64, g.GELO_F32) == "GELO_EINVAL"
    assert status_of(S, ctx, g.GELO_ORTHOGONAL, 16, -1, 64, g.GELO_F32) == "GELO_EINVAL"
    assert status_of(S, ctx, g.GELO_ORTHOGONAL, 16, 0, 60, g.GELO_F32) == "GELO_EALIGN"
    assert status_of(S, ctx, g.GELO_ORTHOGONAL, 16, 0, 64, 5) == "GELO_EINVAL"
    assert status_of(S, ctx, g.GELO_ORTHOGONAL, g.GELO_MAX_N, 1, 64, g.GELO_F32) == "GELO_ESHAPE"
    assert status_of(S, ctx, g.GELO_GAUSSIAN, 16, 0, 64, g.GELO_F32, 0.5, 4) == "GELO_EINVAL"
    assert status_of(S, ctx, g.GELO_GAUSSIAN, 16, 0, 64, g.GELO_F32, 1e3, 0) == "GELO_EINVAL"
    assert status_of(S, ctx, g.GELO_GAUSSIAN, 16, 0, 64, g.GELO_F32, 1e3, 256) == "GELO_EINVAL"
    assert b"max_attempts" in g.load_library().gelo_last_error(ctx)


def test_batch_id_is_never_reused(ctx):
    m = g.gelo_sample_mixing(ctx, g.GELO_ORTHOGONAL, 16, 0, 64, g.GELO_F32, batch_id=3)
    assert status_of(g.gelo_sample_mixing, ctx, g.GELO_ORTHOGONAL, 16, 0, 64, g.GELO_F32, batch_id=3) == "GELO_EREUSE"
    g.gelo_mixing_free(ctx, m)
    assert status_of(g.gelo_sample_mixing, ctx, g.GELO_ORTHOGONAL, 16, 0, 64, g.GELO_F32, batch_id=3) == "GELO_EREUSE"
    m = g.gelo_sample_mixing(ctx, g.GELO_ORTHOGONAL, 16, 0, 64, g.GELO_F32, batch_id=4)
    g.gelo_mixing_free(ctx, m)


def test_mixing_object_life_cycle(ctx):
    H = torch.randn(16, 64, device="cuda")
    W = torch.randn(64, 72, device="cuda")
    U = torch.empty(18, 64, device="cuda")
    Y = torch.empty(18, 72, device="cuda")
    Z = torch.empty(16, 72, device="cuda")
    m = g.gelo_sample_mixing(ctx, g.GELO_ORTHOGONAL, 16, 2, 64, g.GELO_F32, batch_id=10)
    assert status_of(g.gelo_unmix, ctx, m, Y, Z) == "GELO_ESTATE"           # unmix before mix
    assert status_of(g.gelo_mix, ctx, m, H, U, shield_scale=0.0) == "GELO_EINVAL"
    assert status_of(g.gelo_mix, ctx, m, H, U, stat=9) == "GELO_EINVAL"
    g.gelo_mix(ctx, m, H, U)
    assert status_of(g.gelo_mix, ctx, m, H, U) == "GELO_EREUSE"             # one batch per A
    g.gelo_project(ctx, U, W, Y)
    g.gelo_unmix(ctx, m, Y, Z)
    assert status_of(g.gelo_unmix, ctx, m, Y, Z) == "GELO_EREUSE"
    g.gelo_mixing_free(ctx, m)
    assert status_of(g.gelo_mixing_free, ctx, m) == "GELO_EINVAL"           # double free
    assert status_of(g.gelo_mix, ctx, m, H, U) == "GELO_EINVAL"             # use after free
    torch.cuda.synchronize()
    assert torch.allclose(Z, H @ W, rtol=1e-3, atol=1e-3)


def test_alignment_and_shape_checks(ctx):
    lib = g.load_library()
    import ctypes
    m = g.gelo_sample_mixing(ctx, g.GELO_ORTHOGONAL, 16, 0, 64, g.GELO_F32, batch_id=20)
    buf = torch.zeros(64 * 80 + 8, device="cuda")
    base = buf.data_ptr()
    null = ctypes.c_void_p(None)
    s = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    P = ctypes.c_void_p
    # NULL, misaligned pointer, short and odd leading dimensions
    assert lib.gelo_mix(ctx, m, 0, null, 64, 10.0, 0, P(base), 64, s) == 1
    assert lib.gelo_mix(ctx, m, 0, P(base + 4), 64, 10.0, 0, P(base), 64, s) == 4
    assert lib.gelo_mix(ctx, m, 0, P(base), 56, 10.0, 0, P(base), 64, s) == 1
    assert lib.gelo_mix(ctx, m, 0, P(base), 68, 10.0, 0, P(base), 64, s) == 4
    assert lib.gelo_mix(ctx, m, 1, P(base), 64, 10.0, 0, P(base), 64, s) == 3      # bf16 buffers, float mixing object
    assert lib.gelo_mix(ctx, m, 2, P(base), 64, 10.0, 0, P(base), 64, s) == 1
    assert lib.gelo_unmix(ctx, m, 1, 64, P(base), 64, P(base), 64, s) == 3
    assert lib.gelo_project(ctx, 0, 16, 64, 60, P(base), 64, P(base), 64, P(base), 64, s) == 4
    assert lib.gelo_project(ctx, 0, 0, 64, 64, P(base), 64, P(base), 64, P(base), 64, s) == 1
    assert lib.gelo_project(ctx, 3, 16, 64, 64, P(base), 64, P(base), 64, P(base), 64, s) == 1
    assert lib.gelo_unmix(ctx, m, 0, 64, P(base), 64, P(base), 64, s) == 9        # not mixed yet
    assert lib.gelo_unmix(ctx, m, 0, 12, P(base), 64, P(base), 64, s) == 4
    assert lib.gelo_mixing_export(ctx, null, null, null, null, None, None, s) == 1
    g.gelo_mixing_free(ctx, m)
    # a mixing object of another context is refused
    c2 = g.gelo_create(0, 2)
    m2 = g.gelo_sample_mixing(c2, g.GELO_ORTHOGONAL, 16, 0, 64, g.GELO_F32, batch_id=1)
    assert lib.gelo_mix(ctx, m2, 0, P(base), 64, 10.0, 0, P(base), 64, s) == 1
    g.gelo_mixing_free(c2, m2)
    g.gelo_destroy(c2)


def test_dtype_and_shape_mismatch_is_refused_before_any_launch(ctx):
    """A mixing object drawn for float must not meet bf16 buffers (the kernels would run past them), nor
    buffers with too few rows: GELO_EDTYPE / GELO_ESHAPE, nothing enqueued, the object stays usable."""
    m = g.gelo_sample_mixing(ctx, g.GELO_ORTHOGONAL, 16, 2, 64, g.GELO_F32, batch_id=40)
    assert g.gelo_mixing_info(ctx, m) == (16, 2, 64, g.GELO_F32, g.GELO_ORTHOGONAL)
    H = torch.randn(16, 64, device="cuda")
    U = torch.full((18, 64), 5.0, device="cuda")
    Hb, Ub = H.bfloat16(), U.bfloat16()
    assert status_of(g.gelo_mix, ctx, m, Hb, Ub) == "GELO_EDTYPE"
    assert status_of(g.gelo_mix, ctx, m, H, U[:17]) == "GELO_ESHAPE"          # U needs n = 18 rows
    assert status_of(g.gelo_mix, ctx, m, H[:15], U) == "GELO_ESHAPE"
    assert status_of(g.gelo_mix, ctx, m, torch.randn(16, 72, device="cuda"), torch.empty(18, 72, device="cuda")) == "GELO_ESHAPE"
    torch.cuda.synchronize()
    assert torch.all(U == 5.0)                                               # nothing ran
    g.gelo_mix(ctx, m, H, U)
    Y = torch.randn(18, 72, device="cuda")
    Z = torch.full((16, 72), 5.0, device="cuda")
    assert status_of(g.gelo_unmix, ctx, m, Y.bfloat16(), Z.bfloat16()) == "GELO_EDTYPE"
    assert status_of(g.gelo_unmix, ctx, m, Y[:17], Z) == "GELO_ESHAPE"
    assert status_of(g.gelo_unmix, ctx, m, Y, Z[:15]) == "GELO_ESHAPE"
    torch.cuda.synchronize()
    assert torch.all(Z == 5.0)
    g.gelo_unmix(ctx, m, Y, Z)
    g.gelo_mixing_free(ctx, m)
    torch.cuda.synchronize()


def test_batch_window_and_floor(ctx):
    """The record of used batch ids is a high-water mark plus a window of GELO_BATCH_WINDOW ids below it:
    ids above are new, ids inside are remembered one by one, ids further back count as used.  The floor
    lets a restarted process resume from (seed, first unused id)."""
    def draw(b, c=ctx):
        m = g.gelo_sample_mixing(c, g.GELO_ORTHOGONAL, 8, 0, 64, g.GELO_F32, batch_id=b)
        g.gelo_mixing_free(c, m)
    W = g.GELO_BATCH_WINDOW
    assert g.gelo_get_batch_floor(ctx) == 0
    draw(10); draw(7); draw(12)
    assert g.gelo_get_batch_floor(ctx) == 13
    for b in (10, 7, 12):
        assert status_of(draw, b) == "GELO_EREUSE"
    draw(8)                                            # inside the window and unused
    draw(12 + W)                                       # the window slides past 12 and everything below it
    assert status_of(draw, 12) == "GELO_EREUSE"
    assert status_of(draw, 8) == "GELO_EREUSE"
    assert status_of(draw, 11) == "GELO_EREUSE"        # never used, but too far back to know
    draw(13)                                           # the oldest id still inside the window, unused
    draw(12 + W + 5 * W)                               # a jump of more than a window forgets nothing it should keep
    assert status_of(draw, 12 + W) == "GELO_EREUSE"
    draw(12 + 5 * W + 1)
    big = (1 << 63) + 12345
    draw(big)
    assert status_of(draw, big) == "GELO_EREUSE"
    assert status_of(draw, (1 << 64) - 1) == "GELO_EINVAL"
    # resume: same seed, floor restored; everything below is refused, the first unused id works
    first_unused = g.gelo_get_batch_floor(ctx)
    assert first_unused == big + 1
    c2 = g.gelo_create(0, 1, allow_batch_reuse=False)
    try:
        g.gelo_set_batch_floor(c2, first_unused)
        assert status_of(draw, big, c2) == "GELO_EREUSE"
        assert status_of(draw, 0, c2) == "GELO_EREUSE"
        draw(first_unused, c2)
        assert status_of(g.gelo_set_batch_floor, c2, 5) == "GELO_EINVAL"
    finally:
        g.gelo_destroy(c2)


def test_reserve_sizes_the_context_ahead(ctx):
    """After gelo_reserve the per-batch calls of that shape find their memory: device memory in use does not
    grow over a chain (U and Y in context workspace) nor over draws held at the same time."""
    nd, k, d, p = 1000, 24, 1024, 2048       # unreserved, this shape would take about 50 MB on first use
    g.gelo_reserve(ctx, g.GELO_ORTHOGONAL, g.GELO_BF16, nd, k, d, p, mixings=2)
    H = torch.randn(nd, d, device="cuda").bfloat16()
    W = (0.02 * torch.randn(d, p, device="cuda")).bfloat16()
    Z = torch.empty(nd, p, device="cuda", dtype=torch.bfloat16)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    g.gelo_qkv_forward(ctx, g.GELO_ORTHOGONAL, H, W, Z, k_shield=k, batch_id=1)
    m1 = g.gelo_sample_mixing(ctx, g.GELO_ORTHOGONAL, nd, k, d, g.GELO_BF16, batch_id=2)
    m2 = g.gelo_sample_mixing(ctx, g.GELO_ORTHOGONAL, nd, k, d, g.GELO_BF16, batch_id=3)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free0 - (4 << 20)        # a little slack for the runtime's own pools
    g.gelo_mixing_free(ctx, m1)
    g.gelo_mixing_free(ctx, m2)
    assert torch.allclose(Z.float(), H.float() @ W.float(), rtol=5e-2, atol=5e-2)
    assert status_of(g.gelo_reserve, ctx, g.GELO_ORTHOGONAL, g.GELO_BF16, g.GELO_MAX_N, 1, d) == "GELO_ESHAPE"


def test_static_entry_point_argument_checks(ctx):
    H = torch.randn(64, 64, device="cuda")
    W = torch.randn(64, 72, device="cuda")
    Z = torch.empty(64, 72, device="cuda")
    S = g.gelo_qkv_forward_static
    def bufs(n, d=64, p=72):
        return torch.empty(n, d, device="cuda"), torch.empty(n, p, device="cuda")
    U, Y = bufs(68)
    assert status_of(S, ctx, g.GELO_GAUSSIAN, H, W, Z, U, Y, k_shield=4, batch_id=1) == "GELO_EINVAL"
    Hbig = torch.randn(g.GELO_STATIC_MAX_N, 64, device="cuda")
    Zbig = torch.empty(g.GELO_STATIC_MAX_N, 72, device="cuda")
    U2, Y2 = bufs(g.GELO_STATIC_MAX_N + 1)
    assert status_of(S, ctx, g.GELO_ORTHOGONAL, Hbig, W, Zbig, U2, Y2, k_shield=1, batch_id=1) == "GELO_ESHAPE"
    # the shield block alone would not fit the static buffer: 64 x 32768 floats and their rows
    d = 32768
    Hw = torch.randn(64, d, device="cuda")
    Ww = torch.randn(d, 8, device="cuda")
    U3, Y3 = torch.empty(128, d, device="cuda"), torch.empty(128, 8, device="cuda")
    assert status_of(S, ctx, g.GELO_ORTHOGONAL, Hw, Ww, torch.empty(64, 8, device="cuda"), U3, Y3, k_shield=64, batch_id=1) == "GELO_ESHAPE"
    assert b"static buffer" in g.load_library().gelo_last_error(ctx)
    # none of the refused calls consumed the batch id
    S(ctx, g.GELO_ORTHOGONAL, H, W, Z, U, Y, k_shield=4, batch_id=1)
    assert status_of(S, ctx, g.GELO_ORTHOGONAL, H, W, Z, U, Y, k_shield=4, batch_id=1) == "GELO_EREUSE"
    torch.cuda.synchronize()
    assert torch.allclose(Z, H @ W, rtol=1e-3, atol=1e-3)


def test_condition_budget_exhausted(ctx):
    # kappa <= 1.5 never happens for a Gaussian draw: every attempt is rejected, status ECOND
    assert status_of(g.gelo_sample_mixing, ctx, g.GELO_GAUSSIAN, 64, 0, 64, g.GELO_F32, 1.5, 3, 30) == "GELO_ECOND"
    # the failed call consumed nothing: the batch id can still be used
    m = g.gelo_sample_mixing(ctx, g.GELO_GAUSSIAN, 64, 0, 64, g.GELO_F32, 1e6, 3, 30)
    g.gelo_mixing_free(ctx, m)


def test_matrix_rate_measurement(ctx):
    """The measurement aid: a plausible rate for both instruction kinds (between a fifth of the published peak and
    the peak itself), the stated operation count, and argument checks."""
    for fp8, peak in ((False, 2.5e15), (True, 5.0e15)):
        sec, flop = g.gelo_measure_matrix_rate(ctx, fp8, iters=500, launches=3)
        assert flop == 2.0 * 32 * 32 * (64 if fp8 else 16) * 32 * 500 * 8 * 256
        assert 0.2 * peak < flop / sec <= 1.02 * peak, (fp8, flop / sec)
    assert status_of(g.gelo_measure_matrix_rate, ctx, False, 0, 3) == "GELO_EINVAL"
    assert status_of(g.gelo_measure_matrix_rate, ctx, False, 10, 0) == "GELO_EINVAL"
