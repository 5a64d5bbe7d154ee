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
    assert lib.gelo_mix(ctx, m, null, 64, 10.0, 0, P(base), 64, s) == 1
    assert lib.gelo_mix(ctx, m, P(base + 4), 64, 10.0, 0, P(base), 64, s) == 4
    assert lib.gelo_mix(ctx, m, P(base), 56, 10.0, 0, P(base), 64, s) == 1
    assert lib.gelo_mix(ctx, m, P(base), 68, 10.0, 0, P(base), 64, s) == 4
    assert lib.gelo_project(ctx, 0, 16, 64, 60, P(base), 64, P(base), 64, P(base), 64, s) == 4
    assert lib.gelo_project(ctx, 0, 0, 64, 64, P(base), 64, P(base), 64, P(base), 64, s) == 1
    assert lib.gelo_project(ctx, 3, 16, 64, 64, P(base), 64, P(base), 64, P(base), 64, s) == 1
    assert lib.gelo_unmix(ctx, m, 64, P(base), 64, P(base), 64, s) == 9        # not mixed yet
    assert lib.gelo_unmix(ctx, m, 12, P(base), 64, P(base), 64, s) == 4
    assert lib.gelo_mixing_export(ctx, null, null, null, null, None, None, s) == 1
    g.gelo_mixing_free(ctx, m)
    # a mixing object of another context is refused
    c2 = g.gelo_create(0, 2)
    m2 = g.gelo_sample_mixing(c2, g.GELO_ORTHOGONAL, 16, 0, 64, g.GELO_F32, batch_id=1)
    assert lib.gelo_mix(ctx, m2, P(base), 64, 10.0, 0, P(base), 64, s) == 1
    g.gelo_mixing_free(c2, m2)
    g.gelo_destroy(c2)


def test_condition_budget_exhausted(ctx):
    # kappa <= 1.5 never happens for a Gaussian draw: every attempt is rejected, status ECOND
    assert status_of(g.gelo_sample_mixing, ctx, g.GELO_GAUSSIAN, 64, 0, 64, g.GELO_F32, 1.5, 3, 30) == "GELO_ECOND"
    # the failed call consumed nothing: the batch id can still be used
    m = g.gelo_sample_mixing(ctx, g.GELO_GAUSSIAN, 64, 0, 64, g.GELO_F32, 1e6, 3, 30)
    g.gelo_mixing_free(ctx, m)
