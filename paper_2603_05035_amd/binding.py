"""ctypes binding of libgelo.so: the same entry points as include/gelo.h, taking torch
tensors for device memory.  Argument marshalling only: every step runs in the HIP kernels.
There is no fallback: if the shared library is missing or the tensors are not on a GPU,
the calls raise."""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, byref, c_char_p, c_double, c_float, c_int, c_int64, c_uint32, c_uint64,
                    c_void_p)

import torch

GELO_F32, GELO_BF16 = 0, 1
GELO_ORTHOGONAL, GELO_GAUSSIAN, GELO_CONDITIONED, GELO_STRUCTURED, GELO_BLOCK_ORTHOGONAL, GELO_REFLECTOR_PRODUCT = 0, 1, 2, 3, 4, 5
GELO_NORM_MEDIAN, GELO_NORM_MEAN = 0, 1
GELO_OK = 0
STATUS_NAMES = ["GELO_OK", "GELO_EINVAL", "GELO_ESHAPE", "GELO_EDTYPE", "GELO_EALIGN", "GELO_ENOMEM",
                "GELO_ECOND", "GELO_ESINGULAR", "GELO_EREUSE", "GELO_ESTATE", "GELO_EHIP"]
GELO_MAX_N = 5120
GELO_BATCH_WINDOW = 4096
GELO_STATIC_MAX_N = 128
GELO_MAX_BATCH_DRAW = 48
GELO_STATIC_SCRATCH_BYTES = 16 << 20

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libgelo.so")

# name -> (restype, argtypes); mirrors include/gelo.h one to one
SIGNATURES = {
    "gelo_create": (c_int, [POINTER(c_void_p), c_int, c_uint64, c_int]),
    "gelo_destroy": (c_int, [c_void_p]),
    "gelo_last_error": (c_char_p, [c_void_p]),
    "gelo_status_string": (c_char_p, [c_int]),
    "gelo_sample_mixing": (c_int, [c_void_p, c_int, c_int, c_int, c_int, c_int, c_double, c_int, c_uint64,
                                   POINTER(c_void_p), c_void_p]),
    "gelo_set_batch_floor": (c_int, [c_void_p, c_uint64]),
    "gelo_get_batch_floor": (c_int, [c_void_p, POINTER(c_uint64)]),
    "gelo_reserve": (c_int, [c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_int]),
    "gelo_sample_mixing_batch": (c_int, [c_void_p, c_int, c_int, c_int, c_int, c_int, c_uint64, c_int, POINTER(c_void_p), c_void_p]),
    "gelo_chain": (c_int, [c_void_p, c_void_p, c_int, c_int, c_void_p, c_void_p, c_float, c_int, c_void_p, c_void_p, c_void_p,
                           c_void_p]),
    "gelo_mix": (c_int, [c_void_p, c_void_p, c_int, c_void_p, c_int64, c_float, c_int, c_void_p, c_int64, c_void_p]),
    "gelo_project": (c_int, [c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_int64, c_void_p, c_int64,
                             c_void_p, c_int64, c_void_p]),
    "gelo_unmix": (c_int, [c_void_p, c_void_p, c_int, c_int, c_void_p, c_int64, c_void_p, c_int64, c_void_p]),
    "gelo_mixing_free": (c_int, [c_void_p, c_void_p]),
    "gelo_mixing_info": (c_int, [c_void_p, c_void_p, POINTER(c_int), POINTER(c_int), POINTER(c_int), POINTER(c_int),
                                 POINTER(c_int)]),
    "gelo_qkv_forward_static": (c_int, [c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_float,
                                        c_int, c_uint64, c_void_p, c_void_p, c_void_p, c_void_p]),
    "gelo_fp8_weight_bytes": (c_int, [c_int, c_int, POINTER(ctypes.c_size_t)]),
    "gelo_prepare_weight_fp8": (c_int, [c_void_p, c_int, c_int, c_void_p, c_int64, c_void_p, c_void_p]),
    "gelo_project_fp8": (c_int, [c_void_p, c_int, c_int, c_int, c_void_p, c_int64, c_void_p, c_void_p, c_int64, c_void_p]),
    "gelo_debug_quantize_rows_fp8": (c_int, [c_void_p, c_int, c_int, c_void_p, c_int64, c_void_p, c_void_p, c_void_p]),
    "gelo_measure_matrix_rate": (c_int, [c_void_p, c_int, c_int, c_int, POINTER(c_double), POINTER(c_double), c_void_p]),
    "gelo_debug_philox_words": (c_int, [c_void_p, c_uint32, c_uint32, c_uint64, c_uint32, c_uint32, c_void_p, c_void_p]),
    "gelo_mixing_export_table": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p]),
    "gelo_qkv_forward": (c_int, [c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_float,
                                 c_int, c_double, c_int, c_uint64, c_void_p, c_void_p, c_void_p, c_void_p]),
    "gelo_mixing_export": (c_int, [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, POINTER(c_int),
                                   POINTER(c_float), c_void_p]),
}

_lib = None


class GeloError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {message}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Loads libgelo.so (built in-tree by `build.py`); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_05035_amd.build` "
                               "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (restype, argtypes) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = restype
            fn.argtypes = argtypes
        _lib = lib
    return _lib


def _check(ctx, status: int):
    if status != GELO_OK:
        msg = load_library().gelo_last_error(ctx) if ctx else b""
        raise GeloError(status, (msg or b"").decode())


def _stream(stream) -> c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return GELO_F32
    if t.dtype == torch.bfloat16:
        return GELO_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _matrix(t: torch.Tensor, name: str):
    """(pointer, leading dimension) of a 2-D row-major device tensor."""
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be a row-major 2-D tensor")
    return c_void_p(t.data_ptr()), int(t.stride(0)) if t.shape[0] > 1 else int(max(t.stride(0), t.shape[1]))


def gelo_create(device: int = 0, seed: int = 0, allow_batch_reuse: bool = False) -> c_void_p:
    ctx = c_void_p()
    st = load_library().gelo_create(byref(ctx), device, seed, int(allow_batch_reuse))
    if st != GELO_OK:
        raise GeloError(st, "gelo_create failed")
    return ctx


def gelo_destroy(ctx) -> None:
    _check(None, load_library().gelo_destroy(ctx))


def gelo_sample_mixing(ctx, kind: int, n_data: int, k_shield: int, d: int, dtype: int, cond_max: float = 1e3,
                       max_attempts: int = 64, batch_id: int = 0, stream=None) -> c_void_p:
    mixing = c_void_p()
    _check(ctx, load_library().gelo_sample_mixing(ctx, kind, n_data, k_shield, d, dtype, cond_max, max_attempts,
                                                  batch_id, byref(mixing), _stream(stream)))
    return mixing


def gelo_sample_mixing_batch(ctx, kind: int, n_data: int, k_shield: int, d: int, dtype: int, first_batch_id: int,
                             count: int, stream=None):
    """`count` mixing objects for consecutive batch ids from one launch (decode-shaped batches)."""
    arr = (c_void_p * count)()
    _check(ctx, load_library().gelo_sample_mixing_batch(ctx, kind, n_data, k_shield, d, dtype, first_batch_id, count,
                                                        arr, _stream(stream)))
    return [c_void_p(arr[i]) for i in range(count)]


def gelo_chain(ctx, mixing, H: torch.Tensor, W: torch.Tensor, Z: torch.Tensor, U: torch.Tensor, Y: torch.Tensor,
               shield_scale: float = 10.0, stat: int = GELO_NORM_MEDIAN, stream=None) -> torch.Tensor:
    """mix + project + unmix for a mixing object drawn earlier, one call."""
    for name, t in (("H", H), ("W", W), ("Z", Z), ("U", U), ("Y", Y)):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != H.dtype:
            raise ValueError(f"{name} must be a contiguous GPU tensor of H's dtype")
    p = W.shape[1]
    if W.shape[0] != H.shape[1] or Y.shape[1] != p or Z.shape[1] != p:
        raise GeloError(2, "W, Y and Z do not fit together")
    _check_against_mixing(ctx, mixing, (("H", H, "n_data", "d"), ("U", U, "n", "d"), ("Y", Y, "n", None), ("Z", Z, "n_data", None)))
    _check(ctx, load_library().gelo_chain(ctx, mixing, _dtype_code(H), p, c_void_p(H.data_ptr()), c_void_p(W.data_ptr()),
                                          shield_scale, stat, c_void_p(Z.data_ptr()), c_void_p(U.data_ptr()),
                                          c_void_p(Y.data_ptr()), _stream(stream)))
    return Z


def gelo_mixing_info(ctx, mixing):
    """(n_data, k_shield, d, dtype code, kind) the mixing object was drawn for."""
    v = [c_int() for _ in range(5)]
    _check(ctx, load_library().gelo_mixing_info(ctx, mixing, *[byref(x) for x in v]))
    return tuple(x.value for x in v)


def _check_against_mixing(ctx, mixing, tensors):
    """`tensors`: (name, tensor, rows expected ('n' or 'n_data'), width expected ('d' or None)).  The C ABI
    sees raw pointers; here the tensors carry shapes and types, so every mismatch that would make a kernel
    leave the caller's buffers is refused before the call."""
    n_data, k, d, code, _ = gelo_mixing_info(ctx, mixing)
    rows = {"n": n_data + k, "n_data": n_data}
    for name, t, r, w in tensors:
        if _dtype_code(t) != code:
            raise GeloError(3, f"{name} is {t.dtype} but the mixing object was drawn for {'bf16' if code == GELO_BF16 else 'f32'}")
        if t.dim() != 2 or t.shape[0] != rows[r] or (w == "d" and t.shape[1] != d):
            raise GeloError(2, f"{name} has shape {tuple(t.shape)}; this mixing object needs {rows[r]} rows"
                               + (f" of width {d}" if w == "d" else ""))


def gelo_mix(ctx, mixing, H: torch.Tensor, U: torch.Tensor, shield_scale: float = 10.0,
             stat: int = GELO_NORM_MEDIAN, stream=None) -> torch.Tensor:
    hp, ldh = _matrix(H, "H")
    up, ldu = _matrix(U, "U")
    _check_against_mixing(ctx, mixing, (("H", H, "n_data", "d"), ("U", U, "n", "d")))
    _check(ctx, load_library().gelo_mix(ctx, mixing, _dtype_code(H), hp, ldh, shield_scale, stat, up, ldu, _stream(stream)))
    return U


def gelo_project(ctx, U: torch.Tensor, W: torch.Tensor, Y: torch.Tensor, stream=None) -> torch.Tensor:
    up, ldu = _matrix(U, "U")
    wp, ldw = _matrix(W, "W")
    yp, ldy = _matrix(Y, "Y")
    n, d = U.shape
    p = W.shape[1]
    if W.shape[0] != d or tuple(Y.shape) != (n, p) or not (U.dtype == W.dtype == Y.dtype):
        raise ValueError("shape or dtype mismatch in gelo_project")
    _check(ctx, load_library().gelo_project(ctx, _dtype_code(U), n, d, p, up, ldu, wp, ldw, yp, ldy, _stream(stream)))
    return Y


def gelo_unmix(ctx, mixing, Y: torch.Tensor, Z: torch.Tensor, stream=None) -> torch.Tensor:
    yp, ldy = _matrix(Y, "Y")
    zp, ldz = _matrix(Z, "Z")
    if Y.shape[1] != Z.shape[1]:
        raise GeloError(2, "Y and Z must have the same width")
    _check_against_mixing(ctx, mixing, (("Y", Y, "n", None), ("Z", Z, "n_data", None)))
    _check(ctx, load_library().gelo_unmix(ctx, mixing, _dtype_code(Y), Y.shape[1], yp, ldy, zp, ldz, _stream(stream)))
    return Z


def gelo_mixing_free(ctx, mixing) -> None:
    _check(ctx, load_library().gelo_mixing_free(ctx, mixing))


def gelo_qkv_forward(ctx, kind: int, H: torch.Tensor, W: torch.Tensor, Z: torch.Tensor, k_shield: int = 0,
                     shield_scale: float = 10.0, stat: int = GELO_NORM_MEDIAN, cond_max: float = 1e3,
                     max_attempts: int = 64, batch_id: int = 0, U: torch.Tensor | None = None,
                     Y: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    for name, t in (("H", H), ("W", W), ("Z", Z), ("U", U), ("Y", Y)):
        if t is not None and (not t.is_cuda or not t.is_contiguous() or t.dtype != H.dtype):
            raise ValueError(f"{name} must be a contiguous GPU tensor of H's dtype")
    n_data, d = H.shape
    p = W.shape[1]
    n = n_data + k_shield
    if W.shape[0] != d or tuple(Z.shape) != (n_data, p):
        raise ValueError("shape mismatch in gelo_qkv_forward")
    if (U is not None and tuple(U.shape) != (n, d)) or (Y is not None and tuple(Y.shape) != (n, p)):
        raise ValueError("U must be n x d and Y n x p")
    _check(ctx, load_library().gelo_qkv_forward(
        ctx, kind, _dtype_code(H), n_data, k_shield, d, p, c_void_p(H.data_ptr()), c_void_p(W.data_ptr()),
        shield_scale, stat, cond_max, max_attempts, batch_id, c_void_p(Z.data_ptr()),
        c_void_p(U.data_ptr()) if U is not None else None, c_void_p(Y.data_ptr()) if Y is not None else None,
        _stream(stream)))
    return Z


def gelo_qkv_forward_static(ctx, kind: int, H: torch.Tensor, W: torch.Tensor, Z: torch.Tensor, U: torch.Tensor,
                            Y: torch.Tensor, k_shield: int = 0, shield_scale: float = 10.0,
                            stat: int = GELO_NORM_MEDIAN, batch_id: int = 0, stream=None) -> torch.Tensor:
    """The chain for one decode-shaped batch through the entry point that allocates nothing."""
    for name, t in (("H", H), ("W", W), ("Z", Z), ("U", U), ("Y", Y)):
        if not t.is_cuda or not t.is_contiguous() or t.dtype != H.dtype:
            raise ValueError(f"{name} must be a contiguous GPU tensor of H's dtype")
    n_data, d = H.shape
    p = W.shape[1]
    n = n_data + k_shield
    if W.shape[0] != d or tuple(Z.shape) != (n_data, p) or tuple(U.shape) != (n, d) or tuple(Y.shape) != (n, p):
        raise ValueError("shape mismatch in gelo_qkv_forward_static")
    _check(ctx, load_library().gelo_qkv_forward_static(
        ctx, kind, _dtype_code(H), n_data, k_shield, d, p, c_void_p(H.data_ptr()), c_void_p(W.data_ptr()),
        shield_scale, stat, batch_id, c_void_p(Z.data_ptr()), c_void_p(U.data_ptr()), c_void_p(Y.data_ptr()),
        _stream(stream)))
    return Z


def gelo_reserve(ctx, kind: int, dtype: int, n_data: int, k_shield: int, d: int, p: int = 0,
                 max_attempts: int = 64, mixings: int = 1) -> None:
    _check(ctx, load_library().gelo_reserve(ctx, kind, dtype, n_data, k_shield, d, p, max_attempts, mixings))


def gelo_set_batch_floor(ctx, first_unused: int) -> None:
    _check(ctx, load_library().gelo_set_batch_floor(ctx, first_unused))


def gelo_get_batch_floor(ctx) -> int:
    v = c_uint64()
    _check(ctx, load_library().gelo_get_batch_floor(ctx, byref(v)))
    return v.value


def gelo_fp8_weight_bytes(d: int, p: int) -> int:
    v = ctypes.c_size_t()
    st = load_library().gelo_fp8_weight_bytes(d, p, byref(v))
    if st != GELO_OK:
        raise GeloError(st, "gelo_fp8_weight_bytes")
    return v.value


def gelo_prepare_weight_fp8(ctx, W: torch.Tensor, stream=None) -> torch.Tensor:
    """The FP8 form of a bf16 weight (d x p): a uint8 device buffer holding the codes of W^T and the column scales."""
    if W.dtype != torch.bfloat16:
        raise TypeError("the 8-bit projection takes a bf16 weight")
    wp, ldw = _matrix(W, "W")
    d, p = W.shape
    Wq = torch.empty(gelo_fp8_weight_bytes(d, p), dtype=torch.uint8, device="cuda")
    _check(ctx, load_library().gelo_prepare_weight_fp8(ctx, d, p, wp, ldw, c_void_p(Wq.data_ptr()), _stream(stream)))
    return Wq


def gelo_project_fp8(ctx, U: torch.Tensor, Wq: torch.Tensor, p: int, Y: torch.Tensor, stream=None) -> torch.Tensor:
    up, ldu = _matrix(U, "U")
    yp, ldy = _matrix(Y, "Y")
    n, d = U.shape
    if U.dtype != torch.bfloat16 or Y.dtype != torch.bfloat16 or tuple(Y.shape) != (n, p):
        raise ValueError("U and Y must be bf16, Y n x p")
    if Wq.dtype != torch.uint8 or Wq.numel() != gelo_fp8_weight_bytes(d, p):
        raise GeloError(2, "Wq is not the prepared form of a d x p weight")
    _check(ctx, load_library().gelo_project_fp8(ctx, n, d, p, up, ldu, c_void_p(Wq.data_ptr()), yp, ldy, _stream(stream)))
    return Y


def gelo_debug_quantize_rows_fp8(ctx, U: torch.Tensor, stream=None):
    """Test hook: (codes n x d uint8, scales n float32) of the row quantisation of U."""
    up, ldu = _matrix(U, "U")
    n, d = U.shape
    codes = torch.empty((n, d), dtype=torch.uint8, device="cuda")
    scales = torch.empty((n,), dtype=torch.float32, device="cuda")
    _check(ctx, load_library().gelo_debug_quantize_rows_fp8(ctx, n, d, up, ldu, c_void_p(codes.data_ptr()),
                                                            c_void_p(scales.data_ptr()), _stream(stream)))
    return codes, scales


def gelo_measure_matrix_rate(ctx, fp8: bool, iters: int = 2000, launches: int = 5, stream=None):
    """(seconds per launch, FLOP per launch) of the matrix-instruction-only kernel; waits for it."""
    sec, flop = c_double(0.0), c_double(0.0)
    _check(ctx, load_library().gelo_measure_matrix_rate(ctx, 1 if fp8 else 0, iters, launches, byref(sec), byref(flop),
                                                        _stream(stream)))
    return sec.value, flop.value


def gelo_debug_philox_words(ctx, stream_id: int, attempt: int, batch_id: int, first_block: int, blocks: int,
                            stream=None) -> torch.Tensor:
    """Test hook: blocks x 4 raw Philox words (int32 tensor holding the uint32 bit patterns)."""
    words = torch.empty((blocks, 4), dtype=torch.int32, device="cuda")
    _check(ctx, load_library().gelo_debug_philox_words(ctx, stream_id, attempt, batch_id, first_block, blocks,
                                                       c_void_p(words.data_ptr()), _stream(stream)))
    return words


def gelo_mixing_export_table(ctx, mixing, n: int, rounds: int = 3, stream=None) -> torch.Tensor:
    """Test hook: the (rounds + 1) x n table words of a structured mixing object (int32 bit patterns)."""
    table = torch.empty((rounds + 1, n), dtype=torch.int32, device="cuda")
    _check(ctx, load_library().gelo_mixing_export_table(ctx, mixing, c_void_p(table.data_ptr()), _stream(stream)))
    return table


def gelo_mixing_export(ctx, mixing, n: int, k_shield: int, d: int, want_shields: bool = True,
                       want_matrices: bool = True, stream=None):
    """Test hook: (A, A_inv, S, attempt, kappa) with A, A_inv, S float32 GPU tensors (None where not asked for)."""
    A = torch.empty((n, n), dtype=torch.float32, device="cuda") if want_matrices else None
    A_inv = torch.empty((n, n), dtype=torch.float32, device="cuda") if want_matrices else None
    S = torch.empty((k_shield, d), dtype=torch.float32, device="cuda") if (want_shields and k_shield > 0) else None
    attempt, kappa = c_int(-1), c_float(0.0)
    _check(ctx, load_library().gelo_mixing_export(
        ctx, mixing, c_void_p(A.data_ptr()) if A is not None else None,
        c_void_p(A_inv.data_ptr()) if A_inv is not None else None,
        c_void_p(S.data_ptr()) if S is not None else None, byref(attempt), byref(kappa), _stream(stream)))
    return A, A_inv, S, attempt.value, kappa.value
