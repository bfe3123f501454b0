"""ctypes binding of include/gptq.h.  Argument marshalling only: each function takes torch tensors
that live on the GPU, checks dtypes / devices, and passes raw device pointers, sizes and the current
HIP stream to the C entry point of the same name."""
from __future__ import annotations

import ctypes
import os
import re

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgptq_mi355.so")
HEADER_PATH = os.path.join(os.path.dirname(_HERE), "include", "gptq.h")

GPTQ_GRID_MINMAX, GPTQ_GRID_TERNARY = 0, 1
_DTYPE = {torch.float16: 0, torch.bfloat16: 1, torch.float32: 2}

_lib = None


class GptqError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"gptq error {code}: {message}")
        self.code = code


def exported_symbols() -> list[str]:
    """Names of the functions include/gptq.h declares."""
    text = open(HEADER_PATH).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gptq_[a-z0-9_]+)\s*\(", text)))


def load_library(path: str | None = None) -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2210_17323_amd.build` "
                                "(or __graft_entry__.build()); there is no CPU fallback")
    L = ctypes.CDLL(path)
    i64, vp, ci, sz, f32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_float
    L.gptq_version.restype = ci
    L.gptq_last_error.restype = ctypes.c_char_p
    L.gptq_hessian_accumulate.argtypes = [vp, i64, vp, ci, i64, i64, i64, vp, sz, vp]
    L.gptq_hessian_accumulate_workspace_bytes.argtypes = [i64, i64, ci]
    L.gptq_hessian_accumulate_workspace_bytes.restype = sz
    L.gptq_hessian_accumulate_launches.argtypes = [i64, i64, ci]
    L.gptq_hessian_accumulate_launches.restype = i64
    L.gptq_hessian_symmetrize.argtypes = [vp, i64, i64, vp]
    L.gptq_hessian_accumulate_token_major.argtypes = [vp, i64, vp, ci, i64, i64, i64, vp, sz, vp]
    L.gptq_hessian_accumulate_token_major_workspace_bytes.argtypes = [i64, i64, ci]
    L.gptq_hessian_accumulate_token_major_workspace_bytes.restype = sz
    L.gptq_damp_cholesky_inverse_workspace_bytes.argtypes = [i64]
    L.gptq_damp_cholesky_inverse_workspace_bytes.restype = sz
    L.gptq_damp_cholesky_inverse.argtypes = [vp, i64, i64, f32, vp, sz, vp, vp]
    L.gptq_damp_cholesky_inverse_noalloc.argtypes = [vp, i64, i64, f32, vp, vp]
    L.gptq_noalloc_max_n.restype = i64
    L.gptq_check_info.argtypes = [vp, ctypes.POINTER(ci), vp]
    L.gptq_quantize_layer_workspace_bytes.argtypes = [i64, i64, ci, i64]
    L.gptq_quantize_layer_workspace_bytes.restype = sz
    L.gptq_quantize_layer.argtypes = [vp, ci, i64, i64, i64, vp, i64, ci, ci, ci, i64, vp, i64, vp, vp, vp, i64, vp, vp, sz, vp]
    L.gptq_damp_cholesky_workspace_bytes.argtypes = [i64]
    L.gptq_damp_cholesky_workspace_bytes.restype = sz
    L.gptq_damp_cholesky.argtypes = [vp, i64, i64, f32, vp, sz, vp, vp]
    L.gptq_quantize_layer_from_factor.argtypes = L.gptq_quantize_layer.argtypes
    L.gptq_quantize_layer_from_factor_supports.argtypes = [i64]
    L.gptq_quantize_layer_from_factor_supports.restype = ci
    L.gptq_trailing_update.argtypes = [vp, i64, vp, i64, vp, i64, i64, i64, i64, vp]
    L.gptq_trailing_update_split.argtypes = [vp, i64, vp, i64, vp, i64, i64, i64, i64, vp, sz, vp]
    L.gptq_trailing_update_split_workspace_bytes.argtypes = [i64, i64]
    L.gptq_trailing_update_split_workspace_bytes.restype = sz
    L.gptq_symmetric_update_split.argtypes = [vp, i64, vp, i64, i64, i64, vp, sz, vp]
    L.gptq_symmetric_update_split_workspace_bytes.argtypes = [i64]
    L.gptq_symmetric_update_split_workspace_bytes.restype = sz
    L.gptq_set_split_min_tiles.argtypes = [ci]
    L.gptq_set_split_min_tiles.restype = ci
    L.gptq_pack.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp]
    L.gptq_unpack.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp]
    L.gptq_dequantize_packed.argtypes = [vp, i64, i64, i64, ci, vp, vp, i64, vp, ci, i64, vp]
    L.gptq_matvec_packed.argtypes = [vp, i64, i64, i64, ci, vp, vp, i64, vp, ci, vp, vp]
    for name in ("gptq_hessian_accumulate", "gptq_hessian_symmetrize", "gptq_damp_cholesky_inverse", "gptq_check_info",
                 "gptq_quantize_layer", "gptq_pack", "gptq_unpack", "gptq_damp_cholesky_inverse_noalloc",
                 "gptq_hessian_accumulate_token_major", "gptq_dequantize_packed", "gptq_matvec_packed",
                 "gptq_trailing_update_split", "gptq_symmetric_update_split", "gptq_release_thread_resources"):
        getattr(L, name).restype = ci
    if path == LIB_PATH:
        _lib = L
    return L


def lib() -> ctypes.CDLL:
    return load_library()


def version() -> int:
    return lib().gptq_version()


def gptq_release_thread_resources() -> None:
    """Destroys the calling thread's helper streams and events on the current device (the next call recreates them)."""
    _check(lib().gptq_release_thread_resources())


def _check(rc: int):
    if rc != 0:
        raise GptqError(rc, lib().gptq_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: torch.Tensor | None) -> int | None:
    return None if t is None else t.data_ptr()


def _dev2d(t: torch.Tensor, name: str, dtypes) -> None:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-D with contiguous rows")
    if t.dtype not in dtypes:
        raise ValueError(f"{name} has dtype {t.dtype}, expected one of {dtypes}")


def _ld(t: torch.Tensor) -> int:
    return t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))


def packed_words_per_row(n: int, bits: int) -> int:
    return (n * bits + 31) // 32


def gptq_hessian_accumulate_workspace_bytes(n: int, t: int, dtype: torch.dtype = torch.float16) -> int:
    return lib().gptq_hessian_accumulate_workspace_bytes(n, t, _DTYPE[dtype])


def gptq_hessian_accumulate_launches(n: int, t: int, dtype: torch.dtype = torch.float16) -> int:
    """Launches of the matrix-core kernel one gptq_hessian_accumulate call of t tokens makes (1 unless it is sliced)."""
    return int(lib().gptq_hessian_accumulate_launches(n, t, _DTYPE[dtype]))


def gptq_hessian_accumulate(H: torch.Tensor, X: torch.Tensor, ws: torch.Tensor | None = None) -> None:
    """H[upper] += 2 X X^T for one chunk X [n x t] (tokens contiguous); ws: optional uint8 workspace."""
    _dev2d(H, "H", (torch.float32,))
    _dev2d(X, "X", tuple(_DTYPE))
    n, t = X.shape
    if H.shape != (n, n):
        raise ValueError("H must be n x n")
    if ws is not None and (ws.dtype != torch.uint8 or not ws.is_cuda):
        raise ValueError("ws must be a GPU uint8 tensor")
    _check(lib().gptq_hessian_accumulate(_ptr(H), _ld(H), _ptr(X), _DTYPE[X.dtype], n, t, _ld(X),
                                         _ptr(ws), ws.numel() if ws is not None else 0, _stream()))


def gptq_hessian_accumulate_token_major_workspace_bytes(n: int, t: int, dtype: torch.dtype = torch.float16) -> int:
    return lib().gptq_hessian_accumulate_token_major_workspace_bytes(n, t, _DTYPE[dtype])


def gptq_hessian_accumulate_token_major(H: torch.Tensor, X: torch.Tensor, ws: torch.Tensor) -> None:
    """H[upper] += 2 X^T X for one chunk X [t x n] (channels contiguous); ws: uint8 workspace (required)."""
    _dev2d(H, "H", (torch.float32,))
    _dev2d(X, "X", (torch.float16, torch.bfloat16))
    t, n = X.shape
    if H.shape != (n, n):
        raise ValueError("H must be n x n")
    if ws is None or ws.dtype != torch.uint8 or not ws.is_cuda:
        raise ValueError("ws must be a GPU uint8 tensor")
    _check(lib().gptq_hessian_accumulate_token_major(_ptr(H), _ld(H), _ptr(X), _DTYPE[X.dtype], n, t, _ld(X),
                                                     _ptr(ws), ws.numel(), _stream()))


def gptq_hessian_symmetrize(H: torch.Tensor) -> None:
    _dev2d(H, "H", (torch.float32,))
    _check(lib().gptq_hessian_symmetrize(_ptr(H), _ld(H), H.shape[0], _stream()))


def gptq_damp_cholesky_inverse_workspace_bytes(n: int) -> int:
    return lib().gptq_damp_cholesky_inverse_workspace_bytes(n)


def gptq_damp_cholesky_inverse(H_U: torch.Tensor, percdamp: float, ws: torch.Tensor, info: torch.Tensor) -> None:
    """In place: the upper triangle of H becomes U = Cholesky((H + lambda I)^-1)^T."""
    _dev2d(H_U, "H_U", (torch.float32,))
    if info.dtype != torch.int32 or not info.is_cuda or ws.dtype != torch.uint8 or not ws.is_cuda:
        raise ValueError("info must be a GPU int32 tensor and ws a GPU uint8 tensor")
    n = H_U.shape[0]
    _check(lib().gptq_damp_cholesky_inverse(_ptr(H_U), _ld(H_U), n, percdamp, _ptr(ws), ws.numel(), _ptr(info), _stream()))


def gptq_damp_cholesky_workspace_bytes(n: int) -> int:
    return lib().gptq_damp_cholesky_workspace_bytes(n)


def gptq_damp_cholesky(H_R: torch.Tensor, percdamp: float, ws: torch.Tensor, info: torch.Tensor) -> None:
    """In place: the upper triangle of H becomes R with H + lambda I = R R^T (no inverse)."""
    _dev2d(H_R, "H_R", (torch.float32,))
    if info.dtype != torch.int32 or not info.is_cuda or ws.dtype != torch.uint8 or not ws.is_cuda:
        raise ValueError("info must be a GPU int32 tensor and ws a GPU uint8 tensor")
    _check(lib().gptq_damp_cholesky(_ptr(H_R), _ld(H_R), H_R.shape[0], percdamp, _ptr(ws), ws.numel(), _ptr(info), _stream()))


def gptq_noalloc_max_n() -> int:
    return lib().gptq_noalloc_max_n()


def gptq_damp_cholesky_inverse_noalloc(H_U: torch.Tensor, percdamp: float, info: torch.Tensor) -> None:
    """gptq_damp_cholesky_inverse without a workspace argument: scratch lives in the library's own fixed device
    array (n <= gptq_noalloc_max_n()); allocates nothing."""
    _dev2d(H_U, "H_U", (torch.float32,))
    if info.dtype != torch.int32 or not info.is_cuda:
        raise ValueError("info must be a GPU int32 tensor")
    _check(lib().gptq_damp_cholesky_inverse_noalloc(_ptr(H_U), _ld(H_U), H_U.shape[0], percdamp, _ptr(info), _stream()))


def gptq_check_info(info: torch.Tensor) -> int:
    host = ctypes.c_int(0)
    _check(lib().gptq_check_info(_ptr(info), ctypes.byref(host), _stream()))
    return host.value


def gptq_quantize_layer_workspace_bytes(r: int, n: int, block: int = 128, group: int = 0) -> int:
    return lib().gptq_quantize_layer_workspace_bytes(r, n, block, group)


def gptq_quantize_layer(W: torch.Tensor, U: torch.Tensor, bits: int, grid: int, block: int, group: int,
                        codes: torch.Tensor, scales: torch.Tensor, zeros: torch.Tensor, ws: torch.Tensor,
                        Wq: torch.Tensor | None = None, half_E2_rows: torch.Tensor | None = None,
                        from_factor: bool = False) -> None:
    """Alg. 1 with U = Cholesky((H + lambda I)^-1)^T, or -- from_factor=True, gptq_quantize_layer_from_factor -- with
    the Cholesky factor R of H + lambda I in its place."""
    _dev2d(W, "W", tuple(_DTYPE))
    _dev2d(U, "U", (torch.float32,))
    _dev2d(codes, "codes", (torch.uint8,))
    r, n = W.shape
    G = n // group if group else 1
    if codes.shape != (r, n) or U.shape != (n, n):
        raise ValueError("shape mismatch")
    for t, dt, nm in ((scales, torch.float32, "scales"), (zeros, torch.int32, "zeros")):
        if not t.is_cuda or t.dtype != dt or not t.is_contiguous() or t.numel() != r * G:
            raise ValueError(f"{nm} must be a dense GPU {dt} tensor with r * groups elements")
    if Wq is not None:
        _dev2d(Wq, "Wq", (torch.float32,))
    if half_E2_rows is not None and (half_E2_rows.dtype != torch.float64 or half_E2_rows.numel() != r or not half_E2_rows.is_cuda):
        raise ValueError("half_E2_rows must be a GPU float64 tensor of r elements")
    fn = lib().gptq_quantize_layer_from_factor if from_factor else lib().gptq_quantize_layer
    _check(fn(_ptr(W), _DTYPE[W.dtype], _ld(W), r, n, _ptr(U), _ld(U), bits, grid, block, group,
          _ptr(codes), _ld(codes), _ptr(scales), _ptr(zeros),
          _ptr(Wq), _ld(Wq) if Wq is not None else 0, _ptr(half_E2_rows),
          _ptr(ws), ws.numel(), _stream()))


def gptq_quantize_layer_from_factor_supports(group: int) -> bool:
    """Whether gptq_quantize_layer_from_factor takes this group size (0 = one grid per row)."""
    return bool(lib().gptq_quantize_layer_from_factor_supports(int(group)))


def gptq_quantize_layer_from_factor(W, R, bits, grid, block, group, codes, scales, zeros, ws, Wq=None, half_E2_rows=None) -> None:
    gptq_quantize_layer(W, R, bits, grid, block, group, codes, scales, zeros, ws, Wq, half_E2_rows, from_factor=True)


def gptq_trailing_update(W: torch.Tensor, E: torch.Tensor, U: torch.Tensor) -> None:
    """W[r x ncols] -= E[r x k] @ U[k x ncols] (float32): the lazy batch update of Alg. 1."""
    for t, nm in ((W, "W"), (E, "E"), (U, "U")):
        _dev2d(t, nm, (torch.float32,))
    r, ncols = W.shape
    k = E.shape[1]
    if E.shape[0] != r or U.shape != (k, ncols):
        raise ValueError("need E [r x k] and U [k x ncols] for W [r x ncols]")
    _check(lib().gptq_trailing_update(_ptr(W), _ld(W), _ptr(E), _ld(E), _ptr(U), _ld(U), r, ncols, k, _stream()))


def gptq_trailing_update_split_workspace_bytes(r: int, ncols: int) -> int:
    return int(lib().gptq_trailing_update_split_workspace_bytes(int(r), int(ncols)))


def gptq_trailing_update_split(W: torch.Tensor, E: torch.Tensor, U: torch.Tensor, ws: torch.Tensor) -> None:
    """W[r x ncols] -= E[r x 1024] @ U[1024 x ncols] through split float32 products on the bf16 matrix cores."""
    for t, nm in ((W, "W"), (E, "E"), (U, "U")):
        _dev2d(t, nm, (torch.float32,))
    r, ncols = W.shape
    k = E.shape[1]
    if E.shape[0] != r or U.shape != (k, ncols):
        raise ValueError("need E [r x k] and U [k x ncols] for W [r x ncols]")
    _check(lib().gptq_trailing_update_split(_ptr(W), _ld(W), _ptr(E), _ld(E), _ptr(U), _ld(U), r, ncols, k,
                                            _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def gptq_set_split_min_tiles(tiles: int) -> int:
    """Launches of at least `tiles` 256 x 256 tiles take the split products (0: the library's own rule); returns the previous setting."""
    return int(lib().gptq_set_split_min_tiles(int(tiles)))


def gptq_symmetric_update_split_workspace_bytes(n: int) -> int:
    return int(lib().gptq_symmetric_update_split_workspace_bytes(int(n)))


def gptq_symmetric_update_split(H: torch.Tensor, P: torch.Tensor, ws: torch.Tensor) -> None:
    """H[n x n] -= P[n x 1024] @ P^T on the 256 x 256 tiles that touch the upper triangle (split float32 products)."""
    _dev2d(H, "H", (torch.float32,))
    _dev2d(P, "P", (torch.float32,))
    n = H.shape[0]
    if H.shape[1] != n or P.shape[0] != n:
        raise ValueError("need a square H [n x n] and P [n x k]")
    _check(lib().gptq_symmetric_update_split(_ptr(H), _ld(H), _ptr(P), _ld(P), n, P.shape[1],
                                             _ptr(ws), ws.numel() * ws.element_size(), _stream()))


def gptq_pack(codes: torch.Tensor, bits: int, out: torch.Tensor) -> None:
    _dev2d(codes, "codes", (torch.uint8,))
    _dev2d(out, "out", (torch.int32, torch.uint32))
    r, n = codes.shape
    _check(lib().gptq_pack(_ptr(codes), _ld(codes), r, n, bits, _ptr(out), _ld(out), _stream()))


def gptq_unpack(words: torch.Tensor, n: int, bits: int, codes: torch.Tensor) -> None:
    _dev2d(codes, "codes", (torch.uint8,))
    _dev2d(words, "words", (torch.int32, torch.uint32))
    r = codes.shape[0]
    _check(lib().gptq_unpack(_ptr(words), _ld(words), r, n, bits, _ptr(codes), _ld(codes), _stream()))


def _grids(scales: torch.Tensor, zeros: torch.Tensor, r: int, n: int, group: int) -> None:
    G = n // group if group else 1
    for t, name, dt in ((scales, "scales", torch.float32), (zeros, "zeros", torch.int32)):
        if not t.is_cuda or t.dtype != dt or not t.is_contiguous() or t.numel() != r * G:
            raise ValueError(f"{name} must be a dense GPU {dt} tensor of r x {G} entries")


def gptq_dequantize_packed(words: torch.Tensor, n: int, bits: int, scales: torch.Tensor, zeros: torch.Tensor,
                           group: int, out: torch.Tensor) -> None:
    """out[r x n] (float16 or float32) = scale * (code - zero) of the packed layer."""
    _dev2d(words, "words", (torch.int32, torch.uint32))
    _dev2d(out, "out", (torch.float16, torch.float32))
    r = out.shape[0]
    if out.shape[1] != n or words.shape[0] != r:
        raise ValueError("out must be r x n and words must have r rows")
    _grids(scales, zeros, r, n, group)
    _check(lib().gptq_dequantize_packed(_ptr(words), _ld(words), r, n, bits, _ptr(scales), _ptr(zeros), group,
                                        _ptr(out), _DTYPE[out.dtype], _ld(out), _stream()))


def gptq_matvec_packed(words: torch.Tensor, n: int, bits: int, scales: torch.Tensor, zeros: torch.Tensor,
                       group: int, x: torch.Tensor, y: torch.Tensor) -> None:
    """y[r] (float32) = Q x for the packed layer Q and a float16 or float32 vector x[n]."""
    _dev2d(words, "words", (torch.int32, torch.uint32))
    r = words.shape[0]
    if not x.is_cuda or x.dim() != 1 or x.shape[0] != n or not x.is_contiguous() or x.dtype not in (torch.float16, torch.float32):
        raise ValueError("x must be a dense GPU float16 or float32 vector of n entries")
    if not y.is_cuda or y.dim() != 1 or y.shape[0] != r or not y.is_contiguous() or y.dtype != torch.float32:
        raise ValueError("y must be a dense GPU float32 vector of r entries")
    _grids(scales, zeros, r, n, group)
    _check(lib().gptq_matvec_packed(_ptr(words), _ld(words), r, n, bits, _ptr(scales), _ptr(zeros), group,
                                    _ptr(x), _DTYPE[x.dtype], _ptr(y), _stream()))
