"""RotateK hot path for AMD MI355X: thin ctypes binding of librotatek.so.

The functions here have the names and argument order of the C ABI declared in
include/rotatek.h and only marshal arguments (device pointers, strides, sizes);
every step of the path runs in the HIP kernels.  PyTorch is used by callers for
device memory and streams only.  There is no CPU fallback: importing works
without a GPU (so that argument validation can be exercised through a host-only
context), but a missing library is an error.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Any, Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librotatek.so")

RK_OK, RK_ERR_INVALID_ARG, RK_ERR_UNSUPPORTED, RK_ERR_CAPACITY, RK_ERR_WORKSPACE, RK_ERR_HIP, RK_ERR_NO_DEVICE = range(7)
RK_F32, RK_BF16 = 0, 1
RK_FIT_CENTER = 1
RK_OPT_FORCE_GENERIC, RK_OPT_DECODE_SPLITS, RK_OPT_FUSE_MERGE = 1, 2, 3
RK_DEVICE_NONE = -1

EXPORTS = [
    "rk_create", "rk_destroy", "rk_status_str", "rk_last_error", "rk_set_option", "rk_validate_layout",
    "rk_fit_workspace_size", "rk_decode_workspace_size", "rk_decode_plan", "rk_fit_rotation",
    "rk_gather_rotation", "rk_compress", "rk_append", "rk_decode_attn", "rk_cache_bytes", "rk_unpack_cache",
    "rk_decode_attn_dual", "rk_append_text", "rk_fit_subspace", "rk_query_sigma", "rk_append_decode_attn",
    "rk_append_text_decode_attn_dual", "rk_decode_attn_static", "rk_stream_read",
]
RK_STATIC_SCRATCH_BYTES = 8 << 20


class rk_layout(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("keep", C.c_int32), ("dtype", C.c_int32),
                ("capacity", C.c_int32), ("max_seq_len", C.c_int32), ("seq_len", C.c_void_p)]


class rk_rows(C.Structure):
    _fields_ = [("data", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64),
                ("stride_t", C.c_int64), ("n_tokens", C.c_int32), ("n_tokens_dev", C.c_void_p),
                ("tok_idx", C.c_void_p), ("tok_off", C.c_void_p)]


class rk_fit_out(C.Structure):
    _fields_ = [("R", C.c_void_p), ("eigvals", C.c_void_p), ("mask", C.c_void_p), ("keep_idx", C.c_void_p),
                ("R_r", C.c_void_p), ("mu", C.c_void_p), ("delta_mu", C.c_void_p), ("cov", C.c_void_p),
                ("sweeps", C.c_void_p)]


class rk_text(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64),
                ("stride_t", C.c_int64), ("capacity", C.c_int32), ("max_len", C.c_int32), ("len", C.c_void_p)]


class rk_subspace(C.Structure):
    _fields_ = [("v0", C.c_void_p), ("iterations", C.c_int32), ("ridge", C.c_double)]


class RotateKError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"rotatek status {status}: {text}")
        self.status = status


_lib = None


def lib():
    """Load librotatek.so (built by paper_2605_19218_amd/build.py); loud failure if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u32, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_float, C.c_size_t
        PL, PR, PF = C.POINTER(rk_layout), C.POINTER(rk_rows), C.POINTER(rk_fit_out)
        PT = C.POINTER(rk_text)
        L.rk_create.argtypes = [C.POINTER(vp), C.c_int]
        L.rk_destroy.argtypes = [vp]
        L.rk_status_str.argtypes = [C.c_int]
        L.rk_status_str.restype = C.c_char_p
        L.rk_last_error.argtypes = [vp]
        L.rk_last_error.restype = C.c_char_p
        L.rk_set_option.argtypes = [vp, i32, i64]
        L.rk_validate_layout.argtypes = [PL]
        L.rk_fit_workspace_size.argtypes = [PL, i32]
        L.rk_fit_workspace_size.restype = sz
        L.rk_decode_workspace_size.argtypes = [vp, PL]
        L.rk_decode_workspace_size.restype = sz
        L.rk_decode_plan.argtypes = [vp, PL, C.POINTER(i32), C.POINTER(i32)]
        L.rk_cache_bytes.argtypes = [PL, C.POINTER(sz), C.POINTER(sz)]
        L.rk_unpack_cache.argtypes = [vp, PL, vp, vp, vp, vp, vp]
        L.rk_fit_rotation.argtypes = [vp, PL, PR, vp, u32, PF, vp, sz, vp]
        L.rk_gather_rotation.argtypes = [vp, PL, vp, vp, vp, vp]
        L.rk_compress.argtypes = [vp, PL, PR, vp, vp, PR, vp, vp, vp]
        L.rk_append.argtypes = [vp, PL, vp, vp, vp, vp, vp, vp, vp]
        L.rk_decode_attn.argtypes = [vp, PL, vp, vp, vp, vp, vp, f32, vp, vp, sz, vp]
        L.rk_stream_read.argtypes = [vp, vp, sz, vp]
        L.rk_decode_attn_static.argtypes = [vp, PL, vp, vp, vp, vp, vp, f32, vp, vp]
        L.rk_decode_attn_dual.argtypes = [vp, PL, vp, vp, vp, vp, vp, PT, f32, vp, vp, sz, vp]
        L.rk_append_text.argtypes = [vp, PL, PT, vp, vp, vp]
        L.rk_append_text_decode_attn_dual.argtypes = [vp, PL, vp, vp, vp, vp, vp, vp, vp, PT, f32, vp, vp, sz, vp]
        L.rk_append_decode_attn.argtypes = [vp, PL, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, sz, vp]
        L.rk_fit_subspace.argtypes = [vp, PL, PR, vp, u32, C.POINTER(rk_subspace), vp, vp, vp, vp, vp, vp, sz, vp]
        L.rk_query_sigma.argtypes = [vp, PL, vp, i64, i64, i64, i32, vp, vp]
        for name in EXPORTS:
            if name not in ("rk_status_str", "rk_last_error", "rk_fit_workspace_size", "rk_decode_workspace_size"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _ptr(x: Any) -> Optional[int]:
    """Device pointer of a tensor-like (anything with data_ptr()), an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _nbytes(x: Any) -> int:
    return int(x.numel() * x.element_size())


def _stream(stream: Any) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)        # torch.cuda.Stream


def _check(ctx, status: int):
    if status != RK_OK:
        text = lib().rk_last_error(ctx).decode() if ctx else ""
        raise RotateKError(status, text or lib().rk_status_str(status).decode())


# ---- argument holders ------------------------------------------------------
@dataclass
class Layout:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    keep: int
    dtype: int
    capacity: int
    max_seq_len: int
    seq_len: Any = None           # device int32 [batch]
    head_dim: int = 128

    def c(self) -> rk_layout:
        return rk_layout(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.keep, self.dtype,
                         self.capacity, self.max_seq_len, _ptr(self.seq_len))


@dataclass
class Rows:
    """Rows of a [B, H_kv, N, d] tensor-like (any strides, channels contiguous)."""
    data: Any
    n_tokens: int
    n_tokens_dev: Any = None
    tok_idx: Any = None
    tok_off: Any = None
    strides: Optional[tuple] = None      # (stride_b, stride_h, stride_t) in elements

    def c(self) -> rk_rows:
        st = self.strides if self.strides is not None else tuple(self.data.stride()[:3])
        return rk_rows(_ptr(self.data), st[0], st[1], st[2], self.n_tokens, _ptr(self.n_tokens_dev),
                       _ptr(self.tok_idx), _ptr(self.tok_off))


@dataclass
class FitOut:
    R: Any
    eigvals: Any
    mask: Any
    keep_idx: Any
    R_r: Any
    mu: Any
    delta_mu: Any
    cov: Any = None
    sweeps: Any = None

    def c(self) -> rk_fit_out:
        return rk_fit_out(*[_ptr(getattr(self, f)) for f in
                            ("R", "eigvals", "mask", "keep_idx", "R_r", "mu", "delta_mu", "cov", "sweeps")])


@dataclass
class Text:
    """Full-width prompt/text segment: k, v tensor-likes [B, H_kv, capacity, d] sharing one set of strides."""
    k: Any
    v: Any
    max_len: int
    len: Any = None                      # device int32 [B]
    capacity: Optional[int] = None       # rows allocated per (b, h); default: k.shape[2]
    strides: Optional[tuple] = None      # (stride_b, stride_h, stride_t) in elements

    def c(self) -> rk_text:
        st = self.strides if self.strides is not None else tuple(self.k.stride()[:3])
        cap = self.capacity if self.capacity is not None else int(self.k.shape[2])
        return rk_text(_ptr(self.k), _ptr(self.v), st[0], st[1], st[2], cap, self.max_len, _ptr(self.len))


# ---- the ABI, same names -----------------------------------------------------
def rk_create(device: int = 0) -> int:
    h = C.c_void_p()
    st = lib().rk_create(C.byref(h), int(device))
    if st != RK_OK:
        raise RotateKError(st, lib().rk_status_str(st).decode())
    return h.value


def rk_destroy(ctx) -> None:
    lib().rk_destroy(ctx)


def rk_set_option(ctx, key: int, value: int) -> None:
    _check(ctx, lib().rk_set_option(ctx, key, value))


def rk_validate_layout(layout: Layout) -> int:
    return lib().rk_validate_layout(C.byref(layout.c()))


def rk_cache_bytes(layout: Layout):
    """(bytes of the packed-Key cache, bytes of the Value cache)."""
    k, v = C.c_size_t(), C.c_size_t()
    st = lib().rk_cache_bytes(C.byref(layout.c()), C.byref(k), C.byref(v))
    if st != RK_OK:
        raise RotateKError(st, lib().rk_status_str(st).decode())
    return k.value, v.value


def rk_unpack_cache(ctx, layout: Layout, k_packed, v_cache, k_rows, v_rows, stream=None) -> None:
    _check(ctx, lib().rk_unpack_cache(ctx, C.byref(layout.c()), _ptr(k_packed), _ptr(v_cache), _ptr(k_rows),
                                      _ptr(v_rows), _stream(stream)))


def rk_fit_workspace_size(layout: Layout, max_tokens: int) -> int:
    return int(lib().rk_fit_workspace_size(C.byref(layout.c()), int(max_tokens)))


def rk_decode_workspace_size(ctx, layout: Layout) -> int:
    return int(lib().rk_decode_workspace_size(ctx, C.byref(layout.c())))


def rk_decode_plan(ctx, layout: Layout):
    s, t = C.c_int32(), C.c_int32()
    _check(ctx, lib().rk_decode_plan(ctx, C.byref(layout.c()), C.byref(s), C.byref(t)))
    return s.value, t.value


def rk_fit_rotation(ctx, layout: Layout, keys: Rows, sigma, flags: int, out: FitOut, workspace, stream=None,
                    workspace_bytes: Optional[int] = None) -> None:
    wb = workspace_bytes if workspace_bytes is not None else (_nbytes(workspace) if workspace is not None else 0)
    _check(ctx, lib().rk_fit_rotation(ctx, C.byref(layout.c()), C.byref(keys.c()), _ptr(sigma), flags,
                                      C.byref(out.c()), _ptr(workspace), wb, _stream(stream)))


def rk_gather_rotation(ctx, layout: Layout, R, keep_idx, R_r, stream=None) -> None:
    _check(ctx, lib().rk_gather_rotation(ctx, C.byref(layout.c()), _ptr(R), _ptr(keep_idx), _ptr(R_r),
                                         _stream(stream)))


def rk_compress(ctx, layout: Layout, keys: Rows, R_r, k_packed, values: Optional[Rows] = None, v_cache=None,
                seq_len_out=None, stream=None) -> None:
    vrows = C.byref(values.c()) if values is not None else None
    _check(ctx, lib().rk_compress(ctx, C.byref(layout.c()), C.byref(keys.c()), _ptr(R_r), _ptr(k_packed), vrows,
                                  _ptr(v_cache), _ptr(seq_len_out), _stream(stream)))


def rk_append(ctx, layout: Layout, k_new, v_new, R_r, k_packed, v_cache, seq_len, stream=None) -> None:
    _check(ctx, lib().rk_append(ctx, C.byref(layout.c()), _ptr(k_new), _ptr(v_new), _ptr(R_r), _ptr(k_packed),
                                _ptr(v_cache), _ptr(seq_len), _stream(stream)))


def rk_append_decode_attn(ctx, layout: Layout, k_new, v_new, q, R_r, delta_mu, k_packed, v_cache, seq_len,
                          scale: float, out, workspace, stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = workspace_bytes if workspace_bytes is not None else (_nbytes(workspace) if workspace is not None else 0)
    _check(ctx, lib().rk_append_decode_attn(ctx, C.byref(layout.c()), _ptr(k_new), _ptr(v_new), _ptr(q), _ptr(R_r),
                                            _ptr(delta_mu), _ptr(k_packed), _ptr(v_cache), _ptr(seq_len),
                                            float(scale), _ptr(out), _ptr(workspace), wb, _stream(stream)))


def rk_decode_attn(ctx, layout: Layout, q, k_packed, v_cache, R_r, delta_mu, scale: float, out, workspace,
                   stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = workspace_bytes if workspace_bytes is not None else (_nbytes(workspace) if workspace is not None else 0)
    _check(ctx, lib().rk_decode_attn(ctx, C.byref(layout.c()), _ptr(q), _ptr(k_packed), _ptr(v_cache), _ptr(R_r),
                                     _ptr(delta_mu), float(scale), _ptr(out), _ptr(workspace), wb,
                                     _stream(stream)))


def rk_stream_read(ctx, src, nbytes: Optional[int] = None, stream=None) -> None:
    """Calibration: one plain streaming read of a device buffer."""
    _check(ctx, lib().rk_stream_read(ctx, _ptr(src), int(nbytes if nbytes is not None else _nbytes(src)),
                                     _stream(stream)))


def rk_decode_attn_static(ctx, layout: Layout, q, k_packed, v_cache, R_r, delta_mu, scale: float, out,
                          stream=None) -> None:
    """rk_decode_attn without a workspace: the partials live in the library's built-in scratch array."""
    _check(ctx, lib().rk_decode_attn_static(ctx, C.byref(layout.c()), _ptr(q), _ptr(k_packed), _ptr(v_cache),
                                            _ptr(R_r), _ptr(delta_mu), float(scale), _ptr(out), _stream(stream)))


def rk_decode_attn_dual(ctx, layout: Layout, q, k_packed, v_cache, R_r, delta_mu, text: Text, scale: float, out,
                        workspace, stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = workspace_bytes if workspace_bytes is not None else (_nbytes(workspace) if workspace is not None else 0)
    tref = C.byref(text.c()) if text is not None else None
    _check(ctx, lib().rk_decode_attn_dual(ctx, C.byref(layout.c()), _ptr(q), _ptr(k_packed), _ptr(v_cache),
                                          _ptr(R_r), _ptr(delta_mu), tref, float(scale), _ptr(out),
                                          _ptr(workspace), wb, _stream(stream)))


def rk_append_text_decode_attn_dual(ctx, layout: Layout, k_new, v_new, q, k_packed, v_cache, R_r, delta_mu,
                                    text: Text, scale: float, out, workspace, stream=None,
                                    workspace_bytes: Optional[int] = None) -> None:
    wb = workspace_bytes if workspace_bytes is not None else (_nbytes(workspace) if workspace is not None else 0)
    tref = C.byref(text.c()) if text is not None else None
    _check(ctx, lib().rk_append_text_decode_attn_dual(ctx, C.byref(layout.c()), _ptr(k_new), _ptr(v_new), _ptr(q),
                                                      _ptr(k_packed), _ptr(v_cache), _ptr(R_r), _ptr(delta_mu), tref,
                                                      float(scale), _ptr(out), _ptr(workspace), wb,
                                                      _stream(stream)))


def rk_append_text(ctx, layout: Layout, text: Text, k_new, v_new, stream=None) -> None:
    tref = C.byref(text.c()) if text is not None else None
    _check(ctx, lib().rk_append_text(ctx, C.byref(layout.c()), tref, _ptr(k_new), _ptr(v_new), _stream(stream)))


def rk_fit_subspace(ctx, layout: Layout, keys: Rows, sigma, flags: int, v0, iterations: int, ridge: float, R_r, mu,
                    delta_mu, workspace, cov=None, status=None, stream=None,
                    workspace_bytes: Optional[int] = None) -> None:
    wb = workspace_bytes if workspace_bytes is not None else (_nbytes(workspace) if workspace is not None else 0)
    sv = rk_subspace(_ptr(v0), int(iterations), float(ridge))
    _check(ctx, lib().rk_fit_subspace(ctx, C.byref(layout.c()), C.byref(keys.c()), _ptr(sigma), flags, C.byref(sv),
                                      _ptr(R_r), _ptr(mu), _ptr(delta_mu), _ptr(cov), _ptr(status),
                                      _ptr(workspace), wb, _stream(stream)))


def rk_query_sigma(ctx, layout: Layout, q_window, window: int, sigma, strides: Optional[tuple] = None,
                   stream=None) -> None:
    """q_window: tensor-like [B, H_q, window, d]; strides default to its own (elements)."""
    st = strides if strides is not None else tuple(q_window.stride()[:3])
    _check(ctx, lib().rk_query_sigma(ctx, C.byref(layout.c()), _ptr(q_window), st[0], st[1], st[2], int(window),
                                     _ptr(sigma), _stream(stream)))
