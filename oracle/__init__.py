"""ctypes front-end of the RotateK CPU oracle (oracle/rotatek_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg.  The product (paper_2605_19218_amd) never imports
it, and this package never imports the product.

All functions take numpy arrays, promote them to fp64 and call the C routines
one-to-one; `fit()` strings the single-head routines together in the order of
Alg. 1 of the paper.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None

_D = C.POINTER(C.c_double)
_I32 = C.POINTER(C.c_int32)
_U8 = C.POINTER(C.c_uint8)


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.orc_mean_scatter.argtypes = [_D, C.c_int64, C.c_int, _I32, C.c_int, _D, _D]
        L.orc_weight.argtypes = [_D, _D, C.c_int, _D]
        L.orc_jacobi_eigh.argtypes = [_D, C.c_int, C.c_double, C.c_int, _D, _D]
        L.orc_jacobi_eigh.restype = C.c_int
        L.orc_select.argtypes = [_D, C.c_int, C.c_int, _U8, _I32]
        L.orc_gather_rotation.argtypes = [_D, _I32, C.c_int, C.c_int, _D]
        L.orc_delta_mu.argtypes = [_D, _D, C.c_int, C.c_int, _D]
        L.orc_round_bf16.argtypes = [C.c_double]
        L.orc_round_bf16.restype = C.c_double
        L.orc_compress.argtypes = [_D, C.c_int64, C.c_int, _I32, _D, C.c_int, C.c_int, _D]
        L.orc_decode_head.argtypes = [_D, _D, _D, _D, _D, C.c_int64, C.c_int, C.c_int, C.c_double, _D, _D]
        L.orc_full_attn_head.argtypes = [_D, _D, _D, C.c_int64, C.c_int, C.c_double, _D]
        L.orc_fit_batch.argtypes = [_D, C.c_int, C.c_int64, C.c_int, _I32, _D, C.c_int, C.c_int,
                                    _D, _D, _D, _D, _U8, _I32, _D, _D]
        L.orc_fit_batch.restype = C.c_int
        L.orc_compress_batch.argtypes = [_D, C.c_int, C.c_int64, C.c_int, _I32, _D, C.c_int, C.c_int, _D]
        L.orc_decode_batch.argtypes = [_D, _D, _D, _D, _D, _I32, C.c_int, C.c_int, C.c_int, C.c_int64,
                                       C.c_int, C.c_int, C.c_double, _D]
        L.orc_decode_dual_head.argtypes = [_D, _D, _D, C.c_int64, _D, _D, C.c_int64, _D, _D, C.c_int, C.c_int,
                                           C.c_double, _D]
        L.orc_decode_dual_batch.argtypes = [_D, _D, _D, _D, _D, _D, _D, _I32, _I32, C.c_int, C.c_int, C.c_int,
                                            C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_double, _D]
        L.orc_sigma_window.argtypes = [_D, C.c_int64, C.c_int, _D]
        L.orc_subspace_iter.argtypes = [_D, C.c_int, C.c_int, _D, C.c_int, C.c_double, _D]
        L.orc_subspace_iter.restype = C.c_int
        L.orc_num_threads.restype = C.c_int
        _lib = L
    return _lib


def _f64(x):
    return np.ascontiguousarray(x, dtype=np.float64)


def _p(a, t=_D):
    return None if a is None else a.ctypes.data_as(t)


def _i32(x):
    return None if x is None else np.ascontiguousarray(x, dtype=np.int32)


_ROUND = {"none": 0, None: 0, "f32": 1, "bf16": 2}


# --------------------------------------------------------------------------
def mean_scatter(K, tok=None, center=True):
    """Alg. 1 steps 1-3.  K [N,d] -> (mu [d], C [d,d])."""
    K = _f64(K)
    N, d = K.shape
    tok = _i32(tok)
    n = N if tok is None else tok.size
    mu = np.empty(d)
    Cm = np.empty((d, d))
    lib().orc_mean_scatter(_p(K), n, d, _p(tok, _I32), int(bool(center)), _p(mu), _p(Cm))
    return mu, Cm


def weight(Cm, sigma=None):
    """Alg. 1 step 5 / Eq. 4."""
    Cm = _f64(Cm)
    d = Cm.shape[0]
    sigma = None if sigma is None else _f64(sigma)
    out = np.empty((d, d))
    lib().orc_weight(_p(Cm), _p(sigma), d, _p(out))
    return out


def jacobi_eigh(A, tol=1e-14, max_sweeps=60):
    """Symmetric eigendecomposition, eigenvalues decreasing.  -> (R, lam, sweeps)."""
    A = _f64(A)
    d = A.shape[0]
    R = np.empty((d, d))
    lam = np.empty(d)
    sw = lib().orc_jacobi_eigh(_p(A), d, float(tol), int(max_sweeps), _p(R), _p(lam))
    if sw < 0:
        raise RuntimeError("oracle Jacobi did not converge")
    return R, lam, sw


def select(lam, r):
    """Keep-mask from eigenvalues in any column order.  -> (mask u8 [d], keep_idx i32 [r])."""
    lam = _f64(lam)
    d = lam.size
    mask = np.zeros(d, np.uint8)
    keep = np.zeros(r, np.int32)
    lib().orc_select(_p(lam), d, int(r), _p(mask, _U8), _p(keep, _I32))
    return mask, keep


def gather_rotation(R, keep_idx):
    R = _f64(R)
    d = R.shape[0]
    keep_idx = _i32(keep_idx)
    r = keep_idx.size
    Rr = np.empty((d, r))
    lib().orc_gather_rotation(_p(R), _p(keep_idx, _I32), d, r, _p(Rr))
    return Rr


def delta_mu(mu, Rr):
    """Alg. 1 step 15."""
    mu, Rr = _f64(mu), _f64(Rr)
    d, r = Rr.shape
    out = np.empty(d)
    lib().orc_delta_mu(_p(mu), _p(Rr), d, r, _p(out))
    return out


def round_bf16(x):
    L = lib()
    x = _f64(x)
    return np.vectorize(L.orc_round_bf16, otypes=[np.float64])(x) if x.size else x


def compress(K, Rr, tok=None, rounding="none"):
    """Alg. 1 step 14 (+ one storage rounding).  K [N,d], Rr [d,r] -> Kt [n,r]."""
    K, Rr = _f64(K), _f64(Rr)
    N, d = K.shape
    r = Rr.shape[1]
    tok = _i32(tok)
    n = N if tok is None else tok.size
    Kt = np.empty((n, r))
    lib().orc_compress(_p(K), n, d, _p(tok, _I32), _p(Rr), r, _ROUND[rounding], _p(Kt))
    return Kt


def decode_head(q, Kt, V, Rr, dmu=None, scale=0.0, return_lse=False):
    """Alg. 2 steps 1-3, 6 for one query head."""
    q, Kt, V, Rr = _f64(q), _f64(Kt), _f64(V), _f64(Rr)
    L, r = Kt.shape
    d = q.size
    dmu = None if dmu is None else _f64(dmu)
    out = np.empty(d)
    lse = np.empty(2)
    lib().orc_decode_head(_p(q), _p(Kt), _p(V), _p(Rr), _p(dmu), L, d, r, float(scale), _p(out), _p(lse))
    return (out, lse) if return_lse else out


def full_attn_head(q, K, V, scale=0.0):
    q, K, V = _f64(q), _f64(K), _f64(V)
    L, d = K.shape
    out = np.empty(d)
    lib().orc_full_attn_head(_p(q), _p(K), _p(V), L, d, float(scale), _p(out))
    return out


def fit(K, r, sigma=None, center=True, tok=None):
    """Alg. 1 for one head with the full eigendecomposition as the solver.
    Returns dict(mu, C, Cq, R, lam, mask, keep_idx, Rr, dmu, sweeps)."""
    mu, Cm = mean_scatter(K, tok=tok, center=center)
    Cq = weight(Cm, sigma)
    R, lam, sw = jacobi_eigh(Cq)
    mask, keep = select(lam, r)
    Rr = gather_rotation(R, keep)
    dmu = delta_mu(mu, Rr)
    return dict(mu=mu, C=Cm, Cq=Cq, R=R, lam=lam, mask=mask, keep_idx=keep, Rr=Rr, dmu=dmu, sweeps=sw)


def sigma_window(Qw):
    """Alg. 1 step 4: per-channel l2 norm over all leading axes of Qw [..., d] (W rows, or G x W under GQA)."""
    Qw = _f64(Qw)
    d = Qw.shape[-1]
    rows = Qw.size // d
    out = np.empty(d)
    lib().orc_sigma_window(_p(Qw), rows, d, _p(out))
    return out


def subspace_iter(Cq, V0, T=5, eps=1e-6):
    """Alg. 1 steps 6-13: T rounds of V <- Cq V followed by the shifted Cholesky-QR.  Returns V [d,k]."""
    Cq, V0 = _f64(Cq), _f64(V0)
    d, k = V0.shape
    V = np.empty((d, k))
    st = lib().orc_subspace_iter(_p(Cq), d, k, _p(V0), int(T), float(eps), _p(V))
    if st != 0:
        raise RuntimeError(f"oracle Cholesky met a non-positive pivot in iteration {st - 1}")
    return V


def fit_subspace(K, V0, T=5, eps=1e-6, sigma=None, center=True, tok=None):
    """Alg. 1 for one head with the subspace iteration as the solver (the paper's default).
    Returns dict(mu, C, Cq, Rr, dmu); Rr = V^(T) [d,k]."""
    mu, Cm = mean_scatter(K, tok=tok, center=center)
    Cq = weight(Cm, sigma)
    Rr = subspace_iter(Cq, V0, T, eps)
    return dict(mu=mu, C=Cm, Cq=Cq, Rr=Rr, dmu=delta_mu(mu, Rr))


# --------------------------------------------------------------------------
# batched (OpenMP over heads) -- used for full-size parity and cpu_baseline
def fit_batch(K, r, sigma=None, center=True, lens=None):
    """K [U,N,d] -> dict of per-unit arrays."""
    K = _f64(K)
    U, N, d = K.shape
    sigma = None if sigma is None else _f64(sigma)
    lens = _i32(lens)
    o = dict(mu=np.empty((U, d)), C=np.empty((U, d, d)), R=np.empty((U, d, d)), lam=np.empty((U, d)),
             mask=np.zeros((U, d), np.uint8), keep_idx=np.zeros((U, r), np.int32),
             Rr=np.empty((U, d, r)), dmu=np.empty((U, d)))
    sw = lib().orc_fit_batch(_p(K), U, N, d, _p(lens, _I32), _p(sigma), int(bool(center)), int(r),
                             _p(o["mu"]), _p(o["C"]), _p(o["R"]), _p(o["lam"]), _p(o["mask"], _U8),
                             _p(o["keep_idx"], _I32), _p(o["Rr"]), _p(o["dmu"]))
    if sw < 0:
        raise RuntimeError("oracle Jacobi did not converge")
    o["sweeps"] = sw
    return o


def compress_batch(K, Rr, rounding="none", lens=None):
    K, Rr = _f64(K), _f64(Rr)
    U, N, d = K.shape
    r = Rr.shape[2]
    lens = _i32(lens)
    Kt = np.zeros((U, N, r))
    lib().orc_compress_batch(_p(K), U, N, d, _p(lens, _I32), _p(Rr), r, _ROUND[rounding], _p(Kt))
    return Kt


def decode_batch(q, Kt, V, Rr, dmu=None, lens=None, scale=0.0):
    """q [B,Hq,d], Kt [B,Hkv,cap,r], V [B,Hkv,cap,d], Rr [B,Hkv,d,r] -> out [B,Hq,d]."""
    q, Kt, V, Rr = _f64(q), _f64(Kt), _f64(V), _f64(Rr)
    B, Hq, d = q.shape
    _, Hkv, cap, r = Kt.shape
    dmu = None if dmu is None else _f64(dmu)
    lens = _i32(lens)
    out = np.empty((B, Hq, d))
    lib().orc_decode_batch(_p(q), _p(Kt), _p(V), _p(Rr), _p(dmu), _p(lens, _I32), B, Hq, Hkv, cap, d, r,
                           float(scale), _p(out))
    return out


def decode_dual_head(q, Kt, Vvis, Kpt, Vpt, Rr, dmu=None, scale=0.0):
    """Alg. 2 steps 1-6 for one query head: Kt [N,r], Vvis [N,d], Kpt/Vpt [M,d]."""
    q, Kt, Vvis, Kpt, Vpt, Rr = _f64(q), _f64(Kt), _f64(Vvis), _f64(Kpt), _f64(Vpt), _f64(Rr)
    d = q.size
    N, r = Kt.shape if Kt.size else (0, Rr.shape[1])
    M = Kpt.shape[0] if Kpt.size else 0
    dmu = None if dmu is None else _f64(dmu)
    out = np.empty(d)
    lib().orc_decode_dual_head(_p(q), _p(Kt), _p(Vvis), N, _p(Kpt), _p(Vpt), M, _p(Rr), _p(dmu), d, r,
                               float(scale), _p(out))
    return out


def decode_dual_batch(q, Kt, V, Kpt, Vpt, Rr, dmu=None, lens=None, lens_t=None, scale=0.0):
    """decode_batch plus a prompt/text segment Kpt, Vpt [B,Hkv,cap_t,d] with lengths lens_t."""
    q, Kt, V, Kpt, Vpt, Rr = _f64(q), _f64(Kt), _f64(V), _f64(Kpt), _f64(Vpt), _f64(Rr)
    B, Hq, d = q.shape
    _, Hkv, cap, r = Kt.shape
    cap_t = Kpt.shape[2]
    dmu = None if dmu is None else _f64(dmu)
    lens, lens_t = _i32(lens), _i32(lens_t)
    out = np.empty((B, Hq, d))
    lib().orc_decode_dual_batch(_p(q), _p(Kt), _p(V), _p(Kpt), _p(Vpt), _p(Rr), _p(dmu), _p(lens, _I32),
                                _p(lens_t, _I32), B, Hq, Hkv, cap, cap_t, d, r, float(scale), _p(out))
    return out


def num_threads() -> int:
    return int(lib().orc_num_threads())
