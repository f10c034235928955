"""Host<->device marshalling and a small driver object that holds the device buffers
of one attention layer and calls the C ABI binding in the order of the hot path
(fit -> compress -> append -> decode).  Used by the GPU tests, the smoke test and
the benchmark.  Argument plumbing only: no arithmetic of the method lives here, and
PyTorch serves as the allocator of device memory."""
from __future__ import annotations

import numpy as np
import torch

import paper_2605_19218_amd as rk

DEV = "cuda:0"
D = 128


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 numpy array of storage-representable values -> device tensor of the storage dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)             # exact for representable values (round-to-nearest-even otherwise)
    return t.to(DEV)


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor -> fp64 numpy (exact)."""
    if t.dtype == torch.bfloat16:
        return t.detach().cpu().to(torch.float64).numpy()
    return t.detach().cpu().numpy().astype(np.float64) if t.dtype.is_floating_point else t.cpu().numpy()


def rk_dtype(dtype: str) -> int:
    return rk.RK_BF16 if dtype == "bf16" else rk.RK_F32


def torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def bf16_ulp(y: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 at |y| (8 significant bits)."""
    a = np.maximum(np.abs(y), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


class Pipeline:
    """Device buffers of one layer + calls through the binding."""

    def __init__(self, ctx, B, Hq, Hkv, r, dtype, capacity):
        capacity = (capacity + 31) // 32 * 32           # the caches are tiled in 32-token blocks
        self.ctx, self.B, self.Hq, self.Hkv, self.r, self.dtype, self.cap = ctx, B, Hq, Hkv, r, dtype, capacity
        U = B * Hkv
        f32 = dict(device=DEV, dtype=torch.float32)
        self.R = torch.zeros(B, Hkv, D, D, **f32)
        self.lam = torch.zeros(B, Hkv, D, **f32)
        self.mask = torch.zeros(B, Hkv, D, device=DEV, dtype=torch.uint8)
        self.keep_idx = torch.zeros(B, Hkv, r, device=DEV, dtype=torch.int32)
        self.Rr = torch.zeros(B, Hkv, D, r, **f32)
        self.mu = torch.zeros(B, Hkv, D, **f32)
        self.dmu = torch.zeros(B, Hkv, D, **f32)
        self.cov = torch.zeros(B, Hkv, D, D, **f32)
        self.sweeps = torch.zeros(B, Hkv, device=DEV, dtype=torch.int32)
        td = torch_dtype(dtype)
        self.seq_len = torch.zeros(B, device=DEV, dtype=torch.int32)
        self.max_seq_len = 0
        kb, vb = rk.rk_cache_bytes(self.layout())
        self.Kp = torch.zeros(kb, device=DEV, dtype=torch.uint8)     # opaque fragment-major caches
        self.Vc = torch.zeros(vb, device=DEV, dtype=torch.uint8)
        self.out = torch.zeros(B, Hq, D, device=DEV, dtype=td)

    def layout(self):
        return rk.Layout(self.B, self.Hq, self.Hkv, self.r, rk_dtype(self.dtype), self.cap, self.max_seq_len,
                         seq_len=self.seq_len)

    def unpacked(self):
        """(K~ [B,Hkv,cap,r], V [B,Hkv,cap,d]) as fp64 numpy, via rk_unpack_cache."""
        td = torch_dtype(self.dtype)
        k_rows = torch.zeros(self.B, self.Hkv, self.cap, self.r, device=DEV, dtype=td)
        v_rows = torch.zeros(self.B, self.Hkv, self.cap, D, device=DEV, dtype=td)
        rk.rk_unpack_cache(self.ctx, self.layout(), self.Kp, self.Vc, k_rows, v_rows)
        torch.cuda.synchronize()
        return to_host(k_rows), to_host(v_rows)

    def rows(self, t, n_tokens, n_dev=None, tok_idx=None, tok_off=None):
        return rk.Rows(t, n_tokens, n_tokens_dev=n_dev, tok_idx=tok_idx, tok_off=tok_off)

    def fit(self, K_dev, n_tokens, sigma=None, center=True, n_dev=None, tok_idx=None, tok_off=None):
        lay = self.layout()
        ws = torch.empty(rk.rk_fit_workspace_size(lay, n_tokens), device=DEV, dtype=torch.uint8)
        out = rk.FitOut(self.R, self.lam, self.mask, self.keep_idx, self.Rr, self.mu, self.dmu, self.cov, self.sweeps)
        rk.rk_fit_rotation(self.ctx, lay, self.rows(K_dev, n_tokens, n_dev, tok_idx, tok_off), sigma,
                           rk.RK_FIT_CENTER if center else 0, out, ws)
        torch.cuda.synchronize()

    def compress(self, K_dev, n_tokens, V_dev=None, n_dev=None, tok_idx=None, tok_off=None, max_len=None):
        lay = self.layout()
        vrows = self.rows(V_dev, n_tokens, n_dev, tok_idx, tok_off) if V_dev is not None else None
        rk.rk_compress(self.ctx, lay, self.rows(K_dev, n_tokens, n_dev, tok_idx, tok_off), self.Rr, self.Kp,
                       vrows, self.Vc if V_dev is not None else None, self.seq_len)
        torch.cuda.synchronize()
        self.max_seq_len = int(max_len if max_len is not None else n_tokens)

    def append(self, k_new, v_new):
        rk.rk_append(self.ctx, self.layout(), k_new, v_new, self.Rr, self.Kp, self.Vc, self.seq_len)
        torch.cuda.synchronize()
        self.max_seq_len += 1

    def append_decode(self, k_new, v_new, q_dev, use_bias=True, scale=0.0):
        """The fused step: append with the frozen rotation, then attend over the longer cache."""
        lay = self.layout()
        after = rk.Layout(self.B, self.Hq, self.Hkv, self.r, rk_dtype(self.dtype), self.cap,
                          min(self.max_seq_len + 1, self.cap), seq_len=self.seq_len)
        ws = torch.empty(rk.rk_decode_workspace_size(self.ctx, after), device=DEV, dtype=torch.uint8)
        rk.rk_append_decode_attn(self.ctx, lay, k_new, v_new, q_dev, self.Rr, self.dmu if use_bias else None,
                                 self.Kp, self.Vc, self.seq_len, scale, self.out, ws)
        torch.cuda.synchronize()
        self.max_seq_len += 1
        return to_host(self.out)

    def decode(self, q_dev, use_bias=True, scale=0.0):
        lay = self.layout()
        ws = torch.empty(rk.rk_decode_workspace_size(self.ctx, lay), device=DEV, dtype=torch.uint8)
        rk.rk_decode_attn(self.ctx, lay, q_dev, self.Kp, self.Vc, self.Rr, self.dmu if use_bias else None, scale,
                          self.out, ws)
        torch.cuda.synchronize()
        return to_host(self.out)
