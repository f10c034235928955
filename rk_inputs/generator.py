"""Counter-based (Philox) seeded generators for Keys, Values, queries, ragged
lengths and token-keep lists.  No method arithmetic lives here."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_M64 = (1 << 64) - 1

# tensor tags: one independent Philox stream per (config, layer, b, h, tag)
TAG_A, TAG_B, TAG_E, TAG_OUT, TAG_V, TAG_Q, TAG_KNEW, TAG_VNEW, TAG_LEN, TAG_KEEP, TAG_SIGMA = range(11)


def _splitmix64(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _M64
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def stream(config_id: int, layer: int, b: int, h: int, tag: int) -> np.random.Generator:
    """Independent generator for one tensor of one head."""
    s = 0
    for v in (config_id, layer, b, h, tag):
        s = _splitmix64(s ^ (int(v) & _M64))
    key = [s, _splitmix64(s)]
    return np.random.Generator(np.random.Philox(key=np.array(key, dtype=np.uint64)))


# ----------------------------------------------------------------------------
# bf16 storage rounding (round-to-nearest-even on the fp32 bit pattern)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array holding bf16-representable values."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = x.astype(np.float32)
    if dtype == "bf16":
        return bf16_round(x)
    if dtype == "f32":
        return x
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class HeadSpec:
    """Key generator parameters for one head."""
    L: int
    d: int = 128
    rho: int = 16
    noise: float = 0.1
    n_outlier: int = 2
    outlier_scale: float = 10.0
    mean_shift: float = 0.0   # constant added on the outlier channels
    offset_all: float = 0.0   # constant added on every channel


def make_keys(spec: HeadSpec, dtype: str, config_id: int, layer: int, b: int, h: int) -> np.ndarray:
    """[L, d] fp32 array of storage-dtype-representable Key values."""
    A = stream(config_id, layer, b, h, TAG_A).standard_normal((spec.L, spec.rho), dtype=np.float32)
    Bm = stream(config_id, layer, b, h, TAG_B).standard_normal((spec.rho, spec.d), dtype=np.float32)
    K = A @ Bm
    if spec.noise != 0.0:
        E = stream(config_id, layer, b, h, TAG_E).standard_normal((spec.L, spec.d), dtype=np.float32)
        K += np.float32(spec.noise) * E
    if spec.n_outlier > 0:
        ch = stream(config_id, layer, b, h, TAG_OUT).choice(spec.d, size=spec.n_outlier, replace=False)
        K[:, ch] *= np.float32(spec.outlier_scale)
        if spec.mean_shift != 0.0:
            K[:, ch] += np.float32(spec.mean_shift)
    if spec.offset_all != 0.0:
        K += np.float32(spec.offset_all)
    return _store(K, dtype)


def make_normal(shape, dtype: str, config_id: int, layer: int, b: int, h: int, tag: int) -> np.ndarray:
    x = stream(config_id, layer, b, h, tag).standard_normal(shape, dtype=np.float32)
    return _store(x, dtype)


def make_layer(cfg: dict, layer: int = 0, *, lengths=None, spec_overrides: dict | None = None):
    """All tensors of one layer for a config dict from CONFIGS.

    Returns dict with K [B,Hkv,L,d], V [B,Hkv,L,d], q [B,Hq,d],
    k_new/v_new [B,Hkv,d] (fp32 arrays of storage-representable values).
    With `lengths` (one per batch item) rows past a sequence's length are zero.
    """
    B, Hq, Hkv, d, L = cfg["batch"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["L"]
    cid, dtype = cfg["id"], cfg["dtype"]
    rho = cfg.get("rho", 16)
    if "rho_by_layer" in cfg:
        rho = cfg["rho_by_layer"](layer)
    kw = dict(d=d, rho=rho)
    kw.update(spec_overrides or {})
    K = np.zeros((B, Hkv, L, d), np.float32)
    V = np.zeros((B, Hkv, L, d), np.float32)
    for b in range(B):
        Lb = L if lengths is None else int(lengths[b])
        for h in range(Hkv):
            K[b, h, :Lb] = make_keys(HeadSpec(L=Lb, **kw), dtype, cid, layer, b, h)
            V[b, h, :Lb] = make_normal((Lb, d), dtype, cid, layer, b, h, TAG_V)
    q = np.stack([np.stack([make_normal((d,), dtype, cid, layer, b, h, TAG_Q) for h in range(Hq)]) for b in range(B)])
    k_new = np.stack([np.stack([make_keys(HeadSpec(L=1, **kw), dtype, cid + 1000, layer, b, h)[0]
                                for h in range(Hkv)]) for b in range(B)])
    v_new = np.stack([np.stack([make_normal((d,), dtype, cid, layer, b, h, TAG_VNEW) for h in range(Hkv)])
                      for b in range(B)])
    return dict(K=K, V=V, q=q, k_new=k_new, v_new=v_new)


def ragged_lengths(config_id: int, batch: int, lo: int, hi: int) -> np.ndarray:
    """Per-sequence lengths, integer-uniform in [lo, hi]."""
    return stream(config_id, 0, 0, 0, TAG_LEN).integers(lo, hi + 1, size=batch).astype(np.int32)


def token_keep_lists(config_id: int, lengths, n_text: int = 64, keep_frac: float = 0.5):
    """Joint token+channel pruning stand-in: the last `n_text` rows of each
    sequence are text (always kept); of the visual rows before them a seeded
    `keep_frac` subset is kept.  Returns (tok_idx int32 concatenated, ascending
    per sequence; tok_off int64 [B+1])."""
    idx, off = [], [0]
    for b, Lb in enumerate(lengths):
        Lb = int(Lb)
        n_vis = max(Lb - n_text, 0)
        n_keep = int(round(keep_frac * n_vis))
        g = stream(config_id, 0, b, 0, TAG_KEEP)
        vis = np.sort(g.choice(n_vis, size=n_keep, replace=False)) if n_vis > 0 else np.zeros(0, np.int64)
        rows = np.concatenate([vis, np.arange(n_vis, Lb)]).astype(np.int32)
        idx.append(rows)
        off.append(off[-1] + rows.size)
    return np.concatenate(idx).astype(np.int32), np.asarray(off, dtype=np.int64)


# The five workload shapes (tiny fp32; LLaVA-NeXT-7B-shaped MHA; GQA long
# context; ragged joint token+channel pruning; 32-layer prefill+decode).
CONFIGS = {
    "C1": dict(id=1, dtype="f32", batch=1, n_q_heads=2, n_kv_heads=2, head_dim=128, L=512, keep=32),
    "C2": dict(id=2, dtype="bf16", batch=1, n_q_heads=32, n_kv_heads=32, head_dim=128, L=2944, keep=64),
    "C3": dict(id=3, dtype="bf16", batch=8, n_q_heads=28, n_kv_heads=4, head_dim=128, L=16384, keep=64,
               keep_sweep=(32, 64, 96)),
    "C4": dict(id=4, dtype="bf16", batch=16, n_q_heads=32, n_kv_heads=32, head_dim=128, L=32768, keep=64,
               ragged=(1024, 32768), n_text=64, token_keep=0.5),
    "C5": dict(id=5, dtype="bf16", batch=1, n_q_heads=32, n_kv_heads=32, head_dim=128, L=32768, keep=48,
               n_layers=32, decode_steps=128, rho_by_layer=lambda layer: 8 + int(round(24 * layer / 31))),
}
