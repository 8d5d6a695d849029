"""Seeded synthetic inputs shaped like the paper's draft/target models.

This module only draws random tensors and conditions them (RMS normalisation,
rounding to the storage dtype).  It holds none of the method's arithmetic: no
projection, no mask, no softmax.  Both the CPU oracle's tests and the HIP
path's tests/benchmark take their inputs from here so that the two sides see
bit-identical stored values.

The paper trains on ShareGPT states of Vicuna/LLaMA targets (section 5.1);
those are not available, so tensors with the same shapes and comparable value
statistics stand in for them.  NumPy only (PCG64 via default_rng).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


# ---------------------------------------------------------------- bf16 I/O
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = ((u + (0x7FFF + ((u >> 16) & 1))) >> 16).astype(np.uint16)
    r[nan] = ((u[nan] >> 16) | 0x0040).astype(np.uint16)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array whose every value is exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(np.shape(x))


def rmsnorm(x: np.ndarray, eps: float = 1e-5) -> np.ndarray:
    """x / sqrt(mean(x^2, last axis) + eps), no gain."""
    x = np.asarray(x, np.float32)
    ms = np.mean(x.astype(np.float64) ** 2, axis=-1, keepdims=True)
    return (x / np.sqrt(ms + eps)).astype(np.float32)


# ---------------------------------------------------------------- configs
@dataclass(frozen=True)
class XattnConfig:
    name: str
    batch: int
    seq_q: int
    seq_kv: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    block_size: int
    block_offset: int
    dtype: str            # "f32" | "bf16"
    seed_base: int
    recipe: str           # "c1" | "llama" | "outlier" | "decode"

    def with_(self, **kw) -> "XattnConfig":
        return replace(self, **kw)


CONFIGS = {
    # tiny fp32 reference problem
    "c1": XattnConfig("c1", 1, 128, 128, 256, 4, 4, 64, 4, 0, "f32", 0, "c1"),
    # Llama-2-7B-shaped draft head
    "c2": XattnConfig("c2", 4, 2048, 2048, 4096, 32, 32, 128, 4, 0, "bf16", 200, "llama"),
    # Llama-3-8B-shaped GQA draft head
    "c3": XattnConfig("c3", 2, 4096, 4096, 4096, 32, 8, 128, 8, 0, "bf16", 300, "llama"),
    # decode-time draft step; seq_q is overridden with M in {1, 8, 32, 64}
    "c4": XattnConfig("c4", 1, 64, 4096, 4096, 32, 32, 128, 1, 0, "bf16", 400, "decode"),
    # 13B-shaped long-context head with outlier channels
    "c5": XattnConfig("c5", 1, 8192, 8192, 5120, 40, 40, 128, 8, 0, "bf16", 500, "outlier"),
}

W_STD = 0.02
N_OUTLIER_CHANNELS = 8
OUTLIER_GAIN = 20.0
OUTLIER_RATE = 0.01


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


def make_inputs(cfg: XattnConfig, *, peaked_queries: bool = False,
                with_dy: bool = True) -> dict:
    """Tensors for one call, float32 arrays holding the stored (already
    rounded) values.  Seeds: seed_base + i for Xq, Xkv, Wq, Wk, Wv, Wo, dY.

    recipe "c1":     Xq, Xkv ~ N(0,1) then rmsnorm.
    recipe "llama":  Xkv ~ N(0,1) * per-token LogNormal(0, 0.5) then rmsnorm;
                     Xq ~ N(0, 0.02^2) (embedding-like, not normalised).
    recipe "outlier":Xkv ~ N(0,1), 1% of positions get 8 fixed channels x20,
                     then rmsnorm; Xq as "llama".
    recipe "decode": Xq (the M draft states) and Xkv (the target states that
                     the cache is projected from) ~ N(0,1) then rmsnorm.
    peaked_queries:  rmsnorm Xq as well, which gives score std > 1 and a
                     non-trivial softmax (the literal "llama" recipe yields
                     nearly uniform attention).
    Weights ~ N(0, 0.02^2); dY ~ N(0,1).
    """
    B, Sq, L, D = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden
    H, G, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    rng = [np.random.default_rng(cfg.seed_base + i) for i in range(7)]
    f32 = np.float32

    if cfg.recipe in ("c1", "decode"):
        xq = rmsnorm(rng[0].standard_normal((B, Sq, D), dtype=f32))
        xkv = rmsnorm(rng[1].standard_normal((B, L, D), dtype=f32))
    else:
        xq = (W_STD * rng[0].standard_normal((B, Sq, D), dtype=f32)).astype(f32)
        xkv = rng[1].standard_normal((B, L, D), dtype=f32)
        if cfg.recipe == "llama":
            tok = rng[1].lognormal(0.0, 0.5, size=(B, L, 1)).astype(f32)
            xkv = xkv * tok
        elif cfg.recipe == "outlier":
            hit = rng[1].random((B, L)) < OUTLIER_RATE
            chans = rng[1].choice(D, size=N_OUTLIER_CHANNELS, replace=False)
            xkv[..., chans] *= np.where(hit[..., None], OUTLIER_GAIN, 1.0).astype(f32)
        else:
            raise ValueError(cfg.recipe)
        xkv = rmsnorm(xkv)
        if peaked_queries:
            xq = rmsnorm(xq)

    out = dict(
        xq=_store(xq, cfg.dtype), xkv=_store(xkv, cfg.dtype),
        wq=_store(W_STD * rng[2].standard_normal((D, H * d), dtype=f32), cfg.dtype),
        wk=_store(W_STD * rng[3].standard_normal((D, G * d), dtype=f32), cfg.dtype),
        wv=_store(W_STD * rng[4].standard_normal((D, G * d), dtype=f32), cfg.dtype),
        wo=_store(W_STD * rng[5].standard_normal((H * d, D), dtype=f32), cfg.dtype),
    )
    if with_dy:
        out["dy"] = _store(rng[6].standard_normal((B, Sq, D), dtype=f32), cfg.dtype)
    return out


def make_block_inputs(cfg: XattnConfig, ffn: int) -> dict:
    """Tensors for the whole draft block (section 4.1, Eq. 1), float32 arrays of
    stored values.  Unlike make_inputs the activations are NOT normalised (the
    block does that): e ~ N(0, 0.02^2) like an embedding table's rows, hs ~
    3 * N(0,1) * per-token LogNormal(0, 0.5) like a target model's top hidden
    states.  All seven weight matrices ~ N(0, 0.02^2), gains ~ 1 + 0.1 N(0,1),
    dh ~ N(0,1).  Seeds: seed_base + 20 + i in the order below."""
    B, Sq, L, D = cfg.batch, cfg.seq_q, cfg.seq_kv, cfg.hidden
    H, G, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    f32 = np.float32
    rng = [np.random.default_rng(cfg.seed_base + 20 + i) for i in range(14)]
    n = lambda i, *shape: rng[i].standard_normal(shape, dtype=f32)
    hs = 3.0 * n(1, B, L, D) * rng[1].lognormal(0.0, 0.5, size=(B, L, 1)).astype(f32)
    t = dict(e=W_STD * n(0, B, Sq, D), hs=hs,
             wq=W_STD * n(2, D, H * d), wk=W_STD * n(3, D, G * d), wv=W_STD * n(4, D, G * d), wo=W_STD * n(5, H * d, D),
             w_gate=W_STD * n(6, D, ffn), w_up=W_STD * n(7, D, ffn), w_down=W_STD * n(8, ffn, D),
             g_q=1.0 + 0.1 * n(9, D), g_kv=1.0 + 0.1 * n(10, D), g_mlp=1.0 + 0.1 * n(11, D),
             dh=n(12, B, Sq, D))
    return {k: _store(v, cfg.dtype) for k, v in t.items()}
