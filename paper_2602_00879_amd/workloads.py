"""Seeded synthetic inputs shaped like the paper's MoE dLLM workloads.

This module holds NO arithmetic of the method: it only draws random numbers,
rounds them to the storage type and names the shapes.  Both the HIP path's
tests and the CPU oracle's tests take their inputs from here, so that the two
sides see identical bits.

Storage conventions (host side, numpy):
  * fp32 tensors are float32 arrays;
  * bf16 tensors are uint16 arrays holding the bf16 bit patterns (numpy has no
    bf16); `to_f32` / `to_f64` widen either kind exactly.
Layouts (the library's "plain" layout, rows contiguous along the reduction
dimension): x [B, N, D]; w_router [M, D]; bias [M] fp32 or None;
w_gate, w_up [M, F, D]; w_down [M, D, F]; shared expert (wg [Fs, D],
wu [Fs, D], wd [D, Fs]) or None.

The synthetic blocks stand in for the paper's LLaDA2.0-mini / LLaDA-MoE runs
(Sec. 5.1): block length 32, hidden states N(0,1), weights N(0,0.02), and a
Zipf-shaped per-expert router bias that reproduces the concentration of real
routers (Table 1: far fewer unique experts than uniform routing would give).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    name: str
    dtype: str          # "f32" | "bf16"
    n_seqs: int         # B
    n_tokens: int       # N per sequence
    hidden: int         # D
    n_experts: int      # M
    ffn: int            # F
    ffn_shared: int     # Fs (0 = none)
    top_k: int          # K
    coreset: int        # C
    zipf_s: float       # 0 = no router bias
    seed: int
    n_layers: int = 1

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


# The five workloads of the benchmark definition.
CONFIGS: Dict[str, LayerConfig] = {
    "tiny_f32": LayerConfig("tiny_f32", "f32", 1, 8, 256, 16, 128, 0, 2, 4, 0.0, 0),
    "m128_zipf": LayerConfig("m128_zipf", "bf16", 1, 32, 2048, 128, 768, 0, 8, 32, 1.1, 2),
    "m256_shared": LayerConfig("m256_shared", "bf16", 1, 32, 2048, 256, 512, 512, 8, 32, 0.0, 3),
    "m128_sweep": LayerConfig("m128_sweep", "bf16", 1, 32, 2048, 128, 768, 0, 8, 32, 1.1, 4),
    "stack48": LayerConfig("stack48", "bf16", 8, 32, 2048, 128, 768, 0, 8, 32, 1.1, 5, n_layers=48),
}


# ----------------------------------------------------------------------------
# bf16 <-> float helpers (pure type conversion)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round to nearest even); returns uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def to_f32(a: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(a) if a.dtype == np.uint16 else np.asarray(a, dtype=np.float32)


def to_f64(a: np.ndarray) -> np.ndarray:
    return to_f32(a).astype(np.float64)


def _store(a32: np.ndarray, dtype: str) -> np.ndarray:
    return f32_to_bf16_bits(a32) if dtype == "bf16" else np.ascontiguousarray(a32, dtype=np.float32)


def _normal(rng: np.random.Generator, shape, std: float, dtype: str, chunk: int = 1 << 24) -> np.ndarray:
    """N(0, std) in float32, stored as `dtype`; drawn in chunks to bound memory."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16 if dtype == "bf16" else np.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        v = rng.standard_normal(e - s, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        out[s:e] = _store(v, dtype)
    return out.reshape(shape)


def zipf_bias(n_experts: int, s: float, rng: np.random.Generator) -> np.ndarray:
    """Per-expert router bias with Zipf(s) popularity: expert of popularity rank
    r gets ln(r^-s) minus the mean, ranks assigned by a seeded permutation, so
    that the softmax mass of each expert is multiplied by its Zipf popularity."""
    ranks = rng.permutation(n_experts) + 1
    b = -s * np.log(ranks.astype(np.float64))
    return (b - b.mean()).astype(np.float32)


def make_layer(cfg: LayerConfig, layer: int = 0, with_x: bool = True) -> Dict[str, Optional[np.ndarray]]:
    """All tensors of one MoE layer of `cfg`, seeded by (cfg.seed, layer)."""
    rng = np.random.default_rng([cfg.seed, layer])
    B, N, D, M, F = cfg.n_seqs, cfg.n_tokens, cfg.hidden, cfg.n_experts, cfg.ffn
    out: Dict[str, Optional[np.ndarray]] = {}
    out["x"] = _normal(rng, (B, N, D), 1.0, cfg.dtype) if with_x else None
    out["w_router"] = _normal(rng, (M, D), 0.02, cfg.dtype)
    out["bias"] = zipf_bias(M, cfg.zipf_s, rng) if cfg.zipf_s > 0 else None
    out["w_gate"] = _normal(rng, (M, F, D), 0.02, cfg.dtype)
    out["w_up"] = _normal(rng, (M, F, D), 0.02, cfg.dtype)
    out["w_down"] = _normal(rng, (M, D, F), 0.02, cfg.dtype)
    if cfg.ffn_shared > 0:
        Fs = cfg.ffn_shared
        out["shared"] = (_normal(rng, (Fs, D), 0.02, cfg.dtype),
                         _normal(rng, (Fs, D), 0.02, cfg.dtype),
                         _normal(rng, (D, Fs), 0.02, cfg.dtype))
    else:
        out["shared"] = None
    return out


@dataclass(frozen=True)
class AttnConfig:
    """Attention sub-layer around the MoE layer (bf16): H query heads, Hkv key/value
    heads of width dh, n_prefix + n_suffix cached positions (Sec. 5.1 uses 16 + 16)."""
    name: str
    n_seqs: int
    n_tokens: int
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    n_prefix: int
    n_suffix: int
    seed: int


# The per-layer attention shape that goes with the 2048-wide, 128-expert MoE layer of the
# benchmark definition (32 query heads, 4 key/value heads of width 128), and small ones.
ATTN_CONFIGS: Dict[str, AttnConfig] = {
    "attn_block32": AttnConfig("attn_block32", 1, 32, 2048, 32, 4, 128, 16, 16, 31),
    "attn_batch8": AttnConfig("attn_batch8", 8, 32, 2048, 32, 4, 128, 16, 16, 32),
    "attn_small": AttnConfig("attn_small", 1, 8, 256, 4, 2, 64, 3, 2, 33),
    "attn_nocache": AttnConfig("attn_nocache", 3, 20, 256, 4, 4, 32, 0, 0, 34),
    "attn_ragged": AttnConfig("attn_ragged", 2, 70, 384, 8, 2, 48, 5, 9, 35),
    "attn_one_token": AttnConfig("attn_one_token", 1, 1, 128, 2, 1, 64, 7, 0, 36),
    # a long cached context: the per-head values no longer fit the default LDS allowance
    "attn_long_cache": AttnConfig("attn_long_cache", 2, 24, 256, 2, 1, 128, 200, 150, 37),
}


def make_attention(cfg: AttnConfig, layer: int = 0, with_x: bool = True) -> Dict[str, Optional[np.ndarray]]:
    """bf16 tensors of one attention sub-layer, seeded by (cfg.seed, layer): x [B, N, D]
    N(0, 1); wq [H*dh, D], wk, wv [Hkv*dh, D], wo [D, H*dh] N(0, 0.02); cached keys
    and values [B, Hkv, P, dh] N(0, 1) (the scale a projection of N(0, 1) hidden states
    by N(0, 0.02) weights of this width has, to the nearest power of ten)."""
    rng = np.random.default_rng([cfg.seed, layer, 7])
    B, N, D, H, G, dh = cfg.n_seqs, cfg.n_tokens, cfg.hidden, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    P = cfg.n_prefix + cfg.n_suffix
    out: Dict[str, Optional[np.ndarray]] = {}
    out["x"] = _normal(rng, (B, N, D), 1.0, "bf16") if with_x else None
    out["wq"] = _normal(rng, (H * dh, D), 0.02, "bf16")
    out["wk"] = _normal(rng, (G * dh, D), 0.02, "bf16")
    out["wv"] = _normal(rng, (G * dh, D), 0.02, "bf16")
    out["wo"] = _normal(rng, (D, H * dh), 0.02, "bf16")
    out["k_cache"] = _normal(rng, (B, G, P, dh), 1.0, "bf16")
    out["v_cache"] = _normal(rng, (B, G, P, dh), 1.0, "bf16")
    return out


def make_logits(n_tokens: int, n_experts: int, seed: int, zipf_s: float = 0.0,
                scale: float = 1.0) -> np.ndarray:
    """Synthetic fp32 router logits [N, M] for routing-only tests."""
    rng = np.random.default_rng([seed, 977])
    L = rng.standard_normal((n_tokens, n_experts), dtype=np.float32) * np.float32(scale)
    if zipf_s > 0:
        L = L + zipf_bias(n_experts, zipf_s, rng)[None, :]
    return np.ascontiguousarray(L, dtype=np.float32)
