"""Seeded synthetic inputs drawn directly on the GPU, for workloads too large
to draw on the host (the 48-layer stack holds about 58 GB of expert weights).
Like `workloads`, this module holds no arithmetic of the method: it only draws
random numbers, rounds them to the storage type and names the shapes."""
from __future__ import annotations

from typing import Dict

import numpy as np
import torch

from . import workloads as W


def _randn_bf16(shape, std: float, gen: torch.Generator, device) -> torch.Tensor:
    """N(0, std) drawn in fp32, rounded once to bf16; drawn slice by slice along
    dim 0 to bound the fp32 temporary."""
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    for i in range(shape[0]):
        t = torch.randn(shape[1:], generator=gen, dtype=torch.float32, device=device)
        out[i] = (t * std).to(torch.bfloat16)
    return out


def make_stack(cfg: W.LayerConfig, device="cuda") -> Dict[str, torch.Tensor]:
    """Layer-stacked tensors of `cfg.n_layers` layers, seeded per layer by
    (cfg.seed, layer): w_router [L,M,D], bias [L,M] fp32 (Zipf popularity, drawn
    on the host like the single-layer workloads), w_gate/w_up [L,M,F,D],
    w_down [L,M,D,F], x [B,N,D].

    There is no normalisation layer in this stack (attention and norms are
    left out), so with N(0, 0.02) everywhere the residual stream would grow
    layer over layer until bf16 overflows; as GPT-style residual stacks do, the
    projection that writes into the residual stream (w_down) is drawn with
    std 0.02 / sqrt(2 L)."""
    assert cfg.dtype == "bf16"
    L, B, N, D, M, F = cfg.n_layers, cfg.n_seqs, cfg.n_tokens, cfg.hidden, cfg.n_experts, cfg.ffn
    out: Dict[str, torch.Tensor] = {}
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed * 100003 + 17)
    out["x"] = (torch.randn((B, N, D), generator=gen, dtype=torch.float32, device=device)).to(torch.bfloat16)
    out["w_router"] = torch.empty((L, M, D), dtype=torch.bfloat16, device=device)
    out["w_gate"] = torch.empty((L, M, F, D), dtype=torch.bfloat16, device=device)
    out["w_up"] = torch.empty((L, M, F, D), dtype=torch.bfloat16, device=device)
    out["w_down"] = torch.empty((L, M, D, F), dtype=torch.bfloat16, device=device)
    bias = np.zeros((L, M), dtype=np.float32)
    for l in range(L):
        gen.manual_seed(cfg.seed * 100003 + 1000 + l)
        out["w_router"][l] = (torch.randn((M, D), generator=gen, dtype=torch.float32, device=device) * 0.02).to(torch.bfloat16)
        down_std = 0.02 / float(np.sqrt(2.0 * L)) if L > 1 else 0.02
        for name, shp, std in (("w_gate", (M, F, D), 0.02), ("w_up", (M, F, D), 0.02),
                               ("w_down", (M, D, F), down_std)):
            out[name][l] = _randn_bf16(shp, std, gen, device)
        if cfg.zipf_s > 0:
            bias[l] = W.zipf_bias(M, cfg.zipf_s, np.random.default_rng([cfg.seed, l]))
    out["bias"] = torch.from_numpy(bias).to(device) if cfg.zipf_s > 0 else None
    return out


def make_decoder_attention(cfg: W.LayerConfig, attn: W.AttnConfig, device="cuda") -> Dict[str, torch.Tensor]:
    """Layer-stacked attention tensors for `cfg.n_layers` decoder layers: wq [L, H*dh, D],
    wk, wv [L, Hkv*dh, D], wo [L, D, H*dh], k_cache, v_cache [L, B, Hkv, P, dh].  As for
    w_down in make_stack, the projection that writes into the residual stream (wo) is
    drawn with std 0.02 / sqrt(2 L)."""
    L, B, D = cfg.n_layers, cfg.n_seqs, cfg.hidden
    H, G, dh, P = attn.n_heads, attn.n_kv_heads, attn.head_dim, attn.n_prefix + attn.n_suffix
    assert (attn.n_seqs, attn.n_tokens, attn.hidden) == (cfg.n_seqs, cfg.n_tokens, cfg.hidden)
    gen = torch.Generator(device=device)
    gen.manual_seed(attn.seed * 100003 + 29)
    o_std = 0.02 / float(np.sqrt(2.0 * L)) if L > 1 else 0.02
    out = {
        "wq": _randn_bf16((L, H * dh, D), 0.02, gen, device),
        "wk": _randn_bf16((L, G * dh, D), 0.02, gen, device),
        "wv": _randn_bf16((L, G * dh, D), 0.02, gen, device),
        "wo": _randn_bf16((L, D, H * dh), o_std, gen, device),
        "k_cache": _randn_bf16((L, B, G, P, dh), 1.0, gen, device),
        "v_cache": _randn_bf16((L, B, G, P, dh), 1.0, gen, device),
    }
    return out
