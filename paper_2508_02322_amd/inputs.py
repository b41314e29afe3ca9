"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random tensors of the stated shapes and value
distributions; it contains none of the method's arithmetic.  The HIP path and
the CPU oracle both consume the tensors it returns (the oracle after an exact
up-conversion to float64), so both always see the same bytes.

The tensors stand in for the calibration activations and trained weights of
the models the paper analyses (its calibration set is 128 sequences of 2048
tokens of Wikitext2, "Experimental Setup"); neither those activations nor the
weights exist here.

Layout of what ``make_layer`` returns (all row-major, contiguous):
  X       [n, d_model]                 hidden states entering the MoE layer
  W_r     [N_E, d_model]               router weight R
  bias    [N_E] float32 or None        router logit bias
  W_gate  [N_E, d_ff, d_model]         row c of expert e = gate row of micro-expert (e, c)
  W_up    [N_E, d_ff, d_model]
  W_down  [N_E, d_model, d_ff]         column c of expert e = down column of micro-expert (e, c)
  Ws_gate / Ws_up / Ws_down            the same three for the shared experts (or None)
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    name: str
    seed: int
    n_layers: int
    n_tokens: int
    d_model: int
    d_ff: int
    n_experts: int
    top_k: int
    dtype: str = "bf16"            # "bf16" or "f32"
    n_shared: int = 0
    d_ff_shared: int = 0
    alpha: float = 0.95            # balance coefficient used by the paper for this family
    outlier_channels: int = 0      # hidden channels scaled by `outlier_scale`
    outlier_scale: float = 20.0
    router_bias: str = "none"      # "none" | "normal" | "zipf"
    w_std: float = 0.02
    # > 0: every down column (e, c) is scaled by exp(energy_spread * (z_e + z_ec)), z ~ N(0, 1) per expert and per
    # micro-expert: energies spread over orders of magnitude and the experts keep very different numbers of
    # micro-experts, as the paper reports for trained models ("highly non-uniform" energy distribution; the
    # per-expert pruning ratios of its figures).  0: i.i.d. weights, all micro-experts statistically alike.
    energy_spread: float = 0.0

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def n_micro_routed(self):
        return self.n_experts * self.d_ff

    @property
    def n_micro(self):
        return self.n_experts * self.d_ff + self.n_shared * self.d_ff_shared

    def gemm_flops_per_layer(self):
        """4*d_model*d_ff per routed (token, expert) pair plus the shared experts on every token."""
        routed = 4.0 * self.d_model * self.d_ff * self.n_tokens * self.top_k
        shared = 4.0 * self.d_model * self.d_ff_shared * self.n_shared * self.n_tokens
        return routed + shared


CONFIGS = {
    "tiny": LayerConfig("tiny", seed=0, n_layers=1, n_tokens=512, d_model=256, d_ff=512,
                        n_experts=8, top_k=2, dtype="f32"),
    "mixtral": LayerConfig("mixtral", seed=1, n_layers=1, n_tokens=4096, d_model=4096, d_ff=14336,
                           n_experts=8, top_k=2, outlier_channels=8, router_bias="normal"),
    "deepseek-moe-16b": LayerConfig("deepseek-moe-16b", seed=2, n_layers=28, n_tokens=8192,
                                    d_model=2048, d_ff=1408, n_experts=64, top_k=6,
                                    n_shared=2, d_ff_shared=1408),
    "qwen2-57b-a14b": LayerConfig("qwen2-57b-a14b", seed=3, n_layers=28, n_tokens=8192,
                                  d_model=3584, d_ff=2560, n_experts=64, top_k=8,
                                  n_shared=1, d_ff_shared=20480, outlier_channels=8),
    "qwen3-30b-a3b": LayerConfig("qwen3-30b-a3b", seed=4, n_layers=48, n_tokens=16384,
                                 d_model=2048, d_ff=768, n_experts=128, top_k=8,
                                 alpha=1.0, router_bias="zipf"),
}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of a configuration with some sizes replaced (parity tests use reduced copies)."""
    return dataclasses.replace(cfg, **kw)


def _generator(cfg: LayerConfig, layer: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed * 1000003 + layer)
    return g


def _normal(shape, std, dtype, g, device, chunk_rows=None):
    """N(0, std) drawn in float32 and rounded once to `dtype`; large tensors are filled
    slab by slab along the first axis so that the float32 temporary stays small."""
    out = torch.empty(shape, dtype=dtype, device=device)
    if len(shape) == 1 or chunk_rows is None:
        out.copy_(torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std)
        return out
    for lo in range(0, shape[0], chunk_rows):
        hi = min(shape[0], lo + chunk_rows)
        slab = torch.randn((hi - lo,) + tuple(shape[1:]), generator=g, device=device, dtype=torch.float32)
        out[lo:hi].copy_(slab * std)
    return out


def make_layer(cfg: LayerConfig, layer: int = 0, device="cpu") -> dict:
    """Draw every tensor of one MoE layer.  The stream of draws depends on
    (cfg.seed, layer, device type) only."""
    device = torch.device(device)
    g = _generator(cfg, layer, device)
    dt = cfg.torch_dtype
    n, d, f, ne = cfg.n_tokens, cfg.d_model, cfg.d_ff, cfg.n_experts

    X32 = torch.randn((n, d), generator=g, device=device, dtype=torch.float32)
    if cfg.outlier_channels:
        ch = torch.randperm(d, generator=g, device=device)[:cfg.outlier_channels]
        X32[:, ch] *= cfg.outlier_scale          # same channels for every token
    X = X32.to(dt)
    del X32
    W_r = _normal((ne, d), cfg.w_std, dt, g, device)
    bias: Optional[torch.Tensor] = None
    if cfg.router_bias == "normal":
        bias = torch.randn((ne,), generator=g, device=device, dtype=torch.float32)
    elif cfg.router_bias == "zipf":
        order = torch.randperm(ne, generator=g, device=device)
        bias = torch.empty((ne,), device=device, dtype=torch.float32)
        bias[order] = -torch.log1p(torch.arange(ne, device=device, dtype=torch.float32))
    out = {"X": X, "W_r": W_r, "bias": bias,
           "W_gate": _normal((ne, f, d), cfg.w_std, dt, g, device, chunk_rows=max(1, ne // 8)),
           "W_up": _normal((ne, f, d), cfg.w_std, dt, g, device, chunk_rows=max(1, ne // 8)),
           "W_down": _normal((ne, d, f), cfg.w_std, dt, g, device, chunk_rows=max(1, ne // 8)),
           "Ws_gate": None, "Ws_up": None, "Ws_down": None}
    if cfg.n_shared:
        fs, ns = cfg.d_ff_shared, cfg.n_shared
        out["Ws_gate"] = _normal((ns, fs, d), cfg.w_std, dt, g, device)
        out["Ws_up"] = _normal((ns, fs, d), cfg.w_std, dt, g, device)
        out["Ws_down"] = _normal((ns, d, fs), cfg.w_std, dt, g, device)
    if cfg.energy_spread > 0:      # drawn after everything else: the other tensors do not depend on it
        for key, n_e, width in (("W_down", ne, f), ("Ws_down", cfg.n_shared, cfg.d_ff_shared)):
            if n_e == 0:
                continue
            z = torch.randn((n_e, 1, 1), generator=g, device=device) + torch.randn((n_e, 1, width), generator=g, device=device)
            scale = torch.exp(cfg.energy_spread * z)
            for e in range(n_e):   # expert by expert: the float32 temporary stays small
                out[key][e] = (out[key][e].float() * scale[e]).to(dt)
    return out


def segment_offsets(cfg: LayerConfig) -> list:
    """Expert boundaries of the per-layer energy vector: routed experts first, then shared."""
    seg = [e * cfg.d_ff for e in range(cfg.n_experts + 1)]
    for s in range(cfg.n_shared):
        seg.append(seg[-1] + cfg.d_ff_shared)
    return seg


def energy_like(n_micro: int, seed: int, zero_fraction=0.05, tie_fraction=0.02, device="cpu") -> torch.Tensor:
    """A float32 vector shaped like a layer's energies for the rank-kernel tests:
    heavy-tailed positive values, a block of exact zeros (experts without
    tokens) and some repeated values (ties)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    E = torch.randn(n_micro, generator=g).square_() * torch.randn(n_micro, generator=g).square_()
    nz = int(n_micro * zero_fraction)
    nt = int(n_micro * tie_fraction)
    if nz:
        E[torch.randperm(n_micro, generator=g)[:nz]] = 0.0
    if nt and n_micro > 1:
        E[torch.randperm(n_micro, generator=g)[:nt]] = E[n_micro // 2].item()
    return E.to(device)
