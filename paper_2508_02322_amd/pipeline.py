"""The calls of ``binding.Camera`` strung together for one MoE layer: score, decide, apply, run.

Argument marshalling only; every step runs in the HIP library.  A layer is given as a dict with
the tensors of ``inputs.make_layer`` (``X, W_r, bias, W_gate, W_up, W_down`` and, for shared experts,
``Ws_gate, Ws_up, Ws_down``); any caller-made dict of device tensors with those keys works.

  score_layer   Algorithm 1: routing and the energies of every micro-expert of the layer (routed experts first,
                then the shared ones, which every token visits with weight 1)
  prune_layer   Algorithm 2, lines 9-13: the kept micro-experts at a ratio, packed per expert
  CompactLayer  the pruned layer: ``forward`` is Algorithm 2, line 14 (the output recomputed after pruning)
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import torch


@dataclasses.dataclass
class LayerScores:
    topk_idx: torch.Tensor      # int32 [n, k]
    topk_w: torch.Tensor        # float32 [n, k]
    phi2: torch.Tensor          # float32 [n_micro]: routed experts, then shared
    phi_inf: torch.Tensor
    omega2: torch.Tensor
    energy: torch.Tensor
    seg_offsets: List[int]      # expert boundaries inside the vectors above
    n_routed: int               # routed experts
    n_shared: int


def _shared(layer):
    ws = layer.get("Ws_gate")
    return None if ws is None else (layer["Ws_gate"], layer["Ws_up"], layer["Ws_down"])


def score_layer(cam, layer: dict, top_k: int, alpha: float, renorm: bool = True) -> LayerScores:
    X = layer["X"]
    Wg = layer["W_gate"]
    n_routed, d_ff, _ = Wg.shape
    shared = _shared(layer)
    n_shared, d_ff_s = (0, 0) if shared is None else (shared[0].shape[0], shared[0].shape[1])
    n_micro = n_routed * d_ff + n_shared * d_ff_s
    out = {k: torch.empty(n_micro, dtype=torch.float32, device=X.device) for k in ("phi2", "phi_inf", "omega2", "energy")}
    nr = n_routed * d_ff
    idx, w = cam.route_topk(X, layer["W_r"], layer.get("bias"), top_k, renorm)
    cam.score_layer(X, idx, w, Wg, layer["W_up"], layer["W_down"], alpha, out={k: v[:nr] for k, v in out.items()})
    if shared is not None:
        cam.score_layer(X, None, None, shared[0], shared[1], shared[2], alpha, out={k: v[nr:] for k, v in out.items()})
    seg = [e * d_ff for e in range(n_routed + 1)] + [nr + (s + 1) * d_ff_s for s in range(n_shared)]
    return LayerScores(idx, w, out["phi2"], out["phi_inf"], out["omega2"], out["energy"], seg, n_routed, n_shared)


@dataclasses.dataclass
class CompactLayer:
    counts: List[int]           # kept micro-experts per expert: routed, then shared
    n_shared: int
    row_align: int              # row alignment of the W_down blocks
    W_gate: torch.Tensor        # [sum(counts), d_model]
    W_up: torch.Tensor
    W_down: torch.Tensor        # flat: one [d_model][ld(e)] block per expert
    keep_mask: torch.Tensor     # uint8 [n_micro]: what was kept
    kept_idx: torch.Tensor      # int32 [sum(counts)]: the kept micro-experts' indices, ascending

    def forward(self, cam, X, topk_idx, topk_w, Y: Optional[torch.Tensor] = None, accumulate: bool = False):
        """The pruned layer's output for tokens X with routing (topk_idx, topk_w)."""
        return cam.layer_forward_compact(X, topk_idx, topk_w, self.counts, self.W_gate, self.W_up, self.W_down,
                                         n_shared=self.n_shared, down_row_align=self.row_align, Y=Y, accumulate=accumulate)


def prune_layer(cam, layer: dict, scores: LayerScores, ratio: float, row_align: int = 64) -> CompactLayer:
    """Keeps the top (1 - ratio) of the layer's micro-experts by energy and packs their vectors."""
    keep, per, kept_idx, _ = cam.select_prune(scores.energy, scores.seg_offsets, ratio, want_idx=True)
    counts = per.cpu()                                   # the only host round trip: the packed sizes
    ld = (counts + (row_align - 1)) // row_align * row_align
    kept = int(counts.sum())
    Wg = layer["W_gate"]
    d = Wg.shape[2]
    gate_c = torch.empty((kept, d), dtype=Wg.dtype, device=Wg.device)
    up_c = torch.empty_like(gate_c)
    down_c = torch.empty(int(ld.sum()) * d, dtype=Wg.dtype, device=Wg.device)
    groups = [(Wg, layer["W_up"], layer["W_down"], 0, scores.n_routed)]
    shared = _shared(layer)
    if shared is not None:
        groups.append((shared[0], shared[1], shared[2], scores.n_routed, scores.n_shared))
    pos = pos_ld = 0
    for g, u, dn, seg0, n_e in groups:
        n_idx, n_ld = int(counts[seg0:seg0 + n_e].sum()), int(ld[seg0:seg0 + n_e].sum())
        cam.gather_micro_experts(g, u, dn, kept_idx[pos:pos + n_idx], per[seg0:seg0 + n_e], scores.seg_offsets[seg0],
                                 down_row_align=row_align,
                                 out=(gate_c[pos:pos + n_idx], up_c[pos:pos + n_idx], down_c[pos_ld * d:(pos_ld + n_ld) * d]))
        pos, pos_ld = pos + n_idx, pos_ld + n_ld
    return CompactLayer(counts.tolist(), scores.n_shared, row_align, gate_c, up_c, down_c, keep, kept_idx[:kept])
