"""The calls of ``binding.Camera`` strung together for one MoE layer: score, decide, apply, run.

Argument marshalling only; every step runs in the HIP library.  A layer is given as a dict with
the tensors of ``inputs.make_layer`` (``X, W_r, bias, W_gate, W_up, W_down`` and, for shared experts,
``Ws_gate, Ws_up, Ws_down``); any caller-made dict of device tensors with those keys works.

  score_layer   Algorithm 1: routing and the energies of every micro-expert of the layer (routed experts first,
                then the shared ones, which every token visits with weight 1)
  prune_layer   Algorithm 2, lines 9-13: the kept micro-experts at a ratio, packed per expert
  CompactLayer  the pruned layer: ``forward`` is Algorithm 2, line 14 (the output recomputed after pruning)
  cameraq_layer / cameraq_dagger_layer   Algorithm 3, lines 5-8 and the colocation of equal precision: the routed
                experts' matrices reordered by precision class, row-wise for W_up / W_gate (CAMERA-Q: a micro-expert
                keeps one precision) or column-wise (the comparison variant CAMERA-Q-dagger: every matrix sliced along
                its input dimension)
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


@dataclasses.dataclass
class MixedPrecisionLayer:
    """The routed experts' matrices with the members of every precision class side by side inside each expert."""
    bits_down: torch.Tensor     # uint8 [N_E * d_ff]: bit width of every W_down column (= micro-expert)
    count_down: torch.Tensor    # int32 [N_E, L]: class sizes per expert
    W_down: torch.Tensor        # flat [N_E][d_model][d_ff]: columns in class order
    bits_in: torch.Tensor       # uint8: bit width of every W_up / W_gate slice (rows = micro-experts, or input columns)
    count_in: torch.Tensor      # int32 [N_E, L]
    W_gate: torch.Tensor        # CAMERA-Q: [N_E * d_ff, d_model] rows in class order; dagger: flat [N_E][d_ff][d_model], columns in class order
    W_up: torch.Tensor
    column_wise: bool


def cameraq_layer(cam, layer: dict, scores: LayerScores, bits, ratios) -> MixedPrecisionLayer:
    """CAMERA-Q on the routed experts: one ranking of the micro-experts, one precision per micro-expert across its
    gate row, up row and down column."""
    nr = scores.n_routed
    d_ff = layer["W_gate"].shape[1]
    energy, seg = scores.energy[:nr * d_ff], scores.seg_offsets[:nr + 1]
    bit_of, count, perm = cam.alloc_bits(energy, seg, bits, ratios, want_perm=True)
    gate, up, down = cam.gather_micro_experts(layer["W_gate"], layer["W_up"], layer["W_down"], perm)
    return MixedPrecisionLayer(bit_of, count, down, bit_of, count, gate, up, False)


def cameraq_dagger_layer(cam, layer: dict, scores: LayerScores, bits, ratios) -> MixedPrecisionLayer:
    """The comparison variant: W_down split by the micro-expert ranking as above, W_up and W_gate sliced along their
    input dimension by the ranking of the input channels diag(X_e^T X_e) (every micro-expert then mixes precisions)."""
    nr = scores.n_routed
    Wg, Wu = layer["W_gate"], layer["W_up"]
    d_ff, d_model = Wg.shape[1], Wg.shape[2]
    energy, seg = scores.energy[:nr * d_ff], scores.seg_offsets[:nr + 1]
    bits_down, count_down, perm_down = cam.alloc_bits(energy, seg, bits, ratios, want_perm=True)
    _, _, down = cam.gather_micro_experts(None, None, layer["W_down"], perm_down)
    h = cam.input_channel_energy(layer["X"], scores.topk_idx, nr)
    seg_in = [e * d_model for e in range(nr + 1)]
    bits_in, count_in, perm_in = cam.alloc_bits(h.view(-1), seg_in, bits, ratios, want_perm=True)
    # columns of W_gate / W_up: the gather's column path, with the matrix in the place of W_down
    _, _, gate = cam.gather_micro_experts(None, None, Wg, perm_in)
    _, _, up = cam.gather_micro_experts(None, None, Wu, perm_in)
    return MixedPrecisionLayer(bits_down, count_down, down, bits_in, count_in, gate, up, True)
