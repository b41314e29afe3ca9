"""GPU parity of the comparison variant CAMERA-Q-dagger (column-wise slicing of all three matrices): the
input-channel energies against the oracle, then bit widths, class sizes and the column reordering bit-exact on
the same float32 energies, through the same calls pipeline.cameraq_dagger_layer strings together."""
import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc
from paper_2508_02322_amd import inputs, pipeline
from tests import helpers as H

pytestmark = pytest.mark.gpu
# float32 sums of at most a few thousand squares of exactly represented inputs: about sqrt(n) * 2^-24 relative;
# asserted at 1e-4 (the score tolerance 2e-3 would hide a dropped token among thousands)
TOL = 1e-4

CASES = [
    dict(n_tokens=700, d_model=256, d_ff=96, n_experts=8, top_k=2),
    dict(n_tokens=37, d_model=72, d_ff=40, n_experts=3, top_k=2),                       # ragged everything
    dict(n_tokens=2048, d_model=1000, d_ff=64, n_experts=64, top_k=6),
    dict(n_tokens=300, d_model=100, d_ff=52, n_experts=6, top_k=3, dtype="f32"),
    dict(n_tokens=1500, d_model=640, d_ff=48, n_experts=128, top_k=8, router_bias="zipf"),   # experts without tokens
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_input_channel_energy_matches_oracle(cam, case):
    cfg = inputs.scaled(inputs.CONFIGS["mixtral"], n_layers=1, outlier_channels=2, **case)
    layer = inputs.make_layer(cfg, 0)
    dev = H.to_dev(layer)
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    h = cam.input_channel_energy(dev["X"], idx, cfg.n_experts)
    A = orc.dense_routing(idx.cpu().numpy(), np.ones(idx.shape), cfg.n_experts)
    want = orc.input_channel_energy(H.f64(layer["X"]), A)
    got = h.cpu().numpy().astype(np.float64)
    assert got.shape == want.shape
    assert H.rel_err(got, want, max(want.max() * 1e-9, 1e-300)) <= TOL
    assert np.array_equal(got == 0, want == 0)
    # every token through one "expert": the plain column sums of squares; no tokens: zeros
    dense = cam.input_channel_energy(dev["X"], None, 1).cpu().numpy().astype(np.float64)
    want_dense = orc.input_channel_energy(H.f64(layer["X"]), np.ones((cfg.n_tokens, 1)))
    assert H.rel_err(dense, want_dense, want_dense.max() * 1e-9) <= TOL
    none = cam.input_channel_energy(dev["X"][:0], idx[:0], cfg.n_experts)
    assert torch.all(none == 0)
    again = cam.input_channel_energy(dev["X"], idx, cfg.n_experts)
    assert torch.equal(h, again)                       # fixed summation order


def test_dagger_layer_matches_oracle(cam):
    cfg = inputs.scaled(inputs.CONFIGS["deepseek-moe-16b"], n_tokens=900, d_model=192, d_ff=136, n_experts=12, top_k=4,
                        n_shared=0, d_ff_shared=0, n_layers=1)
    layer = inputs.make_layer(cfg, 1)
    dev = H.to_dev(layer)
    scores = pipeline.score_layer(cam, dev, cfg.top_k, cfg.alpha)
    bits, ratios = [4, 3, 2], [0.1, 0.3, 0.6]
    mp = pipeline.cameraq_dagger_layer(cam, dev, scores, bits, ratios)
    torch.cuda.synchronize()
    ne, f, d = cfg.n_experts, cfg.d_ff, cfg.d_model
    # W_down: CAMERA-Q's own split, on the GPU's energies
    E = scores.energy.cpu().numpy()
    o_bits, o_count, o_perm = orc.alloc_bits(E, scores.seg_offsets, bits, ratios)
    np.testing.assert_array_equal(mp.bits_down.cpu().numpy(), o_bits)
    np.testing.assert_array_equal(mp.count_down.cpu().numpy(), o_count)
    raw = lambda t: t.view(torch.int16).cpu().numpy()          # bf16 bit patterns: the gather copies, never recomputes
    down = orc.gather_columns(raw(layer["W_down"]), o_perm, np.full(ne, f))
    np.testing.assert_array_equal(raw(mp.W_down).reshape(ne, d, f), np.stack(down))
    # W_up / W_gate: input channels ranked by the GPU's h, sliced column-wise
    h = cam.input_channel_energy(dev["X"], scores.topk_idx, ne).cpu().numpy().ravel()
    seg_in = [e * d for e in range(ne + 1)]
    i_bits, i_count, i_perm = orc.alloc_bits(h, seg_in, bits, ratios)
    np.testing.assert_array_equal(mp.bits_in.cpu().numpy(), i_bits)
    np.testing.assert_array_equal(mp.count_in.cpu().numpy(), i_count)
    for name, got in (("W_gate", mp.W_gate), ("W_up", mp.W_up)):
        want = orc.gather_columns(raw(layer[name]), i_perm, np.full(ne, d))
        np.testing.assert_array_equal(raw(got).reshape(ne, f, d), np.stack(want))
    assert mp.column_wise
    # and the row-wise method on the same layer: one precision per micro-expert across the three matrices
    q = pipeline.cameraq_layer(cam, dev, scores, bits, ratios)
    gate, up, down_q = orc.gather_micro_experts(raw(layer["W_gate"]), raw(layer["W_up"]), raw(layer["W_down"]), o_perm,
                                                np.full(ne, f))
    np.testing.assert_array_equal(raw(q.W_gate), gate)
    np.testing.assert_array_equal(raw(q.W_up), up)
    np.testing.assert_array_equal(raw(q.W_down).reshape(ne, d, f), np.stack(down_q))
