"""Parity at the full sizes of the benchmark configurations, element by element.

* one layer of every bf16 configuration (first, middle and last layer of the Qwen2-shaped one) through the
  calls and launch shapes that bench.py times: every micro-expert's phi2, phi_inf, omega2 and energy against
  the oracle on the same bytes, then the CAMERA-P masks / CAMERA-Q bit widths by the decidable-band rule
  against the oracle's energies.  The library context is fresh and its workspace has first been used by a
  call on different inputs, so a tile that a launch skipped would read another call's partial statistics
  and fail;
* every layer of the Qwen2-shaped configuration on 64 sampled micro-experts per expert.
"""
import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc
from paper_2508_02322_amd import binding, inputs
from tests import helpers as H
from tests.test_gpu_configs import check_decisions, run_layer

pytestmark = pytest.mark.gpu
TOL = 2e-3


class _PerExpertF64:
    """Expert e of a [N_E, rows, cols] device tensor as an exact float64 array, converted when asked for
    (a whole layer in float64 would be tens of GB)."""

    def __init__(self, t):
        self.t = t

    def __getitem__(self, e):
        return H.f64(self.t[e])


def _poison_workspace(cam, cfg, dev):
    """A scoring call of the same shapes on other hidden states and other routing: the workspace of `cam`
    then holds partial statistics that belong to no micro-expert of the layer under test."""
    g = torch.Generator(device="cuda").manual_seed(99)
    X = (torch.randn(dev["X"].shape, generator=g, device="cuda") * 3.0).to(dev["X"].dtype)
    idx, w = cam.route_topk(X, dev["W_r"], None, cfg.top_k)
    cam.score_layer(X, idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], cfg.alpha)
    if cfg.n_shared:
        cam.score_layer(X, None, None, dev["Ws_gate"], dev["Ws_up"], dev["Ws_down"], cfg.alpha)
    torch.cuda.synchronize()


FULL_LAYERS = [("mixtral", 0), ("deepseek-moe-16b", 27), ("qwen2-57b-a14b", 0), ("qwen2-57b-a14b", 13),
               ("qwen2-57b-a14b", 27), ("qwen3-30b-a3b", 47)]


@pytest.mark.parametrize("name,layer_idx", FULL_LAYERS, ids=[f"{n}-layer{l}" for n, l in FULL_LAYERS])
def test_full_size_layer_every_micro_expert(name, layer_idx):
    cfg = inputs.CONFIGS[name]
    print(f"full-size parity: {name} layer {layer_idx}", flush=True)
    cam = binding.Camera(device=0)
    dev = inputs.make_layer(cfg, layer_idx, device="cuda")      # the bytes bench.py would time
    _poison_workspace(cam, cfg, dev)
    idx, w, out = run_layer(cam, cfg, dev)

    # routing: every token against the oracle, by the margin rule
    host = {"X": dev["X"].cpu(), "W_r": dev["W_r"].cpu(), "bias": None if dev["bias"] is None else dev["bias"].cpu()}
    L, idx_o, w_o, _ = H.oracle_route(host, cfg.top_k)
    flagged, differ = H.check_routing(L, idx_o, w_o, idx.cpu().numpy(), w.cpu().numpy(), cfg.top_k)

    # scores: the oracle on the GPU's routing (identical to its own off the tie margin), every micro-expert
    X = H.f64(host["X"])
    A = orc.dense_routing(idx.cpu().numpy(), w.cpu().numpy().astype(np.float64), cfg.n_experts)
    want = orc.score_layer(X, A, _PerExpertF64(dev["W_gate"]), _PerExpertF64(dev["W_up"]), _PerExpertF64(dev["W_down"]),
                           cfg.alpha)
    if cfg.n_shared:
        shared = orc.score_layer(X, np.ones((cfg.n_tokens, cfg.n_shared)), _PerExpertF64(dev["Ws_gate"]),
                                 _PerExpertF64(dev["Ws_up"]), _PerExpertF64(dev["Ws_down"]), cfg.alpha)
        want = {k: np.concatenate([want[k], shared[k]]) for k in want}
    worst = {}
    for key in ("phi2", "phi_inf", "omega2", "energy"):
        got = out[key].cpu().numpy().astype(np.float64)
        assert got.shape == want[key].shape
        worst[key] = H.rel_err(got, want[key], max(float(want[key].max()) * 1e-9, 1e-300))
        assert worst[key] <= TOL, (key, worst[key])
        assert np.array_equal(got == 0, want[key] == 0), f"{key}: zero pattern differs"
    report = check_decisions(cam, cfg, name, out["energy"], want["energy"])
    counts = torch.bincount(idx.flatten().long(), minlength=cfg.n_experts).cpu().numpy()
    print(f"{name} layer {layer_idx}: {cfg.n_micro} micro-experts, worst rel err {worst}; routing flagged {flagged} "
          f"differ {differ} of {cfg.n_tokens}; tokens per expert min {counts.min()} max {counts.max()}; {report}", flush=True)
    cam.close()


@pytest.mark.parametrize("first", [0, 7, 14, 21])
def test_every_layer_sampled_micro_experts(cam, first):
    """Layers first .. first + 6 of the Qwen2-shaped configuration: 64 seeded micro-experts of every routed
    expert and 64 of the shared one, all tokens."""
    cfg = inputs.CONFIGS["qwen2-57b-a14b"]
    rng = np.random.default_rng(11 + first)
    for layer_idx in range(first, min(first + 7, cfg.n_layers)):
        print(f"sampled parity: {cfg.name} layer {layer_idx}", flush=True)
        dev = inputs.make_layer(cfg, layer_idx, device="cuda")
        idx, w, out = run_layer(cam, cfg, dev)
        X = H.f64(dev["X"])
        A = orc.dense_routing(idx.cpu().numpy(), w.cpu().numpy().astype(np.float64), cfg.n_experts)
        worst = 0.0
        for prefix, n_exp, f, A_mat, base in (("W", cfg.n_experts, cfg.d_ff, A, 0),
                                              ("Ws", cfg.n_shared, cfg.d_ff_shared,
                                               np.ones((cfg.n_tokens, cfg.n_shared)), cfg.n_micro_routed)):
            ch = np.sort(rng.choice(f, size=64, replace=False))
            cht = torch.as_tensor(ch).cuda()
            want = orc.score_layer(X, A_mat, H.f64(dev[prefix + "_gate"][:, cht]), H.f64(dev[prefix + "_up"][:, cht]),
                                   H.f64(dev[prefix + "_down"][:, :, cht]), cfg.alpha)
            index = (base + np.arange(n_exp)[:, None] * f + ch[None, :]).ravel()
            for key in ("phi2", "phi_inf", "omega2", "energy"):
                got = out[key].cpu().numpy().astype(np.float64)[index]
                err = H.rel_err(got, want[key], max(float(want[key].max()) * 1e-9, 1e-300))
                worst = max(worst, err)
                assert err <= TOL, (layer_idx, prefix, key, err)
        print(f"{cfg.name} layer {layer_idx}: worst sampled rel err {worst:.2e}", flush=True)
        del dev, out
