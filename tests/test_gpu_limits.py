"""The built limits of the library, each exercised once against the oracle: CAMERA_MAX_EXPERTS routed
experts, CAMERA_MAX_SEGMENTS segments, CAMERA_MAX_LEVELS precision classes, top_k = n_experts, the longest
W_down row of the gather -- and that one step past each limit is refused before any GPU work."""
import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc
from paper_2508_02322_amd import binding, inputs
from tests import helpers as H
from tests.test_gpu_score import compare_scores, score_on_gpu, TOL

pytestmark = pytest.mark.gpu

BASE = inputs.CONFIGS["qwen3-30b-a3b"]


def test_256_experts_route_score_forward_and_gather(cam):
    cfg = inputs.scaled(BASE, n_tokens=3000, d_model=64, d_ff=24, n_experts=256, top_k=8, n_layers=1, alpha=0.95)
    layer = inputs.make_layer(cfg, 0)
    dev = H.to_dev(layer)
    L, idx_o, w_o, _ = H.oracle_route(layer, cfg.top_k)
    idx_g, w_g = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    H.check_routing(L, idx_o, w_o, idx_g.cpu().numpy(), w_g.cpu().numpy(), cfg.top_k)
    w32 = w_o.astype(np.float32)
    A = orc.dense_routing(idx_o, w32, cfg.n_experts)
    got = score_on_gpu(cam, dev, idx_o, w32, cfg.alpha)
    compare_scores(got, H.oracle_score(layer, A, cfg.alpha), TOL["bf16"])
    # select over 256 segments, gather of the kept micro-experts of all 256 experts
    seg = inputs.segment_offsets(cfg)
    keep, per, kept_idx, _ = cam.select_prune(got["energy"], seg, 0.4, want_idx=True)
    E = got["energy"].cpu().numpy()
    o_keep, o_per, o_idx, _ = orc.select_prune(E, seg, 0.4)
    np.testing.assert_array_equal(keep.cpu().numpy(), o_keep)
    np.testing.assert_array_equal(per.cpu().numpy(), o_per)
    n_keep = o_idx.size
    gate_out, up_out, down_out = cam.gather_micro_experts(dev["W_gate"], dev["W_up"], dev["W_down"], kept_idx[:n_keep], per)
    bits = lambda t: t.detach().cpu().contiguous().view(torch.int16).numpy()
    o_gate, o_up, o_down = orc.gather_micro_experts(bits(layer["W_gate"]), bits(layer["W_up"]), bits(layer["W_down"]),
                                                    o_idx, o_per)
    np.testing.assert_array_equal(bits(gate_out), o_gate)
    np.testing.assert_array_equal(bits(up_out), o_up)
    flat, pos = bits(down_out), 0
    for e in range(cfg.n_experts):
        np.testing.assert_array_equal(flat[pos * cfg.d_model:(pos + o_per[e]) * cfg.d_model].reshape(cfg.d_model, o_per[e]),
                                      o_down[e])
        pos += o_per[e]
    # layer output with all 256 experts in play
    ti = torch.as_tensor(idx_o, dtype=torch.int32).cuda()
    tw = torch.as_tensor(w32).cuda()
    Y = cam.layer_forward(dev["X"], ti, tw, dev["W_gate"], dev["W_up"], dev["W_down"], keep_mask=keep)
    gate = [H.f64(layer["W_gate"][e]) for e in range(cfg.n_experts)]
    up = [H.f64(layer["W_up"][e]) for e in range(cfg.n_experts)]
    down = [H.f64(layer["W_down"][e]) for e in range(cfg.n_experts)]
    O = orc.layer_forward(H.f64(layer["X"]), A, gate, up, down, keep=o_keep, round_hidden=orc.round_to_bf16)
    num = np.linalg.norm(Y.cpu().numpy().astype(np.float64) - O, axis=1)
    assert np.all(num <= 2e-3 * np.linalg.norm(O, axis=1) + 1e-12)   # few terms per token: one bf16 step can show


def test_top_k_equal_to_the_number_of_experts(cam):
    cfg = inputs.scaled(BASE, n_tokens=500, d_model=64, d_ff=40, n_experts=8, top_k=8, n_layers=1)
    layer = inputs.make_layer(cfg, 0)
    dev = H.to_dev(layer)
    L, idx_o, w_o, _ = H.oracle_route(layer, 8)
    idx_g, w_g = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], 8)
    H.check_routing(L, idx_o, w_o, idx_g.cpu().numpy(), w_g.cpu().numpy(), 8)
    w32 = w_o.astype(np.float32)
    got = score_on_gpu(cam, dev, idx_o, w32, cfg.alpha)
    compare_scores(got, H.oracle_score(layer, orc.dense_routing(idx_o, w32, 8), cfg.alpha), TOL["bf16"])


def test_512_segments_and_8_precision_classes(cam):
    n = 100000
    E = inputs.energy_like(n, seed=9, zero_fraction=0.05, tie_fraction=0.1)
    rng = np.random.default_rng(10)
    cuts = np.sort(rng.choice(np.arange(1, n), size=511, replace=False))
    seg = [0] + [int(c) for c in cuts] + [n]
    keep, per, _, _ = cam.select_prune(E.cuda(), seg, 0.37)
    o_keep, o_per, _, _ = orc.select_prune(E.numpy(), seg, 0.37)
    np.testing.assert_array_equal(keep.cpu().numpy(), o_keep)
    np.testing.assert_array_equal(per.cpu().numpy(), o_per)
    bits = [8, 7, 6, 5, 4, 3, 2, 1]
    ratios = [0.05, 0.1, 0.15, 0.2, 0.2, 0.15, 0.1, 0.05]
    bit_of, level_count, perm = cam.alloc_bits(E.cuda(), seg, bits, ratios, want_perm=True)
    o_bits, o_count, o_perm = orc.alloc_bits(E.numpy(), seg, bits, ratios)
    np.testing.assert_array_equal(bit_of.cpu().numpy(), o_bits)
    np.testing.assert_array_equal(level_count.cpu().numpy(), o_count)
    np.testing.assert_array_equal(perm.cpu().numpy(), o_perm)
    keep_bits, per7 = cam.select_prune_multi(E.cuda(), seg, [0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7])
    for k, r in enumerate([0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7]):
        o_keep, o_per, _, _ = orc.select_prune(E.numpy(), seg, r)
        np.testing.assert_array_equal((keep_bits.cpu().numpy() >> k) & 1, o_keep)
        np.testing.assert_array_equal(per7[k].cpu().numpy(), o_per)


def test_one_step_past_each_limit_is_refused(cam):
    E = torch.zeros(1000, device="cuda")
    with pytest.raises(binding.CameraError):
        cam.select_prune(E, list(range(0, 514)) + [1000], 0.5)                   # 514 segments
    with pytest.raises(binding.CameraError):
        cam.alloc_bits(E, [0, 1000], [9, 8, 7, 6, 5, 4, 3, 2, 1], [1 / 9] * 9)     # 9 classes
    with pytest.raises(binding.CameraError):
        cam.select_prune_multi(E, [0, 1000], [0.1 * k for k in range(8)])         # 8 ratios
    X = torch.zeros((8, 64), dtype=torch.bfloat16, device="cuda")
    W_r = torch.zeros((257, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.CameraError):
        cam.route_topk(X, W_r, None, 2)                                            # 257 experts
    W = torch.zeros((1, 32776, 8), dtype=torch.bfloat16, device="cuda")
    Wd = torch.zeros((1, 8, 32776), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.CameraError):
        cam.gather_micro_experts(W, W, Wd, torch.zeros(4, dtype=torch.int32, device="cuda"),
                                 torch.tensor([4], dtype=torch.int32, device="cuda"))   # W_down row of 65552 bytes
