"""One layer through the whole chain on the GPU — score, select, pack, run the pruned layer — against the same
chain in the oracle (Algorithm 1, then Algorithm 2 lines 9-14), each stage fed with what the stage before it
produced on its own side, except where float32 / float64 may legitimately order two energies differently: the
oracle selects on the GPU's float32 energies (the parity rule for the integer stages)."""
import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc
from paper_2508_02322_amd import inputs, pipeline
from tests import helpers as H
from tests.test_gpu_forward import check_output, dense_A, expert_lists, largest_term

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,n_tokens,ratio,spread", [("deepseek-moe-16b", 64, 0.4, 0.0), ("qwen2-57b-a14b", 300, 0.2, 1.0),
                                                         ("mixtral", 1200, 0.6, 1.0)])
def test_score_select_pack_and_run(cam, name, n_tokens, ratio, spread):
    base = inputs.CONFIGS[name]
    cfg = inputs.scaled(base, n_tokens=n_tokens, d_model=128, d_ff=176, n_experts=8, top_k=2, n_layers=1,
                        n_shared=min(base.n_shared, 1), d_ff_shared=264 if base.n_shared else 0,
                        outlier_channels=min(base.outlier_channels, 2), energy_spread=spread)
    layer = inputs.make_layer(cfg, 0, device="cpu")
    dev = H.to_dev(layer)
    scores = pipeline.score_layer(cam, dev, cfg.top_k, cfg.alpha)
    assert scores.seg_offsets == inputs.segment_offsets(cfg)
    compact = pipeline.prune_layer(cam, dev, scores, ratio)
    Y = compact.forward(cam, dev["X"], scores.topk_idx, scores.topk_w)
    torch.cuda.synchronize()

    # Algorithm 1 in the oracle, on the GPU's routing
    A = dense_A(scores.topk_idx.cpu().numpy().astype(np.int64), scores.topk_w.cpu().numpy().astype(np.float64), cfg.n_experts)
    want = [H.oracle_score(layer, A, cfg.alpha)["energy"]]
    ones = np.ones((cfg.n_tokens, max(cfg.n_shared, 1)))
    if cfg.n_shared:
        want.append(H.oracle_score(layer, ones, cfg.alpha, prefix="Ws")["energy"])
    want = np.concatenate(want)
    got = scores.energy.cpu().numpy().astype(np.float64)
    assert H.rel_err(got, want, want.max() * 1e-12) <= 2e-3
    # Algorithm 2, line 9 on the same float32 energies: the same mask, counts and index list
    o_keep, o_per, o_idx, _ = orc.select_prune(scores.energy.cpu().numpy(), scores.seg_offsets, ratio)
    np.testing.assert_array_equal(compact.keep_mask.cpu().numpy(), o_keep)
    assert compact.counts == [int(c) for c in o_per]
    np.testing.assert_array_equal(compact.kept_idx.cpu().numpy(), o_idx)
    # lines 10-14: the layer over the kept micro-experts
    X64 = H.f64(layer["X"])
    gate, up, down = expert_lists(layer, "W")
    nr = cfg.n_micro_routed
    O = orc.layer_forward(X64, A, gate, up, down, keep=o_keep[:nr], round_hidden=orc.round_to_bf16)
    term = largest_term(X64, A, gate, up, down, o_keep[:nr])
    if cfg.n_shared:
        g2, u2, d2 = expert_lists(layer, "Ws")
        O += orc.layer_forward(X64, ones, g2, u2, d2, keep=o_keep[nr:], round_hidden=orc.round_to_bf16)
        term = np.maximum(term, largest_term(X64, ones, g2, u2, d2, o_keep[nr:]))
    err = check_output(Y, O, term)
    print(f"{name}: {n_tokens} tokens, ratio {ratio}, spread {spread}: kept per expert {min(compact.counts)}..{max(compact.counts)}, "
          f"output rel err {err:.2e}")


def test_layer_reordered_by_precision_class_gives_the_same_output(cam):
    """CAMERA-Q's reordering (micro-experts of equal bit width side by side inside every expert) moves the three
    vectors of a micro-expert together, so the layer's output does not change: the reordered layer, run through the
    compacted-layer call with every count equal to d_ff, against the oracle's output of the original layer."""
    cfg = inputs.scaled(inputs.CONFIGS["qwen3-30b-a3b"], n_tokens=90, d_model=128, d_ff=96, n_experts=8, top_k=2, n_layers=1)
    layer = inputs.make_layer(cfg, 0, device="cpu")
    dev = H.to_dev(layer)
    scores = pipeline.score_layer(cam, dev, cfg.top_k, cfg.alpha)
    bit_of, level_count, perm = cam.alloc_bits(scores.energy, scores.seg_offsets, [3, 2, 1], [0.2, 0.6, 0.2], want_perm=True)
    gate_r, up_r, down_r = cam.gather_micro_experts(dev["W_gate"], dev["W_up"], dev["W_down"], perm)
    Y = cam.layer_forward_compact(dev["X"], scores.topk_idx, scores.topk_w, [cfg.d_ff] * cfg.n_experts, gate_r, up_r, down_r)
    torch.cuda.synchronize()
    # inside every expert the classes now sit one after the other, in the order of the bit list
    b = bit_of.cpu().numpy()[perm.cpu().numpy()].reshape(cfg.n_experts, cfg.d_ff)
    assert np.all(np.diff(b.astype(np.int64), axis=1) <= 0)
    assert np.array_equal(np.stack([(b == w).sum(axis=1) for w in (3, 2, 1)], axis=1), level_count.cpu().numpy())
    X64 = H.f64(layer["X"])
    A = dense_A(scores.topk_idx.cpu().numpy().astype(np.int64), scores.topk_w.cpu().numpy().astype(np.float64), cfg.n_experts)
    gate, up, down = expert_lists(layer, "W")
    O = orc.layer_forward(X64, A, gate, up, down, round_hidden=orc.round_to_bf16)
    check_output(Y, O, largest_term(X64, A, gate, up, down))
