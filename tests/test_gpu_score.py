"""GPU parity of camera_route_topk and camera_score_layer against the fp64 oracle on
seeded inputs small enough for the full oracle, with ragged sizes and the degenerate
cases of the method."""
import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc
from paper_2508_02322_amd import binding, inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu

# Relative tolerance on phi2 / phi_inf / omega2 / energy.  bf16: the inputs are exact in both
# paths and products of two bf16 values are exact in float32, so the error is float32
# accumulation (about sqrt(d_model) * 2^-24 per projection, doubled by the square) plus the
# fast exp of SiLU; the budget the task states is 2e-3.  float32 inputs: the same accumulation
# error on 24-bit products; measured values are around 1e-6, the bound used is 5e-5.
TOL = {"bf16": 2e-3, "f32": 5e-5}

BASE = inputs.CONFIGS["mixtral"]


def small(**kw):
    args = dict(n_tokens=300, d_model=128, d_ff=192, n_experts=8, top_k=2, n_layers=1, outlier_channels=2)
    args.update(kw)
    return inputs.scaled(BASE, **args)


def score_on_gpu(cam, dev, idx, w32, alpha, prefix="W", flags=0, out=None):
    ti = None if idx is None else torch.as_tensor(np.asarray(idx), dtype=torch.int32).cuda()
    tw = None if w32 is None else torch.as_tensor(np.asarray(w32), dtype=torch.float32).cuda()
    out = cam.score_layer(dev["X"], ti, tw, dev[prefix + "_gate"], dev[prefix + "_up"], dev[prefix + "_down"], alpha,
                          flags=flags, out=out)
    torch.cuda.synchronize()
    return out


def compare_scores(got, want, tol):
    report = {}
    for key in ("phi2", "phi_inf", "omega2", "energy"):
        g = got[key].cpu().numpy().astype(np.float64)
        floor = max(float(np.max(want[key])) * 1e-9, 1e-300)
        report[key] = H.rel_err(g, want[key], floor)
        assert report[key] <= tol, (key, report[key])
        assert np.all((want[key] == 0) == (g == 0)), f"{key}: zero pattern differs"
    return report


CASES = [
    dict(),                                                        # several M tiles per expert
    dict(n_tokens=37, d_model=72, d_ff=40),                        # everything ragged, K tail
    dict(n_tokens=1000, d_model=256, d_ff=136, n_experts=5, top_k=3),
    dict(n_tokens=513, d_model=64, d_ff=520, n_experts=64, top_k=6, router_bias="none"),
    dict(n_tokens=2048, d_model=512, d_ff=128, n_experts=128, top_k=8, router_bias="zipf", alpha=1.0),
    dict(n_tokens=64, d_model=32, d_ff=16, n_experts=1, top_k=1),  # one expert
    dict(dtype="f32", n_tokens=300, d_model=100, d_ff=52, n_experts=6),
    dict(dtype="f32", n_tokens=129, d_model=64, d_ff=200, n_experts=3, top_k=3),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()) or "base")
def test_route_and_score_match_oracle(cam, case):
    cfg = small(**case)
    layer = inputs.make_layer(cfg, 0)
    dev = H.to_dev(layer)
    L, idx_o, w_o, _ = H.oracle_route(layer, cfg.top_k)
    idx_g, w_g = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    flagged, differ = H.check_routing(L, idx_o, w_o, idx_g.cpu().numpy(), w_g.cpu().numpy(), cfg.top_k)
    # score with the oracle's routing on both sides (weights as the float32 values the GPU reads)
    w32 = w_o.astype(np.float32)
    want = H.oracle_score(layer, orc.dense_routing(idx_o, w32, cfg.n_experts), cfg.alpha)
    got = score_on_gpu(cam, dev, idx_o, w32, cfg.alpha)
    rep = compare_scores(got, want, TOL[cfg.dtype])
    print(f"{cfg.dtype} flagged={flagged} differ={differ} rel_err={rep}")


def test_route_variants(cam):
    cfg = small(n_tokens=200, d_model=64, n_experts=16, top_k=4)
    layer = inputs.make_layer(cfg, 1)
    dev = H.to_dev(layer)
    # no renormalisation: the weights are the softmax probabilities over all experts
    L, idx_o, w_o, _ = H.oracle_route(layer, 4, renorm=False)
    idx_g, w_g = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], 4, renorm=False)
    H.check_routing(L, idx_o, w_o, idx_g.cpu().numpy(), w_g.cpu().numpy(), 4, renorm=False)
    # k = N_E keeps everything
    L, idx_o, w_o, _ = H.oracle_route(layer, 16)
    idx_g, w_g = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], 16)
    H.check_routing(L, idx_o, w_o, idx_g.cpu().numpy(), w_g.cpu().numpy(), 16)
    # two identical router rows: exact ties go to the lower expert index
    W_r = dev["W_r"].clone()
    W_r[9] = W_r[2]
    bias = dev["bias"].clone()
    bias[9] = bias[2]
    idx_g, _ = cam.route_topk(dev["X"], W_r, bias, 4)
    idx_g = idx_g.cpu().numpy()
    has2 = (idx_g == 2).any(axis=1)
    has9 = (idx_g == 9).any(axis=1)
    assert not np.any(has9 & ~has2)
    both = has2 & has9
    pos2 = np.argmax(idx_g == 2, axis=1)
    pos9 = np.argmax(idx_g == 9, axis=1)
    assert np.all(pos9[both] == pos2[both] + 1)
    # strided X (a column slice of a wider buffer)
    wide = torch.zeros((200, 128), dtype=dev["X"].dtype, device="cuda")
    wide[:, :64] = dev["X"]
    idx_s, w_s = cam.route_topk(wide[:, :64], dev["W_r"], dev["bias"], 4)
    idx_c, w_c = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], 4)
    assert torch.equal(idx_s, idx_c) and torch.equal(w_s, w_c)


def test_shared_expert_dense_call(cam):
    cfg = inputs.scaled(inputs.CONFIGS["qwen2-57b-a14b"], n_tokens=333, d_model=96, d_ff=64, n_experts=4, top_k=2,
                        n_shared=2, d_ff_shared=264, n_layers=1)
    layer = inputs.make_layer(cfg, 0)
    dev = H.to_dev(layer)
    want = H.oracle_score(layer, np.ones((cfg.n_tokens, cfg.n_shared)), cfg.alpha, prefix="Ws")
    got = score_on_gpu(cam, dev, None, None, cfg.alpha, prefix="Ws")
    compare_scores(got, want, TOL["bf16"])


def test_degenerate_inputs(cam):
    cfg = small(n_tokens=150, d_model=64, d_ff=96, n_experts=6, top_k=2)
    layer = inputs.make_layer(cfg, 2)
    # expert 4 gets no token; out-of-range indices are ignored; zeroed rows / columns score zero
    _, idx_o, w_o, _ = H.oracle_route(layer, 2)
    idx = idx_o.copy()
    idx[idx == 4] = 5
    idx[::7, 1] = -1
    idx[3::11, 0] = 99
    w32 = w_o.astype(np.float32)
    layer["W_down"][0, :, 3] = 0
    layer["W_up"][1, 7, :] = 0
    layer["W_gate"][2, 9, :] = 0
    dev = H.to_dev(layer)
    valid = (idx >= 0) & (idx < cfg.n_experts)
    # a token may now list expert 5 twice: both pairs count (two rows of Lambda), so build the
    # oracle input pair by pair instead of through a dense matrix
    want = {k: np.zeros(cfg.n_micro_routed) for k in ("phi2", "phi_inf")}
    X = H.f64(layer["X"])
    for e in range(cfg.n_experts):
        rows, cols = np.nonzero(valid & (idx == e))
        p2, pinf = orc.expert_column_stats(X[rows], w32[rows, cols].astype(np.float64), H.f64(layer["W_gate"][e]),
                                           H.f64(layer["W_up"][e]), skip_unrouted=False)
        want["phi2"][e * cfg.d_ff:(e + 1) * cfg.d_ff] = p2
        want["phi_inf"][e * cfg.d_ff:(e + 1) * cfg.d_ff] = pinf
    want["omega2"] = np.concatenate([orc.down_column_sumsq(H.f64(layer["W_down"][e])) for e in range(cfg.n_experts)])
    want["energy"] = orc.energy(want["phi2"], want["phi_inf"], want["omega2"], cfg.alpha)
    got = score_on_gpu(cam, dev, idx, w32, cfg.alpha)
    compare_scores(got, want, TOL["bf16"])
    E = got["energy"].cpu().numpy().reshape(cfg.n_experts, cfg.d_ff)
    assert np.all(E[4] == 0) and E[0, 3] == 0 and E[1, 7] == 0 and E[2, 9] == 0


def test_no_tokens(cam):
    cfg = small(n_tokens=8, d_model=64, d_ff=48, n_experts=3)
    dev = H.to_dev(inputs.make_layer(cfg, 0))
    empty = dev["X"][:0]
    idx = torch.empty((0, 2), dtype=torch.int32, device="cuda")
    w = torch.empty((0, 2), dtype=torch.float32, device="cuda")
    out = cam.score_layer(empty, idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], 0.5)
    assert torch.all(out["phi2"] == 0) and torch.all(out["phi_inf"] == 0) and torch.all(out["energy"] == 0)
    want = np.concatenate([orc.down_column_sumsq(H.f64(dev["W_down"][e])) for e in range(3)])
    assert H.rel_err(out["omega2"].cpu().numpy(), want, 1e-30) < 1e-5
    i2, w2 = cam.route_topk(empty, dev["W_r"], dev["bias"], 2)
    assert i2.shape == (0, 2) and w2.shape == (0, 2)


def test_chunked_accumulation_matches_one_shot(cam):
    cfg = small(n_tokens=700, d_model=128, d_ff=160, n_experts=8, top_k=2)
    layer = inputs.make_layer(cfg, 3)
    dev = H.to_dev(layer)
    _, idx_o, w_o, _ = H.oracle_route(layer, 2)
    w32 = w_o.astype(np.float32)
    want = H.oracle_score(layer, orc.dense_routing(idx_o, w32, cfg.n_experts), cfg.alpha)
    out = None
    bounds = [0, 256, 300, 700]
    for c in range(3):
        lo, hi = bounds[c], bounds[c + 1]
        flags = (binding.ACCUMULATE if c > 0 else 0) | (binding.NO_FINALIZE if c < 2 else 0)
        chunk = dict(dev)
        chunk["X"] = dev["X"][lo:hi]
        out = score_on_gpu(cam, chunk, idx_o[lo:hi], w32[lo:hi], cfg.alpha, flags=flags, out=out)
    compare_scores(out, want, TOL["bf16"])


def test_scores_are_bitwise_repeatable(cam):
    cfg = small(n_tokens=2000, d_model=256, d_ff=256, n_experts=16, top_k=4)
    dev = H.to_dev(inputs.make_layer(cfg, 4))
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], 4)
    a = cam.score_layer(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], 0.95)
    b = cam.score_layer(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], 0.95)
    for k in a:
        assert torch.equal(a[k], b[k]), k


def test_tiny_config_end_to_end(cam):
    """BASELINE config 1: fp32, 8 experts, top-2, 512 tokens, score + 40 % prune mask."""
    cfg = inputs.CONFIGS["tiny"]
    layer = inputs.make_layer(cfg, 0)
    dev = H.to_dev(layer)
    L, idx_o, w_o, A = H.oracle_route(layer, cfg.top_k)
    idx_g, w_g = cam.route_topk(dev["X"], dev["W_r"], None, cfg.top_k)
    flagged, differ = H.check_routing(L, idx_o, w_o, idx_g.cpu().numpy(), w_g.cpu().numpy(), cfg.top_k)
    assert differ == 0
    want = H.oracle_score(layer, A, cfg.alpha)
    got = cam.score_layer(dev["X"], idx_g, w_g, dev["W_gate"], dev["W_up"], dev["W_down"], cfg.alpha)
    compare_scores(got, want, TOL["f32"])
    seg = inputs.segment_offsets(cfg)
    keep, per, _, _ = cam.select_prune(got["energy"], seg, 0.4)
    keep = keep.cpu().numpy().astype(bool)
    n_prune = orc.prune_count(0.4, cfg.n_micro)
    assert n_prune == 1638 and np.count_nonzero(~keep) == n_prune
    must_prune, must_keep = H.decidable_masks(want["energy"], n_prune, TOL["f32"])
    assert not np.any(keep[must_prune]) and np.all(keep[must_keep])
    undecidable = 1.0 - (np.count_nonzero(must_prune) + np.count_nonzero(must_keep)) / cfg.n_micro
    print(f"tiny: undecidable fraction {undecidable:.4f}")
    # same energies -> the mask is bit-exact against the oracle's selection
    o_keep, o_per, _, _ = orc.select_prune(got["energy"].cpu().numpy(), seg, 0.4)
    np.testing.assert_array_equal(keep, o_keep.astype(bool))
    np.testing.assert_array_equal(per.cpu().numpy(), o_per)


def test_machine_probes_report_plausible_ceilings():
    """The probes are measurements, not results: check their range and that random operands are not faster."""
    from paper_2508_02322_amd import bench_probes
    tf_const, mhz_const = bench_probes.mfma_bf16(False, launches=10)
    tf_rand, mhz_rand = bench_probes.mfma_bf16(True, launches=10)
    assert 500.0 < tf_rand <= tf_const * 1.05 and tf_const < 2600.0
    assert 800.0 < mhz_rand < 2600.0 and 800.0 < mhz_const < 2600.0
    gbs = bench_probes.hbm_read(1 << 30, launches=3)
    assert 1000.0 < gbs < 8500.0


def test_non_contiguous_inputs_are_refused_or_honoured(cam):
    """Views the library can describe (a row stride on X, an expert stride on the weights) give the same scores as
    packed tensors; views it cannot (transposed, inner stride) raise instead of scoring the wrong bytes."""
    cfg = small(n_tokens=200, d_model=64, d_ff=48, n_experts=4, top_k=2)
    dev = H.to_dev(inputs.make_layer(cfg, 5))
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], 2)
    want = cam.score_layer(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], 0.95)
    wide = torch.zeros((200, 96), dtype=dev["X"].dtype, device="cuda")
    wide[:, :64] = dev["X"]
    padded = {k: torch.zeros((7, *dev[k].shape[1:]), dtype=dev[k].dtype, device="cuda") for k in ("W_gate", "W_up", "W_down")}
    for k in padded:
        padded[k][::2] = dev[k]                      # experts two slabs apart
    got = cam.score_layer(wide[:, :64], idx, w, padded["W_gate"][::2], padded["W_up"][::2], padded["W_down"][::2], 0.95)
    for k in want:
        assert torch.equal(want[k], got[k]), k
    with pytest.raises(binding.CameraError):
        cam.score_layer(dev["X"].t().contiguous().t(), idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], 0.95)
    with pytest.raises(binding.CameraError):
        cam.score_layer(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"].transpose(1, 2).contiguous().transpose(1, 2), 0.95)
    with pytest.raises(binding.CameraError):
        cam.score_layer(dev["X"], idx.cpu(), w, dev["W_gate"], dev["W_up"], dev["W_down"], 0.95)


def test_row_stride_beyond_32_bit_offsets(cam):
    """Token rows so far apart that a 32-bit byte offset from the start of X cannot reach them: the contraction
    takes its form with a 64-bit address per lane, and scores the same bits."""
    cfg = small(n_tokens=600, d_model=128, d_ff=96, n_experts=4, top_k=2)
    dev = H.to_dev(inputs.make_layer(cfg, 6))
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], 2)
    want = cam.score_layer(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], 0.95)
    ldx = 1 << 21                                    # 600 rows x 4 MiB: 2.5 GB
    wide = torch.zeros((600, ldx), dtype=dev["X"].dtype, device="cuda")
    wide[:, :128] = dev["X"]
    idx2, w2 = cam.route_topk(wide[:, :128], dev["W_r"], dev["bias"], 2)
    assert torch.equal(idx, idx2) and torch.equal(w, w2)
    got = cam.score_layer(wide[:, :128], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], 0.95)
    for k in want:
        assert torch.equal(want[k], got[k]), k

