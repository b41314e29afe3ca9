"""GPU parity of camera_layer_forward / camera_output_error against the fp64 oracle.

The oracle takes the routing the GPU chose (indices and float32 weights, exact in float64), so a
near-tie in the router cannot blur the comparison, and rounds the hidden activations to bf16 as the
kernel does.  What is left is (a) float32 accumulation, a few 1e-7 of the token's norm, and (b) the rare
hidden value whose float32 and float64 forms fall on different sides of a bf16 rounding boundary: it
then differs by one bf16 step, at most 2^-8 of itself, and moves the token's output by that times its
down column.  The bound asserted per token is therefore
    ||y - y_oracle|| <= 2e-5 ||y_oracle|| + 2 * 2^-8 * max_c |Lambda_c| ||w_down_c||
(room for two such values in one token, taken at the largest term); observed values are printed.
"""
import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc
from paper_2508_02322_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu

BASE = inputs.CONFIGS["mixtral"]


def small(**kw):
    args = dict(n_tokens=300, d_model=128, d_ff=192, n_experts=8, top_k=2, n_layers=1, outlier_channels=2)
    args.update(kw)
    return inputs.scaled(BASE, **args)


def dense_A(idx, w, n_experts):
    A = np.zeros((idx.shape[0], n_experts))
    for k in range(idx.shape[1]):
        A[np.arange(idx.shape[0]), idx[:, k]] += w[:, k]
    return A


def expert_lists(layer, prefix):
    Wg, Wu, Wd = layer[prefix + "_gate"], layer[prefix + "_up"], layer[prefix + "_down"]
    n = Wg.shape[0]
    return [H.f64(Wg[e]) for e in range(n)], [H.f64(Wu[e]) for e in range(n)], [H.f64(Wd[e]) for e in range(n)]


def largest_term(X64, A, gate, up, down, keep=None):
    """max over micro-experts of |Lambda[j, c]| * ||w_down_c|| for every token j."""
    best = np.zeros(X64.shape[0])
    pos = 0
    for e in range(len(gate)):
        lam = np.abs(orc.lambda_matrix(X64, A[:, e], gate[e], up[e]))
        if keep is not None:
            lam = lam * np.asarray(keep, dtype=np.float64)[pos:pos + lam.shape[1]][None, :]
        best = np.maximum(best, (lam * np.linalg.norm(down[e], axis=0)[None, :]).max(axis=1))
        pos += lam.shape[1]
    return best


def check_output(Y_gpu, Y_orc, term):
    """Asserts the per-token bound of the module docstring; returns the largest ||y - y_orc|| / ||y_orc||."""
    Y_gpu = Y_gpu.cpu().numpy().astype(np.float64)
    num = np.linalg.norm(Y_gpu - Y_orc, axis=1)
    norm = np.linalg.norm(Y_orc, axis=1)
    allowed = 2e-5 * norm + 2.0 * 2.0 ** -8 * term + 1e-30
    worst = int(np.argmax(num / allowed))
    assert np.all(num <= allowed), (worst, num[worst], allowed[worst], norm[worst])
    return float(np.max(num / np.maximum(norm, 1e-30 + 1e-9 * norm.max())))


CASES = [
    dict(dtype="f32", n_tokens=300, d_model=100, d_ff=52, n_experts=6),    # float32: no rounding of the hidden activations
    dict(dtype="f32", n_tokens=129, d_model=64, d_ff=200, n_experts=3, top_k=3),
    dict(),                                                        # several M tiles per expert, ragged N tile
    dict(n_tokens=37, d_model=72, d_ff=40),                        # everything ragged, K tails in both contractions
    dict(n_tokens=1000, d_model=256, d_ff=136, n_experts=5, top_k=3),
    dict(n_tokens=513, d_model=64, d_ff=520, n_experts=64, top_k=6, router_bias="none"),
    dict(n_tokens=64, d_model=32, d_ff=16, n_experts=1, top_k=1),  # one expert
]


@pytest.mark.parametrize("case", CASES)
def test_layer_output_matches_oracle_with_and_without_a_mask(cam, case):
    cfg = small(**case)
    layer = inputs.make_layer(cfg, 0, device="cpu")
    dev = H.to_dev(layer)
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    A = dense_A(idx.cpu().numpy().astype(np.int64), w.cpu().numpy().astype(np.float64), cfg.n_experts)
    gate, up, down = expert_lists(layer, "W")
    X64 = H.f64(layer["X"])
    Y_full = cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"])
    ones = torch.ones(cfg.n_experts * cfg.d_ff, dtype=torch.uint8, device="cuda")
    Y_ones = cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], keep_mask=ones)
    torch.cuda.synchronize()
    rounding = orc.round_to_bf16 if cfg.dtype == "bf16" else None
    flip = 1.0 if cfg.dtype == "bf16" else 0.0                     # float32: only accumulation error is allowed
    O_full = orc.layer_forward(X64, A, gate, up, down, round_hidden=rounding)
    err_full = check_output(Y_full, O_full, flip * largest_term(X64, A, gate, up, down))
    assert torch.equal(Y_full, Y_ones)                             # NULL mask == every micro-expert kept, bit for bit
    keep = (torch.rand(cfg.n_experts * cfg.d_ff, generator=torch.Generator().manual_seed(3)) < 0.6).to(torch.uint8)
    Y_kept = cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], keep_mask=keep.cuda())
    torch.cuda.synchronize()
    O_kept = orc.layer_forward(X64, A, gate, up, down, keep=keep.numpy(), round_hidden=rounding)
    err_kept = check_output(Y_kept, O_kept, flip * largest_term(X64, A, gate, up, down, keep.numpy()))
    # error measures of the same two outputs
    per_token = cam.output_error(Y_full, Y_kept).cpu().numpy().astype(np.float64)
    want = orc.output_error(Y_full.cpu().numpy(), Y_kept.cpu().numpy())
    for col, key in enumerate(("d2", "yy", "hh", "yh")):
        scale = np.maximum(np.abs(want[key]), 1e-6 * np.sqrt(want["yy"] * want["hh"]) + 1e-30)
        assert np.max(np.abs(per_token[:, col] - want[key]) / scale) <= 2e-5, key
    print(f"{case}: rel err full {err_full:.2e}, masked {err_kept:.2e}")


def test_nothing_kept_gives_zero_and_accumulate_adds_the_shared_experts(cam):
    cfg = small(n_shared=1, d_ff_shared=256)
    layer = inputs.make_layer(cfg, 0, device="cpu")
    dev = H.to_dev(layer)
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    none = torch.zeros(cfg.n_experts * cfg.d_ff, dtype=torch.uint8, device="cuda")
    Y0 = cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], keep_mask=none)
    assert torch.count_nonzero(Y0).item() == 0
    # routed experts, then the shared expert (every token, weight 1) added into the same Y
    Y = cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"])
    Y_routed = Y.clone()
    cam.layer_forward(dev["X"], None, None, dev["Ws_gate"], dev["Ws_up"], dev["Ws_down"], Y=Y, accumulate=True)
    Y_shared = cam.layer_forward(dev["X"], None, None, dev["Ws_gate"], dev["Ws_up"], dev["Ws_down"])
    torch.cuda.synchronize()
    assert torch.equal(Y, Y_routed + Y_shared)
    X64 = H.f64(layer["X"])
    gate, up, down = expert_lists(layer, "Ws")
    O_shared = orc.layer_forward(X64, np.ones((cfg.n_tokens, 1)), gate, up, down, round_hidden=orc.round_to_bf16)
    check_output(Y_shared, O_shared, largest_term(X64, np.ones((cfg.n_tokens, 1)), gate, up, down))


def test_decoding_error_of_one_pruned_micro_expert_is_its_energy(cam):
    """The Lemma with one removed index, on the GPU's own numbers: ||Y - Y_hat||_F^2 = E_i at alpha = 0.
    The hidden activations are rounded to bf16 in the layer output and not in the score, so the two
    agree to bf16 precision (2^-8), not to float32 precision."""
    cfg = small(n_tokens=400, d_ff=64, n_experts=4)
    layer = inputs.make_layer(cfg, 0, device="cpu")
    dev = H.to_dev(layer)
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    E = cam.score_layer(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], 0.0)["energy"].cpu().numpy()
    Y = cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"])
    for i in (0, 70, 130, 255):
        keep = torch.ones(cfg.n_experts * cfg.d_ff, dtype=torch.uint8)
        keep[i] = 0
        Y_hat = cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], keep_mask=keep.cuda())
        d2 = cam.output_error(Y, Y_hat)[:, 0].double().sum().item()
        assert d2 == pytest.approx(float(E[i]), rel=1e-2), (i, d2, E[i])


def test_layer_output_is_bitwise_repeatable(cam):
    cfg = small(n_tokens=700)
    dev = H.to_dev(inputs.make_layer(cfg, 0, device="cpu"))
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    a = cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"]).clone()
    for _ in range(3):
        assert torch.equal(a, cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"]))


@pytest.mark.parametrize("name", ["deepseek-moe-16b", "qwen2-57b-a14b"])
def test_full_size_layer_on_sampled_tokens(cam, name):
    """A whole layer of the benchmark shape at the size bench.py runs; the oracle recomputes a sample of
    token rows (rows of Y only depend on their own token once the routing is fixed)."""
    cfg = inputs.CONFIGS[name]
    layer = inputs.make_layer(cfg, 0, device="cuda")
    idx, w = cam.route_topk(layer["X"], layer["W_r"], layer["bias"], cfg.top_k)
    keep = (torch.rand(cfg.n_micro, generator=torch.Generator().manual_seed(5)) < 0.6).to(torch.uint8).cuda()
    nr = cfg.n_micro_routed
    Y = cam.layer_forward(layer["X"], idx, w, layer["W_gate"], layer["W_up"], layer["W_down"], keep_mask=keep[:nr])
    if cfg.n_shared:
        cam.layer_forward(layer["X"], None, None, layer["Ws_gate"], layer["Ws_up"], layer["Ws_down"],
                          keep_mask=keep[nr:], Y=Y, accumulate=True)
    torch.cuda.synchronize()
    sample = torch.arange(0, cfg.n_tokens, cfg.n_tokens // 24)[:24]
    cpu = {k: (v.cpu() if v is not None else None) for k, v in layer.items()}
    X64 = H.f64(cpu["X"][sample])
    A = dense_A(idx.cpu().numpy().astype(np.int64)[sample], w.cpu().numpy().astype(np.float64)[sample], cfg.n_experts)
    used = np.nonzero(A.sum(axis=0))[0]                         # experts none of the sampled tokens use add nothing
    gate = [H.f64(cpu["W_gate"][e]) for e in used]
    up = [H.f64(cpu["W_up"][e]) for e in used]
    down = [H.f64(cpu["W_down"][e]) for e in used]
    keep_h = keep.cpu().numpy()
    keep_used = np.concatenate([keep_h[e * cfg.d_ff:(e + 1) * cfg.d_ff] for e in used])
    O = orc.layer_forward(X64, A[:, used], gate, up, down, keep=keep_used, round_hidden=orc.round_to_bf16)
    if cfg.n_shared:
        g2, u2, d2 = expert_lists(cpu, "Ws")
        O += orc.layer_forward(X64, np.ones((sample.numel(), cfg.n_shared)), g2, u2, d2, keep=keep_h[nr:],
                               round_hidden=orc.round_to_bf16)
    term = largest_term(X64, A[:, used], gate, up, down, keep_used)
    if cfg.n_shared:
        term = np.maximum(term, largest_term(X64, np.ones((sample.numel(), cfg.n_shared)), g2, u2, d2, keep_h[nr:]))
    err = check_output(Y[sample.cuda()], O, term)
    print(f"{name}: sampled-token rel err {err:.2e}")
