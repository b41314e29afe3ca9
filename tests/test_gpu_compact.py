"""GPU parity of camera_layer_forward_compact (the pruned layer's output from its compacted weights,
Algorithm 2, line 14 after lines 10-13) against the fp64 oracle.

The weights are compacted on the GPU by camera_gather_micro_experts from a keep mask; the oracle computes
the layer with the pruned micro-experts zeroed (its pinned equal of the compacted form), with the GPU's
routing and the hidden activations rounded to bf16.  The per-token bound is that of the uncompacted
layer output (tests/test_gpu_forward.py): float32 accumulation plus at most two bf16 rounding flips.
"""
import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc
from paper_2508_02322_amd import binding, inputs
from tests import helpers as H
from tests.test_gpu_forward import check_output, dense_A, expert_lists, largest_term, small

pytestmark = pytest.mark.gpu


def compact(cam, dev, prefix, keep, n_experts, d_ff, align=1):
    """(count list, gate_c, up_c, down_c) of the experts `prefix` for a 0/1 mask over their micro-experts."""
    keep = np.asarray(keep).astype(bool)
    index = torch.from_numpy(np.flatnonzero(keep).astype(np.int32)).cuda()
    count = keep.reshape(n_experts, d_ff).sum(axis=1).astype(np.int32)
    gate_c, up_c, down_c = cam.gather_micro_experts(dev[prefix + "_gate"], dev[prefix + "_up"], dev[prefix + "_down"],
                                                    index, torch.from_numpy(count).cuda(), down_row_align=align)
    return [int(c) for c in count], gate_c, up_c, down_c


CASES = [
    dict(n_tokens=64),                                                      # the decoding batch; ragged counts (odd row lengths)
    dict(n_tokens=5, d_model=72, d_ff=40),                                  # K tail in the first contraction, d_model % 32 != 0
    dict(n_tokens=33, d_model=64, d_ff=520, n_experts=64, top_k=6, router_bias="none"),   # many experts without a token
    dict(n_tokens=200, d_model=256, d_ff=136, n_experts=4, top_k=3),        # > 64 tokens per expert: several passes, wide tiles
    dict(n_tokens=100, d_model=128, d_ff=96, n_experts=8, top_k=1),         # routed, narrow tiles, some experts above 32 tokens
    dict(n_tokens=1, d_model=32, d_ff=16, n_experts=1, top_k=1),
    dict(n_tokens=1500, d_model=256, d_ff=200, n_experts=8, top_k=2),       # several 256-row tiles per expert (MFMA path when aligned)
    dict(n_tokens=900, d_model=80, d_ff=296, n_experts=3, top_k=2),         # K tails in both contractions, three N tiles
]


@pytest.mark.parametrize("case", CASES)
def test_compacted_layer_output_matches_oracle(cam, case):
    cfg = small(**case)
    layer = inputs.make_layer(cfg, 0, device="cpu")
    dev = H.to_dev(layer)
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    A = dense_A(idx.cpu().numpy().astype(np.int64), w.cpu().numpy().astype(np.float64), cfg.n_experts)
    gate, up, down = expert_lists(layer, "W")
    X64 = H.f64(layer["X"])
    n_micro = cfg.n_experts * cfg.d_ff
    rng = np.random.default_rng(11)
    for frac in (1.0, 0.63, 0.2):
        keep = (rng.random(n_micro) < frac).astype(np.uint8)
        if frac == 0.2 and cfg.n_experts > 1:
            keep[:cfg.d_ff] = 0                                             # an expert that keeps nothing
            keep[cfg.d_ff:cfg.d_ff + 3] = 1                                 # and one with at least three
        count, gate_c, up_c, down_c = compact(cam, dev, "W", keep, cfg.n_experts, cfg.d_ff)
        Y = cam.layer_forward_compact(dev["X"], idx, w, count, gate_c, up_c, down_c)
        mfma = cfg.n_tokens * cfg.top_k // cfg.n_experts > 64 and cfg.d_model % 16 == 0
        for align in (8, 64):   # zero-padded W_down rows
            count_a, gate_a, up_a, down_a = compact(cam, dev, "W", keep, cfg.n_experts, cfg.d_ff, align=align)
            Y_a = cam.layer_forward_compact(dev["X"], idx, w, count_a, gate_a, up_a, down_a, down_row_align=align)
            torch.cuda.synchronize()
            if mfma:            # large batch and aligned rows: the grouped MFMA kernel takes over
                O_a = orc.layer_forward(X64, A, gate, up, down, keep=keep, round_hidden=orc.round_to_bf16)
                check_output(Y_a, O_a, largest_term(X64, A, gate, up, down, keep))
            else:               # the streaming kernels: the same sums, bit for bit
                assert torch.equal(Y, Y_a), align
        Y_masked = cam.layer_forward(dev["X"], idx, w, dev["W_gate"], dev["W_up"], dev["W_down"],
                                     keep_mask=torch.from_numpy(keep).cuda())
        torch.cuda.synchronize()
        O = orc.layer_forward(X64, A, gate, up, down, keep=keep, round_hidden=orc.round_to_bf16)
        term = largest_term(X64, A, gate, up, down, keep)
        err = check_output(Y, O, term)
        # against the masked layer of the grouped MFMA kernel: same values up to summation order and rounding flips
        err_masked = check_output(Y, Y_masked.cpu().numpy().astype(np.float64), term)
        print(f"{case} keep {frac}: rel err {err:.2e}, against the masked layer {err_masked:.2e}, counts {count[:6]}")


def compact_layer(cam, dev, cfg, keep_r, keep_s, align):
    """Routed and shared experts compacted into one set of buffers: the shared group's rows and blocks behind the routed."""
    d = cfg.d_model
    parts = [("W", keep_r, cfg.n_experts, cfg.d_ff), ("Ws", keep_s, cfg.n_shared, cfg.d_ff_shared)]
    per_expert = [np.asarray(keep).astype(bool).reshape(n_e, f).sum(axis=1).astype(np.int32) for _, keep, n_e, f in parts]
    total = int(sum(c.sum() for c in per_expert))
    total_ld = int(sum((-(-int(c) // align) * align) for cs in per_expert for c in cs))
    gate_c = torch.empty((total, d), dtype=torch.bfloat16, device="cuda")
    up_c = torch.empty_like(gate_c)
    down_c = torch.empty(total_ld * d, dtype=torch.bfloat16, device="cuda")
    counts, at, at_ld = [], 0, 0
    for (prefix, keep, n_e, f), count in zip(parts, per_expert):
        index = torch.from_numpy(np.flatnonzero(np.asarray(keep)).astype(np.int32)).cuda()
        k = int(count.sum())
        k_ld = int(sum(-(-int(c) // align) * align for c in count))
        cam.gather_micro_experts(dev[prefix + "_gate"], dev[prefix + "_up"], dev[prefix + "_down"], index,
                                 torch.from_numpy(count).cuda(), down_row_align=align,
                                 out=(gate_c[at:at + k], up_c[at:at + k], down_c[at_ld * d:(at_ld + k_ld) * d]))
        counts += [int(c) for c in count]
        at += k
        at_ld += k_ld
    return counts, gate_c, up_c, down_c


# 700 tokens: more pairs than the one-workgroup bucket kernel takes; a shared expert of 7000: three K chunks in the
# second contraction (ragged: 0.6 * 7000 kept)
@pytest.mark.parametrize("n_tokens,n_shared,d_ff_shared", [(7, 2, 200), (64, 2, 200), (90, 2, 200), (700, 2, 200),
                                                           (64, 1, 7000), (40, 2, 3500)])
def test_shared_experts_in_the_same_call_and_accumulated(cam, n_tokens, n_shared, d_ff_shared):
    cfg = small(n_tokens=n_tokens, n_shared=n_shared, d_ff_shared=d_ff_shared, d_model=64 if d_ff_shared > 1000 else 128)
    layer = inputs.make_layer(cfg, 0, device="cpu")
    dev = H.to_dev(layer)
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    rng = np.random.default_rng(5)
    keep_r = (rng.random(cfg.n_experts * cfg.d_ff) < 0.6).astype(np.uint8)
    keep_s = (rng.random(cfg.n_shared * cfg.d_ff_shared) < 0.6).astype(np.uint8)
    cr, gr, ur, dr = compact(cam, dev, "W", keep_r, cfg.n_experts, cfg.d_ff)
    cs, gs, us, ds = compact(cam, dev, "Ws", keep_s, cfg.n_shared, cfg.d_ff_shared)
    Y = cam.layer_forward_compact(dev["X"], idx, w, cr, gr, ur, dr)
    Y_routed = Y.clone()
    cam.layer_forward_compact(dev["X"], None, None, cs, gs, us, ds, Y=Y, accumulate=True)
    Y_shared = cam.layer_forward_compact(dev["X"], None, None, cs, gs, us, ds)
    align = 64 if n_tokens % 2 == 0 else 1
    call, gc, uc, dc = compact_layer(cam, dev, cfg, keep_r, keep_s, align)
    Y_one = cam.layer_forward_compact(dev["X"], idx, w, call, gc, uc, dc, n_shared=cfg.n_shared, down_row_align=align)
    torch.cuda.synchronize()
    # the same terms in another order of summation: equal up to float32 rounding
    scale = Y.abs().max().item()
    assert (Y - (Y_routed + Y_shared)).abs().max().item() <= 4e-7 * scale
    one_call_on_mfma = align % 8 == 0 and n_tokens * (cfg.top_k + cfg.n_shared) // (cfg.n_experts + cfg.n_shared) > 64
    if not one_call_on_mfma:   # otherwise another kernel, whose hidden values may round to the other bf16 neighbour
        assert (Y - Y_one).abs().max().item() <= 1e-6 * scale
    X64 = H.f64(layer["X"])
    gate, up, down = expert_lists(layer, "Ws")
    ones = np.ones((cfg.n_tokens, cfg.n_shared))
    O_s = orc.layer_forward(X64, ones, gate, up, down, keep=keep_s, round_hidden=orc.round_to_bf16)
    term_s = largest_term(X64, ones, gate, up, down, keep_s)
    check_output(Y_shared, O_s, term_s)
    if n_tokens > 64:          # every token through every shared expert on the tiled path (aligned W_down rows)
        ca, ga, ua, da = compact(cam, dev, "Ws", keep_s, cfg.n_shared, cfg.d_ff_shared, align=8)
        Y_tiled = cam.layer_forward_compact(dev["X"], None, None, ca, ga, ua, da, down_row_align=8)
        torch.cuda.synchronize()
        check_output(Y_tiled, O_s, term_s)
    # the whole layer in one call against the oracle's routed + shared layer
    A = dense_A(idx.cpu().numpy().astype(np.int64), w.cpu().numpy().astype(np.float64), cfg.n_experts)
    gate_r, up_r, down_r = expert_lists(layer, "W")
    O_r = orc.layer_forward(X64, A, gate_r, up_r, down_r, keep=keep_r, round_hidden=orc.round_to_bf16)
    check_output(Y_one, O_r + O_s, np.maximum(term_s, largest_term(X64, A, gate_r, up_r, down_r, keep_r)))


def test_nothing_kept_and_bad_arguments(cam):
    cfg = small(n_tokens=16)
    dev = H.to_dev(inputs.make_layer(cfg, 0, device="cpu"))
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    empty = torch.empty((0, cfg.d_model), dtype=torch.bfloat16, device="cuda")
    Y = cam.layer_forward_compact(dev["X"], idx, w, [0] * cfg.n_experts, empty, empty, empty.reshape(-1))
    torch.cuda.synchronize()
    assert torch.count_nonzero(Y).item() == 0
    with pytest.raises(binding.CameraError, match="count"):
        cam.layer_forward_compact(dev["X"], idx, w, [-1] + [0] * (cfg.n_experts - 1), empty, empty, empty.reshape(-1))
    with pytest.raises(binding.CameraError, match="n_shared"):
        cam.layer_forward_compact(dev["X"], None, None, [0] * cfg.n_experts, empty, empty, empty.reshape(-1), n_shared=1)
    with pytest.raises(binding.CameraError, match="BF16"):
        cam.layer_forward_compact(dev["X"].float(), idx, w, [0] * cfg.n_experts, empty, empty, empty.reshape(-1))


@pytest.mark.parametrize("name", ["deepseek-moe-16b", "qwen2-57b-a14b"])
def test_full_size_layer_decoding_batch(cam, name):
    """A whole layer of the benchmark shape in the launch configuration bench.py times: 64 tokens, routed and
    shared experts compacted into one set of buffers with cache-line-aligned W_down rows, one call.  The oracle
    recomputes every token over the experts the batch uses."""
    cfg = inputs.CONFIGS[name]
    layer = inputs.make_layer(cfg, 0, device="cuda")
    X = layer["X"][:64]
    idx, w = cam.route_topk(X, layer["W_r"], layer["bias"], cfg.top_k)
    keep = (torch.rand(cfg.n_micro, generator=torch.Generator().manual_seed(9)) < 0.6).to(torch.uint8).numpy()
    nr = cfg.n_micro_routed
    counts, gate_c, up_c, down_c = compact_layer(cam, layer, cfg, keep[:nr], keep[nr:], 64)
    Y = cam.layer_forward_compact(X, idx, w, counts, gate_c, up_c, down_c, n_shared=cfg.n_shared, down_row_align=64)
    again = cam.layer_forward_compact(X, idx, w, counts, gate_c, up_c, down_c, n_shared=cfg.n_shared, down_row_align=64)
    torch.cuda.synchronize()
    assert torch.equal(Y, again)                                   # no atomics: the same bits every time
    X64 = H.f64(X)
    A = dense_A(idx.cpu().numpy().astype(np.int64), w.cpu().numpy().astype(np.float64), cfg.n_experts)
    used = np.nonzero(A.sum(axis=0))[0]
    gate = [H.f64(layer["W_gate"][e]) for e in used]
    up = [H.f64(layer["W_up"][e]) for e in used]
    down = [H.f64(layer["W_down"][e]) for e in used]
    keep_used = np.concatenate([keep[e * cfg.d_ff:(e + 1) * cfg.d_ff] for e in used])
    O = orc.layer_forward(X64, A[:, used], gate, up, down, keep=keep_used, round_hidden=orc.round_to_bf16)
    term = largest_term(X64, A[:, used], gate, up, down, keep_used)
    del gate, up, down
    g2, u2, d2 = expert_lists(layer, "Ws")
    ones = np.ones((64, cfg.n_shared))
    O += orc.layer_forward(X64, ones, g2, u2, d2, keep=keep[nr:], round_hidden=orc.round_to_bf16)
    term = np.maximum(term, largest_term(X64, ones, g2, u2, d2, keep[nr:]))
    err = check_output(Y, O, term)
    print(f"{name}: 64-token batch, {len(used)} routed experts used, rel err {err:.2e}")


def run_and_check(cam, cfg, keep_frac, align, seed=3):
    """One merged call (routed + shared, if any) on a small layer against the oracle's masked layer."""
    layer = inputs.make_layer(cfg, 0, device="cpu")
    dev = H.to_dev(layer)
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], cfg.top_k)
    rng = np.random.default_rng(seed)
    keep = (rng.random(cfg.n_micro) < keep_frac).astype(np.uint8)
    nr = cfg.n_micro_routed
    X64 = H.f64(layer["X"])
    A = dense_A(idx.cpu().numpy().astype(np.int64), w.cpu().numpy().astype(np.float64), cfg.n_experts)
    gate, up, down = expert_lists(layer, "W")
    O = orc.layer_forward(X64, A, gate, up, down, keep=keep[:nr], round_hidden=orc.round_to_bf16)
    term = largest_term(X64, A, gate, up, down, keep[:nr])
    if cfg.n_shared:
        counts, gate_c, up_c, down_c = compact_layer(cam, dev, cfg, keep[:nr], keep[nr:], align)
        g2, u2, d2 = expert_lists(layer, "Ws")
        ones = np.ones((cfg.n_tokens, cfg.n_shared))
        O += orc.layer_forward(X64, ones, g2, u2, d2, keep=keep[nr:], round_hidden=orc.round_to_bf16)
        term = np.maximum(term, largest_term(X64, ones, g2, u2, d2, keep[nr:]))
    else:
        counts, gate_c, up_c, down_c = compact(cam, dev, "W", keep, cfg.n_experts, cfg.d_ff, align=align)
    Y = cam.layer_forward_compact(dev["X"], idx, w, counts, gate_c, up_c, down_c, n_shared=cfg.n_shared,
                                  down_row_align=align)
    torch.cuda.synchronize()
    return check_output(Y, O, term), counts


def test_built_limits_of_the_compacted_layer(cam):
    # a shared expert that keeps more than 8 chunks' worth: the chunk count is capped and the chunks grow
    err, counts = run_and_check(cam, small(n_tokens=40, d_model=32, d_ff=64, n_experts=4, n_shared=1, d_ff_shared=32768),
                                0.93, 64)
    assert counts[-1] > 8 * 3072
    # exactly as many pairs as the one-workgroup bucket kernel takes, and one token more (general counting sort)
    run_and_check(cam, small(n_tokens=512, d_model=32, d_ff=40, n_experts=8, top_k=3, n_shared=1, d_ff_shared=48), 0.7, 1)
    run_and_check(cam, small(n_tokens=513, d_model=32, d_ff=40, n_experts=8, top_k=3, n_shared=1, d_ff_shared=48), 0.7, 8)
    # more 32-token groups than the grid has rows (64): the workgroups of the last row walk on
    run_and_check(cam, small(n_tokens=2100, d_model=32, d_ff=24, n_experts=2, top_k=2, n_shared=1, d_ff_shared=40), 0.8, 64)
    # the largest row alignment, and the largest number of experts in one call
    run_and_check(cam, small(n_tokens=9, d_model=32, d_ff=16, n_experts=4, top_k=2), 0.5, 512)
    run_and_check(cam, small(n_tokens=30, d_model=32, d_ff=8, n_experts=250, top_k=4, n_shared=6, d_ff_shared=8,
                             router_bias="none"), 0.6, 1)
    dev = H.to_dev(inputs.make_layer(small(n_tokens=4, d_model=32, d_ff=8, n_experts=250, top_k=4, router_bias="none"), 0))
    idx, w = cam.route_topk(dev["X"], dev["W_r"], dev["bias"], 4)
    empty = torch.empty((0, 32), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.CameraError, match="n_shared"):
        cam.layer_forward_compact(dev["X"], idx, w, [0] * 257, empty, empty, empty.reshape(-1), n_shared=7)
    with pytest.raises(binding.CameraError, match="down_row_align"):
        cam.layer_forward_compact(dev["X"], idx, w, [0] * 250, empty, empty, empty.reshape(-1), down_row_align=513)


@pytest.mark.parametrize("seed", range(16))
def test_seeded_shapes_inside_the_limits(cam, seed):
    """Shapes drawn from a seed (token count, widths, experts, top-k, shared experts, row alignment, kept fraction):
    the streaming kernels, the one-workgroup and the general bucket order and the tiled path all get their share."""
    rng = np.random.default_rng(1000 + seed)
    n_experts = int(rng.integers(1, 13))
    tokens = [1, 3, 17, 64, 65] if seed < 8 else [130, 400, 1100, 2500]   # the second half mostly on the tiled path
    cfg = small(n_tokens=int(rng.choice(tokens)), d_model=int(rng.choice([32, 40, 64, 72, 128, 144])),
                d_ff=8 * int(rng.integers(1, 40)), n_experts=n_experts, top_k=int(rng.integers(1, min(n_experts, 6) + 1)),
                n_shared=int(rng.integers(0, 3)), d_ff_shared=8 * int(rng.integers(1, 60)),
                router_bias=str(rng.choice(["none", "normal", "zipf"])))
    align = int(rng.choice([1, 2, 8, 24, 64, 128]))
    err, counts = run_and_check(cam, cfg, float(rng.uniform(0.05, 1.0)), align, seed=seed)
    print(f"seed {seed}: {cfg.n_tokens} tokens, d_model {cfg.d_model}, d_ff {cfg.d_ff}, {cfg.n_experts} experts top-{cfg.top_k}, "
          f"{cfg.n_shared} shared of {cfg.d_ff_shared}, align {align}: rel err {err:.2e}")
