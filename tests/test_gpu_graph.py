"""The launch sequence of a layer can be captured in a HIP graph once the context workspace has its size
(no allocation, no host synchronisation and no memset node inside the calls): the replays must give what the
eager calls give, also after the inputs changed in place."""
import numpy as np
import pytest
import torch

from paper_2508_02322_amd import inputs
from tests import helpers as H

pytestmark = pytest.mark.gpu


def test_layer_step_replays_from_a_graph(cam):
    cfg = inputs.scaled(inputs.CONFIGS["mixtral"], n_tokens=600, d_model=128, d_ff=192, n_experts=8, top_k=2, n_layers=1,
                        outlier_channels=2)
    dev = H.to_dev(inputs.make_layer(cfg, 0, device="cpu"))
    seg = inputs.segment_offsets(cfg)
    X = dev["X"].clone()
    out = {k: torch.empty(cfg.n_micro, dtype=torch.float32, device="cuda") for k in ("phi2", "phi_inf", "omega2", "energy")}
    prune_out = (torch.empty(cfg.n_micro, dtype=torch.uint8, device="cuda"),
                 torch.empty((3, len(seg) - 1), dtype=torch.int32, device="cuda"))

    def step():
        idx, w = cam.route_topk(X, dev["W_r"], dev["bias"], cfg.top_k)
        cam.score_layer(X, idx, w, dev["W_gate"], dev["W_up"], dev["W_down"], cfg.alpha, out=out)
        cam.select_prune_multi(out["energy"], seg, [0.2, 0.4, 0.6], out=prune_out)

    step()                                   # sizes the workspace (the only allocation the library makes)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            step()
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda").manual_seed(7)
    for trial in range(4):
        if trial:                            # new inputs in place: the graph reads the same buffers
            X.copy_(torch.randn(X.shape, generator=gen, device="cuda").to(X.dtype))
        graph.replay()
        torch.cuda.synchronize()
        got_e, got_bits, got_per = out["energy"].clone(), prune_out[0].clone(), prune_out[1].clone()
        out["energy"].zero_()
        prune_out[0].zero_()
        step()                               # eager work and a synchronisation between the replays
        torch.cuda.synchronize()
        assert torch.equal(got_e, out["energy"]) and torch.equal(got_bits, prune_out[0]) and torch.equal(got_per, prune_out[1])
        assert float(got_e.sum()) > 0


def test_compacted_layer_replays_from_a_graph(cam):
    """The decoding call (routing, bucket order, both streaming contractions, combine) captured once and replayed
    with new tokens in the same buffer."""
    cfg = inputs.scaled(inputs.CONFIGS["deepseek-moe-16b"], n_tokens=64, d_model=128, d_ff=200, n_experts=16, top_k=4,
                        n_shared=1, d_ff_shared=264, n_layers=1)
    dev = H.to_dev(inputs.make_layer(cfg, 0, device="cpu"))
    X = dev["X"].clone()
    rng = np.random.default_rng(2)
    counts, index = [], []
    for prefix, n_e, f, base in (("W", cfg.n_experts, cfg.d_ff, 0), ("Ws", cfg.n_shared, cfg.d_ff_shared, 0)):
        keep = rng.random(n_e * f) < 0.6
        counts.append(keep.reshape(n_e, f).sum(axis=1).astype(np.int32))
        index.append(np.flatnonzero(keep).astype(np.int32))
    align = 64
    ld = [(-(-c // align) * align) for c in counts]
    rows = [int(c.sum()) for c in counts]
    gate_c = torch.empty((sum(rows), cfg.d_model), dtype=torch.bfloat16, device="cuda")
    up_c = torch.empty_like(gate_c)
    down_c = torch.empty(int(sum(l.sum() for l in ld)) * cfg.d_model, dtype=torch.bfloat16, device="cuda")
    at, at_ld = 0, 0
    for g, prefix in enumerate(("W", "Ws")):
        k, k_ld = rows[g], int(ld[g].sum())
        cam.gather_micro_experts(dev[prefix + "_gate"], dev[prefix + "_up"], dev[prefix + "_down"],
                                 torch.from_numpy(index[g]).cuda(), torch.from_numpy(counts[g]).cuda(), down_row_align=align,
                                 out=(gate_c[at:at + k], up_c[at:at + k], down_c[at_ld * cfg.d_model:(at_ld + k_ld) * cfg.d_model]))
        at, at_ld = at + k, at_ld + k_ld
    count_all = [int(c) for cs in counts for c in cs]
    Y = torch.empty((cfg.n_tokens, cfg.d_model), dtype=torch.float32, device="cuda")

    def step():
        idx, w = cam.route_topk(X, dev["W_r"], dev["bias"], cfg.top_k)
        cam.layer_forward_compact(X, idx, w, count_all, gate_c, up_c, down_c, n_shared=cfg.n_shared, down_row_align=align, Y=Y)

    step()
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            step()
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda").manual_seed(11)
    for trial in range(4):
        if trial:
            X.copy_(torch.randn(X.shape, generator=gen, device="cuda").to(X.dtype))
        graph.replay()
        torch.cuda.synchronize()
        got = Y.clone()
        Y.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(got, Y) and float(got.abs().sum()) > 0
