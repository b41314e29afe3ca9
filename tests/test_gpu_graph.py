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
