"""CPU-only checks of the host-side pieces around the kernels: the input generators, the
bench command line, and the package layout rules (the product path never imports the oracle)."""
import os
import re
import subprocess
import sys

import numpy as np
import torch

from paper_2508_02322_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_inputs_are_seeded_and_shaped():
    cfg = inputs.scaled(inputs.CONFIGS["qwen2-57b-a14b"], n_tokens=64, d_model=32, d_ff=16, n_experts=4, top_k=2,
                        n_shared=1, d_ff_shared=48, outlier_channels=2)
    a, b = inputs.make_layer(cfg, 3), inputs.make_layer(cfg, 3)
    for k in a:
        assert (a[k] is None and b[k] is None) or torch.equal(a[k], b[k]), k
    other = inputs.make_layer(cfg, 4)
    assert not torch.equal(a["X"], other["X"])
    assert a["X"].shape == (64, 32) and a["X"].dtype == torch.bfloat16
    assert a["W_gate"].shape == (4, 16, 32) and a["W_down"].shape == (4, 32, 16)
    assert a["Ws_gate"].shape == (1, 48, 32) and a["Ws_down"].shape == (1, 32, 48)
    # two outlier channels, the same for every token, about 20 times larger than the rest
    col = a["X"].float().abs().mean(dim=0)
    top2 = torch.topk(col, 2).values
    assert top2.min() > 8 * col.median()
    assert inputs.segment_offsets(cfg) == [0, 16, 32, 48, 64, 112]
    assert cfg.n_micro == 112 and cfg.n_micro_routed == 64


def test_router_bias_kinds():
    base = inputs.scaled(inputs.CONFIGS["qwen3-30b-a3b"], n_tokens=8, d_model=16, d_ff=8, n_experts=16, top_k=2)
    zipf = inputs.make_layer(base, 0)["bias"].numpy()
    want = -np.log1p(np.arange(16, dtype=np.float32))
    np.testing.assert_allclose(np.sort(zipf)[::-1], want, rtol=1e-6)
    normal = inputs.make_layer(inputs.scaled(inputs.CONFIGS["mixtral"], n_tokens=8, d_model=16, d_ff=8), 0)["bias"]
    assert normal.shape == (8,) and normal.dtype == torch.float32
    assert inputs.make_layer(inputs.CONFIGS["tiny"], 0)["bias"] is None


def test_config_table_matches_the_benchmark_shapes():
    c = inputs.CONFIGS
    assert (c["tiny"].n_experts, c["tiny"].d_model, c["tiny"].d_ff, c["tiny"].top_k, c["tiny"].n_tokens, c["tiny"].dtype) == \
        (8, 256, 512, 2, 512, "f32")
    assert (c["mixtral"].d_model, c["mixtral"].d_ff, c["mixtral"].n_tokens) == (4096, 14336, 4096)
    assert (c["deepseek-moe-16b"].n_layers, c["deepseek-moe-16b"].top_k, c["deepseek-moe-16b"].n_shared) == (28, 6, 2)
    q2 = c["qwen2-57b-a14b"]
    assert q2.n_micro == 64 * 2560 + 20480 == 184320 and q2.alpha == 0.95
    assert abs(q2.gemm_flops_per_layer() - 4.81e12) < 0.01e12
    q3 = c["qwen3-30b-a3b"]
    assert (q3.n_layers, q3.n_experts, q3.d_ff, q3.n_tokens, q3.alpha) == (48, 128, 768, 16384, 1.0)


def test_energy_like_has_ties_and_zeros():
    E = inputs.energy_like(10000, seed=1)
    assert E.dtype == torch.float32 and (E >= 0).all()
    assert (E == 0).sum() >= 400
    vals, counts = torch.unique(E[E > 0], return_counts=True)
    assert counts.max() >= 100


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "one GPU" in res.stderr


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2508_02322_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, name)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), name
                assert "camera_oracle" not in text, name
    oracle_text = open(os.path.join(ROOT, "oracle", "camera_oracle.py")).read()
    assert "paper_2508_02322_amd" not in re.sub(r'""".*?"""', "", oracle_text, flags=re.S)


def test_binding_refuses_layouts_the_library_cannot_see():
    """A transposed or sliced view, a foreign dtype or device: an error, not silently wrong scores.  The checks run
    before anything touches the GPU, so host tensors serve here."""
    import pytest
    from paper_2508_02322_amd import binding
    cam = binding.Camera(device=0)      # creation touches no GPU
    bf = torch.bfloat16
    X = torch.zeros((16, 32), dtype=bf)
    W_r = torch.zeros((4, 32), dtype=bf)
    Wg = torch.zeros((4, 8, 32), dtype=bf)
    Wd = torch.zeros((4, 32, 8), dtype=bf)
    idx = torch.zeros((16, 2), dtype=torch.int32)
    w = torch.zeros((16, 2), dtype=torch.float32)

    def refused(fn, *a, **kw):
        with pytest.raises(binding.CameraError) as exc:
            fn(*a, **kw)
        assert exc.value.code == -2, exc.value
        return exc.value.message

    assert "X" in refused(cam.route_topk, torch.zeros((32, 16), dtype=bf).t(), W_r, None, 2)          # transposed
    assert "W_r" in refused(cam.route_topk, X, torch.zeros((4, 64), dtype=bf)[:, ::2], None, 2)       # inner stride 2
    assert "W_r" in refused(cam.route_topk, X, W_r.float(), None, 2)                                  # dtype differs
    assert "W_gate" in refused(cam.score_layer, X, idx, w, Wg.transpose(1, 2).contiguous().transpose(1, 2), Wg, Wd, 0.5)
    assert "W_up" in refused(cam.score_layer, X, idx, w, Wg, torch.zeros((4, 8, 64), dtype=bf)[:, :, :32], Wd, 0.5)  # rows too far apart
    assert "W_down" in refused(cam.score_layer, X, idx, w, Wg, Wg, Wg, 0.5)                            # not [experts, d_model, d_ff]
    assert "topk_w" in refused(cam.score_layer, X, idx, w.double(), Wg, Wg, Wd, 0.5)
    assert "energy" in refused(cam.select_prune, torch.zeros(64)[::2], [0, 32], 0.5)
    assert "energy" in refused(cam.alloc_bits, torch.zeros(32, dtype=torch.float64), [0, 32], [3, 2], [0.5, 0.5])
    assert "Y" in refused(cam.layer_forward, X, idx, w, Wg, Wg, Wd, Y=torch.zeros((32, 16)).t())
    cam.close()
