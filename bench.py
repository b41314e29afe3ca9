#!/usr/bin/env python3
"""Benchmark of the CAMERA scoring hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole hot path over every MoE layer of the workload:
route (Top&Norm) -> bucket -> grouped gate/up contraction with fused epilogue ->
W_down column norms -> energy -> CAMERA-P masks / CAMERA-Q bit allocation.  All
inputs (seeded synthetic tensors of the model's shapes) are resident in HBM
before the timed region starts.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3       # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

# Decisions taken per layer after scoring: CAMERA-P ratios and CAMERA-Q (bits, ratios) settings.
DECISIONS = {
    "tiny": dict(prune=[0.4], alloc=[]),
    "mixtral": dict(prune=[0.2, 0.4, 0.6], alloc=[]),
    "deepseek-moe-16b": dict(prune=[0.2, 0.4, 0.6], alloc=[]),
    "qwen2-57b-a14b": dict(prune=[0.2, 0.4, 0.6], alloc=[([3, 2, 1], [0.2, 0.6, 0.2])]),
    "qwen3-30b-a3b": dict(prune=[], alloc=[([3, 2, 1], [0.2, 0.6, 0.2]), ([4, 3, 2], [0.1, 0.3, 0.6]),
                                           ([4, 3, 2], [0.0, 0.0, 1.0])]),
}

# HBM-side bytes per grouped-GEMM launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by what the same
# counters read for a plain 1 GiB copy; not measured by this program: the figure and the file it comes from are
# reported side by side (None where no such profile exists).
PMC_TRAFFIC = {"qwen2-57b-a14b": (6.000e9, "profiles/grouped_gemm_bf16_qwen2-57b-a14b_hbm_traffic.txt")}
PMC_NORM_TRAFFIC = {"qwen2-57b-a14b": (6.651e8, "profiles/down_norm_qwen2-57b-a14b_hbm_traffic.txt")}
# The same for the two streaming kernels of the compacted layer on a 64-token batch, unpruned
# (profiles/compact_layer_decode_hbm_traffic.txt): read + written bytes per call.
PMC_DECODE_TRAFFIC_BYTES = {"deepseek-moe-16b": 777.0e6 + 392.5e6 + 5.6e6, "qwen2-57b-a14b": 2976.9e6 + 1522.0e6 + 19.0e6}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="qwen2-57b-a14b", choices=sorted(DECISIONS))
    ap.add_argument("--layers", type=int, default=0, help="debug: only this many layers (the result is then not the named workload)")
    ap.add_argument("--calib-tokens", type=int, default=0,
                    help="calibration tokens per layer (default: the configuration's own); more than that are fed "
                         "in chunks of the configuration's size through CAMERA_ACCUMULATE (the paper calibrates on "
                         "128 x 2048 = 262144 tokens)")
    ap.add_argument("--chunk-tokens", type=int, default=0, help="chunk size for --calib-tokens (default: the configuration's token count)")
    ap.add_argument("--streams", type=int, default=1,
                    help="run consecutive layers on this many HIP streams (one library context each), so that the tail of one "
                         "layer's kernels overlaps the start of the next layer's; per-kernel timings then overlap as well")
    ap.add_argument("--energy-spread", type=float, default=0.0,
                    help="scale every W_down column by a log-normal factor of this sigma (per expert and per micro-expert): "
                         "energies and per-expert kept counts as uneven as on trained models; 0 = the named workload")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short timed runs of the other benchmark configurations after the main one")
    ap.add_argument("--other-steps", type=int, default=5, help="timed steps of each of the other configurations")
    ap.add_argument("--no-streamed", action="store_true",
                    help="skip the streamed calibration of the paper's size (128 x 2048 tokens in chunks) after the main run")
    ap.add_argument("--streamed-tokens", type=int, default=262144)
    ap.add_argument("--streamed-chunk", type=int, default=16384)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the measured MFMA / HBM ceilings (about 1 s)")
    ap.add_argument("--no-forward", action="store_true",
                    help="skip the measurement of the pruned layer's output and its decoding error")
    ap.add_argument("--decode-ratios", default="0,0.2,0.4,0.6",
                    help="pruning ratios of the decode measurement (comma separated; the first is the reference of the speed-ups)")
    ap.add_argument("--no-decode", action="store_true",
                    help="skip the measurement of a pruned layer's output from compacted weights on a 64-token batch")
    ap.add_argument("--no-apply", action="store_true",
                    help="skip the measurement of applying a 40 %% mask (gather of the kept micro-experts)")
    return ap.parse_args()


class LayerRunner:
    """Owns the resident tensors of one layer and its preallocated outputs."""

    def __init__(self, cam, cfg, layer_idx, torch, inputs, calib_tokens, chunk_tokens):
        self.cfg = cfg
        gen_cfg = cfg if calib_tokens == cfg.n_tokens else inputs.scaled(cfg, n_tokens=calib_tokens)
        self.t = inputs.make_layer(gen_cfg, layer_idx, device="cuda")
        self.chunks = [(lo, min(calib_tokens, lo + chunk_tokens)) for lo in range(0, calib_tokens, chunk_tokens)]
        n_micro = cfg.n_micro
        self.out = {k: torch.empty(n_micro, dtype=torch.float32, device="cuda")
                    for k in ("phi2", "phi_inf", "omega2", "energy")}
        nr = cfg.n_micro_routed
        self.out_routed = {k: v[:nr] for k, v in self.out.items()}
        self.out_shared = {k: v[nr:] for k, v in self.out.items()}
        self.seg = inputs.segment_offsets(cfg)
        self.prune_out = None

    def run(self, cam, decisions, binding):
        cfg, t = self.cfg, self.t
        last = len(self.chunks) - 1
        for c, (lo, hi) in enumerate(self.chunks):
            X = t["X"][lo:hi]
            flags = (binding.ACCUMULATE if c > 0 else 0) | (binding.NO_FINALIZE if c < last else 0)
            idx, w = cam.route_topk(X, t["W_r"], t["bias"], cfg.top_k)
            cam.score_layer(X, idx, w, t["W_gate"], t["W_up"], t["W_down"], cfg.alpha, flags=flags, out=self.out_routed)
            if cfg.n_shared:
                cam.score_layer(X, None, None, t["Ws_gate"], t["Ws_up"], t["Ws_down"], cfg.alpha, flags=flags,
                                out=self.out_shared)
        res = []
        alloc = list(decisions["alloc"])
        if decisions["prune"] and alloc:   # masks and the first bit allocation from one pass over the ranking
            bits, ratios = alloc.pop(0)
            res.append(cam.rank_decisions(self.out["energy"], self.seg, decisions["prune"], bits, ratios))
        elif decisions["prune"]:           # every CAMERA-P mask of the workload from one pass
            res.append(cam.select_prune_multi(self.out["energy"], self.seg, decisions["prune"], out=self.prune_out))
        for bits, ratios in alloc:
            res.append(cam.alloc_bits(self.out["energy"], self.seg, bits, ratios))
        return res


def measure_apply(cam, cfg, layers, torch, binding, ratio=0.4, reps=3):
    """Applies a CAMERA-P mask: gathers the kept gate / up rows and down columns of every expert of up to
    four layers (outside the timed step: it is the stage after the scoring path).  Returns the HBM-bound
    roofline of that launch group: algorithmic bytes = each kept vector read once and written once."""
    use = layers[:4]
    es = 2 if cfg.dtype == "bf16" else 4
    n_keep_max = cfg.n_micro
    bufs = [torch.empty(n_keep_max * cfg.d_model, dtype=use[0].t["W_gate"].dtype, device="cuda") for _ in range(3)]
    plans = []
    for lr in use:
        keep, per, kept_idx, _ = cam.select_prune(lr.out["energy"], lr.seg, ratio, want_idx=True)
        per_h = per.cpu()
        groups = [("W", cfg.n_experts, 0, 0)]
        if cfg.n_shared:
            groups.append(("Ws", cfg.n_shared, cfg.n_experts, cfg.n_micro_routed))
        pos, plan = 0, []
        for prefix, n_e, seg0, base in groups:
            n_idx = int(per_h[seg0:seg0 + n_e].sum())
            plan.append((lr.t[prefix + "_gate"], lr.t[prefix + "_up"], lr.t[prefix + "_down"], kept_idx[pos:pos + n_idx],
                         per[seg0:seg0 + n_e], base, n_idx))
            pos += n_idx
        plans.append(plan)
    kept_vectors = 0

    def run():
        total = 0
        for plan in plans:
            at = 0
            for Wg, Wu, Wd, idx, cnt, base, n_idx in plan:
                if n_idx == 0:
                    continue
                d = cfg.d_model
                out = (bufs[0][at * d:(at + n_idx) * d].view(n_idx, d), bufs[1][at * d:(at + n_idx) * d].view(n_idx, d),
                       bufs[2][at * d:(at + n_idx) * d])
                cam.gather_micro_experts(Wg, Wu, Wd, idx, cnt, base, out=out)
                at += n_idx
            total += at
        return total

    run()
    torch.cuda.synchronize()
    cam.profile_read(binding.K_GATHER)
    cam.profile_enable(True)
    for _ in range(reps):
        kept_vectors = run()
    torch.cuda.synchronize()
    cam.profile_enable(False)
    ms, launches = cam.profile_read(binding.K_GATHER)
    ms_per_layer = ms / (reps * len(use))
    bytes_per_layer = 6.0 * (kept_vectors / len(use)) * cfg.d_model * es
    gbs = bytes_per_layer / (ms_per_layer * 1e-3) / 1e9
    return {"what": f"gather of the kept micro-experts at lambda = {ratio} (Algorithm 2, lines 10-13), {len(use)} layers",
            "ms_per_layer": round(ms_per_layer, 4), "bound": "hbm", "achieved": round(gbs, 1), "peak": 8000.0,
            "unit": "GB/s", "frac": round(gbs / 8000.0, 4), "algorithmic_bytes_per_layer": bytes_per_layer}


def measure_forward(cam, cfg, layers, torch, binding, ratio=0.4, reps=3):
    """Output of the original and of the pruned layer (CAMERA-P mask at lambda = ratio) and their distance, for up
    to two layers, outside the timed step.  Roofline: the second contraction Lambda W_down^T on the MFMA peak,
    algorithmic flops = 2 * d_ff * d_model per routed (token, expert) pair (+ per token and shared expert)."""
    if cfg.dtype != "bf16":
        return None
    use = layers[:2]
    n, d = cfg.n_tokens, cfg.d_model
    Y = torch.empty((n, d), dtype=torch.float32, device="cuda")
    Y_hat = torch.empty_like(Y)
    nr = cfg.n_micro_routed
    stats = []

    def forward(lr, keep, out):
        t = lr.t
        X = t["X"][:n]
        idx, w = cam.route_topk(X, t["W_r"], t["bias"], cfg.top_k)
        cam.layer_forward(X, idx, w, t["W_gate"], t["W_up"], t["W_down"], keep_mask=None if keep is None else keep[:nr], Y=out)
        if cfg.n_shared:
            cam.layer_forward(X, None, None, t["Ws_gate"], t["Ws_up"], t["Ws_down"],
                              keep_mask=None if keep is None else keep[nr:], Y=out, accumulate=True)

    def run(record):
        for lr in use:
            keep = cam.select_prune(lr.out["energy"], lr.seg, ratio)[0]
            forward(lr, None, Y)
            forward(lr, keep, Y_hat)
            per_token = cam.output_error(Y, Y_hat)
            if record:
                s4 = per_token.double().sum(dim=0).tolist()
                pruned = keep == 0
                e_sum = float((lr.out["phi2"].double() * lr.out["omega2"].double())[pruned].sum())
                stats.append({"l2": s4[0] ** 0.5, "cosine": s4[3] / max((s4[1] * s4[2]) ** 0.5, 1e-300),
                              "decoding_error_over_sum_of_pruned_energies_alpha0": s4[0] / max(e_sum, 1e-300)})

    run(False)
    torch.cuda.synchronize()
    for k in range(len(binding.KERNEL_NAMES)):
        cam.profile_read(k)
    cam.profile_enable(True)
    for r in range(reps):
        run(r == 0)
    torch.cuda.synchronize()
    cam.profile_enable(False)
    ms = {name: cam.profile_read(k) for k, name in enumerate(binding.KERNEL_NAMES)}
    launches = max(1, ms["down_gemm"][1])
    down_ms = ms["down_gemm"][0] / launches
    pairs = n * cfg.top_k
    flops_routed = 2.0 * cfg.d_ff * d * pairs
    flops_shared = 2.0 * cfg.d_ff_shared * d * n * cfg.n_shared
    calls_per_forward = 2 if cfg.n_shared else 1
    flops_per_launch = (flops_routed + flops_shared) / calls_per_forward
    achieved = flops_per_launch / (down_ms * 1e-3) / 1e12
    forwards = 2 * reps * len(use)
    # the same pruned layer from its compacted weights: work in proportion to what is kept
    lr = use[0]
    align = 64
    _, per, kept_idx, _ = cam.select_prune(lr.out["energy"], lr.seg, ratio, want_idx=True)
    per_h = per.cpu()
    ld = (per_h + (align - 1)) // align * align
    kept = int(per_h.sum())
    dt = lr.t["W_gate"].dtype
    gate_c = torch.empty((kept, d), dtype=dt, device="cuda")
    up_c = torch.empty_like(gate_c)
    down_c = torch.empty(int(ld.sum()) * d, dtype=dt, device="cuda")
    pos, pos_ld = 0, 0
    groups = [("W", cfg.n_experts, 0, 0)] + ([("Ws", cfg.n_shared, cfg.n_experts, cfg.n_micro_routed)] if cfg.n_shared else [])
    for prefix, n_e, seg0, base in groups:
        n_idx, n_ld = int(per_h[seg0:seg0 + n_e].sum()), int(ld[seg0:seg0 + n_e].sum())
        cam.gather_micro_experts(lr.t[prefix + "_gate"], lr.t[prefix + "_up"], lr.t[prefix + "_down"], kept_idx[pos:pos + n_idx],
                                 per[seg0:seg0 + n_e], base, down_row_align=align,
                                 out=(gate_c[pos:pos + n_idx], up_c[pos:pos + n_idx], down_c[pos_ld * d:(pos_ld + n_ld) * d]))
        pos, pos_ld = pos + n_idx, pos_ld + n_ld
    X = lr.t["X"][:n]
    idx, w = cam.route_topk(X, lr.t["W_r"], lr.t["bias"], cfg.top_k)
    Y_c = torch.empty_like(Y)
    run_c = lambda: cam.layer_forward_compact(X, idx, w, per_h.tolist(), gate_c, up_c, down_c, n_shared=cfg.n_shared,
                                              down_row_align=align, Y=Y_c)
    run_c()
    begin, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    begin.record()
    for _ in range(reps):
        run_c()
    end.record()
    torch.cuda.synchronize()
    compact_ms = begin.elapsed_time(end) / reps
    for k in range(len(binding.KERNEL_NAMES)):
        cam.profile_read(k)
    cam.profile_enable(True)
    for _ in range(reps):
        run_c()
    torch.cuda.synchronize()
    cam.profile_enable(False)
    compact_kernels = {name: round(cam.profile_read(k)[0] / reps, 4) for k, name in enumerate(binding.KERNEL_NAMES)
                       if name in ("bucket", "gemm", "down_gemm", "combine")}
    keep0 = cam.select_prune(lr.out["energy"], lr.seg, ratio)[0]
    forward(lr, keep0, Y_hat)
    torch.cuda.synchronize()
    compact_diff = float((Y_c - Y_hat).norm() / Y_hat.norm())
    del gate_c, up_c, down_c
    return {"what": f"layer output of the original and of the pruned layer (lambda = {ratio}) and their distance, {len(use)} layers",
            "ms_per_layer_output": round(sum(ms[k][0] for k in ("route", "bucket", "gemm", "down_gemm", "combine")) / forwards, 3),
            "kernel_ms_per_launch": {k: round(ms[k][0] / max(1, ms[k][1]), 4) for k in ("gemm", "down_gemm", "combine")},
            "roofline": {"kernel": "grouped_gemm_bf16 (Lambda W_down^T)", "bound": "mfma", "achieved": round(achieved, 1),
                         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                         "flops_per_launch": flops_per_launch, "avg_launch_ms": round(down_ms, 4)},
            "from_compacted_weights": {"ms_per_layer_output": round(compact_ms, 3), "tokens": n, "kernel_ms": compact_kernels,
                                       "relative_distance_from_the_masked_layer_output": compact_diff},
            "synthetic_layers": stats}


def measure_decode(cam, cfg, layers, torch, binding, ratios=(0.0, 0.2, 0.4, 0.6), batch=64, reps=30):
    """Output of one pruned layer from its compacted weights for a decoding batch of 64 tokens, at several pruning
    ratios (the setting of the paper's decoding-speed comparison of a pruned MoE layer), outside the timed step.
    The call is bound by reading the kept weights of the experts the batch activates: algorithmic bytes =
    3 * d_model * (kept micro-experts of the activated experts) * 2."""
    if cfg.dtype != "bf16":
        return None
    lr = layers[0]
    t, d = lr.t, cfg.d_model
    X = t["X"][:batch]
    idx, w = cam.route_topk(X, t["W_r"], t["bias"], cfg.top_k)
    active = torch.bincount(idx.flatten().long(), minlength=cfg.n_experts).cpu() > 0
    groups = [("W", cfg.n_experts, 0, 0)]
    if cfg.n_shared:
        groups.append(("Ws", cfg.n_shared, cfg.n_experts, cfg.n_micro_routed))
    Y = torch.empty((batch, d), dtype=torch.float32, device="cuda")
    rows = []
    names = ("bucket", "compact_hidden", "compact_down", "combine")
    dt = t["W_gate"].dtype
    align = 64
    for ratio in ratios:
        _, per, kept_idx, _ = cam.select_prune(lr.out["energy"], lr.seg, ratio, want_idx=True)
        per_h = per.cpu()
        kept = int(per_h.sum())
        ld = (per_h + (align - 1)) // align * align     # row lengths of the W_down blocks: zero-padded to whole cache lines
        # routed and shared experts compacted into one set of buffers: one call then runs the whole layer
        gate_c = torch.empty((kept, d), dtype=dt, device="cuda")
        up_c = torch.empty_like(gate_c)
        down_c = torch.empty(int(ld.sum()) * d, dtype=dt, device="cuda")
        pos, pos_ld, kept_bytes = 0, 0, 0.0
        for prefix, n_e, seg0, base in groups:
            counts = per_h[seg0:seg0 + n_e]
            n_idx, n_ld = int(counts.sum()), int(ld[seg0:seg0 + n_e].sum())
            cam.gather_micro_experts(t[prefix + "_gate"], t[prefix + "_up"], t[prefix + "_down"], kept_idx[pos:pos + n_idx],
                                     per[seg0:seg0 + n_e], base, down_row_align=align,
                                     out=(gate_c[pos:pos + n_idx], up_c[pos:pos + n_idx], down_c[pos_ld * d:(pos_ld + n_ld) * d]))
            read = counts[active] if prefix == "W" else counts
            kept_bytes += 3.0 * d * float(read.sum()) * 2.0
            pos += n_idx
            pos_ld += n_ld
        counts_all = per_h.tolist()

        def run():
            cam.layer_forward_compact(X, idx, w, counts_all, gate_c, up_c, down_c, n_shared=cfg.n_shared,
                                      down_row_align=align, Y=Y)

        for _ in range(3):
            run()
        torch.cuda.synchronize()
        for name in names:
            cam.profile_read(binding.KERNEL_NAMES.index(name))
        cam.profile_enable(True)
        for _ in range(reps):
            run()
        torch.cuda.synchronize()
        cam.profile_enable(False)
        ms = {name: cam.profile_read(binding.KERNEL_NAMES.index(name))[0] / reps for name in names}
        begin, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        begin.record()
        for _ in range(reps):
            run()
        end.record()
        torch.cuda.synchronize()
        stream_ms = begin.elapsed_time(end) / reps
        kernel_ms = ms["compact_hidden"] + ms["compact_down"]
        rows.append({"ratio": ratio, "ms_per_layer": round(stream_ms, 4), "kernel_ms": {k: round(v, 4) for k, v in ms.items()},
                     "kept_per_routed_expert_min_max": [int(per_h[:cfg.n_experts].min()), int(per_h[:cfg.n_experts].max())],
                     "kept_weight_bytes_read": kept_bytes, "gb_per_s": round(kept_bytes / (kernel_ms * 1e-3) / 1e9, 1)})
        del gate_c, up_c, down_c
    base = rows[0]
    for row in rows:
        row["speedup_vs_unpruned"] = round(base["ms_per_layer"] / row["ms_per_layer"], 3)
    return {"what": f"output of layer 0 from compacted weights, {batch} tokens, per pruning ratio (decoding-speed setting)",
            "batch_tokens": batch, "activated_routed_experts": int(active.sum()), "per_ratio": rows,
            "roofline": {"kernel": "compact_hidden + compact_down, unpruned layer", "bound": "hbm", "achieved": base["gb_per_s"],
                         "peak": 8000.0, "unit": "GB/s", "frac": round(base["gb_per_s"] / 8000.0, 4),
                         "traffic": PMC_DECODE_TRAFFIC_BYTES.get(cfg.name) if cfg.energy_spread == 0 and rows[0]["ratio"] == 0 else None,
                         "algorithmic_bytes": base["kept_weight_bytes_read"]}}


def cpu_baseline(cfg, inputs):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload: layer 0 with
    every expert cut down to a slice of its micro-experts (they are scored independently, so
    the cost is proportional to the slice); the time is scaled back to whole layers."""
    import numpy as np
    import torch
    from oracle import camera_oracle as orc

    def f64(t):
        return None if t is None else t.to(torch.float32).numpy().astype(np.float64)

    def score(prefix, A, channels):
        Wg, Wu, Wd = (layer[prefix + s][:, :channels] if s != "_down" else layer[prefix + s][:, :, :channels]
                      for s in ("_gate", "_up", "_down"))
        ne = Wg.shape[0]
        return orc.score_layer(f64(layer["X"]), A, [f64(Wg[e]) for e in range(ne)], [f64(Wu[e]) for e in range(ne)],
                               [f64(Wd[e]) for e in range(ne)], cfg.alpha)["energy"]

    layer = inputs.make_layer(cfg, 0, device="cpu")
    # aim at roughly 10-20 s of float64 matmul on the machine's host cores (measured ~0.5 TFLOP/s)
    budget_flops = 7e12
    frac = min(1.0, budget_flops / cfg.gemm_flops_per_layer())
    ch = max(8, int(cfg.d_ff * frac))
    ch_s = max(8, int(cfg.d_ff_shared * frac)) if cfg.n_shared else 0
    t0 = time.perf_counter()
    L = orc.router_logits(f64(layer["X"]), f64(layer["W_r"]), f64(layer["bias"]))
    _, _, A = orc.top_and_norm(L, cfg.top_k)
    E = [score("W", A, ch)]
    if cfg.n_shared:
        E.append(score("Ws", np.ones((cfg.n_tokens, cfg.n_shared)), ch_s))
    E = np.concatenate(E).astype(np.float32)
    orc.select_prune(E, [0, E.size], 0.4)
    dt = time.perf_counter() - t0
    scored = cfg.n_experts * ch + cfg.n_shared * ch_s
    full_layer_s = dt * cfg.n_micro / scored
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = torch.get_num_threads()
    return {"value": cfg.n_tokens / full_layer_s, "unit": "tokens*layers/s", "cores": int(cores), "kind": "oracle",
            "sample": f"layer 0, first {ch} of {cfg.d_ff} micro-experts of each routed expert"
                      + (f" and first {ch_s} of {cfg.d_ff_shared} of each shared expert" if cfg.n_shared else "")
                      + f", all {cfg.n_tokens} tokens, {dt:.1f} s measured, scaled by {cfg.n_micro / scored:.1f}x to a whole layer"}


def constant_operand_rate(cam, cfg, layer, torch, binding, reps=40):
    """The step's own contractions of one layer (same calls, same routing, same launch shapes) on constant operands
    (every hidden state 1, every weight 1/64): with nothing toggling in the multipliers the chip holds its full clock,
    so this is the rate the kernel's schedule sustains when power does not limit it."""
    t = layer.t
    idx, w = cam.route_topk(t["X"], t["W_r"], t["bias"], cfg.top_k)
    X = torch.ones_like(t["X"])
    def stats(n_micro):   # NO_FINALIZE calls write these two only
        return {k: torch.empty(n_micro, dtype=torch.float32, device="cuda") for k in ("phi2", "phi_inf")}

    groups = [(idx, w, torch.full_like(t["W_gate"], 2.0 ** -6), torch.full_like(t["W_up"], 2.0 ** -6),
               stats(cfg.n_micro_routed))]
    if cfg.n_shared:
        groups.append((None, None, torch.full_like(t["Ws_gate"], 2.0 ** -6), torch.full_like(t["Ws_up"], 2.0 ** -6),
                       stats(cfg.n_micro - cfg.n_micro_routed)))

    def run():
        for gi, gw, Wg, Wu, out in groups:
            cam.score_layer(X, gi, gw, Wg, Wu, None, cfg.alpha, flags=binding.NO_FINALIZE, out=out)

    for _ in range(10):
        run()
    torch.cuda.synchronize()
    k_gemm = binding.KERNEL_NAMES.index("gemm")
    cam.profile_read(k_gemm)
    cam.profile_enable(True)
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    cam.profile_enable(False)
    ms, launches = cam.profile_read(k_gemm)
    tflops = cfg.gemm_flops_per_layer() * reps / ms / 1e9
    return {"what": "the contractions of layer 0 with constant operands (hidden states 1, weights 1/64), its own routing",
            "tflops": round(tflops, 1), "frac_of_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
            "avg_launch_ms": round(ms / max(1, launches), 4)}


def expert_counts(cam, cfg, layers, torch):
    """Routed (token, expert) pairs per expert and layer, from the library's own routing (outside any timed region)."""
    counts = []
    for lr in layers:
        idx, _ = cam.route_topk(lr.t["X"][:cfg.n_tokens], lr.t["W_r"], lr.t["bias"], cfg.top_k)
        counts.append(torch.bincount(idx.flatten().long(), minlength=cfg.n_experts).cpu().double())
    return torch.stack(counts)


def gemm_bound_ms(cfg, counts):
    """Per layer, the time no kernel can beat on the grouped contraction: every expert needs at least
    max(its flops / MFMA peak, its gate + up weight bytes / HBM peak) -- an expert with few tokens is bound by
    streaming its weights, one with many by the matrix pipe (arithmetic intensity ~ tokens of the expert per
    weight byte against a ridge of 312 flop/B).  Shared experts see every token."""
    es = 2 if cfg.dtype == "bf16" else 4
    peak = (PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_F32_TFLOPS) * 1e12
    w_bytes = 2.0 * cfg.d_model * cfg.d_ff * es
    t_routed = (counts * 4.0 * cfg.d_model * cfg.d_ff / peak).clamp(min=w_bytes / (PEAK_HBM_GBS * 1e9))
    t_routed = t_routed * (counts > 0)           # an expert without tokens is not read at all
    t = t_routed.sum(dim=1)
    if cfg.n_shared:
        ws = 2.0 * cfg.d_model * cfg.d_ff_shared * es
        t = t + cfg.n_shared * max(4.0 * cfg.d_model * cfg.d_ff_shared * cfg.n_tokens / peak, ws / (PEAK_HBM_GBS * 1e9))
    return float(t.mean() * 1e3)


def pass_rooflines(cfg, kernel_ms, n_layers, steps, chunks_per_layer):
    """HBM-side rooflines of the passes around the contraction, from the same event brackets: algorithmic bytes of a
    launch group over its average duration.  The small ones are latency-bound and are reported in microseconds too."""
    es = 2 if cfg.dtype == "bf16" else 4
    n, d, k = cfg.n_tokens, cfg.d_model, cfg.top_k
    calls = {  # algorithmic bytes per launch group
        "down_norm": (cfg.n_micro * d * es + 4.0 * cfg.n_micro) / (2 if cfg.n_shared else 1),   # W_down once, omega2 out
        "route": n * d * es + cfg.n_experts * d * es + 8.0 * n * k,                              # X and R once, indices and weights out
        "bucket": 16.0 * n * k / (2 if cfg.n_shared else 1),                                     # 16 B per routed pair; the dense tables are free
        "finalize": 28.0 * cfg.n_micro / (2 if cfg.n_shared else 1),                             # statistics, omega partials, four outputs
        "rank": 6.0 * cfg.n_micro,                                                               # the energies once, two output bytes
    }
    out = {}
    for name, bytes_per_call in calls.items():
        rec = kernel_ms.get(name)
        if not rec or not rec["launches"]:
            continue
        us = rec["ms_total"] / rec["launches"] * 1e3
        gbs = bytes_per_call / (us * 1e-6) / 1e9
        out[name] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(gbs / PEAK_HBM_GBS, 4), "us_per_call": round(us, 2),
                     "algorithmic_bytes_per_call": bytes_per_call, "calls_per_layer": round(rec["launches"] / (n_layers * steps * 1.0), 2),
                     "ms_per_step": round(rec["ms_total"] / steps, 3)}
    if "down_norm" in out:
        traffic = PMC_NORM_TRAFFIC.get(cfg.name)
        out["down_norm"]["traffic"] = traffic[0] if traffic else None
        out["down_norm"]["traffic_source"] = traffic[1] if traffic else None
    for name in ("route", "bucket", "finalize", "rank"):
        if name in out:
            out[name]["note"] = "latency- and launch-bound at this size: microseconds per call is the figure that matters"
    return out


def run_workload(name, args, torch, binding, inputs, steps, warmup, calib_tokens=0, chunk_tokens=0, energy_spread=0.0,
                 n_layers=0, keep_layers=False):
    """Builds the resident layers of one configuration, times `steps` passes of the whole hot path over them with
    the per-kernel event brackets on, and returns the figures (and the layers, when asked to keep them)."""
    cfg = inputs.CONFIGS[name]
    if energy_spread > 0:
        cfg = inputs.scaled(cfg, energy_spread=energy_spread)
    n_layers = n_layers if n_layers > 0 else cfg.n_layers
    decisions = DECISIONS[name]
    cam = binding.Camera(device=0)
    t_gen = time.perf_counter()
    calib_tokens = calib_tokens if calib_tokens > 0 else cfg.n_tokens
    chunk_tokens = chunk_tokens if chunk_tokens > 0 else cfg.n_tokens
    layers = [LayerRunner(cam, cfg, i, torch, inputs, calib_tokens, chunk_tokens) for i in range(n_layers)]
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    n_streams = max(1, args.streams)
    cams = [cam] + [binding.Camera(device=0) for _ in range(n_streams - 1)]
    streams = [torch.cuda.Stream() for _ in range(n_streams)] if n_streams > 1 else [None]

    def step():
        if n_streams == 1:
            for lr in layers:
                lr.run(cam, decisions, binding)
            return
        for i, lr in enumerate(layers):
            with torch.cuda.stream(streams[i % n_streams]):
                lr.run(cams[i % n_streams], decisions, binding)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    for k in range(len(binding.KERNEL_NAMES)):
        cam.profile_read(k)
    cam.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    cam.profile_enable(False)

    kernel_ms = {}
    for k, kname in enumerate(binding.KERNEL_NAMES):
        ms, count = cam.profile_read(k)
        if count:
            kernel_ms[kname] = {"ms_total": round(ms, 3), "launches": count}
    gemm = kernel_ms["gemm"]
    chunks_per_layer = len(layers[0].chunks)
    flops_per_step = cfg.gemm_flops_per_layer() * n_layers * (calib_tokens / cfg.n_tokens)
    flops_per_launch = flops_per_step / max(1.0, gemm["launches"] / max(1, steps))
    avg_launch_s = gemm["ms_total"] / max(1, gemm["launches"]) * 1e-3
    achieved = flops_per_launch / avg_launch_s / 1e12 if avg_launch_s > 0 else 0.0
    bf16 = cfg.dtype == "bf16"
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_TFLOPS
    traffic = PMC_TRAFFIC.get(name) if calib_tokens == cfg.n_tokens and energy_spread == 0 else None
    roofline = {"kernel": "grouped_gemm_" + ("bf16" if bf16 else "f32"), "bound": "mfma" if bf16 else "alu",
                "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "traffic": traffic[0] if traffic else None,
                "traffic_source": (traffic[1] + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE; not measured in this run)") if traffic else None,
                "flops_per_launch": flops_per_launch, "avg_launch_ms": round(avg_launch_s * 1e3, 4)}
    if calib_tokens == cfg.n_tokens:
        # what the skew of the routing allows at best: every expert bound by its flops or by streaming its weights
        counts = expert_counts(cam, cfg, layers[:min(4, n_layers)], torch)
        bound_ms = gemm_bound_ms(cfg, counts)
        gemm_ms_per_layer = gemm["ms_total"] / (steps * n_layers)
        roofline["per_expert_bound"] = {
            "what": "sum over experts of max(flops / MFMA peak, gate + up weight bytes / HBM peak), ms per layer, "
                    f"from the token counts of the first {counts.shape[0]} layers",
            "bound_ms_per_layer": round(bound_ms, 4), "gemm_ms_per_layer": round(gemm_ms_per_layer, 4),
            "frac": round(bound_ms / gemm_ms_per_layer, 4),
            "tokens_per_expert_min_max": [int(counts.min()), int(counts.max())]}
    ms_per_step = elapsed / steps * 1e3
    other = sum(v["ms_total"] for kname, v in kernel_ms.items() if kname != "gemm") / steps
    result = {
        "value": round(calib_tokens * n_layers * steps / elapsed, 1), "unit": "tokens*layers/s", "steps": steps,
        "warmup": warmup, "ms_per_step": round(ms_per_step, 3), "dtype": cfg.dtype,
        "config": {"workload": cfg.name + ("" if n_layers == cfg.n_layers else f"[first {n_layers} layers only]")
                   + ("" if calib_tokens == cfg.n_tokens else f"[{calib_tokens} calibration tokens in chunks of {chunk_tokens}]")
                   + ("" if cfg.energy_spread == 0 else f"[W_down columns scaled log-normally, sigma {cfg.energy_spread}]"),
                   "layers": n_layers, "tokens": calib_tokens, "d_model": cfg.d_model, "d_ff": cfg.d_ff,
                   "experts": cfg.n_experts, "top_k": cfg.top_k, "shared_experts": cfg.n_shared,
                   "d_ff_shared": cfg.d_ff_shared, "alpha": cfg.alpha, "decisions": decisions,
                   "full_analysis_seconds": round(ms_per_step * 1e-3, 4), "input_generation_s": round(t_gen, 1)},
        "mfma_util_pct_of_bf16_peak": round(100.0 * achieved / PEAK_BF16_TFLOPS, 2) if bf16 else None,
        "roofline": roofline,
        "rooflines": pass_rooflines(cfg, kernel_ms, n_layers, steps, chunks_per_layer),
        "non_gemm_share_of_step": round(other / ms_per_step, 4),
        "kernel_ms": kernel_ms,
    }
    if name == "tiny" and n_streams == 1:
        # The one launch-bound configuration: the same step captured once in a HIP graph and replayed (the calls
        # allocate through torch's capture pool only and never synchronise, so the sequence can be captured).
        try:
            side = torch.cuda.Stream()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    step()
            torch.cuda.synchronize()
            for _ in range(5):
                graph.replay()
            torch.cuda.synchronize()
            reps = 200
            t0 = time.perf_counter()
            for _ in range(reps):
                graph.replay()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) / reps * 1e3
            result["graph_replay"] = {"ms_per_step": round(ms, 4), "value": round(calib_tokens * n_layers / (ms * 1e-3), 1),
                                      "what": f"{reps} replays of one captured step"}
            del graph
        except Exception as exc:  # noqa: BLE001 - a side measurement: say so and go on
            print(f"bench.py: graph replay of {name} failed: {exc!r}", file=sys.stderr)
            torch.cuda.synchronize()
            result["graph_replay"] = {"error": repr(exc)}
    if keep_layers:
        return result, cam, cfg, layers
    del layers, cams
    cam.close()
    torch.cuda.empty_cache()
    return result


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no second device); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2508_02322_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)

    main_run, cam, cfg, layers = run_workload(args.workload, args, torch, binding, inputs, args.steps, args.warmup,
                                              calib_tokens=args.calib_tokens, chunk_tokens=args.chunk_tokens,
                                              energy_spread=args.energy_spread, n_layers=args.layers, keep_layers=True)
    calib_tokens = main_run["config"]["tokens"]
    roofline = main_run["roofline"]
    achieved = roofline["achieved"]
    bf16 = cfg.dtype == "bf16"

    if not args.no_probes:
        # Measured ceilings beside the published peak: the register-resident MFMA loop sustains the published rate
        # only with constant operands; with random operand values the chip lowers its clock to hold its power limit.
        from paper_2508_02322_amd import bench_probes
        tf_const, mhz_const = bench_probes.mfma_bf16(False, launches=50)
        tf_rand, mhz_rand = bench_probes.mfma_bf16(True, launches=50)
        hbm = bench_probes.hbm_read(2 << 30, launches=10)
        roofline["measured"] = {
            "mfma_bf16_constant_operands": {"tflops": round(tf_const, 1), "shader_mhz": round(mhz_const)},
            "mfma_bf16_random_operands": {"tflops": round(tf_rand, 1), "shader_mhz": round(mhz_rand)},
            "hbm_read_gbs": round(hbm, 1),
            "achieved_over_random_operand_ceiling": round(achieved / tf_rand, 4) if bf16 and tf_rand > 0 else None}

    def vendor_reference():
        """The vendor library's plain bf16 GEMM (torch.matmul) on the dense equivalent of the routed call -- the same
        flops with no gather, no grouping and no fused epilogue -- as a yardstick for the grouped kernel's rate."""
        M, K, N = cfg.n_tokens * cfg.top_k, cfg.d_model, 2 * cfg.d_ff
        g = torch.Generator(device="cuda").manual_seed(1)
        A = torch.randn((M, K), generator=g, device="cuda").to(torch.bfloat16)
        B = (torch.randn((N, K), generator=g, device="cuda") * cfg.w_std).to(torch.bfloat16)
        C = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
        for _ in range(10):
            torch.matmul(A, B.t(), out=C)
        begin, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        begin.record()
        for _ in range(40):
            torch.matmul(A, B.t(), out=C)
        end.record()
        torch.cuda.synchronize()
        ms = begin.elapsed_time(end) / 40
        return {"what": f"torch.matmul bf16 [{M} x {K}] x [{K} x {N}], random operands", "ms": round(ms, 4),
                "tflops": round(2.0 * M * K * N / ms / 1e9, 1)}

    def stage(name, skip, fn):
        """A follow-on measurement outside the timed step: its failure is reported in its place and on stderr, and
        does not take the headline line with it."""
        if skip:
            return None
        try:
            return fn()
        except Exception as exc:  # noqa: BLE001 - whatever it was, say so
            print(f"bench.py: stage {name} failed: {exc!r}", file=sys.stderr)
            torch.cuda.synchronize()
            return {"error": repr(exc)}

    if "measured" in roofline and bf16:
        roofline["measured"]["vendor_gemm_dense_equivalent"] = stage("vendor_gemm", False, vendor_reference)
        roofline["measured"]["grouped_gemm_constant_operands"] = stage(
            "constant_operands", calib_tokens != cfg.n_tokens, lambda: constant_operand_rate(cam, cfg, layers[0], torch, binding))
    own_size = calib_tokens == cfg.n_tokens
    apply_mask = stage("apply_mask", args.no_apply, lambda: measure_apply(cam, cfg, layers, torch, binding))
    forward = stage("pruned_layer_output", args.no_forward or not own_size,
                    lambda: measure_forward(cam, cfg, layers, torch, binding))
    decode = stage("pruned_layer_decode", args.no_decode or not own_size,
                   lambda: measure_decode(cam, cfg, layers, torch, binding,
                                          ratios=[float(r) for r in args.decode_ratios.split(",")]))
    del layers
    cam.close()
    torch.cuda.empty_cache()

    result = {
        "metric": "calibration tokens x layers scored/sec; MFMA util % of bf16 peak",
        "value": main_run["value"], "unit": main_run["unit"], "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_run["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": main_run["config"],
        "mfma_util_pct_of_bf16_peak": main_run["mfma_util_pct_of_bf16_peak"],
        "roofline": roofline,
        "rooflines": main_run["rooflines"],
        "non_gemm_share_of_step": main_run["non_gemm_share_of_step"],
        "kernel_ms": main_run["kernel_ms"],
    }
    if "graph_replay" in main_run:
        result["graph_replay"] = main_run["graph_replay"]
    if apply_mask is not None:
        result["apply_mask"] = apply_mask
    if forward is not None:
        result["pruned_layer_output"] = forward
    if decode is not None:
        result["pruned_layer_decode"] = decode

    plain = own_size and args.energy_spread == 0 and args.layers == 0
    if plain and not args.no_streamed and bf16 and args.workload == "qwen2-57b-a14b":
        # The paper's calibration size (128 sequences of 2048 tokens), streamed in chunks through CAMERA_ACCUMULATE:
        # the like-for-like token count beside its "under five minutes" (other hardware, whole pipeline: context only).
        def streamed():
            r = run_workload(args.workload, args, torch, binding, inputs, steps=1, warmup=1,
                             calib_tokens=args.streamed_tokens, chunk_tokens=args.streamed_chunk)
            return {"tokens": args.streamed_tokens, "chunk": args.streamed_chunk, "layers": r["config"]["layers"],
                    "seconds": round(r["ms_per_step"] * 1e-3, 4), "tokens_layers_per_s": r["value"],
                    "frac": r["roofline"]["frac"], "gemm_tflops": r["roofline"]["achieved"],
                    "non_gemm_share_of_step": r["non_gemm_share_of_step"],
                    "what": "whole analysis of the configuration on this many calibration tokens per layer, one warm-up pass, one timed pass"}
        result["streamed_calibration"] = stage("streamed_calibration", False, streamed)
    if plain and not args.no_other_workloads:
        others = {}
        for name in ("tiny", "mixtral", "deepseek-moe-16b", "qwen2-57b-a14b", "qwen3-30b-a3b"):
            if name == args.workload:
                continue
            r = stage(name, False, lambda name=name: run_workload(name, args, torch, binding, inputs,
                                                                   steps=max(1, args.other_steps), warmup=2))
            if r is not None and "error" not in r:
                r = {k: r[k] for k in ("value", "unit", "steps", "ms_per_step", "dtype", "mfma_util_pct_of_bf16_peak", "roofline",
                                       "rooflines", "non_gemm_share_of_step", "config", "graph_replay") if k in r}
            others[name] = r
        result["workloads"] = others
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = stage("cpu_baseline", False, lambda: cpu_baseline(cfg, inputs))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
