"""Shared plumbing of the GPU parity tests: exact up-conversion of the seeded
tensors for the oracle and the comparison rules."""
import numpy as np
import torch

from oracle import camera_oracle as orc


def f64(t):
    """Exact float64 copy of a float32 / bf16 tensor (or None)."""
    if t is None:
        return None
    return t.detach().cpu().to(torch.float32).numpy().astype(np.float64)


def to_dev(layer, device="cuda"):
    return {k: (v.to(device) if v is not None else None) for k, v in layer.items()}


def oracle_route(layer, top_k, renorm=True):
    L = orc.router_logits(f64(layer["X"]), f64(layer["W_r"]), f64(layer["bias"]))
    idx, w, A = orc.top_and_norm(L, top_k, renorm)
    return L, idx, w, A


def oracle_score(layer, A, alpha, prefix="W", channels=None):
    """Oracle scores of the routed ("W") or shared ("Ws") experts; `channels` restricts
    every expert to a subset of its micro-experts (they are independent of each other)."""
    Wg, Wu, Wd = layer[prefix + "_gate"], layer[prefix + "_up"], layer[prefix + "_down"]
    if channels is not None:
        ch = torch.as_tensor(channels, dtype=torch.long)
        Wg, Wu, Wd = Wg[:, ch], Wu[:, ch], Wd[:, :, ch]
    n_experts = Wg.shape[0]
    gate = [f64(Wg[e]) for e in range(n_experts)]
    up = [f64(Wu[e]) for e in range(n_experts)]
    down = [f64(Wd[e]) for e in range(n_experts)]
    return orc.score_layer(f64(layer["X"]), A, gate, up, down, alpha)


def rel_err(got, want, floor):
    """max |got - want| / max(want, floor)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.max(np.abs(got - want) / np.maximum(np.abs(want), floor)))


def margin_flags(L, top_k, margin=1e-4):
    """Tokens whose k-th and (k+1)-th largest logits are closer than margin*max(1,|L|):
    float32 and float64 accumulation may legitimately order them differently."""
    if top_k >= L.shape[1]:
        return np.zeros(L.shape[0], dtype=bool)
    s = -np.sort(-L, axis=1)
    gap = s[:, top_k - 1] - s[:, top_k]
    return gap < margin * np.maximum(1.0, np.abs(s[:, top_k - 1]))


def check_routing(L, idx_orc, w_orc, idx_gpu, w_gpu, top_k, renorm=True, w_tol=2e-4):
    """Indices must agree on every token that is not margin-flagged; on flagged tokens the GPU's
    choice must be a valid top-k up to the margin.  Weights are compared where indices agree."""
    idx_gpu = np.asarray(idx_gpu, dtype=np.int64)
    w_gpu = np.asarray(w_gpu, dtype=np.float64)
    flagged = margin_flags(L, top_k)
    same = np.all(idx_gpu == idx_orc, axis=1)
    assert np.all(same | flagged), f"{np.count_nonzero(~same & ~flagged)} unflagged tokens differ"
    for j in np.nonzero(~same)[0]:
        kth = np.sort(L[j])[::-1][top_k - 1]
        chosen = L[j, idx_gpu[j]]
        assert len(set(idx_gpu[j].tolist())) == top_k
        assert np.all(chosen >= kth - 1e-4 * max(1.0, abs(kth)))
    np.testing.assert_allclose(w_gpu[same], w_orc[same], rtol=w_tol, atol=1e-6)
    if renorm:
        np.testing.assert_allclose(w_gpu.sum(axis=1), 1.0, atol=1e-5)
    return int(np.count_nonzero(flagged)), int(np.count_nonzero(~same))


def decidable_masks(E_orc, n_below, tol):
    """Which micro-experts must be below / above a cut at ascending rank n_below when every
    energy is only known to relative tolerance `tol` (others are undecidable)."""
    s = np.sort(E_orc, kind="stable")
    N = s.size
    if n_below <= 0:
        return np.zeros(N, bool), np.ones(N, bool)
    if n_below >= N:
        return np.ones(N, bool), np.zeros(N, bool)
    tau_lo, tau_hi = s[n_below - 1], s[n_below]
    must_below = E_orc < tau_hi * (1 - tol) / (1 + tol)
    must_above = E_orc > tau_lo * (1 + tol) / (1 - tol)
    return must_below, must_above
