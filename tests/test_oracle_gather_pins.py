"""Pins for the oracle's gather of kept micro-experts (Algorithm 2, lines 10-13; CPU only).

The paper says what pruning a micro-expert means: its gate row, up row and
down column are zeroed together.  So the layer rebuilt from the gathered
(compacted) weights must give the output of the layer with those three vectors
zeroed -- computed here by a forward pass written out with loops that shares
nothing with the oracle.  A gather that pairs a gate row with the wrong down
column, drops an entry, or mixes experts fails these.
"""
import math

import numpy as np
import pytest

from oracle import camera_oracle as orc


def layer(seed, n=10, d=7, f=9, n_experts=4):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(n, d))
    A = rng.uniform(0.1, 1.0, size=(n, n_experts)) * (rng.uniform(size=(n, n_experts)) < 0.6)
    Wg = rng.normal(size=(n_experts, f, d)) * 0.5
    Wu = rng.normal(size=(n_experts, f, d)) * 0.5
    Wd = rng.normal(size=(n_experts, d, f)) * 0.5
    return X, A, Wg, Wu, Wd


def forward_loops(X, A, experts):
    """y_j = sum_e A[j, e] * W_down,e [silu(W_gate,e x_j) * (W_up,e x_j)] (Eq. 1-2); experts is a list of
    (gate [f_e, d], up [f_e, d], down [d, f_e]) with its own width f_e per expert."""
    n, d = X.shape
    Y = np.zeros((n, d))
    for j in range(n):
        for e, (g_w, u_w, d_w) in enumerate(experts):
            for c in range(g_w.shape[0]):
                g = float(np.dot(g_w[c], X[j]))
                u = float(np.dot(u_w[c], X[j]))
                Y[j] += A[j, e] * (g / (1.0 + math.exp(-g))) * u * d_w[:, c]
    return Y


def split_by_expert(gate_out, up_out, down_out, count):
    experts, pos = [], 0
    for e, c in enumerate(count):
        experts.append((gate_out[pos:pos + c], up_out[pos:pos + c], down_out[e]))
        pos += c
    return experts


@pytest.mark.parametrize("ratio", [0.0, 0.2, 0.6, 1.0])
def test_compacted_layer_equals_layer_with_pruned_vectors_zeroed(ratio):
    X, A, Wg, Wu, Wd = layer(3)
    n_experts, f, _ = Wg.shape
    E = np.random.default_rng(5).uniform(size=n_experts * f)
    seg = [e * f for e in range(n_experts + 1)]
    keep, kept_per_expert, kept_idx, _ = orc.select_prune(E, seg, ratio)
    gate_out, up_out, down_out = orc.gather_micro_experts(Wg, Wu, Wd, kept_idx, kept_per_expert)
    Y_compact = forward_loops(X, A, split_by_expert(gate_out, up_out, down_out, kept_per_expert))
    mask = keep.reshape(n_experts, f).astype(bool)
    zeroed = [(np.where(mask[e][:, None], Wg[e], 0.0), np.where(mask[e][:, None], Wu[e], 0.0),
               np.where(mask[e][None, :], Wd[e], 0.0)) for e in range(n_experts)]
    Y_zeroed = forward_loops(X, A, zeroed)
    assert np.allclose(Y_compact, Y_zeroed, rtol=1e-12, atol=1e-13)
    assert gate_out.shape == (n_experts * f - orc.prune_count(ratio, n_experts * f), X.shape[1])


def test_reordering_inside_experts_leaves_the_layer_output_unchanged():
    """CAMERA-Q's colocation of equal precision is a permutation inside every expert; a sum over
    micro-experts does not depend on their order, as long as the three vectors move together."""
    X, A, Wg, Wu, Wd = layer(4)
    n_experts, f, _ = Wg.shape
    E = np.random.default_rng(6).uniform(size=n_experts * f)
    seg = [e * f for e in range(n_experts + 1)]
    _, level_count, perm = orc.alloc_bits(E, seg, [3, 2, 1], [0.2, 0.6, 0.2])
    count = np.full(n_experts, f)
    gate_out, up_out, down_out = orc.gather_micro_experts(Wg, Wu, Wd, perm, count)
    Y = forward_loops(X, A, [(Wg[e], Wu[e], Wd[e]) for e in range(n_experts)])
    Y_perm = forward_loops(X, A, split_by_expert(gate_out, up_out, down_out, count))
    assert np.allclose(Y, Y_perm, rtol=1e-12, atol=1e-13)
    # the classes are contiguous inside every expert after the reordering
    bit_of, _, _ = orc.alloc_bits(E, seg, [3, 2, 1], [0.2, 0.6, 0.2])
    for e in range(n_experts):
        bits_in_order = bit_of[perm[e * f:(e + 1) * f]]
        assert list(bits_in_order) == sorted(bits_in_order, reverse=True)
        assert level_count[e].sum() == f


def test_identity_index_copies_and_values_are_never_recomputed():
    _, _, Wg, Wu, Wd = layer(7)
    Wg32, Wu32, Wd32 = Wg.astype(np.float32), Wu.astype(np.float32), Wd.astype(np.float32)
    n_experts, f, d = Wg.shape
    idx = np.arange(n_experts * f)
    g, u, dn = orc.gather_micro_experts(Wg32, Wu32, Wd32, idx, np.full(n_experts, f))
    assert g.dtype == np.float32 and np.array_equal(g, Wg32.reshape(-1, d)) and np.array_equal(u, Wu32.reshape(-1, d))
    assert all(np.array_equal(dn[e], Wd32[e]) for e in range(n_experts))


def test_single_entries_and_base_offset():
    """One kept micro-expert in one expert, none in the others; indices counted from a base (a group of
    experts that sits behind another group in the layer's numbering)."""
    _, _, Wg, Wu, Wd = layer(8)
    n_experts, f, d = Wg.shape
    base = 1000
    e, c = 2, 5
    count = np.zeros(n_experts, dtype=np.int64)
    count[e] = 1
    g, u, dn = orc.gather_micro_experts(Wg, Wu, Wd, [base + e * f + c], count, index_base=base)
    assert np.array_equal(g[0], Wg[e, c]) and np.array_equal(u[0], Wu[e, c])
    assert dn[e].shape == (d, 1) and np.array_equal(dn[e][:, 0], Wd[e, :, c])
    assert all(dn[k].shape == (d, 0) for k in range(n_experts) if k != e)


def test_rejects_indices_outside_their_expert_and_wrong_counts():
    _, _, Wg, Wu, Wd = layer(9)
    n_experts, f, _ = Wg.shape
    with pytest.raises(ValueError):
        orc.gather_micro_experts(Wg, Wu, Wd, [f], [1] + [0] * (n_experts - 1))     # index f belongs to expert 1
    with pytest.raises(ValueError):
        orc.gather_micro_experts(Wg, Wu, Wd, [0, 1], [1] + [0] * (n_experts - 1))  # counts do not add up
