"""Pins for the oracle's layer output, bf16 rounding and output-error measures (CPU only).

The layer output is checked against a forward pass written out with loops
and scalar SiLU (shares nothing with the oracle), the decoding error against
the energies of the scoring oracle (the Lemma with one removed micro-expert is
an equality), the rounding against the library's bfloat16 conversion, and the
error measures against closed forms.
"""
import math

import numpy as np
import pytest
import torch

from oracle import camera_oracle as orc


def layer(seed, n=14, d=9, f=7, n_experts=4, top_k=2):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(n, d))
    R = rng.normal(size=(n_experts, d)) * 0.5
    Wg = rng.normal(size=(n_experts, f, d)) * 0.5
    Wu = rng.normal(size=(n_experts, f, d)) * 0.5
    Wd = rng.normal(size=(n_experts, d, f)) * 0.5
    _, _, A = orc.top_and_norm(orc.router_logits(X, R), top_k)
    return X, A, Wg, Wu, Wd


def forward_loops(X, A, Wg, Wu, Wd, keep=None):
    n, d = X.shape
    n_experts, f, _ = Wg.shape
    Y = np.zeros((n, d))
    for j in range(n):
        for e in range(n_experts):
            for c in range(f):
                if keep is not None and not keep[e * f + c]:
                    continue
                g = float(np.dot(Wg[e, c], X[j]))
                u = float(np.dot(Wu[e, c], X[j]))
                Y[j] += A[j, e] * (g / (1.0 + math.exp(-g))) * u * Wd[e, :, c]
    return Y


def test_forward_equals_the_loop_written_layer_with_and_without_a_mask():
    X, A, Wg, Wu, Wd = layer(1)
    assert np.allclose(orc.layer_forward(X, A, Wg, Wu, Wd), forward_loops(X, A, Wg, Wu, Wd), rtol=1e-12, atol=1e-13)
    keep = np.random.default_rng(2).uniform(size=Wg.shape[0] * Wg.shape[1]) < 0.6
    assert np.allclose(orc.layer_forward(X, A, Wg, Wu, Wd, keep=keep.astype(np.uint8)),
                       forward_loops(X, A, Wg, Wu, Wd, keep), rtol=1e-12, atol=1e-13)
    none = np.zeros(keep.size, dtype=np.uint8)
    assert np.all(orc.layer_forward(X, A, Wg, Wu, Wd, keep=none) == 0.0)


def test_decoding_error_of_one_removed_micro_expert_is_its_energy():
    """epsilon = ||Phi W - Phi_S W_S||_F^2; with S^C = {i} it is ||Phi_i||^2 ||w_i||^2 = E_i at alpha = 0,
    and the largest per-token error is E_i at alpha = 1."""
    X, A, Wg, Wu, Wd = layer(3)
    n_experts, f, _ = Wg.shape
    E0 = orc.score_layer(X, A, Wg, Wu, Wd, 0.0)["energy"]
    E1 = orc.score_layer(X, A, Wg, Wu, Wd, 1.0)["energy"]
    Y = orc.layer_forward(X, A, Wg, Wu, Wd)
    for i in (0, 5, f, 2 * f + 3, n_experts * f - 1):
        keep = np.ones(n_experts * f, dtype=np.uint8)
        keep[i] = 0
        err = orc.output_error(Y, orc.layer_forward(X, A, Wg, Wu, Wd, keep=keep))
        assert err["d2"].sum() == pytest.approx(E0[i], rel=1e-9, abs=1e-18)
        assert err["d2"].max() == pytest.approx(E1[i], rel=1e-9, abs=1e-18)
        assert err["l2"] == pytest.approx(math.sqrt(E0[i]), rel=1e-9, abs=1e-12)


def test_decoding_error_of_a_removed_set_against_its_definition_and_bounds():
    """epsilon = sum_j || sum_{i in S^C} phi_ji w_i ||^2 from the coefficient matrix itself, and the two
    inequalities that hold for sets (the proof's Cauchy-Schwarz line, and |S^C| * sum E_i)."""
    X, A, Wg, Wu, Wd = layer(4)
    n_experts, f, d = Wg.shape
    rng = np.random.default_rng(5)
    keep = (rng.uniform(size=n_experts * f) < 0.5).astype(np.uint8)
    err = orc.output_error(orc.layer_forward(X, A, Wg, Wu, Wd), orc.layer_forward(X, A, Wg, Wu, Wd, keep=keep))
    Phi = np.concatenate([orc.lambda_matrix(X, A[:, e], Wg[e], Wu[e]) for e in range(n_experts)], axis=1)   # [n, N_e]
    W = np.concatenate([Wd[e].T for e in range(n_experts)], axis=0)                                        # [N_e, d]
    removed = np.nonzero(keep == 0)[0]
    eps = float(((Phi[:, removed] @ W[removed]) ** 2).sum())
    assert err["d2"].sum() == pytest.approx(eps, rel=1e-10)
    E0 = orc.score_layer(X, A, Wg, Wu, Wd, 0.0)["energy"]
    assert eps <= removed.size * E0[removed].sum() * (1 + 1e-12)
    assert eps <= (Phi[:, removed] ** 2).sum() * (W[removed] ** 2).sum() * (1 + 1e-12)


def test_round_to_bf16_is_the_library_conversion():
    rng = np.random.default_rng(6)
    vals = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-20, 20, size=4000), [0.0, -0.0, 1.0, -1.0]])
    # exact ties between two bfloat16 neighbours, odd and even lower neighbour: 1 + k/128 + 1/256
    ties = np.array([1.0 + k / 128.0 + 1.0 / 256.0 for k in range(8)] + [-(1.0 + k / 128.0 + 1.0 / 256.0) for k in range(8)])
    vals = np.concatenate([vals, ties]).astype(np.float32)
    want = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.round_to_bf16(vals)
    assert np.array_equal(got, want)
    assert orc.round_to_bf16(1.0 + 1.0 / 256.0) == 1.0 and orc.round_to_bf16(1.0 + 3.0 / 256.0) == 1.0 + 2.0 / 128.0


def test_rounded_hidden_changes_the_output_by_no_more_than_bf16_precision():
    X, A, Wg, Wu, Wd = layer(7, n=30, d=16, f=40)
    Y = orc.layer_forward(X, A, Wg, Wu, Wd)
    Yr = orc.layer_forward(X, A, Wg, Wu, Wd, round_hidden=orc.round_to_bf16)
    Lam_abs = np.concatenate([np.abs(orc.lambda_matrix(X, A[:, e], Wg[e], Wu[e])) for e in range(Wg.shape[0])], axis=1)
    W_abs = np.concatenate([np.abs(Wd[e]).T for e in range(Wg.shape[0])], axis=0)
    bound = 2.0 ** -8 * (Lam_abs @ W_abs)          # each hidden value moves by at most 2^-9 of itself, float32 step on top
    assert np.all(np.abs(Y - Yr) <= bound + 1e-300) and np.any(Y != Yr)


def test_output_error_closed_forms():
    rng = np.random.default_rng(8)
    Y = rng.normal(size=(11, 6))
    same = orc.output_error(Y, Y)
    assert same["l2"] == 0.0 and same["cosine"] == pytest.approx(1.0) and same["cosine_mean"] == pytest.approx(1.0)
    scaled = orc.output_error(Y, 0.25 * Y)
    assert scaled["l2"] == pytest.approx(0.75 * np.linalg.norm(Y)) and scaled["cosine"] == pytest.approx(1.0)
    flipped = orc.output_error(Y, -Y)
    assert flipped["cosine"] == pytest.approx(-1.0) and flipped["l2"] == pytest.approx(2 * np.linalg.norm(Y))
    a = np.array([[1.0, 0.0], [0.0, 2.0], [0.0, 0.0]])
    b = np.array([[0.0, 3.0], [0.0, 2.0], [1.0, 1.0]])
    e = orc.output_error(a, b)
    assert list(e["d2"]) == [10.0, 0.0, 2.0] and list(e["yh"]) == [0.0, 4.0, 0.0]
    assert e["cosine"] == pytest.approx(4.0 / math.sqrt(5.0 * 15.0))
    assert e["cosine_mean"] == pytest.approx((0.0 + 1.0) / 2)      # the all-zero token is left out
