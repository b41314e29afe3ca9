"""Pins for the oracle's routing and scoring functions (CPU only).

Each test checks the oracle against something other than itself: the plain MoE
layer forward (Eq. 1-2) with one micro-expert ablated, the Lemma, library
softmax / SiLU, or a symmetry the definitions imply.
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import camera_oracle as orc


def tiny_layer(seed, n=24, d=12, f=10, n_experts=5):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(n, d))
    R = rng.normal(size=(n_experts, d)) * 0.5
    Wg = rng.normal(size=(n_experts, f, d)) * 0.4
    Wu = rng.normal(size=(n_experts, f, d)) * 0.4
    Wd = rng.normal(size=(n_experts, d, f)) * 0.4
    return X, R, Wg, Wu, Wd


def moe_forward_loops(X, A, Wg, Wu, Wd):
    """The layer output of Eq. 1-2 written out token by token, expert by expert,
    with scalar SiLU from the math module.  Shares nothing with the oracle."""
    n, d = X.shape
    n_experts, f, _ = Wg.shape
    Y = np.zeros((n, d))
    for j in range(n):
        for e in range(n_experts):
            if A[j, e] == 0.0:
                continue
            hidden = np.zeros(f)
            for c in range(f):
                g = float(np.dot(Wg[e, c], X[j]))
                u = float(np.dot(Wu[e, c], X[j]))
                hidden[c] = (g / (1.0 + math.exp(-g))) * u
            Y[j] += A[j, e] * (Wd[e] @ hidden)
    return Y


@pytest.mark.parametrize("alpha", [0.0, 0.3, 0.95, 1.0])
def test_energy_equals_bruteforce_ablation(alpha):
    """Removing micro-expert i changes token j's output by phi_ji * w_i, so
    sum_j ||dy_j||^2 = ||Phi_i||_2^2 ||w_i||^2 and max_j ||dy_j||^2 =
    ||Phi_i||_inf^2 ||w_i||^2 (the Lemma with one removed index)."""
    X, R, Wg, Wu, Wd = tiny_layer(1)
    _, _, A = orc.top_and_norm(orc.router_logits(X, R), top_k=2)
    E = orc.score_layer(X, A, Wg, Wu, Wd, alpha)["energy"]
    Y = moe_forward_loops(X, A, Wg, Wu, Wd)
    n_experts, f, _ = Wg.shape
    for e in range(n_experts):
        for c in range(f):
            Wd_abl = Wd.copy()
            Wd_abl[e, :, c] = 0.0
            dY = Y - moe_forward_loops(X, A, Wg, Wu, Wd_abl)
            per_token = (dY * dY).sum(axis=1)
            want = (1 - alpha) * per_token.sum() + alpha * per_token.max()
            assert E[e * f + c] == pytest.approx(want, rel=1e-9, abs=1e-18)


def test_lemma_bound_for_removed_sets():
    """Decoding error of a removed set S^C against the energies (alpha = 0).

    With one removed index the error equals E_i exactly.  For larger sets the
    proof's chain (Minkowski, then Cauchy-Schwarz) ends at
    (sum_i ||Phi_i||^2) * (sum_i ||w_i||^2); the Lemma's printed right-hand
    side, sum_i E_i, drops the cross terms and is not a bound in general, so
    the checks here are the two inequalities that do hold: the proof's own
    last-but-one line, and |S^C| * sum_i E_i (from ||sum v_i||^2 <= k sum ||v_i||^2).
    """
    X, R, Wg, Wu, Wd = tiny_layer(2)
    _, _, A = orc.top_and_norm(orc.router_logits(X, R), top_k=3)
    out = orc.score_layer(X, A, Wg, Wu, Wd, 0.0)
    E0 = out["energy"]
    Y = moe_forward_loops(X, A, Wg, Wu, Wd)
    n_experts, f, _ = Wg.shape
    rng = np.random.default_rng(0)
    for size in (1, 2, 5, 17):
        removed = rng.choice(n_experts * f, size=size, replace=False)
        Wd_abl = Wd.copy()
        for i in removed:
            Wd_abl[i // f, :, i % f] = 0.0
        err = ((Y - moe_forward_loops(X, A, Wg, Wu, Wd_abl)) ** 2).sum()
        assert err <= size * E0[removed].sum() * (1 + 1e-12)
        assert err <= out["phi2"][removed].sum() * out["omega2"][removed].sum() * (1 + 1e-12)
        if size == 1:
            assert err == pytest.approx(E0[removed].sum(), rel=1e-9)


def test_top_and_norm_is_softmax_over_kept_logits():
    rng = np.random.default_rng(3)
    L = rng.normal(size=(40, 9)) * 3
    idx, w, A = orc.top_and_norm(L, top_k=4)
    for j in range(L.shape[0]):
        want_idx = sorted(range(9), key=lambda e: (-L[j, e], e))[:4]
        assert list(idx[j]) == want_idx
        np.testing.assert_allclose(w[j], scipy.special.softmax(L[j, want_idx]), rtol=1e-12)
        assert A[j].sum() == pytest.approx(1.0)
        assert np.count_nonzero(A[j]) == 4


def test_top_and_norm_special_cases():
    rng = np.random.default_rng(4)
    L = rng.normal(size=(16, 6))
    # k = N_E: every expert kept, weights are the plain softmax
    idx, w, A = orc.top_and_norm(L, top_k=6)
    np.testing.assert_allclose(A, scipy.special.softmax(L, axis=1), rtol=1e-12)
    # without renormalisation the kept weights are the softmax probabilities themselves
    idx, w, _ = orc.top_and_norm(L, top_k=2, renorm=False)
    np.testing.assert_allclose(w, np.take_along_axis(scipy.special.softmax(L, axis=1), idx, 1), rtol=1e-12)
    # one expert: a == 1 (the dense-FFN case)
    _, w1, A1 = orc.top_and_norm(L[:, :1], top_k=1)
    assert np.all(w1 == 1.0) and np.all(A1 == 1.0)
    # exact ties go to the lower expert index
    idx, _, _ = orc.top_and_norm(np.array([[1.0, 2.0, 2.0, 2.0, 0.0]]), top_k=2)
    assert list(idx[0]) == [1, 2]
    # bias enters the logits
    X, R = rng.normal(size=(3, 4)), rng.normal(size=(5, 4))
    b = rng.normal(size=5)
    np.testing.assert_allclose(orc.router_logits(X, R, b), np.einsum("jc,ec->je", X, R) + b, rtol=1e-12)


def test_dense_ffn_case_matches_library_swiglu():
    """One expert with a == 1 is an ordinary SwiGLU FFN: the column statistics
    must be those of torch's silu(X Wg^T) * (X Wu^T) in float64."""
    X, _, Wg, Wu, Wd = tiny_layer(5, n_experts=1)
    out = orc.score_layer(X, np.ones((X.shape[0], 1)), Wg, Wu, Wd, alpha=0.5)
    Xt, Wgt, Wut, Wdt = (torch.from_numpy(a) for a in (X, Wg[0], Wu[0], Wd[0]))
    H = torch.nn.functional.silu(Xt @ Wgt.T) * (Xt @ Wut.T)
    np.testing.assert_allclose(out["phi2"], (H ** 2).sum(0).numpy(), rtol=1e-11)
    np.testing.assert_allclose(out["phi_inf"], (H.abs().max(0).values ** 2).numpy(), rtol=1e-11)
    np.testing.assert_allclose(out["omega2"], torch.linalg.vector_norm(Wdt, dim=0).numpy() ** 2, rtol=1e-11)
    want = (0.5 * out["phi2"] + 0.5 * out["phi_inf"]) * out["omega2"]
    np.testing.assert_allclose(out["energy"], want, rtol=1e-14)
    # alpha = 0 is the plain energy ||Phi_i||^2 ||w_i||^2, alpha = 1 uses the maximum alone
    np.testing.assert_allclose(orc.energy(out["phi2"], out["phi_inf"], out["omega2"], 0.0),
                               out["phi2"] * out["omega2"], rtol=1e-14)
    np.testing.assert_allclose(orc.energy(out["phi2"], out["phi_inf"], out["omega2"], 1.0),
                               out["phi_inf"] * out["omega2"], rtol=1e-14)


def test_unrouted_tokens_do_not_matter():
    """Algorithm 1 as printed (all tokens, masked by A[:, i]) equals the form
    that only visits routed tokens."""
    X, R, Wg, Wu, Wd = tiny_layer(6)
    _, _, A = orc.top_and_norm(orc.router_logits(X, R), top_k=2)
    a = orc.score_layer(X, A, Wg, Wu, Wd, 0.7, skip_unrouted=True)
    b = orc.score_layer(X, A, Wg, Wu, Wd, 0.7, skip_unrouted=False)
    for key in a:
        np.testing.assert_allclose(a[key], b[key], rtol=1e-13, atol=0)


def test_symmetries():
    X, R, Wg, Wu, Wd = tiny_layer(7)
    L = orc.router_logits(X, R)
    _, _, A = orc.top_and_norm(L, top_k=2)
    alpha = 0.6
    base = orc.score_layer(X, A, Wg, Wu, Wd, alpha)["energy"]
    n_experts, f, d = Wg.shape
    rng = np.random.default_rng(11)

    # token order does not matter
    pt = rng.permutation(X.shape[0])
    np.testing.assert_allclose(orc.score_layer(X[pt], A[pt], Wg, Wu, Wd, alpha)["energy"], base, rtol=1e-12)

    # permuting the d_model channels of X, R, gate/up columns and down rows changes nothing
    pc = rng.permutation(d)
    _, _, A2 = orc.top_and_norm(orc.router_logits(X[:, pc], R[:, pc]), top_k=2)
    got = orc.score_layer(X[:, pc], A2, Wg[:, :, pc], Wu[:, :, pc], Wd[:, pc, :], alpha)["energy"]
    np.testing.assert_allclose(got, base, rtol=1e-10)

    # permuting micro-experts inside an expert permutes their scores
    pf = rng.permutation(f)
    got = orc.score_layer(X, A, Wg[:, pf], Wu[:, pf], Wd[:, :, pf], alpha)["energy"]
    np.testing.assert_allclose(got.reshape(n_experts, f), base.reshape(n_experts, f)[:, pf], rtol=1e-12)

    # permuting experts together with the router rows permutes whole blocks
    pe = rng.permutation(n_experts)
    _, _, A3 = orc.top_and_norm(orc.router_logits(X, R[pe]), top_k=2)
    got = orc.score_layer(X, A3, Wg[pe], Wu[pe], Wd[pe], alpha)["energy"]
    np.testing.assert_allclose(got.reshape(n_experts, f), base.reshape(n_experts, f)[pe], rtol=1e-12)

    # homogeneity: scaling a down column or an up row by s scales that score by s^2
    Wd2, Wu2 = Wd.copy(), Wu.copy()
    Wd2[1, :, 3] *= 3.0
    Wu2[2, 4, :] *= -0.5
    got = orc.score_layer(X, A, Wg, Wu2, Wd2, alpha)["energy"].reshape(n_experts, f)
    want = base.reshape(n_experts, f).copy()
    want[1, 3] *= 9.0
    want[2, 4] *= 0.25
    np.testing.assert_allclose(got, want, rtol=1e-12)

    # zero down column / up row / gate row (SiLU(0) = 0) give a zero score
    Wd3, Wu3, Wg3 = Wd.copy(), Wu.copy(), Wg.copy()
    Wd3[0, :, 0] = 0
    Wu3[0, 1, :] = 0
    Wg3[0, 2, :] = 0
    got = orc.score_layer(X, A, Wg3, Wu3, Wd3, alpha)["energy"]
    assert got[0] == 0 and got[1] == 0 and got[2] == 0
    assert np.all(got[3:f] > 0)

    # an expert that receives no tokens has only zero scores
    A4 = A.copy()
    A4[:, 3] = 0
    got = orc.score_layer(X, A4, Wg, Wu, Wd, alpha)["energy"].reshape(n_experts, f)
    assert np.all(got[3] == 0)


def test_expert_split_and_shared_expert():
    """Micro-experts are independent: an expert cut into two halves that keep
    the same routing weight gives the same scores; a shared expert is an
    expert whose routing weight is one for every token."""
    X, R, Wg, Wu, Wd = tiny_layer(8, f=12)
    _, _, A = orc.top_and_norm(orc.router_logits(X, R), top_k=2)
    base = orc.score_layer(X, A, Wg, Wu, Wd, 0.95)["energy"]
    h = 6
    Wg2 = np.concatenate([Wg[:, :h], Wg[:, h:]], axis=0)
    Wu2 = np.concatenate([Wu[:, :h], Wu[:, h:]], axis=0)
    Wd2 = np.concatenate([Wd[:, :, :h], Wd[:, :, h:]], axis=0)
    A2 = np.concatenate([A, A], axis=1)
    got = orc.score_layer(X, A2, Wg2, Wu2, Wd2, 0.95)["energy"]
    n_experts = Wg.shape[0]
    b = base.reshape(n_experts, 12)
    np.testing.assert_allclose(got[:n_experts * h].reshape(n_experts, h), b[:, :h], rtol=1e-12)
    np.testing.assert_allclose(got[n_experts * h:].reshape(n_experts, h), b[:, h:], rtol=1e-12)
    # shared expert: scores equal the brute-force ablation of a layer with a == 1
    ones = np.ones((X.shape[0], 1))
    E = orc.score_layer(X, ones, Wg[:1], Wu[:1], Wd[:1], 0.0)["energy"]
    Y = moe_forward_loops(X, ones, Wg[:1], Wu[:1], Wd[:1])
    Wd_abl = Wd[:1].copy()
    Wd_abl[0, :, 5] = 0
    assert E[5] == pytest.approx(((Y - moe_forward_loops(X, ones, Wg[:1], Wu[:1], Wd_abl)) ** 2).sum(), rel=1e-9)


def test_chunked_tokens_merge():
    """phi^2 adds and phi^inf takes the larger over disjoint token chunks."""
    X, R, Wg, Wu, Wd = tiny_layer(9, n=30)
    _, _, A = orc.top_and_norm(orc.router_logits(X, R), top_k=2)
    whole = orc.score_layer(X, A, Wg, Wu, Wd, 0.8)
    a = orc.score_layer(X[:13], A[:13], Wg, Wu, Wd, 0.8)
    b = orc.score_layer(X[13:], A[13:], Wg, Wu, Wd, 0.8)
    merged = orc.merge_chunks(a, b, 0.8)
    for key in whole:
        np.testing.assert_allclose(merged[key], whole[key], rtol=1e-12)


def test_dense_routing_scatter():
    idx = np.array([[2, 0], [1, 3]])
    w = np.array([[0.75, 0.25], [0.5, 0.5]])
    A = orc.dense_routing(idx, w, 4)
    np.testing.assert_array_equal(A, [[0.25, 0, 0.75, 0], [0, 0.5, 0, 0.5]])
