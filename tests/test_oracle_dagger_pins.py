"""Pins of the oracle's CAMERA-Q-dagger pieces (the column-wise comparison variant of Section "Experimental
Setup" / "Micro-Expert Integrity"): checked against the library's vector norms, a loop-written diagonal of
X_e^T X_e, and what the mathematics fixes (the projections do not change when the input channels of X and the
columns of W_up / W_gate are permuted together; the dagger split of W_down is CAMERA-Q's own)."""
import numpy as np
import torch

from oracle import camera_oracle as orc


def _layer(seed, n=40, d=12, f=7, ne=3, k=2):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d))
    L = rng.standard_normal((n, ne))
    _, _, A = orc.top_and_norm(L, k)
    Wg = rng.standard_normal((ne, f, d))
    Wu = rng.standard_normal((ne, f, d))
    Wd = rng.standard_normal((ne, d, f))
    return X, A, Wg, Wu, Wd


def test_input_channel_energy_is_the_diagonal_of_the_gram_matrix():
    X, A, *_ = _layer(0)
    h = orc.input_channel_energy(X, A)
    for e in range(A.shape[1]):
        rows = [j for j in range(X.shape[0]) if A[j, e] != 0.0]
        gram = np.zeros((X.shape[1], X.shape[1]))
        for j in rows:                       # H_e = sum_j x_j x_j^T, written out
            gram += np.outer(X[j], X[j])
        np.testing.assert_allclose(h[e], np.diag(gram), rtol=1e-12)
        want = torch.linalg.vector_norm(torch.from_numpy(X[rows]), dim=0).numpy() ** 2
        np.testing.assert_allclose(h[e], want, rtol=1e-12)
    # every token, one expert: the plain column sums of squares
    dense = orc.input_channel_energy(X, np.ones((X.shape[0], 1)))
    np.testing.assert_allclose(dense[0], orc.down_column_sumsq(X), rtol=1e-12)
    # an expert without tokens has no input energy; the routing weight's size does not matter
    A0 = A.copy()
    A0[:, 1] = 0.0
    assert np.all(orc.input_channel_energy(X, A0)[1] == 0.0)
    np.testing.assert_array_equal(orc.input_channel_energy(X, A * 3.7), h)
    # token order does not matter
    p = np.random.default_rng(1).permutation(X.shape[0])
    np.testing.assert_allclose(orc.input_channel_energy(X[p], A[p]), h, rtol=1e-12)


def test_column_gather_keeps_the_projections_under_a_joint_permutation():
    X, A, Wg, Wu, Wd = _layer(2)
    ne, f, d = Wg.shape
    h = orc.input_channel_energy(X, A)
    seg = [e * d for e in range(ne + 1)]
    bit_of, level_count, perm = orc.alloc_bits(h.ravel(), seg, [4, 3, 2], [0.25, 0.5, 0.25])
    count = np.full(ne, d)
    g_cols = orc.gather_columns(Wg, perm, count)
    u_cols = orc.gather_columns(Wu, perm, count)
    for e in range(ne):
        mine = perm[e * d:(e + 1) * d] - e * d
        assert sorted(mine.tolist()) == list(range(d))                  # a permutation of the expert's input channels
        np.testing.assert_array_equal(g_cols[e], Wg[e][:, mine])
        # X W^T is unchanged when X's channels and W's columns move together
        np.testing.assert_allclose(X[:, mine] @ g_cols[e].T, X @ Wg[e].T, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(X[:, mine] @ u_cols[e].T, X @ Wu[e].T, rtol=1e-12, atol=1e-12)
        # inside an expert the classes follow one another, highest input energy first, index order inside a class
        widths = bit_of[e * d:(e + 1) * d][mine]
        assert np.all(np.diff(widths.astype(int)) <= 0)
        for b in set(widths.tolist()):
            members = mine[widths == b]
            assert np.all(np.diff(members) > 0)
    assert level_count.sum() == ne * d


def test_dagger_and_cameraq_share_the_split_of_w_down():
    """W_down is sliced along d_ff by both: the dagger variant's W_down[:, s_k] is the W_down half of CAMERA-Q."""
    X, A, Wg, Wu, Wd = _layer(3)
    ne, f, d = Wg.shape
    E = orc.score_layer(X, A, Wg, Wu, Wd, 0.9)["energy"]
    seg = [e * f for e in range(ne + 1)]
    _, _, perm = orc.alloc_bits(E, seg, [3, 2, 1], [0.2, 0.6, 0.2])
    count = np.full(ne, f)
    _, _, down_q = orc.gather_micro_experts(Wg, Wu, Wd, perm, count)
    down_dagger = orc.gather_columns(Wd, perm, count)
    for a, b in zip(down_q, down_dagger):
        np.testing.assert_array_equal(a, b)
    # out-of-range entries are refused, as in the row gather
    bad = perm.copy()
    bad[0] = f * ne + 5
    try:
        orc.gather_columns(Wd, bad, count)
        raise AssertionError("accepted an index outside its expert")
    except ValueError:
        pass
