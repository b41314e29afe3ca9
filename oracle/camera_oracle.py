"""Plain fp64 CPU oracle for CAMERA micro-expert redundancy analysis.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct
definition that the HIP path is checked against.  Only the tests, the smoke
check and the bench's ``cpu_baseline`` leg may import it; it shares no code
with the HIP library and never imports it.  Everything is numpy float64; the
only library primitives used as steps are ``@`` (matmul), ``np.exp``,
``np.argsort(kind="stable")`` and ``np.cumsum``.

What is computed, in the paper's notation (Section "Micro-Expert Redundancy
Analysis"):

* an expert  E_i(x) = W_down,i [ silu(W_gate,i x) * (W_up,i x) ]      (Eq. 1)
* the layer  y = sum_i A_i(x) E_i(x)                                  (Eq. 2)
* micro-expert c of expert i = (gate row c, up row c, down column c)  (Eq. 3)
* its coefficient for a token  phi = a * silu(w_gate x) * (w_up x)    (Eq. 4)
* its energy  E = [(1-alpha)||Phi_col||_2^2 + alpha ||Phi_col||_inf^2]
                  * ||w_down||_2^2              (energy with balance coefficient)
* Algorithm 1 (micro-expert ranking): A = Top&Norm(R X); per expert the
  column statistics of Lambda = A[:,i] * silu(X W_gate^T) * (X W_up^T) and the
  squared column norms of W_down; energy; argsort.
* CAMERA-P's TopSelect (Algorithm 2) and CAMERA-Q's ListSplitByRatio /
  GetSubIndex (Algorithm 3).
* Applying a selection (Algorithm 2, lines 10-13): the kept gate / up rows and
  down columns of every expert, gathered in index order.
* The comparison variant CAMERA-Q-dagger, which slices all three matrices along
  their input dimension: the input-channel statistic diag(X_e^T X_e) that such
  schemes rank by, and the column gather W[:, s_k].
* The layer output with a subset of the micro-experts (Eq. 1-2; the recomputed
  output of Algorithm 2, line 14) and its distance from the original output:
  the Lemma's decoding error, L2 and cosine.

Readings taken where the paper is silent (each is listed in the design notes):
0-based experts and channels with half-open ranges; Top&Norm = softmax over
all experts, keep the k largest, renormalise the kept ones to sum 1; the
selection is taken on the logits (softmax is strictly increasing, so this is
the same set, and it cannot be blurred by exp underflow); exact ties go to the
lower index; a router bias, when given, is added to the logits; the order of
micro-experts is the stable ascending order of (energy, index);
n_prune = floor(lambda*N + 1e-6); class cuts are cumulative floors counted
from the most important end.

Parity pins: every function here is pinned by tests/test_oracle_*.py
(brute-force ablation of the plain layer forward, the Lemma, closed forms,
library softmax / SiLU, symmetries, brute-force sorting; for the gather, the
layer rebuilt from the compacted weights against the layer with the pruned
vectors zeroed; for the layer output, a loop-written forward pass, the
one-removed-index equality of the Lemma and the library's bfloat16 rounding; for the
dagger variant, the library's column norms and the invariance of the projections under
one permutation of the input channels of X and of the matrix columns).  The absolute score
values on the model-shaped configs are not printed anywhere in the paper:
for those, parity is pinned only through this oracle.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


# --------------------------------------------------------------------------
# Router: A = Top&Norm(R X)                                  (Algorithm 1, l.2)
# --------------------------------------------------------------------------
def router_logits(X, R, bias=None):
    """L[j, e] = <X[j, :], R[e, :]> (+ bias[e]).  X [n, d], R [N_E, d]."""
    L = _f64(X) @ _f64(R).T
    if bias is not None:
        L = L + _f64(bias)[None, :]
    return L


def softmax_rows(L):
    """Row-wise softmax with the row maximum subtracted first."""
    L = _f64(L)
    z = np.exp(L - L.max(axis=1, keepdims=True))
    return z / z.sum(axis=1, keepdims=True)


def top_and_norm(L, top_k, renorm=True):
    """Top&Norm of Algorithm 1 line 2 on logits L [n, N_E].

    Returns (idx [n, k] int64, w [n, k] f64, A [n, N_E] f64).  idx[j] lists the
    k experts with the largest logits, largest first, exact ties to the lower
    expert index.  w is the softmax probability of each kept expert, divided
    by the sum of the kept probabilities when ``renorm``.  A is the dense
    routing matrix with zeros for the experts that were not kept.
    """
    L = _f64(L)
    n, n_experts = L.shape
    if not (1 <= top_k <= n_experts):
        raise ValueError("top_k out of range")
    p = softmax_rows(L)
    order = np.argsort(-L, axis=1, kind="stable")  # descending, ties: lower index
    idx = order[:, :top_k]
    w = np.take_along_axis(p, idx, axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    A = np.zeros((n, n_experts), dtype=F64)
    np.put_along_axis(A, idx, w, axis=1)
    return idx.astype(np.int64), w, A


def dense_routing(idx, w, n_experts):
    """Scatter per-token (idx, w) lists [n, k] into the dense A [n, N_E]."""
    idx = np.asarray(idx, dtype=np.int64)
    A = np.zeros((idx.shape[0], n_experts), dtype=F64)
    np.put_along_axis(A, idx, _f64(w), axis=1)
    return A


# --------------------------------------------------------------------------
# Per-expert statistics                                   (Algorithm 1, l.5-8)
# --------------------------------------------------------------------------
def silu(g):
    """sigma(g) = g / (1 + exp(-g))                       (SiLU of Eq. 1)."""
    g = _f64(g)
    return g / (1.0 + np.exp(-g))


def lambda_matrix(X, a_col, W_gate, W_up):
    """Lambda [n, d_ff] = a_col[:, None] * silu(X W_gate^T) * (X W_up^T)   (l.6).

    W_gate, W_up are [d_ff, d_model] (row c belongs to micro-expert c).
    """
    X = _f64(X)
    G = X @ _f64(W_gate).T
    U = X @ _f64(W_up).T
    return _f64(a_col)[:, None] * silu(G) * U


def down_column_sumsq(W_down):
    """omega^2[c] = sum_r W_down[r, c]^2 ;  W_down is [d_model, d_ff]     (l.5)."""
    W = _f64(W_down)
    return (W * W).sum(axis=0)


def expert_column_stats(X, a_col, W_gate, W_up, skip_unrouted=True):
    """phi^2[c] = sum_j Lambda[j,c]^2 ,  phi^inf[c] = (max_j |Lambda[j,c]|)^2  (l.7-8).

    With ``skip_unrouted`` only the tokens whose routing weight is non-zero
    are pushed through the projections; rows of Lambda with a = 0 are zero
    rows, so both statistics are unchanged.  ``skip_unrouted=False`` is
    Algorithm 1 exactly as printed (all n tokens, masked by A[:, i]).
    """
    X = _f64(X)
    a_col = _f64(a_col)
    d_ff = np.asarray(W_gate).shape[0]
    if skip_unrouted:
        rows = np.nonzero(a_col != 0.0)[0]
        X, a_col = X[rows], a_col[rows]
    if X.shape[0] == 0:
        return np.zeros(d_ff, dtype=F64), np.zeros(d_ff, dtype=F64)
    Lam = lambda_matrix(X, a_col, W_gate, W_up)
    phi2 = (Lam * Lam).sum(axis=0)
    phi_inf = np.abs(Lam).max(axis=0) ** 2
    return phi2, phi_inf


def energy(phi2, phi_inf, omega2, alpha):
    """E = [(1 - alpha) phi^2 + alpha phi^inf] * omega^2                  (l.10)."""
    return ((1.0 - alpha) * _f64(phi2) + alpha * _f64(phi_inf)) * _f64(omega2)


def score_layer(X, A, W_gate, W_up, W_down, alpha, skip_unrouted=True):
    """Algorithm 1 lines 1-10 for one group of experts.

    X [n, d_model]; A [n, N_E] dense routing weights (zeros = not routed; a
    shared or dense expert has a column of ones); W_gate, W_up indexable by
    expert, each [d_ff, d_model]; W_down[e] is [d_model, d_ff].  Micro-expert
    (e, c) has global index e*d_ff + c.  Returns a dict of four float64
    vectors of length N_E*d_ff: phi2, phi_inf, omega2, energy.
    """
    X = _f64(X)
    A = _f64(A)
    n_experts = A.shape[1]
    phi2, phi_inf, omega2 = [], [], []
    for e in range(n_experts):
        p2, pinf = expert_column_stats(X, A[:, e], W_gate[e], W_up[e], skip_unrouted)
        phi2.append(p2)
        phi_inf.append(pinf)
        omega2.append(down_column_sumsq(W_down[e]))
    phi2 = np.concatenate(phi2)
    phi_inf = np.concatenate(phi_inf)
    omega2 = np.concatenate(omega2)
    return {"phi2": phi2, "phi_inf": phi_inf, "omega2": omega2,
            "energy": energy(phi2, phi_inf, omega2, alpha)}


def merge_chunks(stats_a, stats_b, alpha):
    """Statistics of the union of two disjoint token sets: phi^2 adds, phi^inf
    takes the larger, omega^2 depends on the weights only."""
    phi2 = stats_a["phi2"] + stats_b["phi2"]
    phi_inf = np.maximum(stats_a["phi_inf"], stats_b["phi_inf"])
    omega2 = stats_a["omega2"]
    return {"phi2": phi2, "phi_inf": phi_inf, "omega2": omega2,
            "energy": energy(phi2, phi_inf, omega2, alpha)}


# --------------------------------------------------------------------------
# Ranking, CAMERA-P selection, CAMERA-Q bit allocation
# --------------------------------------------------------------------------
def ascending_order(E):
    """Argsort of Algorithm 1 line 11: indices from the most redundant (lowest
    energy) to the most important, equal energies ordered by index."""
    return np.argsort(np.asarray(E), kind="stable")


def rank_of(E):
    """rank[i] = position of micro-expert i in ``ascending_order(E)``."""
    order = ascending_order(E)
    rank = np.empty(order.size, dtype=np.int64)
    rank[order] = np.arange(order.size)
    return rank


def prune_count(ratio, n_micro):
    """Number of micro-experts removed at pruning ratio lambda."""
    if not (0.0 <= ratio <= 1.0):
        raise ValueError("ratio outside [0, 1]")
    return int(np.floor(ratio * n_micro + 1e-6))


def _check_segments(seg_offsets, n_micro):
    seg = np.asarray(seg_offsets, dtype=np.int64)
    if seg.ndim != 1 or seg.size < 2 or seg[0] != 0 or seg[-1] != n_micro or np.any(np.diff(seg) < 0):
        raise ValueError("seg_offsets must rise from 0 to n_micro")
    return seg


def select_prune(E, seg_offsets, ratio):
    """TopSelect(R, 1 - lambda) of Algorithm 2 line 9, per layer.

    The ``prune_count`` lowest-ranked micro-experts are removed.  Returns
    keep_mask u8 [N], kept_per_expert i64 [n_seg], kept_idx i64 [N - n_prune]
    (global indices, ascending inside every expert, experts in order) and
    rank i64 [N].
    """
    E = np.asarray(E)
    N = E.size
    seg = _check_segments(seg_offsets, N)
    rank = rank_of(E)
    keep = rank >= prune_count(ratio, N)
    kept_per_expert = np.array([keep[seg[s]:seg[s + 1]].sum() for s in range(seg.size - 1)],
                               dtype=np.int64)
    return keep.astype(np.uint8), kept_per_expert, np.nonzero(keep)[0].astype(np.int64), rank


def class_cuts(ratios, n_micro):
    """Cumulative class boundaries counted from the most important end:
    cut[m] = floor((r_1 + ... + r_m) * N + 1e-6), cut[L] = N."""
    r = _f64(ratios)
    if r.ndim != 1 or r.size < 1 or np.any(r < 0) or abs(r.sum() - 1.0) > 1e-9:
        raise ValueError("ratios must be non-negative and sum to 1")
    acc, cuts = 0.0, []
    for m in range(r.size):
        acc += float(r[m])
        cuts.append(int(np.floor(acc * n_micro + 1e-6)))
    cuts[-1] = n_micro
    return cuts


def alloc_bits(E, seg_offsets, bits, ratios):
    """ListSplitByRatio + GetSubIndex of Algorithm 3 lines 5-8.

    Class 0 is the fraction ratios[0] of micro-experts with the highest energy
    and receives bits[0]; the last class is what remains at the low end.
    Returns bit_of u8 [N], level_count i64 [n_seg, L] and perm i64 [N]: inside
    every expert's range of perm the members of class 0 come first, then
    class 1, ..., each class in ascending index order (the reordering that
    colocates micro-experts of equal precision inside an expert).
    """
    E = np.asarray(E)
    N = E.size
    seg = _check_segments(seg_offsets, N)
    bits = np.asarray(bits, dtype=np.int64)
    cuts = class_cuts(ratios, N)
    L = len(cuts)
    if bits.size != L:
        raise ValueError("bits and ratios differ in length")
    from_top = (N - 1) - rank_of(E)           # 0 = highest energy
    cls = np.zeros(N, dtype=np.int64)
    for m in range(L - 1):
        cls += (from_top >= cuts[m]).astype(np.int64)
    level_count = np.zeros((seg.size - 1, L), dtype=np.int64)
    perm = np.empty(N, dtype=np.int64)
    for s in range(seg.size - 1):
        lo, hi = int(seg[s]), int(seg[s + 1])
        pos = lo
        for m in range(L):
            members = lo + np.nonzero(cls[lo:hi] == m)[0]
            level_count[s, m] = members.size
            perm[pos:pos + members.size] = members
            pos += members.size
    return bits[cls].astype(np.uint8), level_count, perm


# --------------------------------------------------------------------------
# Applying a selection: W_up, W_gate, W_down <- W_up[S,:], W_gate[S,:], W_down[:,S]
#                                                        (Algorithm 2, l.10-13)
# --------------------------------------------------------------------------
def gather_micro_experts(W_gate, W_up, W_down, index, count, index_base=0):
    """Keeps the micro-experts listed in ``index``, in that order.

    W_gate, W_up [N_E, d_ff, d_model]; W_down [N_E, d_model, d_ff].  ``index``
    holds global micro-expert indices index_base + e*d_ff + c grouped by
    expert in expert order, ``count[e]`` of them for expert e (the kept_idx /
    kept_per_expert of ``select_prune``, or the perm of ``alloc_bits`` with
    count = d_ff: the reordering that colocates equal precision, Section
    "Mixed-precision Strategy CAMERA-Q").  Returns

      gate_out, up_out  [len(index), d_model]: row r is the gate / up row of
                        micro-expert index[r];
      down_out          list over experts of [d_model, count[e]] matrices whose
                        column j is the down column of the expert's j-th entry.

    Same dtype as the inputs: the values are copied, never recomputed.
    """
    W_gate, W_up, W_down = np.asarray(W_gate), np.asarray(W_up), np.asarray(W_down)
    n_experts, d_ff, d_model = W_gate.shape
    if W_up.shape != W_gate.shape or W_down.shape != (n_experts, d_model, d_ff):
        raise ValueError("weight shapes disagree")
    index = np.asarray(index, dtype=np.int64)
    count = np.asarray(count, dtype=np.int64)
    if count.shape != (n_experts,) or count.sum() != index.size or np.any(count < 0):
        raise ValueError("count must give the number of entries of every expert")
    gate_out = np.empty((index.size, d_model), dtype=W_gate.dtype)
    up_out = np.empty((index.size, d_model), dtype=W_up.dtype)
    down_out = []
    pos = 0
    for e in range(n_experts):
        mine = index[pos:pos + count[e]] - index_base - e * d_ff      # channels of expert e
        if np.any(mine < 0) or np.any(mine >= d_ff):
            raise ValueError("an index lies outside its expert")
        gate_out[pos:pos + count[e]] = W_gate[e][mine, :]
        up_out[pos:pos + count[e]] = W_up[e][mine, :]
        down_out.append(W_down[e][:, mine].copy())
        pos += int(count[e])
    return gate_out, up_out, down_out


# --------------------------------------------------------------------------
# CAMERA-Q-dagger: the comparison variant that slices every matrix along its
# input dimension (Section "Experimental Setup", mixed-precision paragraph;
# Section "Micro-Expert Integrity")
# --------------------------------------------------------------------------
def input_channel_energy(X, A):
    """h[e, c] = sum over the tokens j routed to expert e of X[j, c]^2: the diagonal of
    H_e = X_e^T X_e, the input-side statistic by which column-wise mixed-precision schemes
    rank the input channels of a matrix.  X [n, d_model]; A [n, N_E] routing weights (only
    whether A[j, e] is zero matters: H depends on the inputs alone).  Returns [N_E, d_model]."""
    X, A = _f64(X), _f64(A)
    h = np.zeros((A.shape[1], X.shape[1]), dtype=F64)
    for e in range(A.shape[1]):
        rows = np.nonzero(A[:, e] != 0.0)[0]
        h[e] = (X[rows] * X[rows]).sum(axis=0)
    return h


def gather_columns(W, index, count, index_base=0):
    """W[e][:, S_e] for every expert: the columns listed in ``index`` (global indices
    index_base + e*cols + c, grouped by expert in expert order, count[e] of them), in that order.
    W [N_E, rows, cols].  With W = W_up or W_gate ([N_E, d_ff, d_model]: columns are input
    channels) and the per-expert reordering that ``alloc_bits`` returns for the input-channel
    energies, this is the column-wise slicing W_{:, s_k} of the dagger variant; with W = W_down it
    is the W_down half of ``gather_micro_experts``.  Returns a list of [rows, count[e]] matrices."""
    W = np.asarray(W)
    n_experts, _, cols = W.shape
    index = np.asarray(index, dtype=np.int64)
    count = np.asarray(count, dtype=np.int64)
    if count.shape != (n_experts,) or count.sum() != index.size or np.any(count < 0):
        raise ValueError("count must give the number of entries of every expert")
    out, pos = [], 0
    for e in range(n_experts):
        mine = index[pos:pos + count[e]] - index_base - e * cols
        if np.any(mine < 0) or np.any(mine >= cols):
            raise ValueError("an index lies outside its expert")
        out.append(W[e][:, mine].copy())
        pos += int(count[e])
    return out


# --------------------------------------------------------------------------
# Layer output with a subset of the micro-experts, and its decoding error
#                    (Eq. 1-2; Algorithm 2, l.14; the Lemma's epsilon; the
#                     L2 / cosine comparison of hidden states after pruning)
# --------------------------------------------------------------------------
def round_to_bf16(a):
    """Nearest bfloat16 (ties to even) of every element, returned as float64.

    bfloat16 is the upper half of a float32: the value is first rounded to
    float32, then the low 16 bits are rounded away.  Finite inputs only."""
    f32 = np.asarray(a, dtype=np.float32)
    u = f32.view(np.uint32).astype(np.uint64)
    keep_odd = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + keep_odd) >> np.uint64(16) << np.uint64(16)
    return u.astype(np.uint32).view(np.float32).astype(F64).reshape(f32.shape)


def layer_forward(X, A, W_gate, W_up, W_down, keep=None, round_hidden=None):
    """y_j = sum_e W_down,e Lambda_e[j, :]  with  Lambda_e = A[:, e] * silu(X W_gate,e^T) * (X W_up,e^T)
    (Eq. 1-2 with the coefficient of Eq. 4), over the kept micro-experts only.

    keep: None or a 0/1 vector over the layer's micro-experts (index e*d_ff + c):
    a pruned micro-expert contributes nothing (its three vectors are zeroed together).
    round_hidden: None, or a function applied to Lambda before the down
    projection (``round_to_bf16`` for a 16-bit model, whose hidden activations
    are stored in that format).  Returns Y [n, d_model].
    """
    X, A = _f64(X), _f64(A)
    n, d_model = X.shape
    Y = np.zeros((n, d_model), dtype=F64)
    pos = 0
    for e in range(len(W_gate)):
        Wd = _f64(W_down[e])
        d_ff = Wd.shape[1]
        lam = lambda_matrix(X, A[:, e], W_gate[e], W_up[e])
        if keep is not None:
            lam = lam * _f64(np.asarray(keep)[pos:pos + d_ff])[None, :]
        if round_hidden is not None:
            lam = round_hidden(lam)
        Y += lam @ Wd.T
        pos += d_ff
    return Y


def output_error(Y, Y_hat):
    """How far the pruned layer's output is from the original one: per token
    d2 = ||y - y_hat||^2, yy = ||y||^2, hh = ||y_hat||^2, yh = <y, y_hat>, and
    from them l2 = ||Y - Y_hat||_F (the square root of the Lemma's epsilon),
    cosine = <Y, Y_hat> / (||Y||_F ||Y_hat||_F) over the whole calibration set, and
    cosine_mean = the mean of the per-token cosines (tokens with a zero norm left out)."""
    Y, Y_hat = _f64(Y), _f64(Y_hat)
    diff = Y - Y_hat
    d2, yy, hh, yh = (diff * diff).sum(1), (Y * Y).sum(1), (Y_hat * Y_hat).sum(1), (Y * Y_hat).sum(1)
    ok = (yy > 0) & (hh > 0)
    flat_den = np.sqrt(yy.sum() * hh.sum())
    return {"d2": d2, "yy": yy, "hh": hh, "yh": yh, "l2": float(np.sqrt(d2.sum())),
            "cosine": float(yh.sum() / flat_den) if flat_den > 0 else float("nan"),
            "cosine_mean": float(np.mean(yh[ok] / np.sqrt(yy[ok] * hh[ok]))) if ok.any() else float("nan")}
