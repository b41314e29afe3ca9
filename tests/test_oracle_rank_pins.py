"""Pins for the oracle's ranking, CAMERA-P selection and CAMERA-Q allocation
(CPU only): brute-force sorting in pure Python, counting identities, nesting,
and the worked bit-width example the paper prints."""
import os

import numpy as np
import pytest

from oracle import camera_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "cameraq_bits_example.txt")


def read_golden():
    out = {}
    with open(GOLDEN) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


def energies_with_ties(seed, n):
    rng = np.random.default_rng(seed)
    E = rng.gamma(0.5, size=n).astype(np.float32)
    E[rng.choice(n, n // 5, replace=False)] = 0.0          # experts without tokens give zeros
    E[rng.choice(n, n // 7, replace=False)] = E[3]         # repeated positive value
    return E


def python_rank(E):
    order = sorted(range(len(E)), key=lambda i: (float(E[i]), i))
    rank = [0] * len(E)
    for pos, i in enumerate(order):
        rank[i] = pos
    return order, rank


def test_order_and_rank_match_python_sort():
    E = energies_with_ties(0, 300)
    order, rank = python_rank(E)
    assert list(orc.ascending_order(E)) == order
    assert list(orc.rank_of(E)) == rank


@pytest.mark.parametrize("ratio", [0.0, 0.2, 0.4, 0.6, 0.333, 1.0])
def test_select_prune_against_python_sort(ratio):
    E = energies_with_ties(1, 240)
    seg = [0, 50, 50, 130, 240]                             # one empty segment
    keep, per_expert, kept_idx, rank = orc.select_prune(E, seg, ratio)
    order, py_rank = python_rank(E)
    n_prune = int(np.floor(ratio * 240 + 1e-6))
    want_keep = np.ones(240, dtype=np.uint8)
    want_keep[order[:n_prune]] = 0
    np.testing.assert_array_equal(keep, want_keep)
    assert keep.sum() == 240 - n_prune
    assert list(rank) == py_rank
    assert list(kept_idx) == [i for i in range(240) if want_keep[i]]
    assert list(per_expert) == [int(want_keep[seg[s]:seg[s + 1]].sum()) for s in range(4)]
    # every kept micro-expert is at least as important as every pruned one
    if 0 < n_prune < 240:
        assert E[keep == 0].max() <= E[keep == 1].min()


def test_select_prune_is_nested_in_ratio():
    E = energies_with_ties(2, 500)
    seg = [0, 250, 500]
    masks = [orc.select_prune(E, seg, r)[0] for r in (0.2, 0.4, 0.6)]
    assert np.all(masks[1] <= masks[0]) and np.all(masks[2] <= masks[1])
    assert orc.select_prune(E, seg, 0.0)[0].all()
    assert not orc.select_prune(E, seg, 1.0)[0].any()


def test_prune_count_values():
    assert orc.prune_count(0.4, 4096) == 1638
    assert orc.prune_count(0.2, 184320) == 36864
    assert orc.prune_count(0.6, 98304) == 58982
    assert orc.prune_count(0.0, 10) == 0 and orc.prune_count(1.0, 10) == 10
    with pytest.raises(ValueError):
        orc.prune_count(1.5, 10)


def test_alloc_bits_paper_example_average():
    g = read_golden()
    bits = [int(b) for b in g["bits"]]
    ratios = g["ratios"]
    E = np.random.default_rng(3).gamma(0.5, size=2000).astype(np.float32)
    bit_of, level_count, perm = orc.alloc_bits(E, [0, 700, 2000], bits, ratios)
    assert level_count.sum() == 2000
    assert list(level_count.sum(axis=0)) == [200, 1600, 200]
    assert bit_of.astype(np.float64).mean() == pytest.approx(g["average_bits"][0], abs=1e-12)
    total = bit_of.astype(np.float64).mean() + g["group_overhead_bits"][0] / g["group_size"][0]
    assert total == pytest.approx(g["total_bits"][0], abs=1e-12)
    # the experiments' r = 0.2 keeps the same average
    r = g["experiment_r"][0]
    bit_of, _, _ = orc.alloc_bits(E, [0, 2000], bits, [r, 1 - 2 * r, r])
    assert bit_of.astype(np.float64).mean() == pytest.approx(2.0, abs=1e-12)


def test_alloc_bits_against_python_sort():
    E = energies_with_ties(4, 360)
    seg = [0, 100, 100, 260, 360]
    bits, ratios = [4, 3, 2], [0.1, 0.3, 0.6]
    bit_of, level_count, perm = orc.alloc_bits(E, seg, bits, ratios)
    order, _ = python_rank(E)
    descending = order[::-1]                               # most important first
    cuts = [int(np.floor(0.1 * 360 + 1e-6)), int(np.floor((0.1 + 0.3) * 360 + 1e-6)), 360]
    want = np.zeros(360, dtype=np.uint8)
    lo = 0
    for m, hi in enumerate(cuts):
        for i in descending[lo:hi]:
            want[i] = bits[m]
        lo = hi
    np.testing.assert_array_equal(bit_of, want)
    # higher energy never gets fewer bits
    o = np.array(order)
    assert np.all(np.diff(bit_of[o].astype(int)) >= 0)
    # per-expert counts and the stable partition
    for s in range(4):
        a, b = seg[s], seg[s + 1]
        want_perm = []
        for m in range(3):
            members = [i for i in range(a, b) if want[i] == bits[m]]
            assert level_count[s, m] == len(members)
            want_perm += members
        assert list(perm[a:b]) == want_perm
    assert sorted(perm) == list(range(360))


def test_alloc_lowest_class_is_the_prune_mask():
    """With ratios [r, 1-2r, r] the lowest class is exactly what CAMERA-P
    removes at lambda = r (same order, same boundary)."""
    E = energies_with_ties(5, 1000)
    seg = [0, 1000]
    bit_of, _, _ = orc.alloc_bits(E, seg, [3, 2, 1], [0.2, 0.6, 0.2])
    keep = orc.select_prune(E, seg, 0.2)[0]
    np.testing.assert_array_equal(bit_of == 1, keep == 0)
    # degenerate split: everything in the last class
    bit_of, level_count, perm = orc.alloc_bits(E, seg, [4, 3, 2], [0.0, 0.0, 1.0])
    assert np.all(bit_of == 2) and list(level_count[0]) == [0, 0, 1000]
    assert list(perm) == list(range(1000))


def test_bad_arguments_raise():
    E = np.ones(10, dtype=np.float32)
    with pytest.raises(ValueError):
        orc.select_prune(E, [0, 5], 0.5)
    with pytest.raises(ValueError):
        orc.alloc_bits(E, [0, 10], [3, 2, 1], [0.5, 0.2, 0.2])
    with pytest.raises(ValueError):
        orc.alloc_bits(E, [0, 10], [3, 2], [0.1, 0.8, 0.1])
