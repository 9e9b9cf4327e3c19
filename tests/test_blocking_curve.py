"""Blocking curves (sections 2.2, 4.3.1) and the selection rule of sections 4.3.2 / 4.4.2.

The oracle's curve is pinned to what the generator fixes: on a noise-free planted matrix whose
groups drew distinct block sets every threshold in (0, 1] recovers the planted blocking, so the
average block height is the planted height and the in-block density the planted fill, exactly;
tau = 1 on any matrix gives the classes of identical quotient rows, whose counts a few lines of
numpy produce.  The library's integer counts must then match the oracle's bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_2202_05868_amd import binding, synth
from helpers import csr_from_rows, random_csr, row_patterns

TAUS = [0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0]


def test_oracle_curve_on_planted_matrix_is_the_planted_blocking():
    rng = np.random.default_rng(11)
    heights = [24] * 20
    a, info = synth.planted(rng, heights, 40 * 8, 8, blocks_per_group=5, fill=1.0, shuffle=True)
    sets = {tuple(b) for b in info["block_sets"]}
    assert len(sets) == 20                      # distinct block sets: nothing merges across groups
    curve = oracle.blocking_curve(a, 8, TAUS, 24)
    for pt in curve["points"]:
        if pt["tau"] >= 0.7:                    # two groups sharing 4 of 5 blocks have Jaccard 4/6 < 0.7
            assert pt["n_groups"] == 20 and pt["n_blocks"] == 100
            assert pt["avg_height"] == 24.0 and pt["rho"] == 1.0 and pt["stored_elems"] == a["nnz"]
    assert curve["points"][curve["selected"]]["avg_height"] == 24.0


def test_oracle_curve_density_with_partial_fill_and_tau_one():
    rng = np.random.default_rng(12)
    a, info = synth.planted(rng, [16] * 12, 30 * 4, 4, blocks_per_group=6, fill=0.5, shuffle=True)
    pt = oracle.blocking_curve(a, 4, [1.0], 16)["points"][0]
    # tau = 1: groups are the classes of identical quotient rows
    pats = row_patterns(a, 4)
    classes = {}
    for i, p in enumerate(pats):
        classes.setdefault(p, []).append(i)
    n_blocks = sum(len(p) for p in classes)
    area = sum(len(p) * len(m) * 4 for p, m in classes.items())
    assert pt["n_groups"] == len(classes) and pt["n_blocks"] == n_blocks and pt["stored_elems"] == area
    assert pt["rho"] == a["nnz"] / area
    assert pt["sum_heights"] == sum(len(p) * len(m) for p, m in classes.items())


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_library_curve_matches_oracle(seed):
    rng = np.random.default_rng(seed)
    a = random_csr(rng, 400, 24 * 4, float(rng.choice([0.03, 0.1])))
    for target in (1, 3, 8, 1000):
        want = oracle.blocking_curve(a, 4, TAUS, target)
        got = binding.sa1_blocking_curve(a, 4, TAUS, target)
        for k in ("n_groups", "n_blocks", "stored_elems", "sum_heights"):
            assert [p[k] for p in want["points"]] == got[k].tolist(), k
        assert got["selected"] == want["selected"]


def test_library_curve_on_reduced_workloads_and_errors():
    w = synth.workload("c2", scale=0.25)
    want = oracle.blocking_curve(w["A"], w["col_block"], TAUS, 64)
    got = binding.sa1_blocking_curve(w["A"], w["col_block"], TAUS, 64)
    assert got["selected"] == want["selected"]
    assert [p["stored_elems"] for p in want["points"]] == got["stored_elems"].tolist()
    with pytest.raises(binding.VbrError):
        binding.sa1_blocking_curve(w["A"], w["col_block"], [0.5, 1.5], 64)
    with pytest.raises(binding.VbrError):
        binding.sa1_blocking_curve(w["A"], w["col_block"], TAUS, 0)


# --------------------------------------------------------------------------- the selection, by hand
def _pair(first_col, k, rows_a, rows_b):
    """Two classes of identical rows over unit-wide column blocks: `rows_a` rows with the k blocks
    first_col .. first_col+k-1 and `rows_b` rows with the first k-1 of them plus block first_col+k.
    Their Jaccard similarity is (k-1)/(k+1) and their union has k+1 blocks, so under the two-step
    condition they merge exactly when tau <= (k-1)/(k+1) and k+1 <= floor(k / (1 - tau/2))."""
    a = list(range(first_col, first_col + k))
    b = a[:-1] + [first_col + k]
    return [a] * rows_a + [b] * rows_b


def _hand_curve_matrix():
    # pair of k=4 (4 + 2 rows): merges for 0.4 <= tau <= 0.6 (Jaccard 3/5; limit floor(4/(1-tau/2)) >= 5)
    # pair of k=9 (3 + 5 rows): merges for 0.2 <= tau <= 0.8 (Jaccard 8/10; limit floor(9/(1-tau/2)) >= 10)
    # the two pairs share no column, so for tau > 0 nothing else can merge
    return csr_from_rows(_pair(0, 4, 4, 2) + _pair(8, 9, 3, 5), n_cols=20)


# (nonzero blocks, sum over blocks of their height) of each pair, apart and merged
K4_APART, K4_MERGED = (4 + 4, 4 * 4 + 2 * 4), (5, 6 * 5)
K9_APART, K9_MERGED = (9 + 9, 3 * 9 + 5 * 9), (10, 8 * 10)
HAND_TAUS = [0.9, 0.7, 0.5, 0.3, 0.1]
HAND_COUNTS = [(K4_APART[0] + K9_APART[0], K4_APART[1] + K9_APART[1]),       # 0.9: 26 blocks, 96 -> 3.69
               (K4_APART[0] + K9_MERGED[0], K4_APART[1] + K9_MERGED[1]),     # 0.7: 18 blocks, 104 -> 5.78
               (K4_MERGED[0] + K9_MERGED[0], K4_MERGED[1] + K9_MERGED[1]),   # 0.5: 15 blocks, 110 -> 7.33
               (K4_APART[0] + K9_MERGED[0], K4_APART[1] + K9_MERGED[1]),     # 0.3: as 0.7 (limit stops the k=4 pair)
               (K4_APART[0] + K9_APART[0], K4_APART[1] + K9_APART[1])]       # 0.1: as 0.9 (limit stops both)
# target average height -> index the rule must select (nearest; of equally near ones the first given)
HAND_SELECTED = {7: 2,       # 7.33 is nearest, unique, neither first nor last
                 1000: 2,    # beyond every point: the tallest
                 6: 1,       # 5.78 twice (indices 1 and 3): the first of the two
                 5: 1,       # |5.78 - 5| = 0.78 < |3.69 - 5| = 1.31
                 4: 0,       # |3.69 - 4| = 0.31 (indices 0 and 4) < |5.78 - 4| = 1.78
                 1: 0}


@pytest.mark.parametrize("which", ["oracle", "library"])
def test_selected_blocking_on_a_curve_derived_by_hand(which):
    a = _hand_curve_matrix()
    assert HAND_COUNTS == [(26, 96), (18, 104), (15, 110), (18, 104), (26, 96)]
    for target, want in HAND_SELECTED.items():
        if which == "oracle":
            cur = oracle.blocking_curve(a, 1, HAND_TAUS, target)
            got = [(p["n_blocks"], p["sum_heights"]) for p in cur["points"]]
        else:
            cur = binding.sa1_blocking_curve(a, 1, HAND_TAUS, target)
            got = list(zip(cur["n_blocks"].tolist(), cur["sum_heights"].tolist()))
        assert got == HAND_COUNTS
        assert cur["selected"] == want, "target %d" % target
    # the same thresholds in the opposite order: equal points swap places, the first given still wins
    rev = HAND_TAUS[::-1]
    for target, want in {7: 2, 6: 1, 4: 0}.items():
        cur = (oracle.blocking_curve if which == "oracle" else binding.sa1_blocking_curve)(a, 1, rev, target)
        assert cur["selected"] == want


@pytest.mark.parametrize("which", ["oracle", "library"])
def test_selected_blocking_on_a_genuine_tie_and_on_a_matrix_without_blocks(which):
    curve = oracle.blocking_curve if which == "oracle" else binding.sa1_blocking_curve
    # one k=4 pair of 3 + 1 rows: apart 8 blocks of heights 3,3,3,3,1,1,1,1 (average 2), merged 5
    # blocks of height 4; the target 3 is exactly half-way: the first threshold given is selected
    a = csr_from_rows(_pair(0, 4, 3, 1), n_cols=8)
    for taus, heights in ([1.0, 0.5], [2, 4]), ([0.5, 1.0], [4, 2]):
        cur = curve(a, 1, taus, 3)
        if which == "oracle":
            got = [p["sum_heights"] / p["n_blocks"] for p in cur["points"]]
        else:
            got = (cur["sum_heights"] / cur["n_blocks"]).tolist()
        assert got == heights and cur["selected"] == 0
        assert curve(a, 1, taus, 4)["selected"] == heights.index(4)
        assert curve(a, 1, taus, 2)["selected"] == heights.index(2)
    # a matrix without entries has no blocks at any threshold (the only way a blocking can have
    # none, as the stored blocks are those with an entry): nothing to choose from, index 0
    empty = csr_from_rows([[], [], []], n_cols=4)
    assert curve(empty, 1, [0.3, 0.6], 2)["selected"] == 0
