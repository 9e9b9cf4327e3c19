"""Blocking curves (sections 4.1, 6.1) and the selection rule of section 6.2.

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
from helpers import random_csr, row_patterns

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
