"""Pins for the oracle's 1-SA reordering and VBR index (CPU only).

Each test checks the C oracle against something other than itself: values the paper states,
a set-based transcription on tiny inputs, a textbook special case, or an invariant the
paper proves.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_2202_05868_amd import synth
from helpers import (check_partition_shape, csr_from_rows, groups_as_sets, random_csr,
                     row_patterns, sa1_sets)

TAUS = [0.0, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0]


def staircase(ell, q):
    """Rows of the pathological example of section 3.2: ell rows {0}, then prefixes {0..j}, j<q."""
    return [[0]] * ell + [list(range(j + 1)) for j in range(q)]


# ------------------------------------------------------------------ the paper's stated outcome
def test_staircase_similarity_only_gives_the_single_block_the_paper_states(golden_dir):
    path = os.path.join(golden_dir, "staircase_section_3_2.txt")
    rows = [tuple(int(x) for x in ln.split()) for ln in open(path) if ln.strip() and ln[0] != "#"]
    assert rows
    for ell, q, brows, bcols, nnz in rows:
        csr = csr_from_rows(staircase(ell, q), n_cols=q + 3)
        assert csr["nnz"] == nnz
        for tau in (0.5,):
            perm, rg = oracle.sa1(csr, 1, tau, similarity_only=True)
            assert len(rg) - 1 == 1                       # ONE group
            assert rg[1] - rg[0] == brows == ell + q
            bp, bc, bo = oracle.vbr_index(csr, perm, rg, 1)
            assert len(bc) == bcols == q                  # q non-empty columns
            density = nnz / (brows * bcols)               # Theta(ell^-1/4): falls with ell
            assert density < 1.7 / q


def test_staircase_with_the_merge_limit_splits_as_derived_by_hand():
    # tau = 0.5: limit floor(lambda0 / 0.75); seeds with lambda0 = 1,2,3,5,7 allow 1,2,4,6,9 columns
    ell, q = 20, 9
    csr = csr_from_rows(staircase(ell, q), n_cols=q)
    perm, rg = oracle.sa1(csr, 1, 0.5)
    s = lambda j: ell + j
    expect = [frozenset(range(ell)) | {s(0)}, {s(1)}, {s(2), s(3)}, {s(4), s(5)}, {s(6), s(7), s(8)}]
    assert groups_as_sets(perm, rg) == [frozenset(x) for x in expect]
    check_partition_shape(perm, rg, ell + q)


# ------------------------------------------------------------------ brute force on tiny inputs
@pytest.mark.parametrize("col_block", [1, 2, 3])
def test_matches_set_based_transcription_on_tiny_random_matrices(col_block):
    rng = np.random.default_rng(7 + col_block)
    for trial in range(60):
        n_rows = int(rng.integers(1, 13))
        kb = int(rng.integers(1, 7))
        dens = float(rng.choice([0.1, 0.3, 0.5, 0.8]))
        csr = random_csr(rng, n_rows, kb * col_block, dens)
        for tau in TAUS:
            for so in (False, True):
                p0, g0 = sa1_sets(csr, col_block, tau, similarity_only=so)
                p1, g1 = oracle.sa1(csr, col_block, tau, similarity_only=so)
                assert np.array_equal(p0, p1) and np.array_equal(g0, g1), (trial, tau, so)
                check_partition_shape(p1, g1, n_rows)


def test_rejected_row_is_not_revisited_and_pattern_grows():
    # seed {0,1}; row1 {2,3} dissimilar now; row2 {0,1,2,3}... with tau=0.5: J({0,1},{0,1,2,3})=0.5,
    # union 4 > floor(2/0.75)=2 -> rejected by the limit; similarity-only merges it and the pattern
    # becomes {0,1,2,3}; row1 was already passed and stays out (single scan per seed).
    csr = csr_from_rows([[0, 1], [2, 3], [0, 1, 2, 3]], n_cols=4)
    perm, rg = oracle.sa1(csr, 1, 0.5, similarity_only=True)
    assert groups_as_sets(perm, rg) == [frozenset({0, 2}), frozenset({1})]
    perm, rg = oracle.sa1(csr, 1, 0.5)
    assert groups_as_sets(perm, rg) == [frozenset({0}), frozenset({1}), frozenset({2})]
    # a later row that only becomes similar thanks to the union IS merged in the same scan
    csr = csr_from_rows([[0, 1, 2], [0, 1, 2, 3], [1, 2, 3, 4]], n_cols=6)
    perm, rg = oracle.sa1(csr, 1, 0.6, similarity_only=True)   # J(P={0..3},{1..4}) = 3/5
    assert groups_as_sets(perm, rg) == [frozenset({0, 1, 2})]


def test_threshold_is_inclusive_at_exact_fractions():
    # I/U equal to tau exactly must merge: 7/10 vs 0.7, 3/5 vs 0.6, 3/10 vs 0.3, 2/5 vs 0.4, 4/5 vs 0.8
    for inter, union, tau in [(7, 10, 0.7), (3, 5, 0.6), (3, 10, 0.3), (2, 5, 0.4), (4, 5, 0.8)]:
        seed = list(range(union))              # lambda0 = union, so the limit never binds
        other = list(range(inter))
        csr = csr_from_rows([seed, other], n_cols=union + 1)
        perm, rg = oracle.sa1(csr, 1, tau)
        assert len(rg) - 1 == 1, (inter, union, tau)
        csr = csr_from_rows([seed, other[:-1]], n_cols=union + 1)   # one less in common: below tau
        perm, rg = oracle.sa1(csr, 1, tau)
        assert len(rg) - 1 == 2, (inter, union, tau)


# ------------------------------------------------------------------ special cases with a plain definition
def test_tau_one_groups_exactly_the_identical_quotient_rows():
    rng = np.random.default_rng(11)
    for col_block in (1, 4, 8):
        csr = random_csr(rng, 200, 8 * col_block, 0.15)
        perm, rg = oracle.sa1(csr, col_block, 1.0)
        pats = row_patterns(csr, col_block)
        # plain unique-rows grouping on a dense 0/1 table
        table = np.zeros((200, 8), dtype=np.uint8)
        for i, p in enumerate(pats):
            table[i, list(p)] = 1
        _, inv = np.unique(table, axis=0, return_inverse=True)
        inv = np.asarray(inv).reshape(-1)
        expect = {}
        for i, k in enumerate(inv):
            expect.setdefault(int(k), set()).add(i)
        assert set(groups_as_sets(perm, rg)) == {frozenset(v) for v in expect.values()}
        check_partition_shape(perm, rg, 200)


def test_single_column_block_gives_nonempty_rows_and_empty_rows():
    rng = np.random.default_rng(5)
    csr = random_csr(rng, 64, 16, 0.05)
    lens = np.diff(csr["row_ptr"])
    assert (lens == 0).any() and (lens > 0).any()
    for tau in (0.1, 0.5, 1.0):
        perm, rg = oracle.sa1(csr, 16, tau)
        assert set(groups_as_sets(perm, rg)) == {frozenset(np.nonzero(lens > 0)[0].tolist()),
                                                 frozenset(np.nonzero(lens == 0)[0].tolist())}


def test_identical_quotient_rows_always_share_a_group():
    rng = np.random.default_rng(3)
    csr = random_csr(rng, 300, 40, 0.08)
    for tau in (0.0, 0.3, 0.7):
        perm, rg = oracle.sa1(csr, 4, tau)
        grp = np.empty(300, dtype=np.int64)
        for g in range(len(rg) - 1):
            grp[perm[rg[g]: rg[g + 1]]] = g
        seen = {}
        for i, p in enumerate(row_patterns(csr, 4)):
            assert seen.setdefault(p, grp[i]) == grp[i]


# ------------------------------------------------------------------ invariants the paper proves
@pytest.mark.parametrize("tau", [0.1, 0.3, 0.5, 0.7, 0.9])
def test_density_bound_and_merge_limit_hold_for_every_group(tau):
    # Theorem 1 on quotient rows: (#(row, block) pairs holding a nonzero) / (h * blocks) >= tau/2,
    # hence element density >= tau / (2 col_block); and blocks <= lambda0 / (1 - tau/2).
    rng = np.random.default_rng(int(tau * 100))
    for col_block, dens in itertools.product((1, 4), (0.02, 0.1, 0.3)):
        csr = random_csr(rng, 250, 24 * col_block, dens)
        pats = row_patterns(csr, col_block)
        perm, rg = oracle.sa1(csr, col_block, tau)
        bp, bc, bo = oracle.vbr_index(csr, perm, rg, col_block)
        for g in range(len(rg) - 1):
            rows = perm[rg[g]: rg[g + 1]]
            nb = bp[g + 1] - bp[g]
            if nb == 0:
                continue
            pairs = sum(len(pats[r]) for r in rows)
            assert pairs / (len(rows) * nb) >= tau / 2 - 1e-12
            nnz_g = sum(csr["row_ptr"][r + 1] - csr["row_ptr"][r] for r in rows)
            assert nnz_g / (len(rows) * nb * col_block) >= tau / (2 * col_block) - 1e-12
            lam0 = len(pats[rows[0]])
            assert nb <= lam0 / (1 - tau / 2) + 1e-9


# ------------------------------------------------------------------ planted structure comes back
def test_noise_free_planted_groups_are_recovered_after_scrambling():
    for name, scale in (("c1", 1.0), ("c2", 0.25), ("c3", 0.125)):
        w = synth.workload(name, scale=scale, noise=False)
        info = w["info"]
        # planted groups that drew the same block set are indistinguishable: expect their union
        expect = {}
        for g, bs in enumerate(info["block_sets"]):
            expect.setdefault(tuple(bs.tolist()), set()).update(np.nonzero(info["label"] == g)[0].tolist())
        for tau in w["taus"]:
            perm, rg = oracle.sa1(w["A"], w["col_block"], tau)
            assert set(groups_as_sets(perm, rg)) == {frozenset(v) for v in expect.values()}
            check_partition_shape(perm, rg, w["A"]["n_rows"])


# ------------------------------------------------------------------ VBR index
def test_vbr_index_covers_every_nonzero_exactly_once_and_stores_no_empty_block():
    rng = np.random.default_rng(21)
    for col_block in (1, 3, 8):
        csr = random_csr(rng, 120, 12 * col_block, 0.07)
        perm, rg = oracle.sa1(csr, col_block, 0.4)
        bp, bc, bo = oracle.vbr_index(csr, perm, rg, col_block)
        assert bp[0] == 0 and bp[-1] == len(bc) and bo[0] == 0
        dense = synth.dense_bits(csr)
        rebuilt = np.zeros_like(dense)
        covered = np.zeros(dense.shape, dtype=np.int32)
        for g in range(len(rg) - 1):
            rows = perm[rg[g]: rg[g + 1]]
            cols = bc[bp[g]: bp[g + 1]]
            assert np.all(np.diff(cols) > 0)
            for t, j in enumerate(cols):
                b = bp[g] + t
                assert bo[b + 1] - bo[b] == len(rows) * col_block
                blk = oracle.block_bits(csr, perm, rg, g, int(j), col_block)
                assert blk.any() or (dense[np.ix_(rows, range(j * col_block, (j + 1) * col_block))] == 0).all()
                sl = np.ix_(rows, np.arange(j * col_block, (j + 1) * col_block))
                mask = np.zeros(dense.shape, dtype=bool)
                mask[sl] = True
                struct = np.zeros(dense.shape, dtype=bool)
                r_idx = np.repeat(np.arange(csr["n_rows"]), np.diff(csr["row_ptr"]))
                struct[r_idx, csr["col_idx"]] = True
                assert (struct & mask).any()          # no stored block is structurally empty
                rebuilt[sl] = blk
                covered[sl] += 1
        r_idx = np.repeat(np.arange(csr["n_rows"]), np.diff(csr["row_ptr"]))
        assert np.all(covered[r_idx, csr["col_idx"]] == 1)
        assert covered.max() <= 1
        assert np.array_equal(rebuilt, dense)
