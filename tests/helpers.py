"""Helpers shared by the tests: tiny matrix builders and a set-based transcription of 1-SA.

``sa1_sets`` is a third, independent implementation of the greedy pass (Python sets, no
compression shortcut other than the one the method prescribes) used to pin both the C oracle
and the library on tiny inputs.
"""
from __future__ import annotations

import math

import numpy as np

from paper_2202_05868_amd import synth


def csr_from_rows(row_sets, n_cols, rng=None, dtype="f16"):
    """CSR from a list of iterables of column indices; values U[-1,1] (or 1.0 without rng)."""
    rows, cols = [], []
    for i, s in enumerate(row_sets):
        for c in sorted(set(s)):
            rows.append(i)
            cols.append(c)
    n = len(rows)
    vals = rng.uniform(-1, 1, size=n).astype(np.float32) if rng is not None else np.ones(n, np.float32)
    return synth.csr_from_coo(len(row_sets), n_cols, np.array(rows, dtype=np.int64),
                              np.array(cols, dtype=np.int64), synth.to_bits(vals, dtype), dtype)


def random_csr(rng, n_rows, n_cols, density, dtype="f16"):
    mask = rng.random((n_rows, n_cols)) < density
    r, c = np.nonzero(mask)
    v = rng.uniform(-1, 1, size=r.size).astype(np.float32)
    return synth.csr_from_coo(n_rows, n_cols, r, c, synth.to_bits(v, dtype), dtype)


def row_patterns(csr, col_block):
    """Quotient pattern of every row as a frozenset of column-block ids (Eq. 4)."""
    out = []
    for i in range(csr["n_rows"]):
        c = csr["col_idx"][csr["row_ptr"][i]: csr["row_ptr"][i + 1]]
        out.append(frozenset(int(x) // col_block for x in c))
    return out


def sa1_sets(csr, col_block, tau, similarity_only=False):
    """Literal set-based 1-SA: classes of identical quotient rows in first-occurrence order,
    one greedy pass per seed with the pattern updated to the union after each merge, merge
    condition = Jaccard >= tau and |union| <= floor(lambda0 / (1 - tau/2))."""
    pats = row_patterns(csr, col_block)
    classes = {}
    for i, p in enumerate(pats):          # dict keeps first-occurrence order
        classes.setdefault(p, []).append(i)
    keys = list(classes.keys())
    group = [-1] * len(keys)
    n_groups = 0
    for i, pi in enumerate(keys):
        if group[i] != -1:
            continue
        group[i] = n_groups
        pattern = set(pi)
        lam_max = math.floor(len(pi) / (1.0 - 0.5 * tau))
        for j in range(i + 1, len(keys)):
            if group[j] != -1:
                continue
            v = keys[j]
            inter = len(pattern & v)
            union = len(pattern | v)
            similar = True if union == 0 else (inter / union >= tau)
            if similar and (similarity_only or union <= lam_max):
                group[j] = n_groups
                pattern |= v
        n_groups += 1
    members = [[] for _ in range(n_groups)]
    for k, g in zip(keys, group):
        members[g].extend(classes[k])
    perm, row_groups = [], [0]
    for g in range(n_groups):
        perm.extend(sorted(members[g]))
        row_groups.append(len(perm))
    return np.array(perm, dtype=np.int32), np.array(row_groups, dtype=np.int32)


def groups_as_sets(perm, row_groups):
    return [frozenset(int(x) for x in perm[row_groups[g]: row_groups[g + 1]])
            for g in range(len(row_groups) - 1)]


def check_partition_shape(perm, row_groups, n_rows):
    """perm is a bijection; offsets strictly increase from 0 to n_rows; groups ordered by their
    smallest row; rows ascend inside a group."""
    assert perm.shape == (n_rows,)
    assert np.array_equal(np.sort(perm), np.arange(n_rows))
    assert row_groups[0] == 0 and row_groups[-1] == n_rows
    assert np.all(np.diff(row_groups) > 0) or n_rows == 0
    firsts = []
    for g in range(len(row_groups) - 1):
        seg = perm[row_groups[g]: row_groups[g + 1]]
        assert np.all(np.diff(seg) > 0)
        firsts.append(seg[0])
    assert np.all(np.diff(firsts) > 0)
