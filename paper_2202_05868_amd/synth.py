"""Seeded synthetic inputs: planted-block sparse matrices in CSR and dense right-hand sides.

This module only *draws inputs*.  It holds none of the method's arithmetic (no quotient
patterns, no similarity, no blocking, no multiply): the CPU oracle and the HIP library are
both fed from here and share nothing else.

The matrices follow the synthetic generator of the paper (section 4.1, "Dataset description
and generation": a grid of blocks, a fraction theta of them flagged nonzero, a fraction rho
of the entries inside a flagged block kept, then the rows scrambled, section 4.3.1) with the
sizes and noise of the five benchmark workloads this build is measured on.

All values are rounded to the 16-bit storage type *here*, so every consumer sees the same
bit patterns.  A matrix is a dict:

    n_rows, n_cols, nnz : int
    row_ptr  : int64  [n_rows+1]
    col_idx  : int32  [nnz]      strictly increasing inside a row
    vals     : uint16 [nnz]      fp16 or bf16 bit patterns (see ``dtype``)
    dtype    : "f16" | "bf16"
"""
from __future__ import annotations

import numpy as np

F16 = "f16"
BF16 = "bf16"


# ----------------------------------------------------------------------------- storage types
def to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float values to the 16-bit storage type (nearest-even) and return the bit patterns."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == F16:
        return x.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        u = x.view(np.uint32).astype(np.uint64)
        # round to nearest, ties to even, on the upper 16 bits of the binary32 pattern
        u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
        return u.astype(np.uint16)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- CSR assembly
def csr_from_coo(n_rows: int, n_cols: int, rows: np.ndarray, cols: np.ndarray,
                 vals_bits: np.ndarray, dtype: str) -> dict:
    """Canonical CSR from coordinate triples; of duplicate coordinates the first one is kept."""
    rows = np.asarray(rows, dtype=np.int64)
    cols = np.asarray(cols, dtype=np.int64)
    lin = rows * n_cols + cols
    lin_u, first = np.unique(lin, return_index=True)
    rows_u = lin_u // n_cols
    cols_u = (lin_u - rows_u * n_cols).astype(np.int32)
    row_ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows_u, minlength=n_rows), out=row_ptr[1:])
    return dict(n_rows=int(n_rows), n_cols=int(n_cols), nnz=int(lin_u.size), row_ptr=row_ptr,
                col_idx=np.ascontiguousarray(cols_u),
                vals=np.ascontiguousarray(np.asarray(vals_bits, dtype=np.uint16)[first]), dtype=dtype)


def permute_rows(csr: dict, order: np.ndarray) -> dict:
    """New matrix whose row i is row order[i] of ``csr``."""
    order = np.asarray(order, dtype=np.int64)
    lens = np.diff(csr["row_ptr"])[order]
    row_ptr = np.zeros(csr["n_rows"] + 1, dtype=np.int64)
    np.cumsum(lens, out=row_ptr[1:])
    starts = csr["row_ptr"][:-1][order]
    idx = np.repeat(starts - row_ptr[:-1], lens) + np.arange(row_ptr[-1], dtype=np.int64)
    out = dict(csr)
    out.update(row_ptr=row_ptr, col_idx=np.ascontiguousarray(csr["col_idx"][idx]),
               vals=np.ascontiguousarray(csr["vals"][idx]))
    return out


def dense_bits(csr: dict) -> np.ndarray:
    """Zero-filled dense copy of the matrix (uint16 bit patterns).  For small cases only."""
    a = np.zeros((csr["n_rows"], csr["n_cols"]), dtype=np.uint16)
    r = np.repeat(np.arange(csr["n_rows"]), np.diff(csr["row_ptr"]))
    a[r, csr["col_idx"]] = csr["vals"]
    return a


# ----------------------------------------------------------------------------- value draws
def _uniform(rng, n):
    return rng.uniform(-1.0, 1.0, size=n).astype(np.float32)


def _normal(rng, n):
    return rng.standard_normal(size=n).astype(np.float32)


def dense_rhs(rng, k: int, n: int, dtype: str, dist: str = "uniform") -> np.ndarray:
    """Dense K x N right-hand side B as bit patterns, row-major."""
    x = _uniform(rng, k * n) if dist == "uniform" else _normal(rng, k * n)
    return to_bits(x, dtype).reshape(k, n)


# ----------------------------------------------------------------------------- planted blocks
def planted(rng, heights, n_cols: int, col_block: int, *, blocks_per_group=None,
            block_prob=None, fill: float = 1.0, dtype: str = F16, value: str = "uniform",
            shuffle: bool = True, noise_frac: float = 0.0, noise_where: str = "anywhere"):
    """Planted-block matrix.

    heights           row-group heights (sum = n_rows)
    blocks_per_group  each group flags this many distinct column blocks, uniformly; or
    block_prob        each (group, column block) cell is flagged independently with this probability
    fill              probability that an entry inside a flagged block is kept
    value             "uniform": U[-1,1];  "lognormal_block": s*Z/16 per block, Z~N(0,1), s~LogNormal(0,1)
    shuffle           scramble the rows with a random permutation afterwards
    noise_frac        extra nonzeros, as a fraction of the planted nnz
    noise_where       "anywhere" | "off_block" (only outside flagged blocks)

    Returns (csr, info) with info = dict(label[n_rows] planted group of each final row,
    block_sets = list of sorted arrays of flagged column blocks per group, heights).
    """
    heights = np.asarray(heights, dtype=np.int64)
    n_rows = int(heights.sum())
    kb = n_cols // col_block
    assert kb * col_block == n_cols
    g_start = np.concatenate([[0], np.cumsum(heights)])
    block_sets = []
    rr, cc, vv = [], [], []
    flagged = np.zeros((len(heights), kb), dtype=bool)
    for g, h in enumerate(heights):
        if blocks_per_group is not None:
            bs = np.sort(rng.choice(kb, size=int(blocks_per_group), replace=False))
        else:
            bs = np.nonzero(rng.random(kb) < block_prob)[0]
        block_sets.append(bs.astype(np.int64))
        flagged[g, bs] = True
        if bs.size == 0:
            continue
        h = int(h)
        cell = h * col_block
        if fill >= 1.0:
            keep = np.ones((bs.size, cell), dtype=bool)
        else:
            keep = rng.random((bs.size, cell)) < fill
        if value == "uniform":
            x = _uniform(rng, bs.size * cell).reshape(bs.size, cell)
        elif value == "lognormal_block":
            s = rng.lognormal(0.0, 1.0, size=bs.size).astype(np.float32)
            x = (_normal(rng, bs.size * cell).reshape(bs.size, cell) * s[:, None]) / np.float32(16.0)
        else:
            raise ValueError(value)
        b_i, e_i = np.nonzero(keep)
        rr.append(g_start[g] + e_i // col_block)
        cc.append(bs[b_i] * col_block + e_i % col_block)
        vv.append(x[b_i, e_i])
    rows = np.concatenate(rr) if rr else np.zeros(0, np.int64)
    cols = np.concatenate(cc) if cc else np.zeros(0, np.int64)
    vals = np.concatenate(vv) if vv else np.zeros(0, np.float32)
    planted_nnz = rows.size
    label = np.repeat(np.arange(len(heights)), heights)
    n_noise = int(round(noise_frac * planted_nnz))
    if n_noise > 0:
        got_r, got_c = [], []
        need = n_noise
        while need > 0:
            r = rng.integers(0, n_rows, size=2 * need + 16)
            c = rng.integers(0, n_cols, size=2 * need + 16)
            if noise_where == "off_block":
                ok = ~flagged[label[r], c // col_block]
                r, c = r[ok], c[ok]
            got_r.append(r[:need])
            got_c.append(c[:need])
            need -= got_r[-1].size
        nr = np.concatenate(got_r)
        nc = np.concatenate(got_c)
        rows = np.concatenate([rows, nr])
        cols = np.concatenate([cols, nc])
        vals = np.concatenate([vals, _uniform(rng, nr.size)])
    csr = csr_from_coo(n_rows, n_cols, rows, cols, to_bits(vals, dtype), dtype)
    if shuffle:
        order = rng.permutation(n_rows)
        csr = permute_rows(csr, order)
        label = label[order]
    info = dict(label=label.astype(np.int64), block_sets=block_sets, heights=heights,
                planted_nnz=int(planted_nnz))
    return csr, info


def erdos_renyi(rng, n_rows: int, n_cols: int, density: float, dtype: str = F16) -> dict:
    """Every cell nonzero independently with probability ``density``; values U[-1,1]."""
    total = n_rows * n_cols
    n = int(rng.binomial(total, density))
    # positions drawn with replacement; the few duplicates (about n^2 / (2 total)) collapse
    lin = np.unique(rng.integers(0, total, size=n, dtype=np.int64))
    rows = lin // n_cols
    cols = lin - rows * n_cols
    return csr_from_coo(n_rows, n_cols, rows, cols, to_bits(_uniform(rng, lin.size), dtype), dtype)


def rmat(rng, log2_n: int, avg_degree: float, probs=(0.57, 0.19, 0.19, 0.05), dtype: str = F16,
         scramble: bool = True) -> dict:
    """Recursive-matrix graph (section 4.1: generating parameters (0.57, 0.19, 0.19, 0.05)): every
    edge picks one quadrant per bit of the node index with the given probabilities; duplicate
    edges collapse.  2^log2_n nodes, about avg_degree entries per row; values U[-1,1]; rows
    scrambled with a random permutation afterwards (as the paper does before blocking)."""
    n = 1 << log2_n
    n_edges = int(round(n * avg_degree))
    rows = np.zeros(n_edges, dtype=np.int64)
    cols = np.zeros(n_edges, dtype=np.int64)
    cum = np.cumsum(probs)
    for _ in range(log2_n):
        quad = np.searchsorted(cum, rng.random(n_edges), side="right").clip(0, 3)
        rows = (rows << 1) | (quad >> 1)
        cols = (cols << 1) | (quad & 1)
    lin = np.unique(rows * n + cols)
    rows = lin // n
    cols = lin - rows * n
    a = csr_from_coo(n, n, rows, cols, to_bits(_uniform(rng, lin.size), dtype), dtype)
    return permute_rows(a, rng.permutation(n)) if scramble else a


def landscape(rng, n: int, delta: int, theta: float, rho: float, dtype: str = F16, scramble: bool = True) -> dict:
    """Synthetic blocked matrix A(Delta, theta, rho) of section 4.1: the n x n matrix is divided into
    Delta x Delta blocks, a fraction theta of ALL blocks (drawn over the whole grid, so block rows
    differ in how many they hold) is flagged nonzero, and inside every flagged block a fraction rho of
    the entries is kept (at least one); values U[-1,1].  The rows are scrambled afterwards (section 4.3.1)."""
    g = n // delta
    assert g * delta == n
    n_flag = max(1, int(round(theta * g * g)))
    flagged = rng.choice(g * g, size=n_flag, replace=False)
    per = max(1, int(round(rho * delta * delta)))
    rr, cc = [], []
    cell = delta * delta
    for start in range(0, n_flag, 4096):                      # in slices, to bound the scratch memory
        blk = flagged[start:start + 4096]
        # per block `per` distinct cells: the smallest `per` of a random key per cell
        if per * 4 >= cell:
            keys = rng.random((blk.size, cell))
            pick = np.argpartition(keys, per - 1, axis=1)[:, :per]
        else:
            pick = np.stack([rng.choice(cell, size=per, replace=False) for _ in range(blk.size)])
        bi = np.repeat(blk // g, per)
        bj = np.repeat(blk % g, per)
        e = pick.reshape(-1)
        rr.append(bi * delta + e // delta)
        cc.append(bj * delta + e % delta)
    rows = np.concatenate(rr)
    cols = np.concatenate(cc)
    a = csr_from_coo(n, n, rows, cols, to_bits(_uniform(rng, rows.size), dtype), dtype)
    return permute_rows(a, rng.permutation(n)) if scramble else a


# ----------------------------------------------------------------------------- the five workloads
WORKLOADS = ("c1", "c2", "c3", "c4", "c5", "rmat")


def workload(name: str, *, scale: float = 1.0, noise: bool = True, seed: int | None = None,
             rmat_degree: float = 32.0, rmat_col_block: int = 64) -> dict:
    """One of the five benchmark workloads (``c1`` .. ``c5``) or the graph workload ``rmat``,
    optionally shrunk.

    ``scale`` multiplies the matrix dimensions and the dense width N (block sizes, densities and
    value distributions stay), so the small cases keep the structure of the full ones.
    ``noise=False`` drops the extra random nonzeros of c1/c2 (the noise-free variant).
    ``rmat_degree`` / ``rmat_col_block``: edges drawn per node and column-block width of ``rmat``
    (the paper's grid: 8 .. 128 and 64, 128, 256; section 4.1 and section 4.4.3).

    Returns dict(name, A=csr, B=bits[K,N], N, col_block, taus, dtype, info).
    """
    idx = WORKLOADS.index(name)
    rng = np.random.default_rng(1001 + idx if seed is None else seed)

    def sc(x, q):  # scaled size, kept a multiple of q
        return max(q, int(round(x * scale / q)) * q)

    if name == "c1":
        cb, h = 32, 32
        m = sc(1024, h)
        k = sc(1024, cb)
        n = sc(256, 16)
        kb = k // cb
        a, info = planted(rng, [h] * (m // h), k, cb, blocks_per_group=max(1, round(0.10 * kb)),
                          noise_frac=0.005 if noise else 0.0, noise_where="anywhere")
        b = dense_rhs(rng, k, n, F16)
        return dict(name=name, A=a, B=b, N=n, col_block=cb, taus=(0.7,), dtype=F16, info=info)
    if name == "c2":
        cb, h = 64, 64
        m = sc(8192, h)
        k = sc(8192, cb)
        n = sc(1024, 16)
        kb = k // cb
        a, info = planted(rng, [h] * (m // h), k, cb, blocks_per_group=max(1, round(0.05 * kb)),
                          noise_frac=0.01 if noise else 0.0, noise_where="off_block")
        b = dense_rhs(rng, k, n, F16)
        return dict(name=name, A=a, B=b, N=n, col_block=cb, taus=(0.6,), dtype=F16, info=info)
    if name == "c3":
        cb = 32
        m = sc(16384, 16)
        k = sc(16384, cb)
        n = sc(512, 16)
        kb = k // cb
        heights = []
        left = m
        while left > 0:
            hh = int(rng.choice([16, 32, 64, 128]))
            hh = min(hh, left)
            heights.append(hh)
            left -= hh
        a, info = planted(rng, heights, k, cb, blocks_per_group=max(1, round(0.02 * kb)), fill=0.7,
                          dtype=BF16)
        b = dense_rhs(rng, k, n, BF16, dist="normal")
        return dict(name=name, A=a, B=b, N=n, col_block=cb, taus=(0.4, 0.6, 0.8), dtype=BF16, info=info)
    if name == "c4":
        cb, h = 16, 16
        m = sc(4096, h)
        k = sc(16384, cb)
        n = sc(4096, 16)
        a, info = planted(rng, [h] * (m // h), k, cb, block_prob=0.10, value="lognormal_block",
                          shuffle=False)
        b = dense_rhs(rng, k, n, F16, dist="normal")
        return dict(name=name, A=a, B=b, N=n, col_block=cb, taus=(0.5,), dtype=F16, info=info)
    if name == "c5":
        cb = 32
        m = sc(32768, 16)
        k = sc(32768, cb)
        n = sc(256, 16)
        a = erdos_renyi(rng, m, k, 5e-4)
        b = dense_rhs(rng, k, n, F16)
        return dict(name=name, A=a, B=b, N=n, col_block=cb, taus=(0.3,), dtype=F16, info=None)
    if name == "rmat":
        # the graph workload of sections 4.1 and 4.4.3: 2^14 nodes, 32 edges per node on average, column
        # partition of 64, dense width 2^12
        cb = int(rmat_col_block)
        lg = max(8, 14 + int(round(np.log2(scale))))
        n = sc(4096, 16)
        a = rmat(rng, lg, float(rmat_degree))
        b = dense_rhs(rng, a["n_cols"], n, F16)
        return dict(name=name, A=a, B=b, N=n, col_block=cb, taus=(0.4,), dtype=F16, info=None)
    raise ValueError(name)
