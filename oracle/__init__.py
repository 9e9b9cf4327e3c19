"""CPU oracle for the 1-SA / VBR / blocked-SpMM path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front for ``vbr_oracle.c`` (compiled with gcc on first use) plus two numpy helpers.
Nothing in the product package imports this; only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg do.  It shares no code with the HIP library.

Pins (see tests/test_oracle_*.py): brute-force dense products, identity right-hand sides, a
set-based transcription of the greedy pass on tiny matrices, the pathological example and the
density bound of section 3.2 of the paper, tau = 1 against a plain unique-rows grouping,
planted-structure recovery; the blocking curve against planted height and fill and a numpy
grouping at tau = 1 (tests/test_blocking_curve.py).  No function here is left unpinned.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vbr_oracle.c")
_LIB = os.path.join(_HERE, "libvbr_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, no fused multiply-add, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-shared",
                               "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, dbl, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_void_p
        lib.oracle_sa1.argtypes = [i64, i64, vp, vp, i32, dbl, i32, vp, vp, vp]
        lib.oracle_sa1.restype = ctypes.c_int
        lib.oracle_vbr_index.argtypes = [i64, i64, vp, vp, i32, vp, vp, i32, vp, vp, vp, vp]
        lib.oracle_vbr_index.restype = ctypes.c_int
        lib.oracle_spmm.argtypes = [i64, vp, vp, vp, vp, i64, vp, i64, vp, vp]
        lib.oracle_spmm.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def bits_to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact value of fp16 / bf16 bit patterns as binary64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def sa1(csr: dict, col_block: int, tau: float, similarity_only: bool = False):
    """1-SA row reordering (Algorithm 2 with the merge condition of section 3.2).

    Returns (perm int32[n_rows], row_groups int32[G+1])."""
    lib = _load()
    m = csr["n_rows"]
    perm = np.empty(m, dtype=np.int32)
    rg = np.empty(m + 1, dtype=np.int32)
    ng = ctypes.c_int32(0)
    rc = lib.oracle_sa1(m, csr["n_cols"], _p(csr["row_ptr"]), _p(csr["col_idx"]), int(col_block),
                        float(tau), int(bool(similarity_only)), _p(perm), _p(rg), ctypes.byref(ng))
    if rc != 0:
        raise ValueError("oracle_sa1 failed: %d" % rc)
    return perm, rg[: ng.value + 1].copy()


def vbr_index(csr: dict, perm: np.ndarray, row_groups: np.ndarray, col_block: int):
    """VBR index arrays of a row partition: (blk_ptr int64[G+1], blk_col int32[NB], blk_off int64[NB+1])."""
    lib = _load()
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    row_groups = np.ascontiguousarray(row_groups, dtype=np.int32)
    g = row_groups.size - 1
    kb = csr["n_cols"] // col_block
    cap = int(min(csr["nnz"], g * kb)) + 1
    blk_ptr = np.empty(g + 1, dtype=np.int64)
    blk_col = np.empty(cap, dtype=np.int32)
    blk_off = np.empty(cap + 1, dtype=np.int64)
    nb = ctypes.c_int64(0)
    rc = lib.oracle_vbr_index(csr["n_rows"], csr["n_cols"], _p(csr["row_ptr"]), _p(csr["col_idx"]),
                              int(col_block), _p(perm), _p(row_groups), g, _p(blk_ptr), _p(blk_col),
                              _p(blk_off), ctypes.byref(nb))
    if rc != 0:
        raise ValueError("oracle_vbr_index failed: %d" % rc)
    return blk_ptr, blk_col[: nb.value].copy(), blk_off[: nb.value + 1].copy()


def block_bits(csr: dict, perm: np.ndarray, row_groups: np.ndarray, g: int, j: int, col_block: int):
    """Zero-filled dense window of block (group g, column block j): uint16 bits, h_g x col_block."""
    rows = perm[row_groups[g]: row_groups[g + 1]]
    out = np.zeros((rows.size, col_block), dtype=np.uint16)
    for t, r in enumerate(rows):
        lo, hi = csr["row_ptr"][r], csr["row_ptr"][r + 1]
        c = csr["col_idx"][lo:hi]
        sel = (c >= j * col_block) & (c < (j + 1) * col_block)
        out[t, c[sel] - j * col_block] = csr["vals"][lo:hi][sel]
    return out


def spmm(csr: dict, b_bits: np.ndarray, rows=None, with_bound: bool = True):
    """C = A.B (and S = |A|.|B|) in binary64 from the CSR matrix; optionally only some rows."""
    lib = _load()
    vals = bits_to_f64(csr["vals"], csr["dtype"])
    b = np.ascontiguousarray(bits_to_f64(b_bits, csr["dtype"]))
    k, n = b.shape
    assert k == csr["n_cols"]
    if rows is None:
        n_sel, rows_a = csr["n_rows"], None
    else:
        rows_a = np.ascontiguousarray(rows, dtype=np.int64)
        n_sel = rows_a.size
    c = np.empty((n_sel, n), dtype=np.float64)
    s = np.empty((n_sel, n), dtype=np.float64) if with_bound else None
    rc = lib.oracle_spmm(csr["n_rows"], _p(csr["row_ptr"]), _p(csr["col_idx"]), _p(vals), _p(b), n,
                         _p(rows_a), n_sel, _p(c), _p(s))
    if rc != 0:
        raise ValueError("oracle_spmm failed: %d" % rc)
    return c, s


def blocking_curve(csr: dict, col_block: int, taus, target_height: int) -> dict:
    """Blocking curve of sections 2.2 and 4.3.1: for every threshold the blocking of ``sa1`` and, from its
    VBR index, the number of nonzero blocks, the nonzero area, the in-block density
    rho' = nnz / area and the average height Delta'_H of the nonzero blocks; ``selected`` is the
    threshold whose Delta'_H is nearest to ``target_height`` (sections 4.3.2 and 4.4.2 take the blocking with
    Delta'_H ~ Delta; ties go to the first threshold given, empty blockings are skipped)."""
    from fractions import Fraction
    rows = []
    best, best_d = 0, None
    for i, tau in enumerate(taus):
        perm, rg = sa1(csr, col_block, float(tau))
        blk_ptr, blk_col, blk_off = vbr_index(csr, perm, rg, col_block)
        heights = np.repeat(np.diff(rg).astype(np.int64), np.diff(blk_ptr))     # height of every stored block
        nb = int(blk_col.size)
        area = int(blk_off[-1])
        rows.append(dict(tau=float(tau), n_groups=int(rg.size - 1), n_blocks=nb, stored_elems=area,
                         sum_heights=int(heights.sum()),
                         rho=(csr["nnz"] / area) if area else 0.0,
                         avg_height=(float(heights.mean()) if nb else 0.0)))
        if nb:
            d = abs(Fraction(int(heights.sum()), nb) - target_height)
            if best_d is None or d < best_d:
                best, best_d = i, d
    return dict(points=rows, selected=best)
