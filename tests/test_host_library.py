"""Host side of the C-ABI library against the oracle (CPU only, no GPU calls).

sa1_reorder / vbr_build / vbr_get_index / vbr_unpack_block are host code inside the same shared
library as the kernels; perm, row_groups and the VBR index arrays must match the oracle bit for
bit.  Also: the library loads and exports every symbol the header declares, and the error paths.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2202_05868_amd import binding, synth
from helpers import check_partition_shape, csr_from_rows, random_csr, sa1_sets

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TAUS = [0.0, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0]


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "vbr_spmm.h")).read()
    declared = set(re.findall(r"^(?:const char \*|int64_t |int |void )\s*(\w+)\s*\(", header, flags=re.M))
    assert declared == set(binding.EXPORTS), declared ^ set(binding.EXPORTS)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def assert_same_blocking(csr, col_block, tau):
    p0, g0 = oracle.sa1(csr, col_block, tau)
    p1, g1 = binding.sa1_reorder(csr, col_block, tau)
    assert np.array_equal(p0, p1), "perm differs"
    assert np.array_equal(g0, g1), "row_groups differ"
    return p1, g1


def assert_same_index(csr, perm, rg, col_block, check_values=True):
    bp0, bc0, bo0 = oracle.vbr_index(csr, perm, rg, col_block)
    v = binding.vbr_build(csr, perm, rg, col_block)
    v.audit()                       # every index the kernels use lies inside what it indexes
    ix = v.index()
    assert np.array_equal(ix["perm"], perm) and np.array_equal(ix["row_groups"], rg)
    assert np.array_equal(ix["blk_ptr"], bp0)
    assert np.array_equal(ix["blk_col"], bc0)
    assert np.array_equal(ix["blk_off"], bo0)
    assert ix["stored_elems"] == bo0[-1] and ix["n_blocks"] == len(bc0)
    if check_values:
        for g in range(len(rg) - 1):
            h = int(rg[g + 1] - rg[g])
            for b in range(int(bp0[g]), int(bp0[g + 1])):
                got = v.unpack_block(b, h, col_block)
                want = oracle.block_bits(csr, perm, rg, g, int(bc0[b]), col_block)
                assert np.array_equal(got, want), (g, b)
    return v


@pytest.mark.parametrize("col_block", [1, 2, 3, 8, 16])
def test_reorder_and_index_match_oracle_on_random_matrices(col_block):
    rng = np.random.default_rng(100 + col_block)
    for trial in range(12):
        n_rows = int(rng.integers(1, 90))
        kb = int(rng.integers(1, 20))
        csr = random_csr(rng, n_rows, kb * col_block, float(rng.choice([0.02, 0.1, 0.3, 0.7])),
                         dtype="bf16" if trial % 2 else "f16")
        for tau in TAUS:
            perm, rg = assert_same_blocking(csr, col_block, tau)
            check_partition_shape(perm, rg, n_rows)
        assert_same_index(csr, perm, rg, col_block)


def test_reorder_matches_set_based_transcription_too():
    rng = np.random.default_rng(9)
    for trial in range(40):
        csr = random_csr(rng, int(rng.integers(1, 12)), 12, 0.3)
        for tau in TAUS:
            p0, g0 = sa1_sets(csr, 2, tau)
            p1, g1 = binding.sa1_reorder(csr, 2, tau)
            assert np.array_equal(p0, p1) and np.array_equal(g0, g1)


def test_more_than_64_column_blocks_and_hash_collisions():
    # patterns {0,3} and {1,2} share the Eq. 5 hash (3) and the length: they must stay apart
    csr = csr_from_rows([[0, 3], [1, 2], [0, 3], [1, 2], [0, 1, 2]], n_cols=4)
    perm, rg = assert_same_blocking(csr, 1, 1.0)
    assert len(rg) - 1 == 3
    rng = np.random.default_rng(2)
    csr = random_csr(rng, 300, 200 * 2, 0.03)        # 200 column blocks: bitsets of 4 words
    for tau in (0.2, 0.5):
        perm, rg = assert_same_blocking(csr, 2, tau)
    assert_same_index(csr, perm, rg, 2)


@pytest.mark.parametrize("n_rows,n_blocks,density", [(3000, 600, 0.004), (3000, 600, 0.02), (2500, 40, 0.5),
                                                     (2000, 130, 0.08)])
def test_reorder_at_sizes_where_both_scan_strategies_run(n_rows, n_blocks, density):
    # sparse quotient rows over many column blocks: candidates come from the column blocks' row
    # lists; dense ones over few blocks: every remaining row is compared.  Rows are drawn from a
    # few hundred base patterns with noise so that merges, refusals and the size cap all occur.
    rng = np.random.default_rng(n_rows + n_blocks)
    base = rng.random((300, n_blocks)) < density
    rows = []
    for i in range(n_rows):
        pat = base[rng.integers(0, 300)] ^ (rng.random(n_blocks) < density * 0.15)
        rows.append((np.nonzero(pat)[0] * 2 + rng.integers(0, 2)).tolist())
    csr = csr_from_rows(rows, n_cols=2 * n_blocks, rng=rng)
    for tau in (0.0, 0.05, 0.3, 0.6, 0.9, 1.0):
        perm, rg = assert_same_blocking(csr, 2, tau)
        check_partition_shape(perm, rg, n_rows)


@pytest.mark.parametrize("threads", ["1", "3", "8"])
@pytest.mark.parametrize("n_rows,n_blocks,density", [(3000, 600, 0.004), (3000, 600, 0.02), (2500, 40, 0.5),
                                                     (2000, 130, 0.08)])
def test_reorder_with_several_host_threads_is_the_sequential_result(monkeypatch, threads, n_rows, n_blocks, density):
    # the candidate search that runs ahead of the greedy pass on several threads must not change
    # a single decision: same inputs as above (merges, refusals and the size cap all occur), the
    # thread count forced through the environment, compared with the oracle
    monkeypatch.setenv("VBR_SA1_THREADS", threads)
    rng = np.random.default_rng(n_rows + n_blocks)
    base = rng.random((300, n_blocks)) < density
    rows = []
    for i in range(n_rows):
        pat = base[rng.integers(0, 300)] ^ (rng.random(n_blocks) < density * 0.15)
        rows.append((np.nonzero(pat)[0] * 2 + rng.integers(0, 2)).tolist())
    csr = csr_from_rows(rows, n_cols=2 * n_blocks, rng=rng)
    for tau in (0.05, 0.3, 0.6, 0.9, 1.0):
        perm, rg = assert_same_blocking(csr, 2, tau)
        check_partition_shape(perm, rg, n_rows)


def test_reorder_threads_on_the_unstructured_workload_reduced(monkeypatch):
    # the workload the parallel search is for: Erdos-Renyi rows, next to no merges
    w = synth.workload("c5", scale=0.25)
    for threads in ("1", "4"):
        monkeypatch.setenv("VBR_SA1_THREADS", threads)
        for tau in (0.1, 0.3):
            assert_same_blocking(w["A"], w["col_block"], tau)


@pytest.mark.parametrize("name,scale,noise", [("c1", 1.0, True), ("c1", 1.0, False), ("c2", 0.25, True),
                                               ("c3", 0.125, True), ("c4", 0.125, True), ("c5", 0.0625, True)])
def test_workloads_small_scale_bit_exact(name, scale, noise):
    w = synth.workload(name, scale=scale, noise=noise)
    for tau in w["taus"]:
        perm, rg = assert_same_blocking(w["A"], w["col_block"], tau)
    v = assert_same_index(w["A"], perm, rg, w["col_block"], check_values=False)
    # values: sampled blocks
    ix = v.index()
    rng = np.random.default_rng(0)
    grp_of_blk = np.repeat(np.arange(ix["n_groups"]), np.diff(ix["blk_ptr"]))
    for b in rng.choice(ix["n_blocks"], size=min(40, ix["n_blocks"]), replace=False):
        g = int(grp_of_blk[b])
        h = int(rg[g + 1] - rg[g])
        assert np.array_equal(v.unpack_block(int(b), h, w["col_block"]),
                              oracle.block_bits(w["A"], perm, rg, g, int(ix["blk_col"][b]), w["col_block"]))


def test_build_accepts_any_valid_partition_and_tall_groups():
    rng = np.random.default_rng(4)
    csr = random_csr(rng, 300, 64, 0.1)
    perm = rng.permutation(300).astype(np.int32)
    rg = np.array([0, 1, 18, 150, 151, 300], dtype=np.int32)     # heights 1, 17, 132, 1, 149
    assert_same_index(csr, perm, rg, 16)
    assert_same_index(csr, np.arange(300, dtype=np.int32), np.array([0, 300], dtype=np.int32), 4)


def test_panels_unpack_exactly():
    # more than 4096 rows in groups shorter than a slab: they are packed as panels; 12 column
    # blocks at high density make nearly every slab present in every K-step (full masks); every
    # stored block must unpack bit-exactly
    rng = np.random.default_rng(77)
    csr = random_csr(rng, 6000, 12 * 8, 0.08)
    perm, rg = assert_same_blocking(csr, 8, 0.9)
    h = np.diff(rg)
    assert h[h < 16].sum() >= 4096
    v = assert_same_index(csr, perm, rg, 8, check_values=False)
    ix = v.index()
    grp_of_blk = np.repeat(np.arange(ix["n_groups"]), np.diff(ix["blk_ptr"]))
    for b in rng.choice(ix["n_blocks"], size=400, replace=False):
        g = int(grp_of_blk[b])
        assert np.array_equal(v.unpack_block(int(b), int(rg[g + 1] - rg[g]), 8),
                              oracle.block_bits(csr, perm, rg, g, int(ix["blk_col"][b]), 8))


def test_empty_rows_and_empty_matrix():
    csr = csr_from_rows([[], [1], [], [1, 5]], n_cols=8)
    perm, rg = assert_same_blocking(csr, 2, 0.5)
    assert_same_index(csr, perm, rg, 2)
    empty = csr_from_rows([[], [], []], n_cols=8)
    perm, rg = assert_same_blocking(empty, 4, 0.5)
    assert len(rg) == 2
    v = assert_same_index(empty, perm, rg, 4)
    assert v.index()["n_blocks"] == 0 and v.device_bytes() >= 256
    none = csr_from_rows([], n_cols=8)                    # no rows at all
    perm, rg = assert_same_blocking(none, 4, 0.5)
    assert perm.size == 0 and rg.tolist() == [0]
    v = binding.vbr_build(none, perm, rg, 4)
    assert v.index()["n_groups"] == 0 and v.device_bytes() >= 256


def test_graph_workload_reduced_bit_exact():
    w = synth.workload("rmat", scale=0.125)
    a = w["A"]
    assert a["n_rows"] == 2048 and 20 < a["nnz"] / a["n_rows"] < 33      # duplicate edges collapse
    for tau in (0.2, 0.4):
        perm, rg = assert_same_blocking(a, w["col_block"], tau)
    assert_same_index(a, perm, rg, w["col_block"], check_values=False)


def test_comparator_handle_checks_its_input():
    csr = csr_from_rows([[0, 1], [2]], n_cols=4)
    h = binding.CsrDev(csr)
    assert binding._lib.csr_device_bytes(h._h) % 256 == 0
    assert binding._lib.csr_spmm(h._h, 256, 8, 256, 8, 8, 0) == -4       # before upload: state error, no GPU touched
    bad = dict(csr)
    bad["col_idx"] = np.array([1, 0, 2], dtype=np.int32)
    with pytest.raises(binding.VbrError):
        binding.CsrDev(bad)


def test_error_paths():
    csr = csr_from_rows([[0, 1], [2]], n_cols=4)
    with pytest.raises(binding.VbrError):
        binding.sa1_reorder(csr, 3, 0.5)                 # 4 % 3 != 0
    with pytest.raises(binding.VbrError):
        binding.sa1_reorder(csr, 2, 1.5)                 # tau out of range
    with pytest.raises(binding.VbrError):
        binding.sa1_reorder(csr, 0, 0.5)
    bad = dict(csr)
    bad["col_idx"] = np.array([1, 0, 2], dtype=np.int32)  # unsorted inside a row
    with pytest.raises(binding.VbrError):
        binding.sa1_reorder(bad, 2, 0.5)
    bad["col_idx"] = np.array([0, 1, 7], dtype=np.int32)  # out of range
    with pytest.raises(binding.VbrError):
        binding.sa1_reorder(bad, 2, 0.5)
    with pytest.raises(binding.VbrError):
        binding.vbr_build(csr, np.array([0, 0], dtype=np.int32), np.array([0, 2], dtype=np.int32), 2)  # not a bijection
    with pytest.raises(binding.VbrError):
        binding.vbr_build(csr, np.array([0, 1], dtype=np.int32), np.array([0, 1, 1, 2], dtype=np.int32), 2)  # empty group
    v = binding.vbr_build(csr, np.array([1, 0], dtype=np.int32), np.array([0, 2], dtype=np.int32), 2)
    # spmm before upload: state error, no GPU touched
    assert binding.vbr_spmm_raw(v, 256, 8, 256, 8, 8, 0) == -4
    assert binding._lib.vbr_strerror(-4) == b"call out of order"


def test_binding_rejects_operands_the_kernels_would_read_or_write_out_of_bounds():
    # the C ABI gets raw addresses; shapes, types and the device are checked in the binding,
    # before anything is launched (CPU tensors suffice: every check precedes the launch)
    import torch
    csr = csr_from_rows([[0, 1], [2], [5]], n_cols=8)
    v = binding.vbr_build(csr, np.arange(3, dtype=np.int32), np.array([0, 3], dtype=np.int32), 2)
    h = binding.CsrDev(csr)
    fake_dev = torch.empty(1, dtype=torch.uint8)          # stands for the uploaded buffer (CPU "device")
    for what, obj in (("vbr_spmm", v), ("csr_spmm", h)):
        def check(b, c, dev=fake_dev):
            return binding._check_operands(what, "f16", obj.n_rows, obj.n_cols, dev, b, c)
        good_b = torch.zeros((8, 16), dtype=torch.float16)
        good_c = torch.zeros((3, 16), dtype=torch.float32)
        assert check(good_b, good_c) is good_c
        assert tuple(check(good_b, None).shape) == (3, 16)
        for b, c in [(torch.zeros((7, 16), dtype=torch.float16), good_c),            # B too short
                     (good_b.to(torch.bfloat16), good_c),                            # wrong type
                     (torch.zeros((16, 8), dtype=torch.float16).t(), good_c),        # column stride
                     (good_b, torch.zeros((2, 16), dtype=torch.float32)),            # C too short
                     (good_b, torch.zeros((4, 16), dtype=torch.float32)),            # C too tall
                     (good_b, torch.zeros((3, 8), dtype=torch.float32)),             # C too narrow
                     (good_b, torch.zeros((3, 16), dtype=torch.float64)),            # C type
                     (good_b, torch.zeros((3, 1), dtype=torch.float32).expand(3, 16)),   # C rows overlap
                     (good_b[:, :8].expand(8, 8)[:, :8].as_strided((8, 8), (0, 1)), torch.zeros((3, 8), dtype=torch.float32))]:
            with pytest.raises(ValueError):
                check(b, c)
        with pytest.raises(binding.VbrError):            # not uploaded
            check(good_b, good_c, dev=None)
        if torch.cuda.is_available():
            with pytest.raises(ValueError):              # uploaded elsewhere than where B and C live
                check(good_b, good_c, dev=torch.empty(1, dtype=torch.uint8, device="cuda:0"))
    # through the public methods: shape errors surface before the state error
    with pytest.raises(ValueError):
        v.spmm(torch.zeros((4, 16), dtype=torch.float16))
    with pytest.raises(binding.VbrError):
        v.spmm(torch.zeros((8, 16), dtype=torch.float16))
    with pytest.raises(ValueError):
        h.spmm(torch.zeros((8, 16), dtype=torch.float16), torch.zeros((9, 16), dtype=torch.float32))


def test_launch_plan_lists_what_a_call_issues():
    # one-slab groups only: one launch of the one-slab tile kernel, 8 tiles x ceil(N / 256) column tiles
    rng = np.random.default_rng(3)
    csr = random_csr(rng, 128, 64, 0.2)
    v = binding.vbr_build(csr, np.arange(128, dtype=np.int32), np.arange(0, 129, 16, dtype=np.int32), 16)
    plan = v.launches(4096)
    assert [p["kernel"] for p in plan] == ["vbr_spmm_kernel<1 slab>"] and plan[0]["tiles"] == 8
    assert plan[0]["workgroups"] == 8 * 16
    assert v.launches(0) == []
    # groups of 16 and of 100 rows: two classes, few tiles -> one mixed launch, which also takes the
    # column-gathered slab the 12 rows left over (a low group) form
    v = binding.vbr_build(csr, np.arange(128, dtype=np.int32), np.array([0, 16, 116, 128], dtype=np.int32), 16)
    plan = v.launches(256)
    assert [p["kernel"] for p in plan] == ["vbr_spmm_mixed_kernel"] and plan[0]["tiles"] == 3
    # thousands of single-row groups over 4 column blocks, every row touching most of them: one
    # panel per 128 rows shares the few B rows there are; the same number of rows with one entry
    # each over many columns: column-gathered slabs, 16 rows each
    big = random_csr(rng, 6000, 64, 0.2)
    v = binding.vbr_build(big, np.arange(6000, dtype=np.int32), np.arange(0, 6001, dtype=np.int32), 16)
    plan = v.launches(256)
    assert [p["kernel"] for p in plan] == ["vbr_spmm_panel_kernel"] and plan[0]["tiles"] == (6000 + 127) // 128
    wide = csr_from_rows([[int(c)] for c in rng.integers(0, 16384, size=6000)], n_cols=16384)
    v = binding.vbr_build(wide, np.arange(6000, dtype=np.int32), np.arange(0, 6001, dtype=np.int32), 16)
    plan = v.launches(256)
    assert [p["kernel"] for p in plan] == ["vbr_spmm_kernel<1 slab, column-gathered>"] and plan[0]["tiles"] == 6000 // 16
    v.audit()
