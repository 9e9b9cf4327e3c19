"""GPU parity: the HIP path through the C ABI against the CPU oracle on the same seeded inputs.

Bar: perm, row_groups and the VBR index arrays bit-exact; |C - C_ref| <= 1e-4 * sum_k |a_ik||b_kj|
elementwise (C_ref and the bound in binary64 from the original CSR).  Every case, the full-size
workloads included, is compared element by element.
"""
import numpy as np
import pytest

import oracle
from paper_2202_05868_amd import binding, synth, torch_io
from helpers import csr_from_rows, random_csr

pytestmark = pytest.mark.gpu
TOL = 1e-4


def gpu_spmm(csr, perm, rg, col_block, b_bits, ldb_pad=0, ldc_pad=0):
    import torch
    v = binding.vbr_build(csr, perm, rg, col_block)
    v.audit()                       # bounds of everything the kernels index, before anything is launched
    v.upload("cuda:0")
    k, n = b_bits.shape
    if ldb_pad:
        full = np.zeros((k, n + ldb_pad), dtype=np.uint16)
        full[:, :n] = b_bits
        b = torch_io.bits_to_device(full, csr["dtype"])[:, :n]
    else:
        b = torch_io.bits_to_device(b_bits, csr["dtype"])
    c_full = torch.full((csr["n_rows"], n + ldc_pad), float("nan"), dtype=torch.float32, device="cuda:0")
    c = c_full[:, :n]
    v.spmm(b, c)
    torch.cuda.synchronize()
    out = c_full.cpu().numpy()
    if ldc_pad:
        assert np.isnan(out[:, n:]).all(), "wrote outside the N columns"
    return out[:, :n].astype(np.float64), v


def check_c(c, c_ref, s, what=""):
    assert not np.isnan(c).any(), what + ": NaN left in C (rows not written)"
    err = np.abs(c - c_ref)
    bad = err > TOL * s
    assert not bad.any(), "%s: %d elements outside the bound, worst err/bound %.3g" % (
        what, int(bad.sum()), float(np.max(err / np.maximum(s, 1e-300))))


def blocking_bit_exact(csr, col_block, tau):
    p0, g0 = oracle.sa1(csr, col_block, tau)
    perm, rg = binding.sa1_reorder(csr, col_block, tau)
    assert np.array_equal(perm, p0) and np.array_equal(rg, g0)
    return perm, rg


def index_bit_exact(v, csr, perm, rg, col_block):
    bp, bc, bo = oracle.vbr_index(csr, perm, rg, col_block)
    ix = v.index()
    assert np.array_equal(ix["blk_ptr"], bp) and np.array_equal(ix["blk_col"], bc) and np.array_equal(ix["blk_off"], bo)


# --------------------------------------------------------------------------- small, element by element
@pytest.mark.parametrize("col_block", [1, 3, 8, 16, 32, 64])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_random_matrices_all_column_block_widths(col_block, dtype):
    rng = np.random.default_rng(col_block * 7 + (dtype == "bf16"))
    for m, kb, n, dens, tau in [(70, 9, 64, 0.2, 0.4), (300, 5, 264, 0.05, 0.2), (33, 12, 8, 0.6, 0.7)]:
        csr = random_csr(rng, m, kb * col_block, dens, dtype=dtype)
        b = synth.dense_rhs(rng, kb * col_block, n, dtype)
        perm, rg = blocking_bit_exact(csr, col_block, tau)
        c, v = gpu_spmm(csr, perm, rg, col_block, b)
        index_bit_exact(v, csr, perm, rg, col_block)
        c_ref, s = oracle.spmm(csr, b)
        check_c(c, c_ref, s, "cb=%d %s m=%d n=%d" % (col_block, dtype, m, n))


def test_result_does_not_depend_on_the_row_partition_used():
    rng = np.random.default_rng(5)
    csr = random_csr(rng, 500, 256, 0.04)
    b = synth.dense_rhs(rng, 256, 520, "f16")           # 520: two full column tiles + ragged tail
    c_ref, s = oracle.spmm(csr, b)
    ident = (np.arange(500, dtype=np.int32), np.arange(501, dtype=np.int32))          # every row its own group
    one = (np.arange(500, dtype=np.int32), np.array([0, 500], dtype=np.int32))        # one group of 500 rows
    rnd = (rng.permutation(500).astype(np.int32), np.array([0, 1, 18, 150, 151, 300, 500], dtype=np.int32))
    sa = blocking_bit_exact(csr, 16, 0.3)
    for name, (perm, rg) in [("identity", ident), ("one group", one), ("random", rnd), ("1-SA", sa)]:
        c, v = gpu_spmm(csr, perm, rg, 16, b)
        index_bit_exact(v, csr, perm, rg, 16)
        check_c(c, c_ref, s, name)


def test_short_groups_in_panels():
    # more than 4096 rows in groups shorter than a slab: the panel kernel; few column blocks at
    # high density make nearly every slab present in every K-step (full masks)
    rng = np.random.default_rng(12)
    csr = random_csr(rng, 6000, 12 * 8, 0.08)
    b = synth.dense_rhs(rng, 96, 136, "f16")            # one full 128-column tile + a ragged one
    perm, rg = blocking_bit_exact(csr, 8, 0.9)
    h = np.diff(rg)
    assert h[h < 16].sum() >= 4096                       # enough short rows for panels to be used
    c, v = gpu_spmm(csr, perm, rg, 8, b)
    index_bit_exact(v, csr, perm, rg, 8)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "panels")
    # tall and short groups in one matrix: tiles and panels side by side
    csr = random_csr(rng, 5000, 256, 0.02, dtype="bf16")
    b = synth.dense_rhs(rng, 256, 264, "bf16")
    perm = rng.permutation(5000).astype(np.int32)
    # heights 3, 16, 181, 16, 1, 283, then 4500 rows in groups of 9 (short: they form the panels)
    rg = np.concatenate([[0, 3, 19, 200, 216, 217, 500], np.arange(509, 5001, 9)]).astype(np.int32)
    assert rg[-1] == 5000
    c, v = gpu_spmm(csr, perm, rg, 32, b)
    index_bit_exact(v, csr, perm, rg, 32)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "tiles and panels mixed")


def test_low_rows_packed_both_ways_in_one_matrix():
    # 3072 single-row groups that all touch the same 6 column blocks (one shared panel per 128 rows
    # needs fewest loads), then 3072 rows with two entries each anywhere in 16384 columns (slabs that
    # gather their own columns do), then one tall group: three kernels in one call; the low groups
    # are handed over in scrambled order, so the packing's own ordering of them is at work too
    rng = np.random.default_rng(91)
    n_cols, cb = 16384, 16
    dense_cols = np.concatenate([np.arange(b * cb, (b + 1) * cb) for b in (3, 70, 200, 511, 800, 1023)])
    rows = [sorted(rng.choice(dense_cols, size=40, replace=False).tolist()) for _ in range(3072)]
    rows += [sorted(set(rng.integers(0, n_cols, size=2).tolist())) for _ in range(3072)]
    rows += [sorted(rng.choice(n_cols, size=30, replace=False).tolist()) for _ in range(40)]
    csr = csr_from_rows(rows, n_cols=n_cols, rng=rng)
    m = len(rows)
    low = rng.permutation(6144).astype(np.int32)
    perm = np.concatenate([low, np.arange(6144, m, dtype=np.int32)])
    rg = np.concatenate([np.arange(0, 6145), [m]]).astype(np.int32)
    b = synth.dense_rhs(rng, n_cols, 264, "f16")
    c, v = gpu_spmm(csr, perm, rg, cb, b, ldb_pad=8, ldc_pad=4)
    plan = v.launches(264)
    # some twenty panels, then one launch with the ~200 gathered slabs and the tile of the tall group
    assert plan[0]["kernel"] == "vbr_spmm_panel_kernel" and plan[0]["tiles"] >= 16
    assert len(plan) == 2 and plan[1]["kernel"] == "vbr_spmm_mixed_kernel" and plan[1]["tiles"] >= 150
    index_bit_exact(v, csr, perm, rg, cb)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "panels and gathered slabs")
    ix = v.index()
    for blk in rng.choice(ix["n_blocks"], size=300, replace=False):
        g = int(np.searchsorted(ix["blk_ptr"], blk, side="right") - 1)
        assert np.array_equal(v.unpack_block(int(blk), int(rg[g + 1] - rg[g]), cb),
                              oracle.block_bits(csr, perm, rg, g, int(ix["blk_col"][blk]), cb))


@pytest.mark.parametrize("col_block,n_blocks,density,dtype,n", [(16, 12, 0.03, "f16", 136), (32, 40, 0.01, "bf16", 264),
                                                              (16, 200, 0.004, "f16", 128)])
def test_short_groups_wider_blocks_and_padded_leading_dimensions(col_block, n_blocks, density, dtype, n):
    # thousands of short groups with blocks of 16 and 32 columns (granules of 16 and 32 B rows), few
    # and many column blocks, B and C with padded leading dimensions
    rng = np.random.default_rng(col_block + n_blocks)
    csr = random_csr(rng, 6000, n_blocks * col_block, density, dtype=dtype)
    b = synth.dense_rhs(rng, n_blocks * col_block, n, dtype)
    perm, rg = blocking_bit_exact(csr, col_block, 0.9)
    c, v = gpu_spmm(csr, perm, rg, col_block, b, ldb_pad=8, ldc_pad=4)
    index_bit_exact(v, csr, perm, rg, col_block)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "short groups cb=%d" % col_block)


def test_block_rows_of_exactly_one_slab():
    # the shape of the pruned-weight workload at a size the oracle multiplies whole: 16 x 16 blocks
    # kept at 10 %, every block row is one group of exactly one slab
    rng = np.random.default_rng(31)
    keep = rng.random((256, 64)) < 0.10
    mask = np.kron(keep, np.ones((16, 16), dtype=bool))
    r, cc = np.nonzero(mask)
    vals = synth.to_bits(rng.standard_normal(r.size).astype(np.float32) / 4, "f16")
    csr = synth.csr_from_coo(4096, 1024, r, cc, vals, "f16")
    b = synth.dense_rhs(rng, 1024, 264, "f16", dist="normal")
    perm, rg = blocking_bit_exact(csr, 16, 0.5)
    c, v = gpu_spmm(csr, perm, rg, 16, b)
    index_bit_exact(v, csr, perm, rg, 16)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "block rows of one slab")


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_partitions_and_widths(seed):
    # random everything: size, block width (fast and slow gather paths), density, dtype, dense
    # width with and without a column tail, padded leading dimensions, and an arbitrary valid row
    # partition with heights from 1 row to several tiles
    rng = np.random.default_rng(1000 + seed)
    col_block = int(rng.choice([1, 2, 4, 5, 8, 12, 16, 24, 32, 48, 64]))
    kb = int(rng.integers(1, 30))
    m = int(rng.integers(1, 700))
    n = 8 * int(rng.integers(1, 80))
    dtype = "bf16" if seed % 2 else "f16"
    csr = random_csr(rng, m, kb * col_block, float(rng.choice([0.01, 0.05, 0.3])), dtype=dtype)
    b = synth.dense_rhs(rng, kb * col_block, n, dtype, dist="normal" if seed % 3 else "uniform")
    cuts = np.unique(np.concatenate([[0, m], rng.integers(0, m + 1, size=int(rng.integers(0, 12)))]))
    if rng.random() < 0.4:                     # plus a run of single-row groups
        lo = int(rng.integers(0, m)); hi = min(m, lo + int(rng.integers(1, 60)))
        cuts = np.unique(np.concatenate([cuts, np.arange(lo, hi + 1)]))
    rg = cuts.astype(np.int32)
    perm = rng.permutation(m).astype(np.int32)
    c, v = gpu_spmm(csr, perm, rg, col_block, b, ldb_pad=8 * int(rng.integers(0, 3)), ldc_pad=4 * int(rng.integers(0, 3)))
    index_bit_exact(v, csr, perm, rg, col_block)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "seed %d cb=%d m=%d n=%d groups=%d" % (seed, col_block, m, n, rg.size - 1))


def test_leading_dimensions_and_overwrite():
    rng = np.random.default_rng(6)
    csr = random_csr(rng, 90, 128, 0.1, dtype="bf16")
    b = synth.dense_rhs(rng, 128, 72, "bf16", dist="normal")
    perm, rg = blocking_bit_exact(csr, 32, 0.5)
    c, _ = gpu_spmm(csr, perm, rg, 32, b, ldb_pad=24, ldc_pad=12)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "padded leading dimensions")


def test_empty_rows_get_zeros_and_single_dense_block_is_a_gemm():
    rng = np.random.default_rng(7)
    csr = csr_from_rows([[], [1, 40], [], [2], []], n_cols=64, rng=rng)
    b = synth.dense_rhs(rng, 64, 16, "f16")
    perm, rg = blocking_bit_exact(csr, 16, 0.5)
    c, _ = gpu_spmm(csr, perm, rg, 16, b)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "empty rows")
    assert np.all(c[[0, 2, 4]] == 0.0)
    dense = random_csr(rng, 48, 96, 1.0)
    b = synth.dense_rhs(rng, 96, 128, "f16")
    perm, rg = blocking_bit_exact(dense, 32, 0.5)
    assert len(rg) == 2                                   # one group, three full blocks
    c, _ = gpu_spmm(dense, perm, rg, 32, b)
    a64 = oracle.bits_to_f64(synth.dense_bits(dense), "f16")
    b64 = oracle.bits_to_f64(b, "f16")
    check_c(c, a64 @ b64, np.abs(a64) @ np.abs(b64), "dense block vs numpy GEMM")


def test_identity_like_right_hand_side_reproduces_rows_exactly():
    rng = np.random.default_rng(8)
    csr = random_csr(rng, 64, 64, 0.2)
    eye = synth.to_bits(np.eye(64, dtype=np.float32), "f16")
    perm, rg = blocking_bit_exact(csr, 16, 0.4)
    c, _ = gpu_spmm(csr, perm, rg, 16, eye)
    assert np.array_equal(c, oracle.bits_to_f64(synth.dense_bits(csr), "f16"))


def test_argument_checks_on_the_gpu_entry():
    import torch
    rng = np.random.default_rng(9)
    csr = random_csr(rng, 20, 32, 0.3)
    perm, rg = binding.sa1_reorder(csr, 16, 0.5)
    v = binding.vbr_build(csr, perm, rg, 16).upload("cuda:0")
    b = torch.zeros((32, 16), dtype=torch.float16, device="cuda:0")
    c = torch.zeros((20, 16), dtype=torch.float32, device="cuda:0")
    s = torch.cuda.current_stream().cuda_stream
    assert binding.vbr_spmm_raw(v, b.data_ptr(), 16, c.data_ptr(), 16, 12, s) == -1       # N % 8
    assert binding.vbr_spmm_raw(v, b.data_ptr(), 8, c.data_ptr(), 16, 16, s) == -1        # ldb < N
    assert binding.vbr_spmm_raw(v, b.data_ptr() + 2, 16, c.data_ptr(), 16, 16, s) == -1   # alignment
    assert binding.vbr_spmm_raw(v, b.data_ptr(), 16, c.data_ptr(), 16, 0, s) == 0         # N = 0: nothing to do
    assert binding.vbr_spmm_raw(v, b.data_ptr(), 16, c.data_ptr(), 16, 16, s) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("col_block,short", [(16, False), (8, True), (3, False)])
def test_b_rows_no_block_touches_never_reach_c(col_block, short):
    # Column blocks no row of A enters hold NaN and Inf in B.  Padding of K-steps, of partial slabs
    # and of absent slabs must come from zeros, never from whatever B rows happen to be near: C
    # stays finite and within the bound.  (B rows inside a STORED block do meet the block's
    # fill-in zeros: that is the format's semantics, not tested here.)
    import torch
    rng = np.random.default_rng(50 + col_block)
    kb, n = 40, 136
    m = 6000 if short else 300
    dens = 0.004 if short else 0.05
    csr = random_csr(rng, m, kb * col_block, dens)
    # empty the odd column blocks of A
    keep = (csr["col_idx"] // col_block) % 2 == 0
    rows = np.repeat(np.arange(m), np.diff(csr["row_ptr"]))[keep]
    csr = synth.csr_from_coo(m, kb * col_block, rows, csr["col_idx"][keep], csr["vals"][keep], "f16")
    b_bits = synth.dense_rhs(rng, kb * col_block, n, "f16")
    poison = b_bits.copy()
    odd = (np.arange(kb * col_block) // col_block) % 2 == 1
    poison[odd] = np.where(rng.random((int(odd.sum()), n)) < 0.5, 0x7E00, 0x7C00).astype(np.uint16)   # NaN / +Inf
    perm, rg = blocking_bit_exact(csr, col_block, 0.9 if short else 0.4)
    c, v = gpu_spmm(csr, perm, rg, col_block, poison)
    c_ref, s = oracle.spmm(csr, b_bits)          # the clean B: A never reads the poisoned rows
    assert np.isfinite(c).all()
    check_c(c, c_ref, s, "poisoned B rows, cb=%d" % col_block)


def test_runs_on_the_given_stream_and_in_a_captured_graph():
    # vbr_spmm only enqueues kernels on the stream it is given (no allocation, no memset, no
    # synchronisation), so it can run on a side stream and be captured into a graph; every replay
    # must reproduce the eager result for the B that is in place at that moment
    import torch
    rng = np.random.default_rng(60)
    w = synth.workload("c3", scale=0.125)            # tall and low groups: several kernels per call
    a, cb = w["A"], w["col_block"]
    perm, rg = binding.sa1_reorder(a, cb, w["taus"][1])
    v = binding.vbr_build(a, perm, rg, cb).upload("cuda:0")
    k, n = w["B"].shape
    b = torch_io.bits_to_device(w["B"], w["dtype"])
    c_ref, s_ref = oracle.spmm(a, w["B"])
    side = torch.cuda.Stream()                        # default priority
    c_side = torch.full((a["n_rows"], n), float("nan"), dtype=torch.float32, device="cuda:0")
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        v.spmm(b, c_side)
    side.synchronize()
    check_c(c_side.cpu().numpy().astype(np.float64), c_ref, s_ref, "side stream")

    c_graph = torch.full_like(c_side, float("nan"))
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        v.spmm(b, c_graph)
    for rep in range(3):
        b_bits = synth.dense_rhs(rng, k, n, w["dtype"], dist="normal")
        b.copy_(torch_io.bits_to_device(b_bits, w["dtype"]))       # eager work between the replays
        c_graph.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        c_eager = v.spmm(b, torch.empty_like(c_graph))
        torch.cuda.synchronize()
        assert torch.equal(c_graph, c_eager), "replay %d differs from the eager launch" % rep
        c_ref, s_ref = oracle.spmm(a, b_bits)
        check_c(c_graph.cpu().numpy().astype(np.float64), c_ref, s_ref, "graph replay %d" % rep)


def test_forked_launches_keep_the_order_of_the_callers_stream_and_replay_in_a_graph():
    # a multiply of several launches spreads them over the handle's own streams between an event
    # recorded on the caller's stream and waits of the caller's stream: work queued before the call
    # (the NaN fill) must be over before any launch writes, work queued after it (the clone) must
    # see every row; a captured graph must carry the same fork and join
    import torch
    rng = np.random.default_rng(61)
    w = synth.workload("rmat")
    a, cb = w["A"], w["col_block"]
    perm, rg = binding.sa1_reorder(a, cb, w["taus"][0])
    v = binding.vbr_build(a, perm, rg, cb).upload("cuda:0")
    k, n = w["B"].shape
    assert len(v.launches(n)) >= 2, v.launches(n)
    b = torch_io.bits_to_device(w["B"], w["dtype"])
    c_ref, s_ref = oracle.spmm(a, w["B"])
    side = torch.cuda.Stream()                        # default priority
    c = torch.empty((a["n_rows"], n), dtype=torch.float32, device="cuda:0")
    side.wait_stream(torch.cuda.current_stream())
    results = []
    with torch.cuda.stream(side):
        for _ in range(6):
            c.fill_(float("nan"))
            v.spmm(b, c)
            results.append(c.clone())
    side.synchronize()
    check_c(results[0].cpu().numpy().astype(np.float64), c_ref, s_ref, "forked launches, first call")
    for i, r in enumerate(results[1:]):
        assert torch.equal(r, results[0]), "call %d differs from the first" % (i + 1)

    c_graph = torch.full_like(c, float("nan"))
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        v.spmm(b, c_graph)
    for rep in range(3):
        b_bits = synth.dense_rhs(rng, k, n, w["dtype"])
        b.copy_(torch_io.bits_to_device(b_bits, w["dtype"]))       # eager work between the replays
        c_graph.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        c_eager = v.spmm(b, torch.empty_like(c_graph))
        torch.cuda.synchronize()
        assert torch.equal(c_graph, c_eager), "replay %d differs from the eager launches" % rep
    c_ref, s_ref = oracle.spmm(a, b_bits)
    check_c(c_graph.cpu().numpy().astype(np.float64), c_ref, s_ref, "graph replay")


def test_two_handles_on_two_streams_at_the_same_time():
    # every handle has its own side streams and events, so two multiplies of several launches each
    # may be in flight at once from different caller streams
    import torch
    rng = np.random.default_rng(62)
    w = synth.workload("rmat")
    a, cb = w["A"], w["col_block"]
    perm, rg = binding.sa1_reorder(a, cb, w["taus"][0])
    k, n = w["B"].shape
    hs = [binding.vbr_build(a, perm, rg, cb).upload("cuda:0") for _ in range(2)]
    assert len(hs[0].launches(n)) >= 2
    bs = [torch_io.bits_to_device(synth.dense_rhs(rng, k, n, w["dtype"]), w["dtype"]) for _ in range(2)]
    alone = [hs[i].spmm(bs[i], torch.empty((a["n_rows"], n), dtype=torch.float32, device="cuda:0")) for i in range(2)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]          # default priority
    cs = [torch.full_like(alone[0], float("nan")) for _ in range(2)]
    for st in streams:
        st.wait_stream(torch.cuda.current_stream())
    for _ in range(5):
        for i in range(2):
            with torch.cuda.stream(streams[i]):
                cs[i].fill_(float("nan"))
                hs[i].spmm(bs[i], cs[i])
    for st in streams:
        st.synchronize()
    for i in range(2):
        assert torch.equal(cs[i], alone[i]), "handle %d: concurrent result differs from the one computed alone" % i
        hs[i].close()


def test_right_hand_side_larger_than_4_gib():
    # B is a 256-column window of a 70 000 x 32 776 tensor (4.6 GB): row bases need 64 bits
    import torch
    rng = np.random.default_rng(41)
    k, n, ld = 70000, 256, 32776
    rows = [sorted(set(rng.integers(0, k, size=40).tolist()) | {0, k - 1}) for _ in range(48)]
    csr = csr_from_rows(rows, n_cols=k, rng=rng)
    b_bits = synth.dense_rhs(rng, k, n, "f16")
    big = torch.zeros((k, ld), dtype=torch.float16, device="cuda:0")
    b = big[:, 1024:1024 + n]
    b.copy_(torch_io.bits_to_device(b_bits, "f16"))
    assert k * ld * 2 > (1 << 32) and b.stride(0) == ld
    for col_block, perm, rg in [(16, np.arange(48, dtype=np.int32), np.array([0, 16, 48], dtype=np.int32)),
                                (8, *binding.sa1_reorder(csr, 8, 0.3))]:
        v = binding.vbr_build(csr, perm, rg, col_block).upload("cuda:0")
        c = torch.full((48, n), float("nan"), dtype=torch.float32, device="cuda:0")
        v.spmm(b, c)
        torch.cuda.synchronize()
        c_ref, s = oracle.spmm(csr, b_bits)
        check_c(c.cpu().numpy().astype(np.float64), c_ref, s, "B beyond 4 GiB, cb=%d" % col_block)
    del big


# --------------------------------------------------------------------------- the CSR comparator kernel
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_csr_comparator_matches_oracle(dtype):
    import torch
    rng = np.random.default_rng(21)
    for m, k, n, dens in [(70, 96, 64, 0.2), (301, 160, 520, 0.05), (33, 64, 8, 0.6), (5, 32, 1032, 0.0)]:
        csr = random_csr(rng, m, k, dens, dtype=dtype)
        b_bits = synth.dense_rhs(rng, k, n, dtype)
        h = binding.CsrDev(csr).upload("cuda:0")
        full = np.zeros((k, n + 8), dtype=np.uint16)
        full[:, :n] = b_bits
        b = torch_io.bits_to_device(full, dtype)[:, :n]                      # padded leading dimension
        c_full = torch.full((m, n + 4), float("nan"), dtype=torch.float32, device="cuda:0")
        h.spmm(b, c_full[:, :n])
        torch.cuda.synchronize()
        out = c_full.cpu().numpy()
        assert np.isnan(out[:, n:]).all()
        c_ref, s = oracle.spmm(csr, b_bits)
        check_c(out[:, :n].astype(np.float64), c_ref, s, "csr %s m=%d n=%d" % (dtype, m, n))


def test_csr_comparator_and_blocked_path_agree_on_the_graph_workload():
    import torch
    w = synth.workload("rmat", scale=0.125)
    a, cb = w["A"], w["col_block"]
    perm, rg = blocking_bit_exact(a, cb, w["taus"][0])
    c, v = gpu_spmm(a, perm, rg, cb, w["B"])
    index_bit_exact(v, a, perm, rg, cb)
    c_ref, s = oracle.spmm(a, w["B"])
    check_c(c, c_ref, s, "rmat blocked")
    b = torch_io.bits_to_device(w["B"], w["dtype"])
    c2 = binding.CsrDev(a).upload("cuda:0").spmm(b)
    torch.cuda.synchronize()
    check_c(c2.cpu().numpy().astype(np.float64), c_ref, s, "rmat csr")


# --------------------------------------------------------------------------- the five workloads, reduced
@pytest.mark.parametrize("name,scale,noise", [("c1", 1.0, True), ("c1", 1.0, False), ("c2", 0.25, True),
                                               ("c2", 0.25, False), ("c3", 0.125, True), ("c4", 0.125, True),
                                               ("c5", 0.0625, True)])
def test_workloads_reduced_elementwise(name, scale, noise):
    w = synth.workload(name, scale=scale, noise=noise)
    c_ref, s = oracle.spmm(w["A"], w["B"])
    for tau in w["taus"]:
        perm, rg = blocking_bit_exact(w["A"], w["col_block"], tau)
        c, v = gpu_spmm(w["A"], perm, rg, w["col_block"], w["B"])
        index_bit_exact(v, w["A"], perm, rg, w["col_block"])
        check_c(c, c_ref, s, "%s tau=%g" % (name, tau))


# --------------------------------------------------------------------------- wide dense matrices, small A
def test_one_slab_groups_with_eight_or_more_column_tiles():
    # N = 2056: nine 256-column tiles (the last one ragged), so the workgroup -> (tile, column
    # tile) map takes the branch it takes at the full size of the pruned-weight workload
    rng = np.random.default_rng(77)
    keep = rng.random((40, 48)) < 0.15
    mask = np.kron(keep, np.ones((16, 16), dtype=bool))
    r, cc = np.nonzero(mask)
    vals = synth.to_bits(rng.standard_normal(r.size).astype(np.float32) / 4, "f16")
    csr = synth.csr_from_coo(640, 768, r, cc, vals, "f16")
    b = synth.dense_rhs(rng, 768, 2056, "f16", dist="normal")
    perm, rg = blocking_bit_exact(csr, 16, 0.5)
    c, v = gpu_spmm(csr, perm, rg, 16, b)
    index_bit_exact(v, csr, perm, rg, 16)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "one-slab groups, N=2056")


def test_short_groups_with_eight_or_more_column_tiles():
    # short groups (panels) with N = 1032: nine 128-column tiles, the last one 8 columns wide
    rng = np.random.default_rng(78)
    csr = random_csr(rng, 6000, 20 * 16, 0.01)
    b = synth.dense_rhs(rng, 320, 1032, "f16")
    perm, rg = blocking_bit_exact(csr, 16, 0.9)
    h = np.diff(rg)
    assert h[h < 16].sum() >= 4096
    c, v = gpu_spmm(csr, perm, rg, 16, b)
    index_bit_exact(v, csr, perm, rg, 16)
    c_ref, s = oracle.spmm(csr, b)
    check_c(c, c_ref, s, "short groups, N=1032")


# --------------------------------------------------------------------------- full sizes, every element
@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5", "rmat"])
def test_workloads_full_size_every_element(name):
    # the launch configuration bench.py times, at the full size, every element of C against the
    # oracle; c3 at all three of its thresholds
    w = synth.workload(name)
    a, cb = w["A"], w["col_block"]
    print("full size %s: oracle multiply" % name, flush=True)
    c_ref, s = oracle.spmm(a, w["B"])
    empty = np.nonzero(np.diff(a["row_ptr"]) == 0)[0]
    for tau in w["taus"]:
        print("full size %s tau=%g: library" % (name, tau), flush=True)
        perm, rg = blocking_bit_exact(a, cb, tau)
        c, v = gpu_spmm(a, perm, rg, cb, w["B"])
        index_bit_exact(v, a, perm, rg, cb)
        check_c(c, c_ref, s, "%s full size tau=%g" % (name, tau))
        # rows without entries are exactly zero
        assert np.all(c[empty] == 0.0)
        del c, v


# --------------------------------------------------------------------------- the comparison experiments, reduced
CURVE_TAUS = [0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0]


def blocked_and_csr_against_oracle(a, col_block, tau, b_bits, what):
    import torch
    perm, rg = blocking_bit_exact(a, col_block, tau)
    c, v = gpu_spmm(a, perm, rg, col_block, b_bits)
    index_bit_exact(v, a, perm, rg, col_block)
    c_ref, s = oracle.spmm(a, b_bits)
    check_c(c, c_ref, s, what + " blocked")
    b = torch_io.bits_to_device(b_bits, a["dtype"])
    c2 = binding.CsrDev(a).upload("cuda:0").spmm(b)
    torch.cuda.synchronize()
    check_c(c2.cpu().numpy().astype(np.float64), c_ref, s, what + " csr")


@pytest.mark.parametrize("theta,rho", [(0.1, 0.05), (0.3, 0.5), (0.02, 0.2)])
def test_landscape_point_at_the_selected_threshold(theta, rho):
    # one point of the synthetic landscape A(Delta, theta, rho) at reduced size: the threshold the
    # selection rule picks (same as the oracle's), then both kernels against the oracle
    rng = np.random.default_rng(int(theta * 1000 + rho * 100))
    a = synth.landscape(rng, 1024, 32, theta, rho)
    b_bits = synth.dense_rhs(rng, 1024, 264, "f16")
    sel = binding.sa1_blocking_curve(a, 32, CURVE_TAUS, 32)["selected"]
    assert sel == oracle.blocking_curve(a, 32, CURVE_TAUS, 32)["selected"]
    blocked_and_csr_against_oracle(a, 32, CURVE_TAUS[sel], b_bits, "landscape theta=%g rho=%g" % (theta, rho))


@pytest.mark.parametrize("degree,col_block", [(8, 64), (8, 256), (128, 64), (128, 256), (32, 128)])
def test_graph_grid_points_reduced(degree, col_block):
    # corners and centre of the graph grid (edges per node x column-block width) at 2^11 nodes
    w = synth.workload("rmat", scale=0.125, rmat_degree=degree, rmat_col_block=col_block)
    a = w["A"]
    sel = binding.sa1_blocking_curve(a, col_block, CURVE_TAUS, col_block)["selected"]
    assert sel == oracle.blocking_curve(a, col_block, CURVE_TAUS, col_block)["selected"]
    for tau in {CURVE_TAUS[sel], 0.4}:
        blocked_and_csr_against_oracle(a, col_block, tau, w["B"], "rmat degree=%d cb=%d tau=%g" % (degree, col_block, tau))
