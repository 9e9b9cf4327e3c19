#!/usr/bin/env python3
"""Benchmark of the blocked SpMM path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--clean] [--select-tau] [--no-cpu-baseline]
    python bench.py --landscape | --rmat-grid [--small]       (the paper's two comparison experiments instead)

Prints ONE JSON line.  The metric is VBR-SpMM throughput in TFLOP/s on stored-block flops
(2 * stored elements * N per multiply); a step is one ``vbr_spmm`` launch on the resident VBR
matrix with A (packed), B and C already in HBM.  The one-off host work of the path (1-SA
reordering, VBR build, upload), which the method discounts over many multiplications (section 6
of the paper), is timed once and reported under ``setup``.  The CPU oracle is timed beside it on
a bounded sample of the same workload (``cpu_baseline``); it is a checker, not a target.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2500.0   # MI355X dense fp16 / bf16 matrix peak
PEAK_HBM_GBS = 8000.0

WORKLOAD_TEXT = {
    "c1": "configs[0]: A 1024x1024 fp16, 32x32 planted blocks at 10%, +0.5% noise, N=256, tau=0.7",
    "c2": "configs[1]: A 8192x8192 fp16, 64x64 planted blocks at 5%, +1% off-block noise, N=1024, tau=0.6",
    "c3": "configs[2]: A 16384x16384 bf16, heights {16,32,64,128} x 32 blocks at 2%, fill 0.7, N=512, tau=0.6",
    "c4": "configs[3]: pruned-weight-like A 4096x16384 fp16, 16x16 blocks kept at 10%, N=4096, tau=0.5",
    "c5": "configs[4]: Erdos-Renyi A 32768x32768 fp16 density 0.05%, column block 32, N=256, tau=0.3",
    "rmat": "graph workload of the paper's sections 4.1 / 4.4.3: RMAT (0.57,0.19,0.19,0.05), 2^14 nodes, 32 edges per node, "
            "rows scrambled, column block 64, N=4096, tau=0.4",
}


def measure_denominators(torch, binding, dev) -> dict:
    """Rates of the single units the kernels lean on, measured on this GPU with the library's probe
    loops (HIP events around the third of three launches each): flop/s for the matrix
    instructions, bytes/s otherwise."""
    buf = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    iters = {"mfma_16x16x32_f16": 20000, "mfma_16x16x16_f16": 20000, "mfma_32x32x16_f16": 10000,
             "lds_read_tr_b64": 4000, "lds_read_b64": 4000, "lds_read_b128": 4000, "lds_dma_b128": 2000, "hbm_copy": 1}
    res = {}
    for kind, it in iters.items():
        best = None
        for _ in range(3):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            work = binding.vbr_probe_launch(kind, buf, it)
            e1.record(stream)
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3
            best = t if best is None else min(best, t)
        res[kind] = {"rate": work / best, "unit": "flop/s" if kind.startswith("mfma") else "B/s", "ms": best * 1e3}
        if kind.startswith("lds"):
            res[kind]["bytes_per_clk_per_cu_at_2.4GHz"] = work / best / 256 / 2.4e9
    del buf
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c4", choices=sorted(WORKLOAD_TEXT))
    ap.add_argument("--clean", action="store_true", help="noise-free variant of c1/c2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ramp", action="store_true",
                    help="skip the clock-ramp launches before the warm-up (for counter-collection runs, where every "
                         "dispatch is slow and the clocks do not matter)")
    ap.add_argument("--timed-only", action="store_true",
                    help="only the warm-up and the timed region (what the rocprofv3 summaries under profiles/ are "
                         "made from): no single-launch, cold-cache, comparator, dense or CPU legs")
    ap.add_argument("--no-csr-baseline", action="store_true",
                    help="skip the CSR comparator kernel (the stand-in for the sparse-library routine)")
    ap.add_argument("--no-dense-baseline", action="store_true",
                    help="skip the dense product on the zero-filled matrix (run by default for c2 and c4)")
    ap.add_argument("--dense", action="store_true",
                    help="measure the dense product on the zero-filled matrix instead (A stored as one dense VBR, groups "
                         "of 128 rows, every block kept, no reordering): the comparison the target configuration names, "
                         "as a workload of its own so that it can be profiled; no CSR / dense / CPU baselines")
    ap.add_argument("--select-tau", action="store_true",
                    help="take the threshold from the blocking curve (tau = 0.1 .. 1) by the paper's rule, average block "
                         "height nearest to the matrix's own block height, instead of the workload's fixed tau")
    ap.add_argument("--landscape", action="store_true",
                    help="instead of the benchmark: blocked multiply vs CSR multiply over the synthetic landscape "
                         "A(Delta, theta, rho) of the paper's Table 2 (section 4.4.2); prints one JSON line")
    ap.add_argument("--rmat-grid", action="store_true",
                    help="instead of the benchmark: blocked multiply vs CSR multiply on RMAT graphs, 8 .. 128 edges per "
                         "node x column blocks 64 / 128 / 256 (section 4.4.3); prints one JSON line")
    ap.add_argument("--small", action="store_true", help="with --landscape / --rmat-grid: a reduced grid (a minute)")
    ap.add_argument("--denominators", action="store_true",
                    help="instead of the benchmark: only the measured denominators, as one JSON line")
    ap.add_argument("--no-denominators", action="store_true",
                    help="skip the measured denominators (matrix-instruction issue rates, LDS operand rates, "
                         "direct-to-LDS load rate, HBM copy), which run outside the timed region")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 256 MiB streaming kernel, out = 2*in (outside the timed region): the known-size "
                         "kernel the rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.timed_only:
        args.no_cpu_baseline = args.no_csr_baseline = args.no_dense_baseline = args.no_denominators = True
    if args.dense:
        args.no_cpu_baseline = args.no_csr_baseline = args.no_dense_baseline = True
        args.select_tau = False
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (row groups shard "
              "without any exchange step; nothing here uses a second GPU)" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2202_05868_amd import binding, synth, torch_io

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    torch.cuda.set_device(0)
    torch.zeros(1, device=dev)
    torch.cuda.synchronize()              # the context exists before anything is timed (setup.upload_s)

    if args.denominators:
        print(json.dumps({"denominators": measure_denominators(torch, binding, dev),
                          "note": "rates of single units measured with the library's probe loops (vbr_probe_launch), "
                                  "16 waves per CU; flop/s for the matrix instructions, bytes/s otherwise"}))
        return 0
    if args.landscape or args.rmat_grid:
        from paper_2202_05868_amd import experiments
        say = lambda msg: print(msg, file=sys.stderr, flush=True)
        if args.landscape:
            res = (experiments.landscape(n=2048, delta=64, widths=(512, 2048), thetas=(0.1, 0.4), rhos=(0.02, 0.2), progress=say)
                   if args.small else experiments.landscape(progress=say))
        else:
            res = (experiments.rmat_grid(degrees=(8, 64), col_blocks=(64,), log2_nodes=12, width=1024, progress=say)
                   if args.small else experiments.rmat_grid(progress=say))
        say(experiments.landscape_table(res) if args.landscape else experiments.rmat_table(res))
        print(json.dumps(res))
        return 0

    w = synth.workload(args.workload, noise=not args.clean)
    a, cb, n = w["A"], w["col_block"], w["N"]
    tau = w["taus"][len(w["taus"]) // 2]
    selection = None
    if args.select_tau:
        # the matrix's own block height: the planted one, or the column-block width where nothing is planted
        info = w.get("info")
        target = int(round(float(np.mean(info["heights"])))) if info else cb
        taus = [0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0]
        ts = time.perf_counter()
        cur = binding.sa1_blocking_curve(a, cb, taus, target)
        tau = taus[cur["selected"]]
        selection = {"rule": "average block height nearest to %d" % target, "taus": taus,
                     "avg_block_height": (cur["sum_heights"] / np.maximum(cur["n_blocks"], 1)).tolist(),
                     "rho_after": (a["nnz"] / np.maximum(cur["stored_elems"], 1)).tolist(),
                     "selected_tau": tau, "curve_s": time.perf_counter() - ts}

    def zero_filled(m):
        """the matrix with every entry stored (explicit zeros), as CSR"""
        rows, cols = m["n_rows"], m["n_cols"]
        d = dict(m)
        d["row_ptr"] = np.arange(rows + 1, dtype=np.int64) * cols
        d["col_idx"] = np.tile(np.arange(cols, dtype=np.int32), rows)
        d["vals"] = np.ascontiguousarray(synth.dense_bits(m).reshape(-1))
        d["nnz"] = rows * cols
        return d

    # ---- one-off host work of the path
    t0 = time.perf_counter()
    if args.dense:
        a = zero_filled(a)
        tau = None
        perm = np.arange(a["n_rows"], dtype=np.int32)
        rg = np.arange(0, a["n_rows"] + 128, 128, dtype=np.int32).clip(max=a["n_rows"])
    else:
        perm, rg = binding.sa1_reorder(a, cb, tau)
    t1 = time.perf_counter()
    v = binding.vbr_build(a, perm, rg, cb)
    t2 = time.perf_counter()
    v.upload(dev)
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    ix = v.index()
    stored = int(ix["stored_elems"])
    h = np.diff(rg)

    b = torch_io.bits_to_device(w["B"], w["dtype"], dev)
    c = torch.empty((a["n_rows"], n), dtype=torch.float32, device=dev)

    if args.calib_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)      # 256 MiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 2.0, out=dst)       # one streaming elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- clock ramp: the GPU raises its clocks only under sustained load (the first tens of
    # milliseconds run 10-15 % slower); launches are repeated in batches until a batch stops getting
    # faster, so that the W warm-up steps and the K timed steps see the steady state a real job sees
    stream = torch.cuda.current_stream()

    def clock_ramp(launch, batch=50, budget_ms=2000.0):
        n, best, stale, spent = 0, float("inf"), 0, 0.0
        while not args.no_ramp and n < 4000 and stale < 3:
            r0 = torch.cuda.Event(enable_timing=True)
            r1 = torch.cuda.Event(enable_timing=True)
            r0.record(stream)
            for _ in range(batch):
                launch()
            r1.record(stream)
            torch.cuda.synchronize()
            t = r0.elapsed_time(r1)
            n += batch
            if t < 0.99 * best:
                best, stale = t, 0
            else:
                stale += 1
            spent += t
            if spent + t > budget_ms:                    # never more than the budget (about 2 s) of ramp
                break
        return n
    ramp_launches = clock_ramp(lambda: v.spmm(b, c))

    # ---- timed region: K launches between HIP events on the launch stream
    for _ in range(args.warmup):
        v.spmm(b, c)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        v.spmm(b, c)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall1 = time.perf_counter()
    ms = ev0.elapsed_time(ev1) / args.steps
    wall_ms = (wall1 - wall0) * 1e3 / args.steps

    # ---- outside the timed region: single launches (median, min), then with cold caches
    def time_single(reps, flush=None):
        out = []
        for _ in range(reps):
            if flush is not None:
                flush.add_(1.0)            # streams 1 GiB through L2 and the memory-side cache
            a0 = torch.cuda.Event(enable_timing=True)
            a1 = torch.cuda.Event(enable_timing=True)
            a0.record(stream)
            v.spmm(b, c)
            a1.record(stream)
            torch.cuda.synchronize()
            out.append(a0.elapsed_time(a1))
        return out
    if args.timed_only:
        single, cold = [ms], [float("nan")]
    else:
        single = time_single(20)
        flush_buf = torch.zeros(256 * 1024 * 1024, dtype=torch.float32, device=dev)
        cold = time_single(5, flush_buf)
        del flush_buf

    flops_stored = 2.0 * stored * n
    flops_nnz = 2.0 * a["nnz"] * n
    tflops = flops_stored / (ms * 1e-3) * 1e-12
    tflops_nnz = flops_nnz / (ms * 1e-3) * 1e-12
    # What the matrix units are actually given: the packed fragments.  Tiles that gather single
    # columns leave out the columns of a stored block that hold only fill-in, so for matrices with
    # much fill-in this is less than the stored-block count the metric credits; the roofline below
    # is priced on the smaller of the two, never on flops that were not executed.
    packed = v.schedule()["packed_elems"]
    flops_exec = min(flops_stored, 2.0 * packed * n)
    tflops_exec = flops_exec / (ms * 1e-3) * 1e-12
    # compulsory HBM bytes of one multiply: packed A once, B once, C once
    hbm_min = packed * 2 + a["n_cols"] * n * 2 + a["n_rows"] * n * 4
    # the bound: the MFMA time of the executed flops against the compulsory HBM time
    t_mfma = flops_exec / (PEAK_MFMA_F16_TFLOPS * 1e12)
    t_hbm = hbm_min / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        roofline = dict(bound="mfma", achieved=tflops_exec, peak=PEAK_MFMA_F16_TFLOPS, unit="TFLOP/s",
                        frac=tflops_exec / PEAK_MFMA_F16_TFLOPS, traffic=None)
    else:
        gbs = hbm_min / (ms * 1e-3) * 1e-9
        roofline = dict(bound="hbm", achieved=gbs, peak=PEAK_HBM_GBS, unit="GB/s", frac=gbs / PEAK_HBM_GBS,
                        traffic=None)
    # the kernels one vbr_spmm call launches for this workload, from the library's own launch plan;
    # the time between the events is the whole call's
    roofline["kernel"] = v.launches(n)
    roofline["ms_per_launch"] = ms
    roofline["algorithmic_flops"] = flops_exec
    roofline["algorithmic_hbm_bytes"] = hbm_min
    # B rows gathered from the caches into LDS when no two row groups share a staged row: one panel
    # per stored block and column tile (sum over blocks of col_block * N * 2 bytes); priced below
    # against the measured rate of direct-to-LDS loads
    gathered = float(ix["n_blocks"]) * cb * n * 2
    roofline["cache_to_lds_gather"] = {"bytes": gathered, "achieved_TBs": gathered / (ms * 1e-3) * 1e-12}
    # HBM bytes per launch measured with rocprofv3 --pmc: the figure the summary under profiles/ ends with
    tr_name = "vbr_spmm_%s%s.txt" % (args.workload, "_clean" if args.clean else "")
    tr = os.path.join(ROOT, "profiles", tr_name)
    if os.path.exists(tr):
        import re
        m = re.search(r"^HBM traffic per launch: ([0-9.]+) MB", open(tr).read(), flags=re.M)
        if m:
            roofline["traffic"] = float(m.group(1)) * 1e6
            roofline["traffic_source"] = "profiles/" + tr_name + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command)"

    # ---- measured denominators (outside the timed region): what the chip delivers per unit
    denominators = None
    if not args.no_denominators:
        denominators = measure_denominators(torch, binding, dev)
        dma = denominators["lds_dma_b128"]["rate"]
        roofline["cache_to_lds_gather"]["measured_load_rate_TBs"] = dma * 1e-12
        roofline["cache_to_lds_gather"]["frac_of_measured_load_rate"] = gathered / (ms * 1e-3) / dma
        roofline["frac_of_measured_mfma_16x16x32"] = tflops_exec * 1e12 / denominators["mfma_16x16x32_f16"]["rate"]
        roofline["frac_of_measured_hbm_copy"] = hbm_min / (ms * 1e-3) / denominators["hbm_copy"]["rate"]

    out = {
        "metric": "VBR-SpMM TFLOP/s (stored-block flops 2*stored_elems*N)",
        "value": tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w["dtype"],
        "accumulate_dtype": "f32 (MFMA)",
        "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload] + ("" if not args.clean else " (noise-free)") +
                               ("" if not args.dense else " -- ZERO-FILLED: every entry stored, groups of 128 rows, no reordering"),
                   "N": n, "col_block": cb, "tau": tau, "parallelism": "1 GPU"},
        "nnz_effective_tflops": tflops_nnz,
        "executed_tflops": tflops_exec,
        "fill_in_not_multiplied": 1.0 - flops_exec / flops_stored if flops_stored else 0.0,
        "pct_mfma_fp16_peak": 100.0 * tflops_exec / PEAK_MFMA_F16_TFLOPS,
        "pct_hbm_peak_compulsory": 100.0 * (hbm_min / (ms * 1e-3) * 1e-9) / PEAK_HBM_GBS,
        "wall_ms_per_step": wall_ms,
        "clock_ramp_launches": ramp_launches,
        "single_launch_ms": {"median": float(np.median(single)), "min": float(np.min(single)),
                             "cold_caches_median": float(np.median(cold))},
        "blocking": {"groups": int(len(h)), "mean_height": float(h.mean()) if len(h) else 0.0,
                     "max_height": int(h.max()) if len(h) else 0, "blocks": int(ix["n_blocks"]),
                     "stored_elems": stored, "nnz": int(a["nnz"]),
                     "fill_overhead": stored / max(1, a["nnz"]), **v.schedule()},
        "setup": {"sa1_reorder_s": t1 - t0, "vbr_build_s": t2 - t1, "upload_s": t3 - t2,
                  "host_threads": os.cpu_count()},
        "roofline": roofline,
    }
    if denominators is not None:
        out["denominators"] = denominators
    if selection is not None:
        out["tau_selection"] = selection

    if not args.no_csr_baseline:
        # the comparison of the paper's section 4.4.2: the same product straight from CSR (own kernel,
        # fp32 FMAs on the vector units), timed the same way
        hcsr = binding.CsrDev(a).upload(dev)
        cc = torch.empty_like(c)
        for _ in range(2):
            hcsr.spmm(b, cc)
        torch.cuda.synchronize()
        s0 = torch.cuda.Event(enable_timing=True)
        s1 = torch.cuda.Event(enable_timing=True)
        s0.record(stream)
        for _ in range(5):
            hcsr.spmm(b, cc)
        s1.record(stream)
        torch.cuda.synchronize()
        cms = s0.elapsed_time(s1) / 5
        out["csr_spmm_baseline"] = {
            "kind": "own CSR x dense kernel on the same GPU, one wave per row and 512 columns, fp32 accumulation",
            "ms": cms, "nnz_tflops": flops_nnz / (cms * 1e-3) * 1e-12,
            "gathered_B_GBs": a["nnz"] * n * 2 / (cms * 1e-3) * 1e-9,
            "speedup_of_vbr_over_csr": cms / ms,
            "max_abs_diff_vs_vbr": float((cc - c).abs().max()),
        }
        del hcsr, cc

    if args.workload in ("c2", "c4") and not args.no_dense_baseline:
        # the dense product on the zero-filled matrix (the comparison the target config names): the
        # same hand-written tile kernel, A stored as one dense VBR (128-row groups, every block kept)
        m_rows, k_cols = a["n_rows"], a["n_cols"]
        dense = zero_filled(a)
        vd = binding.vbr_build(dense, np.arange(m_rows, dtype=np.int32),
                               np.arange(0, m_rows + 1, 128, dtype=np.int32), cb)
        del dense
        vd.upload(dev)
        cd = torch.empty_like(c)
        for _ in range(3):
            vd.spmm(b, cd)
        torch.cuda.synchronize()
        dense_ramp = clock_ramp(lambda: vd.spmm(b, cd), batch=20, budget_ms=1000.0)     # same steady-state clocks as the timed region
        d0 = torch.cuda.Event(enable_timing=True)
        d1 = torch.cuda.Event(enable_timing=True)
        d0.record(stream)
        for _ in range(10):
            vd.spmm(b, cd)
        d1.record(stream)
        torch.cuda.synchronize()
        dms = d0.elapsed_time(d1) / 10
        dfl = 2.0 * m_rows * k_cols * n
        out["dense_baseline"] = {
            "kind": "same tile kernel, zero-filled A stored as one dense VBR (groups of 128 rows, every block stored)",
            "ms": dms, "tflops": dfl / (dms * 1e-3) * 1e-12, "clock_ramp_launches": dense_ramp,
            "pct_mfma_fp16_peak": 100.0 * dfl / (dms * 1e-3) * 1e-12 / PEAK_MFMA_F16_TFLOPS,
            "speedup_of_vbr_over_dense": dms / ms,
            "max_abs_diff_vs_vbr": float((cd - c).abs().max()),
        }
        del vd, cd

    if not args.no_cpu_baseline:
        import oracle
        t = time.perf_counter()
        oracle.sa1(a, cb, tau)
        out["setup"]["oracle_sa1_reorder_s"] = time.perf_counter() - t
        # bounded sample: as many whole rows of the same workload as take roughly 10-20 s
        rows_all = np.arange(a["n_rows"])
        probe = rows_all[:: max(1, a["n_rows"] // 64)][:64]
        t = time.perf_counter()
        oracle.spmm(a, w["B"], rows=probe)
        dt = max(time.perf_counter() - t, 1e-4)   # includes the 16-bit -> binary64 conversion of B
        nnz_probe = int(np.diff(a["row_ptr"])[probe].sum())
        t = time.perf_counter()
        oracle.spmm(a, w["B"], rows=probe)
        dt = max(time.perf_counter() - t, 1e-4)
        per_nnz = dt / max(1, nnz_probe)
        target_nnz = 12.0 / per_nnz
        lens = np.diff(a["row_ptr"])
        k = int(np.searchsorted(np.cumsum(lens), target_nnz)) + 1
        sample = rows_all[: min(k, a["n_rows"])]
        t = time.perf_counter()
        oracle.spmm(a, w["B"], rows=sample)
        dt = time.perf_counter() - t
        nnz_s = int(lens[sample].sum())
        out["cpu_baseline"] = {
            "value": 2.0 * nnz_s * n / dt * 1e-12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "first %d of %d rows (%d nonzeros), fp64 C = A.B and bound |A|.|B| from CSR, OpenMP over rows, "
                      "%.1f s incl. 16-bit->fp64 conversion of B; flops counted as 2*nnz*N" % (
                          sample.size, a["n_rows"], nnz_s, dt),
        }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
