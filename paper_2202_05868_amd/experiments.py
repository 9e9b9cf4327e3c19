"""The two comparison experiments of the paper's section 4.4 on this GPU, with the library's own
kernels on both sides: the blocked multiply (1-SA blocking -> VBR -> ``vbr_spmm``) against the
multiply straight from CSR (``csr_spmm``, which stands where the sparse-library routine stands
in the paper).

``landscape``   section 4.4.2: synthetic blocked matrices A(Delta, theta, rho) over the grid of the
                paper's Table 2, rows scrambled, blocked with 1-SA for tau = 0.1 .. 1, the blocking
                whose average block height is nearest to Delta taken as the representative
                (sections 4.3.2, 4.4.2), multiplied by dense matrices of several widths.
``rmat_grid``   section 4.4.3: RMAT graphs of 2^14 nodes, 8 .. 128 edges per node, column blocks of
                64 / 128 / 256, dense width 2^12.  The paper states no threshold for this
                experiment; the same rule is used with the column-block width as the target
                height, and the fastest threshold of the sweep is reported beside it.

Both return plain dicts (``bench.py --landscape`` / ``--rmat-grid`` print them as one JSON line).
Inputs are drawn by ``synth``; everything else goes through the binding.  Needs the GPU.
"""
from __future__ import annotations

import time

import numpy as np

from . import binding, synth, torch_io

TAUS = [0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.7, 0.8, 0.9, 1.0]
THETAS = [0.01, 0.1, 0.2, 0.3, 0.4]                 # Table 2: fraction of nonzero blocks
RHOS = [0.01, 0.02, 0.05, 0.1, 0.2, 0.5]            # Table 2: in-block density


def _time_ms(fn, warm: int, reps: int) -> float:
    import torch
    stream = torch.cuda.current_stream()
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        fn()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _compare(a: dict, col_block: int, tau: float, b_full, widths, dev: str, reps: int) -> dict:
    """Block ``a`` at ``tau``, multiply by the first N columns of ``b_full`` for every N in
    ``widths`` with both kernels; returns times and the largest difference between the two results."""
    import torch
    perm, rg = binding.sa1_reorder(a, col_block, tau)
    v = binding.vbr_build(a, perm, rg, col_block).upload(dev)
    h = binding.CsrDev(a).upload(dev)
    ix = v.index()
    out = {"tau": tau, "groups": int(rg.size - 1), "blocks": int(ix["n_blocks"]),
           "fill_in": ix["stored_elems"] / max(1, a["nnz"]), "N": {}}
    for n in widths:
        b = b_full[:, :n]
        c1 = torch.empty((a["n_rows"], n), dtype=torch.float32, device=dev)
        c2 = torch.empty_like(c1)
        t_vbr = _time_ms(lambda: v.spmm(b, c1), 3, reps)
        t_csr = _time_ms(lambda: h.spmm(b, c2), 2, max(2, reps // 2))
        out["N"][str(n)] = {"vbr_ms": t_vbr, "csr_ms": t_csr, "speedup": t_csr / t_vbr,
                            "max_abs_diff": float((c1 - c2).abs().max())}
        del c1, c2
    v.close()
    h.close()
    return out


def landscape(n: int = 8192, delta: int = 64, widths=(2048, 4096, 8192), thetas=THETAS, rhos=RHOS,
              dev: str = "cuda:0", reps: int = 10, seed: int = 2024, progress=None) -> dict:
    rng = np.random.default_rng(seed)
    b_full = torch_io.bits_to_device(synth.dense_rhs(rng, n, max(widths), synth.F16), synth.F16, dev)
    points = []
    for theta in thetas:
        for rho in rhos:
            t0 = time.perf_counter()
            a = synth.landscape(rng, n, delta, theta, rho)
            t1 = time.perf_counter()
            cur = binding.sa1_blocking_curve(a, delta, TAUS, delta)
            t2 = time.perf_counter()
            sel = cur["selected"]
            pt = _compare(a, delta, TAUS[sel], b_full, widths, dev, reps)
            nb = int(cur["n_blocks"][sel])
            pt.update(theta=theta, rho=rho, nnz=int(a["nnz"]), density=a["nnz"] / float(n) / n,
                      avg_block_height=float(cur["sum_heights"][sel]) / max(1, nb),
                      rho_after=a["nnz"] / max(1, int(cur["stored_elems"][sel])),
                      generate_s=t1 - t0, blocking_curve_s=t2 - t1)
            points.append(pt)
            if progress:
                progress("landscape theta=%g rho=%g tau=%g height=%.1f rho'=%.3f speedup %s" % (
                    theta, rho, pt["tau"], pt["avg_block_height"], pt["rho_after"],
                    " ".join("N=%s:%.2f" % (k, x["speedup"]) for k, x in pt["N"].items())))
    return {"experiment": "blocked multiply vs CSR multiply over A(Delta, theta, rho), section 4.4.2",
            "n": n, "delta": delta, "taus": TAUS, "selection": "average block height nearest to delta", "points": points}


def rmat_grid(degrees=(8, 16, 32, 64, 128), col_blocks=(64, 128, 256), log2_nodes: int = 14, width: int = 4096,
              dev: str = "cuda:0", reps: int = 10, seed: int = 2025, progress=None) -> dict:
    rng = np.random.default_rng(seed)
    n = 1 << log2_nodes
    b_full = torch_io.bits_to_device(synth.dense_rhs(rng, n, width, synth.F16), synth.F16, dev)
    points = []
    for deg in degrees:
        a = synth.rmat(rng, log2_nodes, float(deg))
        for cb in col_blocks:
            cur = binding.sa1_blocking_curve(a, cb, TAUS, cb)
            sel = cur["selected"]
            runs = {}
            for tau in TAUS:
                runs[tau] = _compare(a, cb, tau, b_full, (width,), dev, reps)
            best = min(TAUS, key=lambda t: runs[t]["N"][str(width)]["vbr_ms"])
            pt = {"avg_degree_drawn": deg, "nnz": int(a["nnz"]), "col_block": cb,
                  "selected_by_height": runs[TAUS[sel]], "fastest": runs[best],
                  "avg_block_height_selected": float(cur["sum_heights"][sel]) / max(1, int(cur["n_blocks"][sel]))}
            points.append(pt)
            if progress:
                progress("rmat degree=%d col_block=%d: rule tau=%g speedup %.2f | fastest tau=%g speedup %.2f (fill-in %.1f)" % (
                    deg, cb, TAUS[sel], runs[TAUS[sel]]["N"][str(width)]["speedup"], best,
                    runs[best]["N"][str(width)]["speedup"], runs[best]["fill_in"]))
    return {"experiment": "blocked multiply vs CSR multiply on RMAT graphs, section 4.4.3", "nodes": n, "N": width,
            "taus": TAUS, "points": points}


def landscape_table(res: dict) -> str:
    """The landscape result as a text table (what is kept under profiles/)."""
    widths = [k for k in res["points"][0]["N"]]
    out = ["# Blocked multiply (1-SA -> VBR -> vbr_spmm) against the CSR multiply (csr_spmm) over the synthetic landscape",
           "# A(Delta=%d, theta, rho), %d x %d, rows scrambled, tau of the blocking whose average block height is nearest to Delta" % (
               res["delta"], res["n"], res["n"]),
           "# (paper: section 4.4.2, Table 2).  fp16 -> fp32.  x = csr_ms / vbr_ms per dense width N.",
           "command: python bench.py --landscape",
           "",
           "%-6s %-5s %9s %4s %8s %7s %8s" % ("theta", "rho", "nnz", "tau", "height", "rho'", "fill-in") +
           "".join(" | N=%-5s vbr ms  csr ms      x" % n for n in widths)]
    for p in res["points"]:
        line = "%-6g %-5g %9d %4g %8.1f %7.3f %8.2f" % (p["theta"], p["rho"], p["nnz"], p["tau"], p["avg_block_height"],
                                                        p["rho_after"], p["fill_in"])
        for n in widths:
            x = p["N"][n]
            line += " | %14.3f %7.3f %6.2f" % (x["vbr_ms"], x["csr_ms"], x["speedup"])
        out.append(line)
    out.append("")
    out.append("largest |C_vbr - C_csr| over all points: %.3g" % max(x["max_abs_diff"] for p in res["points"] for x in p["N"].values()))
    return "\n".join(out) + "\n"


def rmat_table(res: dict) -> str:
    n = str(res["N"])
    out = ["# Blocked multiply against the CSR multiply on RMAT graphs (0.57, 0.19, 0.19, 0.05), %d nodes, rows scrambled," % res["nodes"],
           "# dense width N = %s (paper: section 4.1 Table 2, section 4.4.3).  The paper states no threshold for this experiment:" % n,
           "# 'rule' = the tau of {0.1 .. 1} whose average block height is nearest to the column-block width, 'fastest' = the tau",
           "# of the sweep with the shortest blocked multiply.  fp16 -> fp32.  x = csr_ms / vbr_ms.",
           "command: python bench.py --rmat-grid",
           "",
           "%-7s %9s %-6s | %-4s %8s %8s %8s %6s | %-4s %8s %8s %6s" % ("degree", "nnz", "Dw", "tau", "fill-in", "vbr ms", "csr ms", "x",
                                                                          "tau", "fill-in", "vbr ms", "x")]
    for p in res["points"]:
        a, b = p["selected_by_height"], p["fastest"]
        xa, xb = a["N"][n], b["N"][n]
        out.append("%-7d %9d %-6d | %-4g %8.1f %8.3f %8.3f %6.2f | %-4g %8.1f %8.3f %6.2f" % (
            p["avg_degree_drawn"], p["nnz"], p["col_block"], a["tau"], a["fill_in"], xa["vbr_ms"], xa["csr_ms"], xa["speedup"],
            b["tau"], b["fill_in"], xb["vbr_ms"], xb["speedup"]))
    return "\n".join(out) + "\n"
