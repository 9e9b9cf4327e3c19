"""Collect the rocprofv3 evidence behind one ``bench.py`` line and write the short text summary
that is kept under ``profiles/``.

    python -m paper_2202_05868_amd.rocprof_summary --workload c4 --out gpurun_out/prof_c4

Runs, one after the other, each as its own process and under its own time limit:

  1. ``rocprofv3 --kernel-trace --stats``  on  ``python3 bench.py --workload W --timed-only``
  2. ``rocprofv3 --pmc FETCH_SIZE``        on the same command with ``--no-ramp --steps 5 --warmup 2 --calib-copy``
  3. ``rocprofv3 --pmc WRITE_SIZE``        likewise
  4. ``rocprofv3 --pmc SQ_BUSY_CU_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_WAVE_CYCLES SQ_LDS_BANK_CONFLICT``  likewise
  5. ``rocprofv3 --pmc TA_BUSY_avr SQ_BUSY_CU_CYCLES SQ_INSTS_VMEM_RD SQ_WAIT_ANY SQ_WAVE_CYCLES``  likewise

and writes ``<out>/summary.txt``.  The kernel trace holds every dispatch of the run: the launches
that let the clocks settle, the warm-up and the timed steps.  The summary therefore gives the
average over the dispatches of the TIMED steps (the last ``steps`` calls) beside the average over
all dispatches, and the ``ms_per_step`` the benchmark printed in that same run.  HBM bytes are the
counters scaled by what they read for a plain 256 MiB streaming kernel in the same process.
This process never touches the GPU itself; the profiled program is the one named after ``--``.
"""
from __future__ import annotations

import argparse
import json
import os
import sqlite3
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = 256 * 1024 * 1024


def run(cmd, log, limit):
    print("[rocprof_summary] " + " ".join(cmd), flush=True)
    env = dict(os.environ, TMPDIR="/tmp")
    with open(log, "w") as f:
        rc = subprocess.run(["timeout", "-s", "KILL", str(limit)] + cmd, cwd="/tmp", env=env, stdout=subprocess.PIPE,
                            stderr=f, text=True)
    if rc.returncode != 0:
        raise SystemExit("pass failed (%d): see %s" % (rc.returncode, log))
    lines = [ln for ln in rc.stdout.splitlines() if ln.startswith("{")]
    return json.loads(lines[-1]) if lines else None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c4")
    ap.add_argument("--clean", action="store_true")
    ap.add_argument("--dense", action="store_true", help="the dense product on the zero-filled matrix (bench.py --dense)")
    ap.add_argument("--out", required=True)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--no-counters", action="store_true", help="kernel trace only")
    args = ap.parse_args()
    out_dir = os.path.abspath(args.out)
    os.makedirs(out_dir, exist_ok=True)
    bench = ["python3", os.path.join(ROOT, "bench.py"), "--workload", args.workload, "--timed-only"]
    flags = (" --clean" if args.clean else "") + (" --dense" if args.dense else "")
    bench += flags.split()
    shown = "python3 bench.py --workload %s --timed-only%s" % (args.workload, flags)
    pmc_tail = ["--no-ramp", "--steps", "5", "--warmup", "2", "--calib-copy"]
    text = ["# rocprofv3 summary: vbr_spmm on workload %s%s (MI355X, gfx950)" % (
                args.workload, (" (noise-free)" if args.clean else "") + (" stored zero-filled: the dense product" if args.dense else "")),
            "",
            "made by             : python -m paper_2202_05868_amd.rocprof_summary --workload %s%s --out <out>" % (
                args.workload, flags),
            "kernel trace command: cd /tmp && export TMPDIR=/tmp && rocprofv3 --kernel-trace --stats -d <out>/trace -o t -- %s --steps %d" % (shown, args.steps)]

    bj = run(["rocprofv3", "--kernel-trace", "--stats", "-d", os.path.join(out_dir, "trace"), "-o", "t", "--"] + bench +
             ["--steps", str(args.steps)], os.path.join(out_dir, "trace.err"), 400)
    con = sqlite3.connect(os.path.join(out_dir, "trace", "t_results.db"))
    rows = con.execute("select name, start, end from kernels where name like '%vbr_spmm%' order by start").fetchall()
    per_step = len(bj["roofline"]["kernel"])
    timed = rows[-args.steps * per_step:] if per_step else []
    text += ["", "## kernel trace: per kernel, dispatches / average us, over ALL dispatches of the run and over the",
             "## dispatches of the %d timed steps (the last %d dispatches)" % (args.steps, len(timed))]
    names = []
    for r in rows:
        if r[0] not in names:
            names.append(r[0])
    step_us = 0.0
    for nm in names:
        all_d = [(e - s) / 1e3 for k, s, e in rows if k == nm]
        tim_d = [(e - s) / 1e3 for k, s, e in timed if k == nm]
        short = nm[nm.find("vbr_spmm"):][:70]
        text.append("  %-70s all %5d / %9.3f us    timed %4d / %9.3f us" % (
            short, len(all_d), sum(all_d) / len(all_d), len(tim_d), sum(tim_d) / max(1, len(tim_d))))
        step_us += sum(tim_d) / max(1, args.steps)
    text.append("  kernel time per timed step (sum over its launches): %.3f us" % step_us)
    if per_step > 1:
        spans = [max(e for _, _, e in timed[i:i + per_step]) - min(b for _, b, _ in timed[i:i + per_step])
                 for i in range(0, len(timed), per_step)]
        text.append("  the launches of one call run side by side (the first on the caller's stream, the others on the handle's own")
        text.append("  streams), so their durations overlap: first start to last end of a timed step, average %.3f us" % (
            sum(spans) / len(spans) / 1e3))
    text.append("bench.py in the same run: ms_per_step %.4f (HIP events around the %d timed steps), value %.1f %s, clock-ramp launches %d" % (
        bj["ms_per_step"], args.steps, bj["value"], bj["unit"], bj["clock_ramp_launches"]))
    text.append("(under the profiler every dispatch is followed by a completion signal, so the GPU idles between launches and")
    text.append(" its clocks settle lower than in an unprofiled run; compare with the ms_per_step of this run, not of another)")

    if not args.no_counters:
        res, spmm_sum = {}, {}
        for tag, sub in (("FETCH_SIZE", "fetch"), ("WRITE_SIZE", "write")):
            run(["rocprofv3", "--pmc", tag, "-d", os.path.join(out_dir, sub), "-o", "p", "--"] + bench + pmc_tail,
                os.path.join(out_dir, sub + ".err"), 180)
            con = sqlite3.connect(os.path.join(out_dir, sub, "p_results.db"))
            q = con.execute("select kernel_name, avg(value), count(*) from counters_collection where counter_name=? "
                            "group by kernel_name", (tag,)).fetchall()
            text += ["", "## %s (KiB per dispatch, average over dispatches): rocprofv3 --pmc %s -d <out>/%s -o p -- %s %s" % (
                tag, tag, sub, shown, " ".join(pmc_tail))]
            spmm_sum[tag] = 0.0
            for k, val, cnt in q:
                if "vbr_spmm" in k:
                    text.append("  %-70s %14.1f KiB (n=%d)" % (k[k.find("vbr_spmm"):][:70], val, cnt))
                    spmm_sum[tag] += val
                elif "elementwise" in k and "Fill" not in k:
                    text.append("  %-70s %14.1f KiB (n=%d)" % ("256 MiB streaming kernel (torch.mul out=)", val, cnt))
                    res[tag] = val
        if "FETCH_SIZE" in res and "WRITE_SIZE" in res:
            sf = COPY_BYTES / (res["FETCH_SIZE"] * 1024)
            sw = COPY_BYTES / (res["WRITE_SIZE"] * 1024)
            fb = spmm_sum["FETCH_SIZE"] * 1024 * sf
            wb = spmm_sum["WRITE_SIZE"] * 1024 * sw
            text += ["", "calibration: the streaming kernel reads 256 MiB and writes 256 MiB -> scale factors %.4f (fetch), %.4f (write)" % (sf, sw),
                     "vbr_spmm FETCH_SIZE per call (all its launches): %.1f MB scaled" % (fb / 1e6),
                     "vbr_spmm WRITE_SIZE per call (all its launches): %.1f MB scaled" % (wb / 1e6),
                     "HBM traffic per launch: %.1f MB (algorithmic: %.1f MB)" % ((fb + wb) / 1e6, bj["roofline"]["algorithmic_hbm_bytes"] / 1e6)]
        ctrs = ["SQ_BUSY_CU_CYCLES", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_WAVE_CYCLES", "SQ_LDS_BANK_CONFLICT"]
        run(["rocprofv3", "--pmc"] + ctrs + ["-d", os.path.join(out_dir, "mfma"), "-o", "p", "--"] + bench + pmc_tail[:-1],
            os.path.join(out_dir, "mfma.err"), 180)
        con = sqlite3.connect(os.path.join(out_dir, "mfma", "p_results.db"))
        q = con.execute("select kernel_name, counter_name, avg(value), count(*) from counters_collection "
                        "where kernel_name like '%vbr_spmm%' group by kernel_name, counter_name").fetchall()
        text += ["", "## matrix-unit and LDS counters (per dispatch, average): rocprofv3 --pmc %s -d <out>/mfma -o p -- %s %s" % (
            " ".join(ctrs), shown, " ".join(pmc_tail[:-1]))]
        per = {}
        for k, c, val, cnt in q:
            text.append("  %-60s %-28s %16.1f (n=%d)" % (k[k.find("vbr_spmm"):][:60], c, val, cnt))
            per.setdefault(k, {})[c] = val
        for k, cs in per.items():
            if cs.get("SQ_BUSY_CU_CYCLES"):
                text.append("  -> MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x SQ_BUSY_CU_CYCLES) = %.1f %%  (%s)" % (
                    100.0 * cs.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / (4.0 * cs["SQ_BUSY_CU_CYCLES"]), k[k.find("vbr_spmm"):][:50]))
        # the load path: how busy the texture-address unit is (every direct-to-LDS load goes through it)
        ctrs = ["TA_BUSY_avr", "SQ_BUSY_CU_CYCLES", "SQ_INSTS_VMEM_RD", "SQ_WAIT_ANY", "SQ_WAVE_CYCLES"]
        run(["rocprofv3", "--pmc"] + ctrs + ["-d", os.path.join(out_dir, "ta"), "-o", "p", "--"] + bench + pmc_tail[:-1],
            os.path.join(out_dir, "ta.err"), 180)
        con = sqlite3.connect(os.path.join(out_dir, "ta", "p_results.db"))
        q = con.execute("select kernel_name, counter_name, avg(value), count(*) from counters_collection "
                        "where kernel_name like '%vbr_spmm%' group by kernel_name, counter_name").fetchall()
        text += ["", "## load path (per dispatch, average): rocprofv3 --pmc %s -d <out>/ta -o p -- %s %s" % (
            " ".join(ctrs), shown, " ".join(pmc_tail[:-1]))]
        per = {}
        for k, c, val, cnt in q:
            text.append("  %-60s %-28s %16.1f (n=%d)" % (k[k.find("vbr_spmm"):][:60], c, val, cnt))
            per.setdefault(k, {})[c] = val
        for k, cs in per.items():
            if cs.get("SQ_BUSY_CU_CYCLES") and cs.get("SQ_INSTS_VMEM_RD"):
                per_cu = cs["SQ_BUSY_CU_CYCLES"] / 256.0
                text.append("  -> TA busy %.0f %% of the kernel's cycles (TA_BUSY_avr / (SQ_BUSY_CU_CYCLES / 256 CUs)); %.1f busy cycles and "
                            "%.1f kernel cycles per vector-memory load instruction and CU; waves waiting %.0f %% of their time  (%s)" % (
                                100.0 * cs.get("TA_BUSY_avr", 0.0) / per_cu, cs.get("TA_BUSY_avr", 0.0) * 256.0 / cs["SQ_INSTS_VMEM_RD"],
                                cs["SQ_BUSY_CU_CYCLES"] / cs["SQ_INSTS_VMEM_RD"],
                                100.0 * cs.get("SQ_WAIT_ANY", 0.0) / max(1.0, cs.get("SQ_WAVE_CYCLES", 1.0)), k[k.find("vbr_spmm"):][:50]))
    with open(os.path.join(out_dir, "summary.txt"), "w") as f:
        f.write("\n".join(text) + "\n")
    print("\n".join(text))
    return 0


if __name__ == "__main__":
    sys.exit(main())
