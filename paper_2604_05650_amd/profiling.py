"""Turn a rocprofv3 result database (rocpd SQLite, the default output of rocprofv3 7.x) into the
short text summaries kept under profiles/.

    python -m paper_2604_05650_amd.profiling kernels  <results.db>
    python -m paper_2604_05650_amd.profiling counters <results.db> <COUNTER>

`kernels`  : calls / average / min / max duration per kernel (what --kernel-trace --stats shows).
`counters` : per-kernel average of one hardware counter per dispatch (from a --pmc run), plus the
             same counter for the 1 GiB + 1 GiB calibration kernel of `bench.py --calibrate-copy`.

    python -m paper_2604_05650_amd.profiling traffic <fetch.db> <write.db> <workload name>

    python -m paper_2604_05650_amd.profiling mfma <results.db>

`mfma`     : matrix-core use per kernel from a run with
             --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 GRBM_GUI_ACTIVE:
             executed bf16 MFMA flops (MOPS x 512) per launch, the rate over the kernel's
             duration as a fraction of the 2.5 PFLOP/s dense bf16 peak, and the share of
             SIMD-cycles the MFMA unit was busy (256 CUs x 4 SIMDs at 2.4 GHz).

    python -m paper_2604_05650_amd.profiling summary <dir with the runs> <out dir> <workload> ...

`summary`  : the text files kept under profiles/ for the named workloads, from the result
             databases and bench.py lines of `profiles/README.md`'s commands (kt_<w>, fetch_<w>,
             write_<w>, mfma_<w>), and traffic.json: the per-call HBM bytes and matrix-core
             figures bench.py replays, stamped with the commit, the library version and the
             launch plan of every workload they were taken at.

`traffic`  : HBM bytes per library call from a FETCH_SIZE run and a WRITE_SIZE run of
             `bench.py --calibrate-copy`: each counter is scaled by what it reads for the
             calibration kernel (which moves exactly 1 GiB each way); printed as the JSON that
             bench.py loads from profiles/traffic.json.
"""
from __future__ import annotations

import re
import sqlite3
import sys


def _short(name: str) -> str:
    m = re.search(r"(\w+_kernel(<[^>]*>)?)", name)
    return (m.group(1) if m else name)[:72]


def kernels(db_path: str) -> str:
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute(
        "select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
        "from kernels group by name order by sum(end-start) desc").fetchall()
    tot = sum(r[5] for r in rows) or 1
    out = [f"{'kernel':72s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'time%':>6s}"]
    for n, c, a, mi, ma, s in rows:
        out.append(f"{_short(n):72s} {c:6d} {a / 1e3:9.2f} {mi / 1e3:9.2f} {ma / 1e3:9.2f} "
                   f"{100 * s / tot:6.1f}")
    return "\n".join(out)


def counters(db_path: str, counter: str) -> str:
    con = sqlite3.connect(db_path)
    cur = con.cursor()
    cols = [r[1] for r in cur.execute("pragma table_info(counters_collection)")]
    name_col = "kernel_name" if "kernel_name" in cols else "name"
    rows = cur.execute(
        f"select {name_col}, count(*), avg(value), min(value), max(value) from counters_collection "
        "where counter_name = ? group by 1 order by avg(value) desc", (counter,)).fetchall()
    out = [f"counter {counter} per dispatch",
           f"{'kernel':72s} {'calls':>6s} {'avg':>14s} {'min':>14s} {'max':>14s}"]
    for n, c, a, mi, ma in rows:
        out.append(f"{_short(n):72s} {c:6d} {a:14.1f} {mi:14.1f} {ma:14.1f}")
    return "\n".join(out)


MFMA_PEAK_BF16 = 2.5e15     # MI355X dense bf16, FLOP/s
SIMDS = 256 * 4
CLOCK_HZ = 2.4e9


def mfma_table(db_path: str) -> list:
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute(
        "select kernel_name, counter_name, avg(value), avg(duration), count(*) "
        "from counters_collection group by 1, 2").fetchall()
    per = {}
    for n, c, v, d, k in rows:
        e = per.setdefault(n, {"calls": k, "dur_ns": d})
        e[c] = v
    out = []
    for n, e in per.items():
        mops = e.get("SQ_INSTS_VALU_MFMA_MOPS_BF16", 0.0)
        if mops <= 0:
            continue
        flops = mops * 512.0
        dur = e["dur_ns"] * 1e-9
        busy = e.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / (dur * CLOCK_HZ * SIMDS)
        out.append({"kernel": _short(n), "calls": e["calls"], "avg_us": e["dur_ns"] / 1e3,
                    "mfma_flops_per_launch": flops, "tflops": flops / dur / 1e12,
                    "frac_of_bf16_peak": flops / dur / MFMA_PEAK_BF16, "mfma_busy_frac": busy})
    return sorted(out, key=lambda r: -r["mfma_flops_per_launch"] * r["calls"])


def mfma(db_path: str) -> str:
    out = [f"{'kernel':44s} {'calls':>6s} {'avg_us':>9s} {'GFLOP/launch':>13s} {'TFLOP/s':>9s} "
           f"{'of 2.5 PF':>10s} {'MFMA busy':>10s}"]
    for r in mfma_table(db_path):
        out.append(f"{r['kernel'][:44]:44s} {r['calls']:6d} {r['avg_us']:9.2f} "
                   f"{r['mfma_flops_per_launch'] / 1e9:13.3f} {r['tflops']:9.1f} "
                   f"{100 * r['frac_of_bf16_peak']:9.2f}% {100 * r['mfma_busy_frac']:9.2f}%")
    return "\n".join(out)


GROUPS = {   # kernels launched by one call of each entry point
    "verify_attn": ("attn_split_kernel", "attn_combine_kernel"),
    "visual_relevance": ("gemm_stream_kernel<0", "gemm_stream_kernel<2", "rel_finalize_kernel",
                         "rel_cand_kernel", "rel_merge_kernel"),
    "lm_head_accept": ("gemm_stream_kernel<1", "accept_finalize_kernel",
                       "accept_finalize_general_kernel", "accept_decide_kernel"),
}
CALIBRATION_KERNEL = "CUDAFunctorOnSelf_add<int>"
GIB = float(1 << 30)


def _avg_by_kernel(db_path: str, counter: str) -> dict:
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select kernel_name, avg(value) from counters_collection "
                       "where counter_name = ? group by 1", (counter,)).fetchall()
    return {n: v for n, v in rows}


def traffic(fetch_db: str, write_db: str, workload: str) -> str:
    import json
    fetch = _avg_by_kernel(fetch_db, "FETCH_SIZE")
    write = _avg_by_kernel(write_db, "WRITE_SIZE")
    cal_f = next(v for n, v in fetch.items() if CALIBRATION_KERNEL in n)
    cal_w = next(v for n, v in write.items() if CALIBRATION_KERNEL in n)
    res = {"calibration": {"kernel": "torch.add on 2^28 int32 (reads 1 GiB, writes 1 GiB)",
                           "FETCH_SIZE_reading": cal_f, "WRITE_SIZE_reading": cal_w,
                           "bytes_per_FETCH_SIZE_unit": GIB / cal_f,
                           "bytes_per_WRITE_SIZE_unit": GIB / cal_w}}
    per = {}
    detail = {}
    for call, kerns in GROUPS.items():
        tot = 0.0
        for k in kerns:
            f = sum(v for n, v in fetch.items() if k in n) * GIB / cal_f
            w = sum(v for n, v in write.items() if k in n) * GIB / cal_w
            detail[k] = {"fetch_bytes": round(f), "write_bytes": round(w)}
            tot += f + w
        per[call] = round(tot)
    res[workload] = per
    res[workload + ":kernels"] = detail
    return json.dumps(res, indent=1)


def _own(text: str, keep_add: bool = False) -> str:
    """drop torch's input-generation kernels from a listing"""
    return "\n".join(l for l in text.split("\n")
                     if ("at::native" not in l or (keep_add and CALIBRATION_KERNEL in l))
                     and "rocclr" not in l)


def summary(run_dir: str, out_dir: str, workloads: list) -> None:
    import json
    import os
    import subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    try:
        commit = subprocess.run(["git", "-C", here, "rev-parse", "--short", "HEAD"],
                                capture_output=True, text=True).stdout.strip() or None
    except OSError:
        commit = None
    commit = commit or os.environ.get("LVSPEC_COMMIT") or None   # a box without the .git folder
    tpath = os.path.join(out_dir, "traffic.json")
    tr = json.load(open(tpath)) if os.path.exists(tpath) else {}
    stamp = {"commit": commit, "library_version": None, "plans": dict(tr.get("stamp", {}).get("plans", {}))}
    tr = {k: v for k, v in tr.items() if k != "stamp"}
    for w in workloads:
        bench = json.loads(open(os.path.join(run_dir, f"kt_{w}.json")).read().strip().splitlines()[-1])
        name = bench["config"]["workload"]
        flags = f"--workload {w} --only --no-cpu-baseline"
        db = lambda kind: os.path.join(run_dir, f"{kind}_{w}_results.db")
        roof = "\n".join(f"  {k}: avg {v['avg_us']} us per call (median {v['median_us']}, min {v['min_us']}), "
                         f"{v['achieved']} GB/s algorithmic = {v['frac']} of 8 TB/s"
                         for k, v in bench["rooflines"].items())
        open(os.path.join(out_dir, f"kernel_trace_{w}.txt"), "w").write(
            f"rocprofv3 kernel trace, workload {name} (bench.py {flags}), MI355X, one GPU, commit {commit}.\n\n"
            "Command (run from /tmp with TMPDIR=/tmp, repository at $R):\n"
            f"  rocprofv3 --kernel-trace --stats -d <out> -o kt_{w} -- python3 $R/bench.py {flags} --steps 10 --warmup 3\n"
            "Summary made with:\n"
            f"  python -m paper_2604_05650_amd.profiling summary <out> profiles {w}\n"
            "(torch's input-generation kernels removed from the listing; durations in microseconds)\n\n"
            + _own(kernels(db("kt"))) + "\n\n"
            "bench.py line of the same run (HIP-event timing inside the timed region; the profiler's per-launch\n"
            "bookkeeping adds several microseconds between kernels, so a workload made of many short launches reads\n"
            "slower here than without the profiler; the unprofiled per-call figures are in the last lines):\n"
            f"  ms_per_step {bench['ms_per_step']}  tokens/s {bench['value']}\n" + roof + "\n"
            + _unprofiled(run_dir, w))
        t = json.loads(traffic(db("fetch"), db("write"), name))
        tr["calibration"] = t["calibration"]
        tr[name] = t[name]
        tr[name + ":kernels"] = t[name + ":kernels"]
        ratio = "\n".join(
            f"  {k}: measured {t[name][k]:,} B, algorithmic {bench['rooflines'][k]['algorithmic_bytes']:,} B, "
            f"ratio {t[name][k] / bench['rooflines'][k]['algorithmic_bytes']:.3f}" for k in t[name])
        open(os.path.join(out_dir, f"hbm_counters_{w}.txt"), "w").write(
            f"rocprofv3 HBM byte counters, workload {name} (bench.py {flags}), MI355X, one GPU, commit {commit}.\n\n"
            "Commands (run from /tmp with TMPDIR=/tmp, repository at $R; one counter per run):\n"
            f"  rocprofv3 --pmc FETCH_SIZE -d <out> -o fetch_{w} -- python3 $R/bench.py {flags} --steps 3 --warmup 1 --calibrate-copy\n"
            f"  rocprofv3 --pmc WRITE_SIZE -d <out> -o write_{w} -- python3 $R/bench.py {flags} --steps 3 --warmup 1 --calibrate-copy\n"
            "Summary made with:\n"
            f"  python -m paper_2604_05650_amd.profiling summary <out> profiles {w}\n\n"
            "Calibration: the elementwise kernel CUDAFunctorOnSelf_add<int> (torch.add on 2^28 int32) reads exactly 1 GiB and\n"
            f"writes exactly 1 GiB; its readings give {t['calibration']['bytes_per_FETCH_SIZE_unit']:.1f} bytes per FETCH_SIZE unit and\n"
            f"{t['calibration']['bytes_per_WRITE_SIZE_unit']:.1f} bytes per WRITE_SIZE unit.  (torch input-generation kernels removed.)\n\n"
            + _own(counters(db("fetch"), "FETCH_SIZE"), True) + "\n\n"
            + _own(counters(db("write"), "WRITE_SIZE"), True) + "\n\n"
            "HBM bytes per library call (fetch + write, scaled) vs algorithmic bytes:\n" + ratio + "\n")
        tab = mfma_table(db("mfma"))
        key = {"verify_attn": "attn_split_kernel", "visual_relevance": "gemm_stream_kernel<0",
               "lm_head_accept": "gemm_stream_kernel<1"}
        tr[name + ":mfma"] = {
            k: {"kernel": r["kernel"], "mfma_flops_per_launch": round(r["mfma_flops_per_launch"]),
                "frac_of_bf16_peak": round(r["frac_of_bf16_peak"], 4),
                "mfma_busy_frac": round(r["mfma_busy_frac"], 4)}
            for k, pref in key.items() for r in tab if r["kernel"].startswith(pref)}
        open(os.path.join(out_dir, f"mfma_counters_{w}.txt"), "w").write(
            f"rocprofv3 matrix-core counters, workload {name} (bench.py {flags}), MI355X, one GPU, commit {commit}.\n\n"
            "Command (run from /tmp with TMPDIR=/tmp, repository at $R):\n"
            f"  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 GRBM_GUI_ACTIVE -d <out> -o mfma_{w} -- python3 $R/bench.py {flags} --steps 3 --warmup 1\n"
            "Summary made with:\n"
            f"  python -m paper_2604_05650_amd.profiling summary <out> profiles {w}\n"
            "GFLOP/launch = SQ_INSTS_VALU_MFMA_MOPS_BF16 x 512 (executed, padding rows included); TFLOP/s over the kernel's\n"
            "duration in the same run; \"of 2.5 PF\" = fraction of the dense bf16 MFMA peak; \"MFMA busy\" =\n"
            "SQ_VALU_MFMA_BUSY_CYCLES / (duration x 2.4 GHz x 1024 SIMDs).  All three kernels are HBM-bound: the matrix cores\n"
            "are needed to stay under the HBM roof, not to fill it.\n\n" + mfma(db("mfma")) + "\n")
        if os.path.exists(db("lds")):
            open(os.path.join(out_dir, f"lds_counters_{w}.txt"), "w").write(
                f"rocprofv3 LDS counters, workload {name} (bench.py {flags}), MI355X, one GPU, commit {commit}.\n\n"
                "Command (run from /tmp with TMPDIR=/tmp, repository at $R):\n"
                f"  rocprofv3 --pmc {' '.join(LDS_COUNTERS)} -d <out> -o lds_{w} -- python3 $R/bench.py {flags} --steps 3 --warmup 1\n"
                "Summary made with:\n"
                f"  python -m paper_2604_05650_amd.profiling summary <out> profiles {w}\n"
                "Per launch, summed over the chip: LDS instructions issued, cycles the LDS index unit was active, cycles\n"
                "lost to bank conflicts and their share of the active cycles.  Tiles are stored with the 16-byte chunks\n"
                "of a row XOR-permuted by a key of the row index, so that the rows of an MFMA operand read fall into\n"
                "different banks; direct-to-LDS copies write whole 1 KiB lines.\n\n" + lds(db("lds")) + "\n")
        stamp["plans"][name] = bench["plan"]
        stamp["library_version"] = bench.get("library_version")
    tr["stamp"] = stamp
    json.dump(tr, open(tpath, "w"), indent=1)


LDS_COUNTERS = ("SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE", "SQ_LDS_ADDR_CONFLICT", "SQ_INSTS_LDS",
                "SQ_ACTIVE_INST_LDS", "SQ_WAIT_INST_LDS")


def lds(db_path: str) -> str:
    """LDS use per kernel from a run with --pmc <LDS_COUNTERS>: cycles the LDS spent on bank
    conflicts as a share of its active cycles, per launch."""
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select kernel_name, counter_name, avg(value), count(*) "
                       "from counters_collection group by 1, 2").fetchall()
    per = {}
    for n, c, v, k in rows:
        per.setdefault(n, {"calls": k})[c] = v
    out = [f"{'kernel':44s} {'calls':>6s} {'LDS instr':>12s} {'active cyc':>13s} {'conflict cyc':>13s} "
           f"{'conflict %':>10s} {'addr confl':>11s}"]
    for n, e in sorted(per.items(), key=lambda kv: -kv[1].get("SQ_LDS_IDX_ACTIVE", 0.0)):
        act = e.get("SQ_LDS_IDX_ACTIVE", 0.0)
        if act <= 0 or "at::native" in n or "rocclr" in n:
            continue
        bc = e.get("SQ_LDS_BANK_CONFLICT", 0.0)
        out.append(f"{_short(n)[:44]:44s} {e['calls']:6d} {e.get('SQ_INSTS_LDS', 0.0):12.0f} {act:13.0f} "
                   f"{bc:13.0f} {100.0 * bc / act:9.2f}% {e.get('SQ_LDS_ADDR_CONFLICT', 0.0):11.0f}")
    return "\n".join(out)


def _unprofiled(run_dir: str, w: str) -> str:
    """per-call figures of the same command without the profiler, when that run is there"""
    import json
    import os
    path = os.path.join(run_dir, f"plain_{w}.json")
    if not os.path.exists(path):
        return ""
    b = json.loads(open(path).read().strip().splitlines()[-1])
    return ("\nThe same command without the profiler (HIP events around each call, median of "
            f"{b['steps']} steps):\n  ms_per_step {b['ms_per_step']}\n" + "\n".join(
                f"  {k}: median {v['median_us']} us per call, min {v['min_us']}, {v['frac']} of 8 TB/s"
                for k, v in b["rooflines"].items()) + "\n")


if __name__ == "__main__":
    if len(sys.argv) >= 5 and sys.argv[1] == "summary":
        summary(sys.argv[2], sys.argv[3], sys.argv[4:])
        sys.exit(0)
    if len(sys.argv) >= 5 and sys.argv[1] == "traffic":
        print(traffic(sys.argv[2], sys.argv[3], sys.argv[4]))
        sys.exit(0)
    if len(sys.argv) >= 3 and sys.argv[1] == "mfma":
        print(mfma(sys.argv[2]))
        sys.exit(0)
    if len(sys.argv) >= 3 and sys.argv[1] == "kernels":
        print(kernels(sys.argv[2]))
    elif len(sys.argv) >= 4 and sys.argv[1] == "counters":
        print(counters(sys.argv[2], sys.argv[3]))
    else:
        print(__doc__)
        sys.exit(2)
