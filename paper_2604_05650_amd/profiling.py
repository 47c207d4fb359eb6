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
    "visual_relevance": ("gemm_stream_kernel<0", "rel_finalize_kernel", "rel_cand_kernel",
                         "rel_merge_kernel"),
    "lm_head_accept": ("gemm_stream_kernel<1", "accept_finalize_kernel", "accept_decide_kernel"),
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


if __name__ == "__main__":
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
