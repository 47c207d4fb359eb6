"""The profiling helper turns a rocprofv3 result database into the short text kept under
profiles/: checked here on a small hand-made database with the same tables."""
import json
import sqlite3

from paper_2604_05650_amd import profiling as P


def _db(path, kernels=(), counters=()):
    con = sqlite3.connect(path)
    con.execute("create table kernels (name text, start integer, end integer)")
    con.executemany("insert into kernels values (?, ?, ?)", kernels)
    con.execute("create table counters_collection (kernel_name text, counter_name text, "
                "value real, duration integer)")
    con.executemany("insert into counters_collection values (?, ?, ?, ?)", counters)
    con.commit()
    con.close()


SPLIT = "void lvspec::(anonymous namespace)::attn_split_kernel<2, 1>(lvspec::AttnKernelArgs)"
COMB = "void lvspec::(anonymous namespace)::attn_combine_kernel<1, 2>(lvspec::AttnKernelArgs)"
ADD = "void at::native::vectorized_elementwise_kernel<4, at::native::CUDAFunctorOnSelf_add<int>, x>"


def test_kernel_table(tmp_path):
    db = str(tmp_path / "k.db")
    _db(db, kernels=[(SPLIT, 0, 16000), (SPLIT, 20000, 38000), (COMB, 40000, 43000)])
    txt = P.kernels(db)
    rows = {l.split()[0] + l.split()[1]: l.split() for l in txt.splitlines()[1:]}
    split = next(v for k, v in rows.items() if k.startswith("attn_split_kernel"))
    assert split[-5:] == ["2", "17.00", "16.00", "18.00", "91.9"]


def test_traffic_is_scaled_by_the_copy_kernel(tmp_path):
    f, w = str(tmp_path / "f.db"), str(tmp_path / "w.db")
    # the calibration kernel moves 1 GiB each way: 524288 fetch units of 2 KiB, 1048576 write
    # units of 1 KiB; the split kernel reads 32768 fetch units = 64 MiB and writes 4 MiB
    _db(f, counters=[(ADD, "FETCH_SIZE", 524288.0, 1), (SPLIT, "FETCH_SIZE", 32768.0, 1),
                     (COMB, "FETCH_SIZE", 2048.0, 1)])
    _db(w, counters=[(ADD, "WRITE_SIZE", 1048576.0, 1), (SPLIT, "WRITE_SIZE", 4096.0, 1),
                     (COMB, "WRITE_SIZE", 50.0, 1)])
    t = json.loads(P.traffic(f, w, "wl"))
    assert t["calibration"]["bytes_per_FETCH_SIZE_unit"] == 2048.0
    assert t["calibration"]["bytes_per_WRITE_SIZE_unit"] == 1024.0
    assert t["wl:kernels"]["attn_split_kernel"] == {"fetch_bytes": 64 << 20, "write_bytes": 4 << 20}
    assert t["wl"]["verify_attn"] == (64 << 20) + (4 << 20) + (4 << 20) + 50 * 1024
    assert t["wl"]["visual_relevance"] == 0


def test_mfma_utilisation(tmp_path):
    db = str(tmp_path / "m.db")
    # 4 194 304 MOPS x 512 = 2.147 GFLOP in 16 us = 134.2 TFLOP/s = 5.37 % of 2.5 PFLOP/s;
    # 1 966 080 busy SIMD-cycles of 16 us x 2.4 GHz x 1024 SIMDs = 5 %
    _db(db, counters=[(SPLIT, "SQ_INSTS_VALU_MFMA_MOPS_BF16", 4194304.0, 16000),
                      (SPLIT, "SQ_VALU_MFMA_BUSY_CYCLES", 1966080.0, 16000),
                      (SPLIT, "GRBM_GUI_ACTIVE", 1.0, 16000),
                      (COMB, "SQ_INSTS_VALU_MFMA_MOPS_BF16", 0.0, 3000)])
    tab = P.mfma_table(db)
    assert len(tab) == 1 and tab[0]["kernel"].startswith("attn_split_kernel")
    assert abs(tab[0]["frac_of_bf16_peak"] - 0.05369) < 1e-4
    assert abs(tab[0]["mfma_busy_frac"] - 0.05) < 1e-6
    assert "attn_split_kernel" in P.mfma(db)
