"""Host-only checks of the benchmark's command line and of the seeded input recipe."""
import os
import subprocess
import sys

import numpy as np

from paper_2604_05650_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 2
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_configs_have_the_stated_shapes():
    c = synth.CONFIGS
    assert (c["c1"].Hq, c["c1"].Hkv, c["c1"].gamma, c["c1"].kv_len, c["c1"].pst_window) == \
        (8, 2, 4, (2048,), 2)
    assert (c["c1"].vis_begin, c["c1"].vis_len, c["c1"].d, c["c1"].V) == ((16,), 1568, 1024, 8192)
    assert (c["c2"].Hq, c["c2"].Hkv, c["c2"].d, c["c2"].V, c["c2"].gamma) == (40, 8, 5120, 152064, 5)
    assert c["c2"].kv_len == (16384,) and c["c2"].vis_len == 14336
    assert (c["c3"].Hq, c["c3"].d, c["c3"].kv_len, c["c3"].vis_len) == (64, 8192, (7296,), 6272)
    assert c["c4"].layers == 64 and c["c4"].kv_bytes_per_layer == 2 * (16384 + 5) * 8 * 128 * 2
    assert (c["c5"].B, c["c5"].gamma, c["c5"].kv_len[0], c["c5"].vis_len) == (4, 8, 65536, 63488)
    assert len(set(c["c5"].vis_begin)) == 4
    # loosened-set sizes written into the configurations: what lambda = 0.7 gives (Eq. 9's slice)
    from oracle import lvspec_oracle as oracle
    for k, cfg in c.items():
        assert cfg.n_loose == oracle.n_loose(cfg.lam, cfg.chain_len), k
    assert [c[k].n_loose for k in ("c1", "c2", "c5")] == [2, 3, 5]
    # the draft-tree variants: two chains of ten, ranking local to a chain
    assert (c["c2t"].gamma, c["c2t"].n_branches, c["c2t"].chain_len, c["c2t"].n_loose) == (20, 2, 10, 7)


def test_generators_are_seeded_and_bf16_exact():
    a = synth.normal_bf16((1, 2, 3), (64, 128), 1.0)
    b = synth.normal_bf16((1, 2, 3), (64, 128), 1.0)
    c = synth.normal_bf16((1, 2, 4), (64, 128), 1.0)
    assert a.dtype == np.uint16 and np.array_equal(a, b) and not np.array_equal(a, c)
    f = synth.bf16_bits_to_f32(a)
    assert np.array_equal(synth.f32_to_bf16_bits(f), a)          # round trip is exact
    assert abs(float(f.std()) - 1.0) < 0.05 and abs(float(f.mean())) < 0.05
    # round to nearest even at the bf16 boundary
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], np.float32)   # ties
    assert synth.f32_to_bf16_bits(x).tolist() == [0x3F80, 0x3F82]


def test_branch_mask_is_block_diagonal_lower_triangular():
    m = synth.branch_mask(2, 3)
    assert [int(x) for x in m] == [0b000001, 0b000011, 0b000111, 0b001000, 0b011000, 0b111000]
    assert synth.CONFIGS["c1"].tree_mask() is None


def test_shifted_drafts_follow_the_recipe():
    y = np.arange(40, dtype=np.int32).reshape(4, 10) + 100
    d = synth.draft_ids_from_target(y, (9,), p_shift=0.5)
    same = d == y
    prev = np.empty_like(y)
    prev[:, 1:] = y[:, :-1]
    prev[:, 0] = y[:, 1]
    assert np.all(same | (d == prev)) and 0.2 < same.mean() < 0.8


def test_counter_summary_is_only_replayed_when_its_stamp_matches(tmp_path):
    """bench.py replays HBM bytes and matrix-core figures from profiles/traffic.json; they must
    reach the line only when the file was taken with the same library version and launch plan."""
    import json
    import types
    sys.path.insert(0, ROOT)
    import bench
    plan = {"attn_rows_padded": 32, "attn_splits": 32}
    name = "c4-qwen2.5-vl-32b-64layer-step"
    data = {"stamp": {"commit": "abc1234", "library_version": 106, "plans": {name: plan}},
            name: {"verify_attn": 74000000, "visual_relevance": 1, "lm_head_accept": 2},
            name + ":mfma": {"verify_attn": {"frac_of_bf16_peak": 0.05}}}
    path = tmp_path / "traffic.json"
    path.write_text(json.dumps(data))
    wl = types.SimpleNamespace(cfg=types.SimpleNamespace(name=name), plan=dict(plan))
    out, info = bench.load_counters(str(path), wl, 106)
    assert info["match"] and info["commit"] == "abc1234" and info["replayed"]
    assert out["verify_attn"] == {"traffic": 74000000, "mfma_frac_of_peak": 0.05}
    # another library version, another plan, another workload, a missing or broken file: nothing
    assert bench.load_counters(str(path), wl, 107) == ({}, dict(info, match=False))
    wl2 = types.SimpleNamespace(cfg=wl.cfg, plan=dict(plan, attn_splits=16))
    assert bench.load_counters(str(path), wl2, 106)[0] == {}
    wl3 = types.SimpleNamespace(cfg=types.SimpleNamespace(name="other"), plan=plan)
    assert bench.load_counters(str(path), wl3, 106)[0] == {}
    out, info = bench.load_counters(str(tmp_path / "missing.json"), wl, 106)
    assert out == {} and not info["match"] and "error" in info
    path.write_text("{not json")
    out, info = bench.load_counters(str(path), wl, 106)
    assert out == {} and "error" in info


def test_tracked_counter_summary_matches_the_library():
    """The committed profiles/traffic.json carries a stamp for every profiled workload and was
    taken with the library version this tree builds."""
    import json
    from paper_2604_05650_amd import binding as L
    data = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
    stamp = data["stamp"]
    assert stamp["library_version"] == L.version()
    for key in ("c2", "c3", "c4", "c4t", "c5"):
        name = synth.CONFIGS[key].name
        assert name in stamp["plans"] and name in data and name + ":mfma" in data
        cfg = synth.CONFIGS[key]
        # the plan recorded for the attention call is what the planner says today
        a = L.AttnArgs()
        a.B, a.gamma, a.Hq, a.Hkv, a.D, a.cap = cfg.B, cfg.gamma, cfg.Hq, cfg.Hkv, cfg.D, cfg.cap
        a.max_kv_len = max(cfg.kv_len)
        now = L.describe_plan(attn=a)
        assert {k: stamp["plans"][name][k] for k in now} == now, key


def test_lds_summary_reads_conflict_share_per_kernel(tmp_path):
    # a counters_collection table shaped like rocprofv3's, two launches of one kernel
    import sqlite3
    from paper_2604_05650_amd import profiling
    db = tmp_path / "lds_results.db"
    con = sqlite3.connect(db)
    con.execute("create table counters_collection (kernel_name text, counter_name text, value real)")
    rows = []
    for launch in range(2):
        rows += [("void lvspec::(anonymous namespace)::attn_split_kernel<2, 1>(x)", "SQ_LDS_IDX_ACTIVE", 1000.0),
                 ("void lvspec::(anonymous namespace)::attn_split_kernel<2, 1>(x)", "SQ_LDS_BANK_CONFLICT", 250.0),
                 ("void lvspec::(anonymous namespace)::attn_split_kernel<2, 1>(x)", "SQ_INSTS_LDS", 200.0),
                 ("void at::native::fill(x)", "SQ_LDS_IDX_ACTIVE", 5.0)]
    con.executemany("insert into counters_collection values (?, ?, ?)", rows)
    con.commit()
    con.close()
    text = profiling.lds(str(db))
    lines = [ln for ln in text.splitlines() if "attn_split_kernel" in ln]
    assert len(lines) == 1 and "25.00%" in lines[0] and " 2 " in lines[0]
    assert "at::native" not in text
