"""Host-only tests of the C ABI: the library loads, exports every declared symbol, and rejects
bad arguments with the documented codes before touching a device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2604_05650_amd import binding
    return binding


def test_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "lvspec.h")).read()
    declared = set(re.findall(r"\b(lvspec_[a-z_]+)\s*\(", header))
    assert declared == set(L.EXPORTS)
    for name in declared:
        assert hasattr(L.raw(), name), name


def test_version_and_strings(L):
    assert L.version() == 106
    assert L.status_string(0) == "ok"
    assert "workspace" in L.status_string(L.EWORKSPACE)
    assert L.status_string(-99) == "unknown status"


def test_n_loose_matches_the_slice_length(L):
    assert [L.n_loose(0.7, g) for g in (3, 4, 5, 8, 10)] == [2, 2, 3, 5, 7]
    assert L.n_loose(0.0, 10) == 0 and L.n_loose(1.0, 16) == 16 and L.n_loose(2.0, 4) == 4
    assert L.n_loose(-1.0, 4) == 0


def _attn(L, **kw):
    a = L.AttnArgs()
    a.B, a.gamma, a.Hq, a.Hkv, a.D, a.cap = 1, 5, 40, 8, 128, 16389
    a.q = a.k = a.v = a.out = a.kv_len = 0x1000
    a.q_sb, a.q_sg, a.q_sh = 5 * 40 * 128, 40 * 128, 128
    a.kv_sb, a.kv_sh, a.kv_sl = 8 * 16389 * 128, 16389 * 128, 128
    a.o_sb, a.o_sg, a.o_sh = 5 * 40 * 128, 40 * 128, 128
    a.workspace, a.workspace_bytes = 0x10000, 1 << 40
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_attention_argument_checks(L):
    lib = L.raw()
    ok = _attn(L)
    assert lib.lvspec_verify_attn_workspace(C.byref(ok)) > 0
    bad = [
        (dict(gamma=0), L.EINVAL), (dict(gamma=33), L.EINVAL), (dict(Hq=41), L.EINVAL),
        (dict(D=64), L.EUNSUPPORTED), (dict(cap=3), L.EINVAL), (dict(max_kv_len=16385), L.EINVAL),
        (dict(q=0), L.EINVAL), (dict(kv_len=0), L.EINVAL), (dict(out=0), L.EINVAL),
        (dict(q=0x1008), L.EINVAL), (dict(kv_sl=100), L.EINVAL), (dict(q_sh=132), L.EINVAL),
        (dict(vis_begin=0x1000), L.EINVAL), (dict(vis_mass=0x1000), L.EINVAL),
        (dict(scale=-1.0), L.EINVAL),
        (dict(workspace=0), L.EWORKSPACE), (dict(workspace=0x10010), L.EWORKSPACE),
        (dict(workspace_bytes=16), L.EWORKSPACE),
    ]
    for kw, code in bad:
        a = _attn(L, **kw)
        assert lib.lvspec_verify_attn(C.byref(a), None) == code, kw
        if code != L.EWORKSPACE and not set(kw) & {"q", "kv_len", "out", "kv_sl", "q_sh",
                                                   "vis_begin", "vis_mass"}:
            assert lib.lvspec_verify_attn_workspace(C.byref(a)) == 0, kw
    # a draft row must see itself and nothing beyond gamma
    a = _attn(L)
    arr = (C.c_uint32 * 5)(1, 3, 7, 15, 15)
    a.draft_mask = C.cast(arr, C.POINTER(C.c_uint32))
    assert lib.lvspec_verify_attn(C.byref(a), None) == L.EINVAL
    arr = (C.c_uint32 * 5)(1, 3, 7, 15, 63)
    a.draft_mask = C.cast(arr, C.POINTER(C.c_uint32))
    assert lib.lvspec_verify_attn(C.byref(a), None) == L.EINVAL
    assert lib.lvspec_verify_attn(None, None) == L.EINVAL
    # host lengths: validated against the bound, and a device array becomes optional
    a = _attn(L, kv_len=0)
    lens = (C.c_int32 * 1)(16385)
    a.kv_len_host = C.cast(lens, C.POINTER(C.c_int32))
    assert lib.lvspec_verify_attn(C.byref(a), None) == L.EINVAL
    lens[0] = -1
    assert lib.lvspec_verify_attn(C.byref(a), None) == L.EINVAL


def test_static_scratch_limit_is_checked_on_the_host(L):
    lib = L.raw()
    big = _attn(L, B=64, Hq=64, gamma=8, cap=4104, workspace=0, workspace_bytes=0)
    assert lib.lvspec_verify_attn_workspace(C.byref(big)) > L.STATIC_SCRATCH_BYTES
    assert lib.lvspec_verify_attn_static(C.byref(big), None) == L.ESCRATCH
    assert lib.lvspec_verify_attn_static(C.byref(_attn(L, gamma=0)), None) == L.EINVAL
    assert lib.lvspec_verify_attn_static(C.byref(_attn(L, q=0)), None) == L.EINVAL
    assert lib.lvspec_verify_attn_static(None, None) == L.EINVAL
    assert "scratch" in L.status_string(L.ESCRATCH)


def test_workspace_size_scales_with_shape(L):
    lib = L.raw()
    small = lib.lvspec_verify_attn_workspace(C.byref(_attn(L)))
    big = lib.lvspec_verify_attn_workspace(C.byref(_attn(L, B=4)))
    assert big >= small
    # 128 query rows per kv head need two row chunks
    a = _attn(L, Hq=64, gamma=16)
    assert lib.lvspec_verify_attn_workspace(C.byref(a)) > 0


def _rel(L, **kw):
    a = L.RelArgs()
    a.B, a.gamma, a.d, a.top_n, a.lv_max = 1, 5, 5120, 10, 14336
    a.h_d = a.h_v = a.l_v = a.relevance = 0x1000
    a.hd_sb, a.hd_sg, a.hv_sb, a.hv_sl = 5 * 5120, 5120, 14336 * 5120, 5120
    a.workspace, a.workspace_bytes = 0x10000, 1 << 40
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_relevance_argument_checks(L):
    lib = L.raw()
    assert lib.lvspec_visual_relevance_workspace(C.byref(_rel(L))) > 0
    bad = [(dict(top_n=0), L.EINVAL), (dict(top_n=1025), L.EINVAL), (dict(gamma=33), L.EINVAL),
           (dict(d=5000), L.EUNSUPPORTED), (dict(h_d=0), L.EINVAL), (dict(h_v=0), L.EINVAL),
           (dict(l_v=0), L.EINVAL), (dict(relevance=0), L.EINVAL), (dict(hv_sl=5000), L.EINVAL),
           (dict(lv_max=-1), L.EINVAL), (dict(workspace_bytes=1024), L.EWORKSPACE),
           (dict(B=65536), L.EUNSUPPORTED), (dict(B=4096, lv_max=1 << 24), L.EUNSUPPORTED)]
    for kw, code in bad:
        assert lib.lvspec_visual_relevance(C.byref(_rel(L, **kw)), None) == code, kw
    assert lib.lvspec_visual_relevance(None, None) == L.EINVAL


def test_hv_prepare_argument_checks(L):
    lib = L.raw()

    def hv(**kw):
        a = L.HvArgs()
        a.B, a.d, a.lv_max = 1, 5120, 14336
        a.h_v = a.hv_inv_norm = 0x1000
        a.hv_sb, a.hv_sl = 14336 * 5120, 5120
        for k, v in kw.items():
            setattr(a, k, v)
        return a

    bad = [(dict(B=0), L.EINVAL), (dict(d=0), L.EINVAL), (dict(d=5000), L.EUNSUPPORTED),
           (dict(lv_max=-1), L.EINVAL), (dict(lv_max=(1 << 30) + 1), L.EUNSUPPORTED),
           (dict(h_v=0), L.EINVAL), (dict(hv_inv_norm=0), L.EINVAL), (dict(h_v=0x1004), L.EINVAL),
           (dict(hv_sl=5000), L.EINVAL), (dict(hv_sl=5124), L.EINVAL)]
    for kw, code in bad:
        assert lib.lvspec_hv_prepare(C.byref(hv(**kw)), None) == code, kw
    assert lib.lvspec_hv_prepare(None, None) == L.EINVAL
    # no rows: nothing to do, nothing launched
    assert lib.lvspec_hv_prepare(C.byref(hv(lv_max=0, h_v=0)), None) == L.OK


def _acc(L, **kw):
    a = L.AcceptArgs()
    a.B, a.gamma, a.d, a.V, a.topk = 1, 5, 5120, 152064, 4
    a.h_d = a.lm_head = a.draft_ids = a.relevance = 0x1000
    a.target_ids = a.verdict = a.accept_len = a.bonus_id = 0x1000
    a.hd_sb, a.hd_sg = 5 * 5120, 5120
    a.n_loose, a.pst_window = 3, 5
    a.workspace, a.workspace_bytes = 0x10000, 1 << 40
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_accept_argument_checks(L):
    lib = L.raw()
    assert lib.lvspec_loose_accept_workspace(C.byref(_acc(L))) > 0
    bad = [(dict(n_loose=6), L.EINVAL), (dict(n_loose=-1), L.EINVAL), (dict(pst_window=-1), L.EINVAL),
           (dict(topk=0), L.EINVAL), (dict(topk=17), L.EINVAL), (dict(loose_topk_gate=5), L.EINVAL),
           (dict(V=0), L.EINVAL), (dict(d=100), L.EUNSUPPORTED), (dict(B=5000), L.EUNSUPPORTED),
           (dict(gamma=16, n_loose=0, B=5, n_branches=5), L.EUNSUPPORTED),
           (dict(lm_head=0), L.EINVAL), (dict(draft_ids=0), L.EINVAL), (dict(verdict=0), L.EINVAL),
           (dict(w_sv=64), L.EINVAL), (dict(workspace=0), L.EWORKSPACE),
           (dict(gamma=17, n_loose=0), L.EINVAL), (dict(n_branches=-1), L.EINVAL),
           (dict(n_branches=9), L.EINVAL), (dict(n_branches=2), L.EINVAL),
           (dict(B=3, n_branches=2), L.EINVAL), (dict(bonus_row=2), L.EINVAL),
           (dict(bonus_row=-1), L.EINVAL), (dict(relevance=0), L.EINVAL),
           (dict(rule=3), L.EINVAL), (dict(rule=-1), L.EINVAL),
           (dict(rule=1, entropy_threshold=-0.5), L.EINVAL),
           (dict(rule=2, entropy_threshold=float("nan")), L.EINVAL),
           (dict(rule=2, defer_window=17), L.EINVAL), (dict(rule=2, defer_window=-1), L.EINVAL),
           # a tree of four chains of sixteen tokens fits one pass, with the extra rows it does not
           (dict(gamma=16, n_loose=0, B=4, n_branches=4, bonus_row=1), L.EUNSUPPORTED)]
    for kw, code in bad:
        assert lib.lvspec_loose_accept(C.byref(_acc(L, **kw)), None) == code, kw
    assert lib.lvspec_loose_accept_workspace(
        C.byref(_acc(L, gamma=16, n_loose=0, B=4, n_branches=4))) > 0
    # the extra row enlarges the per-pass workspace
    assert (lib.lvspec_loose_accept_workspace(C.byref(_acc(L, bonus_row=1))) >
            lib.lvspec_loose_accept_workspace(C.byref(_acc(L))))
    assert lib.lvspec_loose_accept(None, None) == L.EINVAL
    # with an entropy rule the relevance scores are not read and may be missing: the call gets
    # past validation (the tiny workspace is what stops it here, before any launch)
    ok = _acc(L, rule=2, entropy_threshold=0.1, defer_window=4, relevance=0, workspace_bytes=16)
    assert lib.lvspec_loose_accept(C.byref(ok), None) == L.EWORKSPACE


def _commit(L, **kw):
    a = L.CommitArgs()
    a.B, a.Hkv, a.D, a.n_layers, a.n_branches, a.chain_len = 1, 8, 128, 64, 2, 10
    a.k = a.v = 0x1000
    a.kv_slayer, a.kv_sb, a.kv_sh, a.kv_sl, a.cap = 8 * 4096 * 128, 8 * 4096 * 128, 4096 * 128, 128, 4096
    a.kv_len, a.accept_len, a.best_branch, a.new_len = 0x2000, 0x3000, 0x4000, 0x5000
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_commit_argument_checks(L):
    lib = L.raw()
    bad = [dict(B=0), dict(D=12), dict(D=0), dict(n_layers=0), dict(n_branches=9),
           dict(chain_len=0), dict(chain_len=17), dict(n_branches=4, chain_len=10), dict(k=0),
           dict(v=0x1004), dict(kv_len=0), dict(accept_len=0), dict(new_len=0),
           dict(new_len=0x2000), dict(kv_sl=64), dict(kv_sl=132), dict(kv_slayer=0), dict(cap=19)]
    for kw in bad:
        assert lib.lvspec_kv_commit(C.byref(_commit(L, **kw)), None) == L.EINVAL, kw
    assert lib.lvspec_kv_commit(None, None) == L.EINVAL


def test_launch_planning(L):
    """The planner's choices for the benchmark shapes (256 compute units assumed when no device
    can be queried): they encode measurements, so a change here should come with new ones."""
    # 32B shape, one layer: 25 query rows per kv head -> 32-row workgroups, 8 kv heads x 32 splits
    p = L.describe_plan(attn=_attn(L))
    assert p == dict(attn_rows_padded=32, attn_row_chunks=1, attn_splits=32)
    # gamma = 8: 40 rows -> the 48-row variant; a tree of 2 x 10 tokens: two chunks of 64
    assert L.describe_plan(attn=_attn(L, gamma=8, cap=16392))["attn_rows_padded"] == 48
    p = L.describe_plan(attn=_attn(L, gamma=20, cap=16404))
    assert p == dict(attn_rows_padded=64, attn_row_chunks=2, attn_splits=16)
    # relevance: 224 row blocks leave the workgroups half idle -> two splits of d;
    # the long-video shape (3968 row blocks on 512 slots) runs unsplit
    p = L.describe_plan(rel=_rel(L))
    assert p == dict(rel_splits=2, rel_stage_bytes=512, rel_slices=14, rel_slice_rows=1024)
    c5 = dict(B=4, gamma=8, d=8192, lv_max=63488, hd_sb=8 * 8192, hd_sg=8192,
              hv_sb=63488 * 8192, hv_sl=8192)
    p = L.describe_plan(rel=_rel(L, **c5))
    assert p == dict(rel_splits=1, rel_stage_bytes=512, rel_slices=62, rel_slice_rows=1024)
    # more than 16 draft rows: 256-byte stages; more than 65536 video rows: slices of several
    # 1024-row chunks; more than a million, or N > 16: single-kernel selection
    assert L.describe_plan(rel=_rel(L, gamma=20, hd_sb=20 * 5120))["rel_stage_bytes"] == 256
    p = L.describe_plan(rel=_rel(L, lv_max=152064, hv_sb=152064 * 5120))
    assert (p["rel_slices"], p["rel_slice_rows"]) == (50, 3072)
    assert L.describe_plan(rel=_rel(L, lv_max=1 << 21, hv_sb=(1 << 21) * 5120))["rel_slices"] == 0
    assert L.describe_plan(rel=_rel(L, top_n=100))["rel_slices"] == 0
    # lm_head: 64-row tasks at d = 5120, 128-row tasks at a row pitch that is a multiple of
    # 8 KiB, or when the merge kernel could not keep the candidates in registers (top-k > 8)
    assert L.describe_plan(accept=_acc(L)) == dict(acc_rows_per_task=64, acc_chains_per_pass=1,
                                                   acc_passes=1)
    assert L.describe_plan(accept=_acc(L, d=8192, hd_sb=5 * 8192, hd_sg=8192))[
        "acc_rows_per_task"] == 128
    assert L.describe_plan(accept=_acc(L, topk=16))["acc_rows_per_task"] == 128
    assert L.describe_plan(accept=_acc(L, topk=8))["acc_rows_per_task"] == 64
    # four chains of eight tokens: 32 rows in one pass; with bonus rows 36 -> the 48-column
    # variant, still one pass; nine chains of five with bonus rows: 54 rows, one pass; twelve:
    # two passes of six chains
    c5a = dict(B=4, gamma=8, d=8192, hd_sb=8 * 8192, hd_sg=8192, n_loose=5, pst_window=8)
    assert L.describe_plan(accept=_acc(L, **c5a)) == dict(
        acc_rows_per_task=128, acc_chains_per_pass=4, acc_passes=1)
    c5b = dict(c5a, bonus_row=1, hd_sb=9 * 8192)
    assert L.describe_plan(accept=_acc(L, **c5b)) == dict(
        acc_rows_per_task=64, acc_chains_per_pass=4, acc_passes=1)
    assert L.describe_plan(accept=_acc(L, B=9, bonus_row=1, hd_sb=6 * 5120)) == dict(
        acc_rows_per_task=64, acc_chains_per_pass=9, acc_passes=1)
    assert L.describe_plan(accept=_acc(L, B=12, bonus_row=1, hd_sb=6 * 5120)) == dict(
        acc_rows_per_task=64, acc_chains_per_pass=6, acc_passes=2)
    # errors come back as the planning status; nothing is launched
    lib = L.raw()
    info = L.PlanInfo()
    assert lib.lvspec_describe_plan(C.byref(_attn(L, D=64)), None, None, C.byref(info)) == L.EUNSUPPORTED
    assert lib.lvspec_describe_plan(None, C.byref(_rel(L, top_n=0)), None, C.byref(info)) == L.EINVAL
    assert lib.lvspec_describe_plan(None, None, None, None) == L.EINVAL


def test_planning_from_several_threads(L):
    # the planners and the plan description share per-device caches (compute-unit count, kernel
    # attributes); concurrent first calls must agree with a serial call
    import threading
    lib = L.raw()
    want = (lib.lvspec_verify_attn_workspace(C.byref(_attn(L))),
            lib.lvspec_visual_relevance_workspace(C.byref(_rel(L))))
    got, errs = [], []

    def work():
        try:
            for _ in range(200):
                got.append((lib.lvspec_verify_attn_workspace(C.byref(_attn(L))),
                            lib.lvspec_visual_relevance_workspace(C.byref(_rel(L)))))
        except Exception as e:   # pragma: no cover
            errs.append(e)

    threads = [threading.Thread(target=work) for _ in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errs and len(got) == 1600 and set(got) == {want}
