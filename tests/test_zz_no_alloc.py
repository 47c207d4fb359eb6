"""lvspec_verify_attn_static (the entry point that allocates nothing: its split partials live
in a static device array of the library) against lvspec_verify_attn, through the C ABI, on two
calls in a row, the second with a smaller input.  Same kernels, so the results are bit-equal."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_2604_05650_amd import synth
from parity import assert_rows_close, bf16_out_to_f64, dev, t_bf16, t_i32

pytestmark = pytest.mark.gpu


def _both(L, B, gamma, Hq, Hkv, Lk, seed):
    D = 128
    cap = Lk + gamma
    q = synth.normal_bf16((401, seed, 0), (B, gamma, Hq, D), 1.0)
    k = synth.normal_bf16((401, seed, 1), (B, Hkv, cap, D), 1.0)
    v = synth.normal_bf16((401, seed, 2), (B, Hkv, cap, D), 1.0)
    kv_len = [Lk - 7 * b for b in range(B)]
    tq, tk, tv, tl = t_bf16(q), t_bf16(k), t_bf16(v), t_i32(kv_len)
    vb, ve = t_i32([3] * B), t_i32([Lk // 2] * B)
    outs = []
    for static in (False, True):
        out = torch.zeros((B, gamma, Hq, D), dtype=torch.bfloat16, device=dev())
        lse = torch.zeros((B, Hq, gamma), dtype=torch.float32, device=dev())
        vm = torch.zeros((B, Hq, gamma), dtype=torch.float32, device=dev())
        a = L.verify_attn_args(tq, tk, tv, tl, out=out, vis_begin=vb, vis_end=ve, lse=lse,
                               vis_mass=vm)
        stream = torch.cuda.current_stream().cuda_stream
        if static:
            a.workspace, a.workspace_bytes = None, 0       # ignored by the static entry point
            print(f"[static] lvspec_verify_attn_static B{B} g{gamma} Hq{Hq} Hkv{Hkv} L{Lk}",
                  flush=True)
            rc = L.raw().lvspec_verify_attn_static(C.byref(a), stream)
        else:
            need = L.raw().lvspec_verify_attn_workspace(C.byref(a))
            assert 0 < need <= L.STATIC_SCRATCH_BYTES
            ws = torch.empty((need,), dtype=torch.uint8, device=dev())
            a.workspace, a.workspace_bytes = ws.data_ptr(), need
            rc = L.raw().lvspec_verify_attn(C.byref(a), stream)
        assert rc == L.OK, L.status_string(rc)
        torch.cuda.synchronize()
        outs.append((out, lse, vm))
    (o0, l0, m0), (o1, l1, m1) = outs
    assert torch.equal(o0, o1) and torch.equal(l0, l1) and torch.equal(m0, m1)
    o_out, _, _ = oracle.verify_attn(q, k, v, kv_len, [3] * B, [Lk // 2] * B)
    assert_rows_close(bf16_out_to_f64(o1), o_out, "static scratch vs oracle")


def test_static_scratch_two_calls_second_smaller():
    from paper_2604_05650_amd import binding as L
    # first call: several splits per kv head and two sequences; second: smaller in every way, so
    # stale partials of the first call lie beyond and between what the second one writes
    _both(L, B=2, gamma=5, Hq=16, Hkv=4, Lk=3000, seed=1)
    _both(L, B=1, gamma=3, Hq=8, Hkv=2, Lk=700, seed=2)
    # and a larger one again (more rows per kv head: another kernel variant, same array)
    _both(L, B=1, gamma=8, Hq=40, Hkv=8, Lk=1500, seed=3)


def test_static_scratch_rejects_what_does_not_fit():
    from paper_2604_05650_amd import binding as L
    # 64 sequences x 8 kv heads x 64 padded rows of partials exceed the 16 MiB array: the call
    # must say so before launching anything (the pointers are never dereferenced)
    a = L.AttnArgs()
    a.B, a.gamma, a.Hq, a.Hkv, a.D, a.cap = 64, 8, 64, 8, 128, 4104
    a.q = a.k = a.v = a.out = a.kv_len = 0x1000
    a.q_sb, a.q_sg, a.q_sh = 8 * 64 * 128, 64 * 128, 128
    a.kv_sb, a.kv_sh, a.kv_sl = 8 * 4104 * 128, 4104 * 128, 128
    a.o_sb, a.o_sg, a.o_sh = 8 * 64 * 128, 64 * 128, 128
    assert L.raw().lvspec_verify_attn_workspace(C.byref(a)) > L.STATIC_SCRATCH_BYTES
    assert L.raw().lvspec_verify_attn_static(C.byref(a), None) == L.ESCRATCH
    assert "scratch" in L.status_string(L.ESCRATCH)
