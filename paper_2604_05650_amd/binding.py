"""Thin ctypes binding of liblvspec.so: argument marshalling only.

Every step of the verify path runs inside the library's HIP kernels; torch supplies device
memory, the current stream and nothing else.  There is no CPU fallback: if the shared library
is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblvspec.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} not found: build it with `python -m paper_2604_05650_amd.build` "
        "(there is no fallback path)")

_lib = C.CDLL(LIB_PATH)

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP, ESCRATCH = 0, -1, -2, -3, -4, -5
STATIC_SCRATCH_BYTES = 16 << 20
REJECT, EXACT, LOOSE, SHIFT, GATED = 0, 1, 2, 3, 4
RULE_VISUAL, RULE_ENTROPY_GATE, RULE_ENTROPY_WINDOW = 0, 1, 2
MAX_GAMMA, MAX_TOPK, MAX_TOPN = 16, 16, 1024


class AttnArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("gamma", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32),
        ("D", C.c_int32),
        ("q", C.c_void_p), ("q_sb", C.c_int64), ("q_sg", C.c_int64), ("q_sh", C.c_int64),
        ("k", C.c_void_p), ("v", C.c_void_p),
        ("kv_sb", C.c_int64), ("kv_sh", C.c_int64), ("kv_sl", C.c_int64),
        ("cap", C.c_int64),
        ("kv_len", C.c_void_p), ("kv_len_host", C.POINTER(C.c_int32)), ("max_kv_len", C.c_int64),
        ("vis_begin", C.c_void_p), ("vis_end", C.c_void_p),
        ("draft_mask", C.POINTER(C.c_uint32)),
        ("scale", C.c_float),
        ("out", C.c_void_p), ("o_sb", C.c_int64), ("o_sg", C.c_int64), ("o_sh", C.c_int64),
        ("lse", C.c_void_p), ("vis_mass", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


class RelArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("gamma", C.c_int32), ("d", C.c_int32), ("top_n", C.c_int32),
        ("h_d", C.c_void_p), ("hd_sb", C.c_int64), ("hd_sg", C.c_int64),
        ("h_v", C.c_void_p), ("hv_sb", C.c_int64), ("hv_sl", C.c_int64),
        ("lv_max", C.c_int64),
        ("l_v", C.c_void_p),
        ("hv_inv_norm", C.c_void_p),
        ("relevance", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


class HvArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("d", C.c_int32),
        ("h_v", C.c_void_p), ("hv_sb", C.c_int64), ("hv_sl", C.c_int64),
        ("lv_max", C.c_int64),
        ("hv_inv_norm", C.c_void_p),
    ]


class AcceptArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("gamma", C.c_int32), ("d", C.c_int32), ("V", C.c_int32),
        ("topk", C.c_int32),
        ("h_d", C.c_void_p), ("hd_sb", C.c_int64), ("hd_sg", C.c_int64),
        ("lm_head", C.c_void_p), ("w_sv", C.c_int64),
        ("draft_ids", C.c_void_p), ("relevance", C.c_void_p),
        ("n_loose", C.c_int32), ("pst_window", C.c_int32), ("loose_topk_gate", C.c_int32),
        ("n_branches", C.c_int32),
        ("bonus_row", C.c_int32),
        ("rule", C.c_int32), ("entropy_threshold", C.c_float), ("defer_window", C.c_int32),
        ("target_ids", C.c_void_p), ("topk_ids", C.c_void_p), ("topk_probs", C.c_void_p),
        ("verdict", C.c_void_p), ("accept_len", C.c_void_p), ("bonus_id", C.c_void_p),
        ("best_branch", C.c_void_p),
        ("logits", C.c_void_p), ("entropy", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


class CommitArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32), ("n_layers", C.c_int32),
        ("n_branches", C.c_int32), ("chain_len", C.c_int32),
        ("k", C.c_void_p), ("v", C.c_void_p),
        ("kv_slayer", C.c_int64), ("kv_sb", C.c_int64), ("kv_sh", C.c_int64), ("kv_sl", C.c_int64),
        ("cap", C.c_int64),
        ("kv_len", C.c_void_p), ("accept_len", C.c_void_p), ("best_branch", C.c_void_p),
        ("new_len", C.c_void_p),
    ]


class PlanInfo(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "attn_rows_padded", "attn_row_chunks", "attn_splits", "rel_splits", "rel_stage_bytes",
        "rel_slices", "rel_slice_rows", "acc_rows_per_task", "acc_chains_per_pass", "acc_passes")]


_lib.lvspec_status_string.restype = C.c_char_p
_lib.lvspec_status_string.argtypes = [C.c_int]
_lib.lvspec_version.restype = C.c_int
_lib.lvspec_last_hip_error.restype = C.c_int
_lib.lvspec_n_loose.restype = C.c_int
_lib.lvspec_n_loose.argtypes = [C.c_float, C.c_int]
_lib.lvspec_describe_plan.restype = C.c_int
_lib.lvspec_describe_plan.argtypes = [C.POINTER(AttnArgs), C.POINTER(RelArgs),
                                      C.POINTER(AcceptArgs), C.POINTER(PlanInfo)]
_lib.lvspec_kv_commit.restype = C.c_int
_lib.lvspec_kv_commit.argtypes = [C.POINTER(CommitArgs), C.c_void_p]
for _name, _t in (("verify_attn", AttnArgs), ("visual_relevance", RelArgs),
                  ("loose_accept", AcceptArgs)):
    getattr(_lib, f"lvspec_{_name}_workspace").restype = C.c_size_t
    getattr(_lib, f"lvspec_{_name}_workspace").argtypes = [C.POINTER(_t)]
    getattr(_lib, f"lvspec_{_name}").restype = C.c_int
    getattr(_lib, f"lvspec_{_name}").argtypes = [C.POINTER(_t), C.c_void_p]

_lib.lvspec_hv_prepare.restype = C.c_int
_lib.lvspec_hv_prepare.argtypes = [C.POINTER(HvArgs), C.c_void_p]
_lib.lvspec_verify_attn_static.restype = C.c_int
_lib.lvspec_verify_attn_static.argtypes = [C.POINTER(AttnArgs), C.c_void_p]

EXPORTS = ["lvspec_hv_prepare", "lvspec_verify_attn_static", "lvspec_status_string", "lvspec_version", "lvspec_last_hip_error", "lvspec_n_loose",
           "lvspec_verify_attn_workspace", "lvspec_verify_attn",
           "lvspec_visual_relevance_workspace", "lvspec_visual_relevance",
           "lvspec_loose_accept_workspace", "lvspec_loose_accept", "lvspec_kv_commit",
           "lvspec_describe_plan"]


class LvspecError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        msg = _lib.lvspec_status_string(status).decode()
        if status == EHIP:
            msg += f" (hipError_t {_lib.lvspec_last_hip_error()})"
        super().__init__(f"lvspec status {status}: {msg}")


def raw():
    """The ctypes library handle (tests of the C ABI call it directly)."""
    return _lib


def version() -> int:
    return int(_lib.lvspec_version())


def status_string(status: int) -> str:
    return _lib.lvspec_status_string(status).decode()


def n_loose(lam: float, gamma: int) -> int:
    return int(_lib.lvspec_n_loose(float(lam), int(gamma)))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(status: int):
    if status != OK:
        raise LvspecError(status)


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> torch.Tensor:
    if workspace is not None:
        return workspace
    return torch.empty((max(int(nbytes), 256),), dtype=torch.uint8, device=device)


def verify_attn_args(q, k, v, kv_len, *, out, vis_begin=None, vis_end=None, draft_mask=None,
                     scale=0.0, lse=None, vis_mass=None, max_kv_len=0,
                     kv_len_host=None) -> AttnArgs:
    """Fill the C struct from torch tensors: q [B,gamma,Hq,D], k/v [B,Hkv,cap,D] (bf16, last dim
    contiguous), kv_len / vis_begin / vis_end int32 [B] on the device; kv_len_host an optional
    host sequence with the same lengths."""
    B, gamma, Hq, D = q.shape
    a = AttnArgs()
    a.B, a.gamma, a.Hq, a.Hkv, a.D = B, gamma, Hq, k.shape[1], D
    a.q, a.q_sb, a.q_sg, a.q_sh = q.data_ptr(), q.stride(0), q.stride(1), q.stride(2)
    a.k, a.v = k.data_ptr(), v.data_ptr()
    a.kv_sb, a.kv_sh, a.kv_sl = k.stride(0), k.stride(1), k.stride(2)
    a.cap = k.shape[2]
    a.kv_len, a.max_kv_len = _ptr(kv_len), int(max_kv_len)
    if kv_len_host is not None:
        lens = (C.c_int32 * B)(*[int(x) for x in kv_len_host])
        a._keep_len = lens
        a.kv_len_host = C.cast(lens, C.POINTER(C.c_int32))
    a.vis_begin, a.vis_end = _ptr(vis_begin), _ptr(vis_end)
    if draft_mask is not None:
        arr = (C.c_uint32 * gamma)(*[int(m) for m in draft_mask])
        a._keep = arr
        a.draft_mask = C.cast(arr, C.POINTER(C.c_uint32))
    a.scale = float(scale)
    a.out, a.o_sb, a.o_sg, a.o_sh = out.data_ptr(), out.stride(0), out.stride(1), out.stride(2)
    a.lse, a.vis_mass = _ptr(lse), _ptr(vis_mass)
    return a


def verify_attn(q, k, v, kv_len, *, vis_begin=None, vis_end=None, draft_mask=None, scale=0.0,
                out=None, return_lse=False, return_vis_mass=False, workspace=None,
                max_kv_len=0, kv_len_host=None, stream=None):
    """lvspec_verify_attn.  Returns out, or (out, lse, vis_mass) when either extra is asked for
    (the one not asked for is None)."""
    assert q.dtype == torch.bfloat16 and k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16
    assert q.stride(-1) == 1 and k.stride(-1) == 1 and v.stride(-1) == 1
    assert k.stride() == v.stride() and k.shape == v.shape
    B, gamma, Hq, D = q.shape
    if out is None:
        out = torch.empty((B, gamma, Hq, D), dtype=torch.bfloat16, device=q.device)
    lse = torch.empty((B, Hq, gamma), dtype=torch.float32, device=q.device) if return_lse else None
    vm = (torch.empty((B, Hq, gamma), dtype=torch.float32, device=q.device)
          if return_vis_mass else None)
    a = verify_attn_args(q, k, v, kv_len, out=out, vis_begin=vis_begin, vis_end=vis_end,
                         draft_mask=draft_mask, scale=scale, lse=lse, vis_mass=vm,
                         max_kv_len=max_kv_len, kv_len_host=kv_len_host)
    need = _lib.lvspec_verify_attn_workspace(C.byref(a))
    ws = _workspace(need, q.device, workspace)
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel() * ws.element_size()
    _check(_lib.lvspec_verify_attn(C.byref(a), _stream(stream)))
    if return_lse or return_vis_mass:
        return out, lse, vm
    return out


def verify_attn_static(q, k, v, kv_len, *, out, vis_begin=None, vis_end=None, draft_mask=None,
                       scale=0.0, lse=None, vis_mass=None, max_kv_len=0, kv_len_host=None,
                       stream=None):
    """lvspec_verify_attn_static: the same attention with the library's static scratch; every
    output tensor is the caller's, nothing is allocated here."""
    a = verify_attn_args(q, k, v, kv_len, out=out, vis_begin=vis_begin, vis_end=vis_end,
                         draft_mask=draft_mask, scale=scale, lse=lse, vis_mass=vis_mass,
                         max_kv_len=max_kv_len, kv_len_host=kv_len_host)
    _check(_lib.lvspec_verify_attn_static(C.byref(a), _stream(stream)))
    return out


def hv_prepare(h_v, *, hv_inv_norm=None, stream=None):
    """lvspec_hv_prepare: h_v [B,lv_max,d] bf16 -> fp32 [B,lv_max] inverse row norms (once, at
    prefill), to be handed to visual_relevance at every step."""
    assert h_v.dtype == torch.bfloat16 and h_v.stride(-1) == 1
    B, lv_max, d = h_v.shape
    if hv_inv_norm is None:
        hv_inv_norm = torch.empty((B, lv_max), dtype=torch.float32, device=h_v.device)
    assert hv_inv_norm.is_contiguous() and hv_inv_norm.shape == (B, lv_max)
    a = HvArgs()
    a.B, a.d = B, d
    a.h_v, a.hv_sb, a.hv_sl = h_v.data_ptr(), h_v.stride(0), h_v.stride(1)
    a.lv_max = lv_max
    a.hv_inv_norm = hv_inv_norm.data_ptr()
    _check(_lib.lvspec_hv_prepare(C.byref(a), _stream(stream)))
    return hv_inv_norm


def visual_relevance_args(h_d, h_v, l_v, top_n, *, relevance, hv_inv_norm=None) -> RelArgs:
    B, gamma, d = h_d.shape
    a = RelArgs()
    a.B, a.gamma, a.d, a.top_n = B, gamma, d, int(top_n)
    a.h_d, a.hd_sb, a.hd_sg = h_d.data_ptr(), h_d.stride(0), h_d.stride(1)
    a.h_v, a.hv_sb, a.hv_sl = h_v.data_ptr(), h_v.stride(0), h_v.stride(1)
    a.lv_max = h_v.shape[1]
    a.l_v = l_v.data_ptr()
    if hv_inv_norm is not None:
        assert hv_inv_norm.dtype == torch.float32 and hv_inv_norm.is_contiguous()
        assert hv_inv_norm.shape == (B, h_v.shape[1])
        a.hv_inv_norm = hv_inv_norm.data_ptr()
    a.relevance = relevance.data_ptr()
    return a


def visual_relevance(h_d, h_v, l_v, top_n=10, *, relevance=None, workspace=None, stream=None,
                     hv_inv_norm=None):
    """lvspec_visual_relevance.  h_d [B,gamma,d], h_v [B,lv_max,d] bf16; l_v int32 [B] (device);
    hv_inv_norm optional fp32 [B,lv_max] from hv_prepare.  Returns fp32 [B,gamma]."""
    assert h_d.dtype == torch.bfloat16 and h_v.dtype == torch.bfloat16
    assert h_d.stride(-1) == 1 and h_v.stride(-1) == 1
    B, gamma, d = h_d.shape
    if relevance is None:
        relevance = torch.empty((B, gamma), dtype=torch.float32, device=h_d.device)
    a = visual_relevance_args(h_d, h_v, l_v, top_n, relevance=relevance, hv_inv_norm=hv_inv_norm)
    need = _lib.lvspec_visual_relevance_workspace(C.byref(a))
    ws = _workspace(need, h_d.device, workspace)
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel() * ws.element_size()
    _check(_lib.lvspec_visual_relevance(C.byref(a), _stream(stream)))
    return relevance


def loose_accept_args(h_d, lm_head, draft_ids, relevance, n_loose_, pst_window, *, topk,
                      loose_topk_gate, outs, n_branches=1, bonus_row=False, rule=RULE_VISUAL,
                      entropy_threshold=0.0, defer_window=0) -> AcceptArgs:
    B, rows, d = h_d.shape
    gamma = rows - 1 if bonus_row else rows
    a = AcceptArgs()
    a.B, a.gamma, a.d, a.V, a.topk = B, gamma, d, lm_head.shape[0], int(topk)
    a.h_d, a.hd_sb, a.hd_sg = h_d.data_ptr(), h_d.stride(0), h_d.stride(1)
    a.lm_head, a.w_sv = lm_head.data_ptr(), lm_head.stride(0)
    a.draft_ids, a.relevance = draft_ids.data_ptr(), _ptr(relevance)
    a.rule, a.entropy_threshold, a.defer_window = int(rule), float(entropy_threshold), int(defer_window)
    a.n_loose, a.pst_window, a.loose_topk_gate = int(n_loose_), int(pst_window), int(loose_topk_gate)
    a.target_ids = outs["target_ids"].data_ptr()
    a.topk_ids, a.topk_probs = _ptr(outs.get("topk_ids")), _ptr(outs.get("topk_probs"))
    a.verdict = outs["verdict"].data_ptr()
    a.accept_len = outs["accept_len"].data_ptr()
    a.bonus_id = outs["bonus_id"].data_ptr()
    a.n_branches = int(n_branches)
    a.bonus_row = 1 if bonus_row else 0
    a.best_branch = _ptr(outs.get("best_branch"))
    a.logits = _ptr(outs.get("logits"))
    a.entropy = _ptr(outs.get("entropy"))
    return a


def alloc_accept_outputs(B, gamma, V, topk, device, return_logits=False, return_topk=True,
                         n_branches=1, return_entropy=False, bonus_row=False):
    rows = gamma + (1 if bonus_row else 0)   # hidden rows per chain
    outs = dict(
        target_ids=torch.empty((B, rows), dtype=torch.int32, device=device),
        verdict=torch.empty((B, gamma), dtype=torch.uint8, device=device),
        accept_len=torch.empty((B,), dtype=torch.int32, device=device),
        bonus_id=torch.empty((B,), dtype=torch.int32, device=device))
    if return_topk:
        outs["topk_ids"] = torch.empty((B, rows, topk), dtype=torch.int32, device=device)
        outs["topk_probs"] = torch.empty((B, rows, topk), dtype=torch.float32, device=device)
    if return_logits:
        outs["logits"] = torch.empty((B, rows, V), dtype=torch.float32, device=device)
    if n_branches > 1:
        outs["best_branch"] = torch.empty((B // n_branches,), dtype=torch.int32, device=device)
    if return_entropy:
        outs["entropy"] = torch.empty((B, rows), dtype=torch.float32, device=device)
    return outs


def loose_accept(h_d, lm_head, draft_ids, relevance, n_loose_, pst_window, *, topk=1,
                 loose_topk_gate=0, return_logits=False, outs=None, workspace=None, stream=None,
                 n_branches=1, return_entropy=False, bonus_row=False, rule=RULE_VISUAL,
                 entropy_threshold=0.0, defer_window=0):
    """lvspec_loose_accept.  h_d [B,gamma,d] bf16 ([B,gamma+1,d] with bonus_row), lm_head [V,d]
    bf16, draft_ids int32 [B,gamma], relevance fp32 [B,gamma] (all on the device); B counts
    chains, n_branches of them per sequence.  Returns a dict of device tensors: target_ids,
    topk_ids, topk_probs, verdict, accept_len, bonus_id (+ logits, + best_branch when
    n_branches > 1, + entropy)."""
    assert h_d.dtype == torch.bfloat16 and lm_head.dtype == torch.bfloat16
    assert draft_ids.dtype == torch.int32
    assert relevance is None or relevance.dtype == torch.float32
    assert h_d.stride(-1) == 1 and lm_head.stride(-1) == 1
    assert draft_ids.is_contiguous() and (relevance is None or relevance.is_contiguous())
    B, rows, d = h_d.shape
    gamma = rows - 1 if bonus_row else rows
    assert draft_ids.shape == (B, gamma) and (relevance is None or relevance.shape == (B, gamma))
    if outs is None:
        outs = alloc_accept_outputs(B, gamma, lm_head.shape[0], topk, h_d.device, return_logits,
                                    n_branches=n_branches, return_entropy=return_entropy,
                                    bonus_row=bonus_row)
    a = loose_accept_args(h_d, lm_head, draft_ids, relevance, n_loose_, pst_window, topk=topk,
                          loose_topk_gate=loose_topk_gate, outs=outs, n_branches=n_branches,
                          bonus_row=bonus_row, rule=rule, entropy_threshold=entropy_threshold,
                          defer_window=defer_window)
    need = _lib.lvspec_loose_accept_workspace(C.byref(a))
    ws = _workspace(need, h_d.device, workspace)
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel() * ws.element_size()
    _check(_lib.lvspec_loose_accept(C.byref(a), _stream(stream)))
    return outs


def kv_commit(k, v, kv_len, accept_len, chain_len, *, best_branch=None, n_branches=1, new_len=None,
              stream=None):
    """lvspec_kv_commit.  k, v bf16 [B,Hkv,cap,D] or [layers,B,Hkv,cap,D] (changed in place),
    kv_len int32 [B], accept_len int32 [B*n_branches], best_branch int32 [B] (trees).
    Returns new_len int32 [B]."""
    assert k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16 and k.shape == v.shape
    assert k.stride() == v.stride() and k.stride(-1) == 1
    if k.dim() == 4:
        k, v = k.unsqueeze(0), v.unsqueeze(0)
    layers, B, Hkv, cap, D = k.shape
    assert kv_len.dtype == torch.int32 and accept_len.dtype == torch.int32
    if new_len is None:
        new_len = torch.empty((B,), dtype=torch.int32, device=k.device)
    a = CommitArgs()
    a.B, a.Hkv, a.D, a.n_layers = B, Hkv, D, layers
    a.n_branches, a.chain_len = int(n_branches), int(chain_len)
    a.k, a.v = k.data_ptr(), v.data_ptr()
    a.kv_slayer, a.kv_sb, a.kv_sh, a.kv_sl = k.stride(0), k.stride(1), k.stride(2), k.stride(3)
    a.cap = cap
    a.kv_len, a.accept_len = kv_len.data_ptr(), accept_len.data_ptr()
    a.best_branch = _ptr(best_branch)
    a.new_len = new_len.data_ptr()
    _check(_lib.lvspec_kv_commit(C.byref(a), _stream(stream)))
    return new_len


def describe_plan(attn: Optional[AttnArgs] = None, rel: Optional[RelArgs] = None,
                  accept: Optional[AcceptArgs] = None) -> dict:
    """lvspec_describe_plan: the launch planning for the given argument structures (shape fields
    only are read).  Returns the fields of the structures that were given."""
    info = PlanInfo()
    _check(_lib.lvspec_describe_plan(C.byref(attn) if attn is not None else None,
                                     C.byref(rel) if rel is not None else None,
                                     C.byref(accept) if accept is not None else None,
                                     C.byref(info)))
    out = {}
    for name, _ in PlanInfo._fields_:
        if ((name.startswith("attn_") and attn is not None) or
                (name.startswith("rel_") and rel is not None) or
                (name.startswith("acc_") and accept is not None)):
            out[name] = int(getattr(info, name))
    return out
