"""ctypes front end of ``lvspec_oracle.c`` (test infrastructure; fp64 from bf16 bit patterns).

All tensors are numpy arrays.  bf16 tensors are passed as ``uint16`` bit patterns.  Nothing here
does arithmetic of the method except the composition of the C steps in ``loose_accept`` (which
chains O3 -> O4 -> O5 exactly in the order of the paper's Sec. 3.2 / 3.3).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lvspec_oracle.c")
_LIB = os.path.join(_HERE, "liblvspec_oracle.so")

REJECT, EXACT, LOOSE, PST, GATED = 0, 1, 2, 3, 4
RULE_VISUAL, RULE_ENTROPY_GATE, RULE_ENTROPY_WINDOW = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99 + OpenMP across independent output units)."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _l():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.lvo_n_loose.restype = C.c_int
        _lib.lvo_n_loose.argtypes = [C.c_double, C.c_int]
        _lib.lvo_num_threads.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bf16 tensors are passed as uint16 bit patterns"
    return a


def _i32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(_l().lvo_num_threads())


def set_num_threads(n: int) -> None:
    _l().lvo_set_num_threads(C.c_int(int(n)))


def n_loose(lam: float, gamma: int) -> int:
    """floor(lambda*K) of Eq. 9's slice."""
    return int(_l().lvo_n_loose(float(lam), int(gamma)))


def verify_attn(q, k, v, kv_len, vis_begin=None, vis_end=None, scale=None, draft_mask=None,
                rows=None):
    """O1.  q [B,gamma,Hq,D], k/v [B,Hkv,cap,D] (uint16 bf16 bits), kv_len [B].

    Returns (out, lse, vis_mass) as float64: out [B,gamma,Hq,D], lse/vis_mass [B,Hq,gamma];
    with ``rows`` = int array [n,3] of (b,i,h): out [n,D], lse/vis_mass [n].
    """
    q, k, v = _u16(q), _u16(k), _u16(v)
    B, gamma, Hq, D = q.shape
    Bk, Hkv, cap, Dk = k.shape
    assert (Bk, Dk) == (B, D) and v.shape == k.shape and Hq % Hkv == 0
    kv_len = _i32(kv_len)
    assert kv_len.shape == (B,) and int(kv_len.max(initial=0)) + gamma <= cap
    vb, ve = _i32(vis_begin), _i32(vis_end)
    if scale is None:
        scale = 1.0 / np.sqrt(float(D))
    dm = None if draft_mask is None else np.ascontiguousarray(draft_mask, dtype=np.uint32)
    if rows is None:
        out = np.empty((B, gamma, Hq, D), np.float64)
        lse = np.empty((B, Hq, gamma), np.float64)
        vm = np.empty((B, Hq, gamma), np.float64)
        _l().lvo_verify_attn(C.c_int(B), C.c_int(gamma), C.c_int(Hq), C.c_int(Hkv), C.c_int(D),
                             C.c_int64(cap), _p(q), _p(k), _p(v), _p(kv_len), _p(vb), _p(ve),
                             _p(dm), C.c_double(scale), _p(out), _p(lse), _p(vm))
        return out, lse, vm
    sel = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    n = sel.shape[0]
    out = np.empty((n, D), np.float64)
    lse = np.empty((n,), np.float64)
    vm = np.empty((n,), np.float64)
    _l().lvo_verify_attn_rows(C.c_int(gamma), C.c_int(Hq), C.c_int(Hkv), C.c_int(D),
                              C.c_int64(cap), _p(q), _p(k), _p(v), _p(kv_len), _p(vb), _p(ve),
                              _p(dm), C.c_double(scale), C.c_int(n), _p(sel), _p(out), _p(lse),
                              _p(vm))
    return out, lse, vm


def hv_inv_norm(h_v):
    """O2p: 1 / max(|h_v row|, 1e-8) for every visual row (what Eq. 7's prefill-side H_V carries
    along).  h_v [B,lv_max,d] uint16 bf16 bits -> float64 [B,lv_max]."""
    h_v = _u16(h_v)
    B, lv_max, d = h_v.shape
    out = np.empty((B, lv_max), np.float64)
    _l().lvo_hv_inv_norm(C.c_int(B), C.c_int64(lv_max), C.c_int(d), _p(h_v), _p(out))
    return out


def visual_relevance(h_d, h_v, l_v, top_n, return_cos=False, hv_inv_norm=None):
    """O2 (Eq. 8).  h_d [B,gamma,d], h_v [B,lv_max,d] uint16 bf16 bits, l_v [B].  With
    ``hv_inv_norm`` (float32 [B,lv_max]) the visual rows' inverse norms are taken as given."""
    h_d, h_v = _u16(h_d), _u16(h_v)
    B, gamma, d = h_d.shape
    Bv, lv_max, dv = h_v.shape
    assert (Bv, dv) == (B, d)
    l_v = _i32(l_v)
    assert l_v.shape == (B,) and int(l_v.max(initial=0)) <= lv_max
    rel = np.empty((B, gamma), np.float64)
    cos = np.zeros((B, gamma, lv_max), np.float64) if return_cos else None
    if hv_inv_norm is not None:
        r = np.ascontiguousarray(hv_inv_norm, dtype=np.float32)
        assert r.shape == (B, lv_max)
        _l().lvo_visual_relevance_prepared(C.c_int(B), C.c_int(gamma), C.c_int(d),
                                           C.c_int(int(top_n)), _p(h_d), _p(h_v), _p(r), _p(l_v),
                                           C.c_int64(lv_max), _p(rel), _p(cos))
        return (rel, cos) if return_cos else rel
    _l().lvo_visual_relevance(C.c_int(B), C.c_int(gamma), C.c_int(d), C.c_int(int(top_n)),
                              _p(h_d), _p(h_v), _p(l_v), C.c_int64(lv_max), _p(rel), _p(cos))
    return (rel, cos) if return_cos else rel


def logits(h, w, cols=None):
    """O3 (Eq. 6).  h [rows,d], w [V,d] uint16 bf16 bits -> z [rows,V] float64."""
    h, w = _u16(h), _u16(w)
    rows, d = h.shape
    V, dw = w.shape
    assert dw == d
    if cols is None:
        z = np.empty((rows, V), np.float64)
        _l().lvo_logits(C.c_int64(rows), C.c_int(d), C.c_int64(V), _p(h), _p(w), _p(z))
        return z
    vs = np.ascontiguousarray(cols, dtype=np.int64)
    z = np.empty((rows, vs.size), np.float64)
    _l().lvo_logits_cols(C.c_int64(rows), C.c_int(d), _p(h), _p(w), C.c_int(vs.size), _p(vs),
                         _p(z))
    return z


def softmax_topk(z_row, k):
    """Greedy token, ln-sum-exp, top-k (ids, probs), argmax margin and entropy of one row."""
    z_row = np.ascontiguousarray(z_row, dtype=np.float64)
    V = z_row.shape[0]
    y = C.c_int32()
    lse = C.c_double()
    margin = C.c_double()
    ent = C.c_double()
    ids = np.empty((k,), np.int32)
    probs = np.empty((k,), np.float64)
    _l().lvo_softmax_topk(C.c_int64(V), _p(z_row), C.c_int(k), C.byref(y), C.byref(lse),
                          _p(ids), _p(probs), C.byref(margin), C.byref(ent))
    return dict(y=int(y.value), lse=float(lse.value), topk_ids=ids, topk_probs=probs,
                margin=float(margin.value), entropy=float(ent.value))


def loosened_set(a, n_loose_):
    """O4 (Eq. 9).  a [gamma] float32 -> (mask uint8 [gamma], ascending stable order)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    g = a.shape[0]
    mask = np.zeros((g,), np.uint8)
    order = np.zeros((g,), np.int32)
    _l().lvo_loosened_set(C.c_int(g), _p(a), C.c_int(int(n_loose_)), _p(mask), _p(order))
    return mask, order


def verdicts(draft, target, loose_mask, pst_window, gate_ok=None):
    """O5 (Eq. 10/11, Eq. 2) -> (verdict uint8 [gamma], tau, bonus).  ``target`` holds gamma
    tokens, or gamma + 1 when the row after the last draft is given (then bonus is never -1)."""
    draft, target = _i32(draft), _i32(target)
    g = draft.shape[0]
    assert target.shape[0] in (g, g + 1)
    loose_mask = np.ascontiguousarray(loose_mask, dtype=np.uint8)
    gate = None if gate_ok is None else np.ascontiguousarray(gate_ok, dtype=np.uint8)
    vd = np.zeros((g,), np.uint8)
    tau = C.c_int32()
    bonus = C.c_int32()
    _l().lvo_verdicts(C.c_int(g), C.c_int(target.shape[0]), _p(draft), _p(target), _p(loose_mask),
                      _p(gate),
                      C.c_int(int(pst_window)), _p(vd), C.byref(tau), C.byref(bonus))
    return vd, int(tau.value), int(bonus.value)


def verdicts_entropy(draft, target, entropy, threshold, window):
    """O5e (entropy gate, alone or with a deferred window: the text-only loose rules of the
    paper's comparison) -> (verdict uint8 [gamma], tau, bonus).  entropy [>= gamma] float32."""
    draft, target = _i32(draft), _i32(target)
    g = draft.shape[0]
    assert target.shape[0] in (g, g + 1)
    ent = np.ascontiguousarray(entropy, dtype=np.float32)
    assert ent.shape[0] >= g
    vd = np.zeros((g,), np.uint8)
    tau = C.c_int32()
    bonus = C.c_int32()
    _l().lvo_verdicts_entropy(C.c_int(g), C.c_int(target.shape[0]), _p(draft), _p(target),
                              _p(ent), C.c_float(float(threshold)), C.c_int(int(window)), _p(vd),
                              C.byref(tau), C.byref(bonus))
    return vd, int(tau.value), int(bonus.value)


def select_branch(tau):
    """O6 (draft-tree appendix): index of the chain with the longest accepted length."""
    tau = _i32(tau).reshape(-1)
    _l().lvo_select_branch.restype = C.c_int32
    return int(_l().lvo_select_branch(C.c_int(tau.size), _p(tau)))


def loose_accept(h_d, w, draft_ids, relevance, n_loose_, pst_window, topk=1, loose_topk_gate=0,
                 return_logits=False, n_branches=1, bonus_row=False, rule=RULE_VISUAL,
                 entropy_threshold=0.0, defer_window=0):
    """Chain O3 -> O4 -> O5 for B chains of gamma rows (Sec. 3.2 / 3.3 of the paper).

    With ``bonus_row`` every chain has gamma + 1 hidden rows: row i < gamma yields the target's
    token at draft position i, row gamma the token after the last draft; target_ids, topk_*,
    lse, entropy, margin and logits then have gamma + 1 rows, and bonus_id is always a token.

    ``rule`` other than RULE_VISUAL replaces O4/O5 by O5e (entropy gate; RULE_ENTROPY_WINDOW adds
    the deferred window ``defer_window``); relevance may then be None.  ``entropy_margin``
    [B,gamma] is |H - threshold| / max(|H|, 1e-3) for mismatching positions (inf elsewhere).

    With ``n_branches`` > 1, chains s*n_branches .. (s+1)*n_branches-1 are the branches of one
    sequence's draft tree; ``best_branch`` [B/n_branches] is the branch kept (O6).

    h_d [B,gamma,d] bf16 bits, w [V,d] bf16 bits, draft_ids [B,gamma] int32, relevance
    [B,gamma] float32.  Returns a dict of numpy arrays; ``margin`` [B,gamma] is the argmax
    margin, ``loose_margin`` [B] the gap between the last loosened and the first strict score
    relative to max|A| (inf when the set is empty or full).
    """
    h_d = _u16(h_d)
    B, rows, d = h_d.shape
    gamma = rows - 1 if bonus_row else rows
    assert gamma >= 1
    V = w.shape[0]
    draft_ids = _i32(draft_ids).reshape(B, gamma)
    if relevance is None:
        assert rule != RULE_VISUAL
        relevance = np.zeros((B, gamma), np.float32)
    relevance = np.ascontiguousarray(relevance, dtype=np.float32).reshape(B, gamma)
    z = logits(h_d.reshape(B * rows, d), w).reshape(B, rows, V)
    out = dict(target_ids=np.zeros((B, rows), np.int32),
               topk_ids=np.zeros((B, rows, topk), np.int32),
               topk_probs=np.zeros((B, rows, topk), np.float64),
               lse=np.zeros((B, rows), np.float64),
               entropy=np.zeros((B, rows), np.float64),
               margin=np.zeros((B, rows), np.float64),
               verdict=np.zeros((B, gamma), np.uint8),
               loose_mask=np.zeros((B, gamma), np.uint8),
               accept_len=np.zeros((B,), np.int32),
               bonus_id=np.zeros((B,), np.int32),
               loose_margin=np.full((B,), np.inf),
               entropy_margin=np.full((B, gamma), np.inf))
    for b in range(B):
        for i in range(rows):
            r = softmax_topk(z[b, i], topk)
            out["target_ids"][b, i] = r["y"]
            out["topk_ids"][b, i] = r["topk_ids"]
            out["topk_probs"][b, i] = r["topk_probs"]
            out["lse"][b, i] = r["lse"]
            out["entropy"][b, i] = r["entropy"]
            out["margin"][b, i] = r["margin"]
        mask, order = loosened_set(relevance[b], n_loose_)
        out["loose_mask"][b] = mask
        if 0 < n_loose_ < gamma:
            a = relevance[b].astype(np.float64)
            amax = max(float(np.abs(a).max()), 1e-30)
            out["loose_margin"][b] = (a[order[n_loose_]] - a[order[n_loose_ - 1]]) / amax
        gate = None
        if loose_topk_gate > 0:
            g = min(loose_topk_gate, topk)
            gate = np.array([draft_ids[b, i] in out["topk_ids"][b, i, :g] for i in range(gamma)],
                            np.uint8)
        if rule == RULE_VISUAL:
            vd, tau, bonus = verdicts(draft_ids[b], out["target_ids"][b], mask, pst_window, gate)
        else:
            ent = out["entropy"][b].astype(np.float32)
            win = defer_window if rule == RULE_ENTROPY_WINDOW else 0
            vd, tau, bonus = verdicts_entropy(draft_ids[b], out["target_ids"][b], ent,
                                              entropy_threshold, win)
            miss = draft_ids[b] != out["target_ids"][b, :gamma]
            h = out["entropy"][b, :gamma]
            out["entropy_margin"][b, miss] = (np.abs(h - entropy_threshold) /
                                              np.maximum(np.abs(h), 1e-3))[miss]
        out["verdict"][b] = vd
        out["accept_len"][b] = tau
        out["bonus_id"][b] = bonus
    if n_branches > 1:
        assert B % n_branches == 0
        out["best_branch"] = np.array(
            [select_branch(out["accept_len"][s * n_branches:(s + 1) * n_branches])
             for s in range(B // n_branches)], np.int32)
    if return_logits:
        out["logits"] = z
    return out


def kv_commit(k, v, kv_len, accept_len, chain_len, best_branch=None, n_branches=1):
    """O7: the KV cache after a verified step (the accepted drafts join the history of Eq. 1).

    k, v [..., B, Hkv, cap, D] (any dtype; leading axes are layers).  Chain c's draft token i sits
    at cache row kv_len[b] + c*chain_len + i.  The kept chain (best_branch[b], else 0) has
    tau = accept_len[b*n_branches + kept] accepted tokens; they become rows kv_len[b] ..
    kv_len[b]+tau-1 and the sequence grows by tau.  All other rows stay as they are.
    Returns (k', v', new_len)."""
    k, v = np.array(k, copy=True), np.array(v, copy=True)
    B = k.shape[-4]
    new_len = np.zeros((B,), np.int32)
    for b in range(B):
        kept = int(best_branch[b]) if (best_branch is not None and n_branches > 1) else 0
        tau = int(accept_len[b * n_branches + kept])
        ctx = int(kv_len[b])
        for t in (k, v):
            accepted = t[..., b, :, ctx + kept * chain_len: ctx + kept * chain_len + tau, :].copy()
            t[..., b, :, ctx: ctx + tau, :] = accepted
        new_len[b] = ctx + tau
    return k, v, new_len
