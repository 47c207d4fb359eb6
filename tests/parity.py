"""Shared helpers of the GPU parity tests: tolerances and flag rules.

Tolerance (max-abs-rel 1e-2, bf16 inputs / fp32 accumulation):
  * vector outputs (attention rows, logits rows): max_t |gpu - oracle| <= 1e-2 * max_t |oracle|
    per row (error relative to the row's largest magnitude)
  * scalar outputs (relevance, log-sum-exp, visual mass, probabilities):
    |gpu - oracle| <= 1e-2 * max(|oracle|, 1e-3)
Integer outputs are bit-exact, except that a decision which hinges on two oracle values closer
than the tolerance is *flagged* and not counted.
"""
import numpy as np
import torch

TOL = 1e-2


def dev():
    return torch.device("cuda:0")


def t_bf16(bits, device=None):
    from paper_2604_05650_amd import synth
    return synth.to_torch_bf16(bits, device or dev())


def t_i32(a, device=None):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(device or dev())


def t_f32(a, device=None):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device or dev())


def bf16_out_to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rows_rel_err(gpu, ref):
    """per-row max-abs error relative to the row's max magnitude; rows along all but last dim"""
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    num = np.abs(gpu - ref).max(axis=-1)
    den = np.maximum(np.abs(ref).max(axis=-1), 1e-30)
    return num / den


def assert_rows_close(gpu, ref, what, tol=TOL):
    err = rows_rel_err(gpu, ref)
    worst = float(err.max()) if err.size else 0.0
    assert np.all(np.isfinite(np.asarray(gpu, np.float64))), f"{what}: non-finite output"
    assert worst <= tol, f"{what}: max-abs-rel {worst:.3e} > {tol}"
    return worst


def assert_scalars_close(gpu, ref, what, tol=TOL, floor=1e-3):
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    assert np.all(np.isfinite(gpu)), f"{what}: non-finite output"
    err = np.abs(gpu - ref) / np.maximum(np.abs(ref), floor)
    worst = float(err.max()) if err.size else 0.0
    assert worst <= tol, f"{what}: rel err {worst:.3e} > {tol}"
    return worst


def compare_accept(gpu, orc, draft_ids, gamma, extra_flag=None, check_topk=True, tol=TOL):
    """Bit-exact comparison of the acceptance outputs with oracle-margin flagging.

    gpu: dict of numpy arrays from the library; orc: dict from oracle.loose_accept.
    A position is flagged when the oracle's argmax margin is below tol (or extra_flag[b,i]).
    A sequence's verdicts / accepted length / bonus are counted only if none of its positions
    is flagged.  Returns dict(flagged_positions, counted_sequences, flagged_mismatch)."""
    B = orc["target_ids"].shape[0]
    flag = orc["margin"] < tol
    if extra_flag is not None:
        flag = flag | extra_flag
    same = gpu["target_ids"] == orc["target_ids"]
    assert np.all(same | flag), (
        f"target ids differ at unflagged positions: gpu {gpu['target_ids'][~(same | flag)]} "
        f"oracle {orc['target_ids'][~(same | flag)]}")
    counted = 0
    for b in range(B):
        if flag[b].any():
            continue
        counted += 1
        np.testing.assert_array_equal(gpu["verdict"][b], orc["verdict"][b], f"verdict seq {b}")
        assert gpu["accept_len"][b] == orc["accept_len"][b], f"accept_len seq {b}"
        assert gpu["bonus_id"][b] == orc["bonus_id"][b], f"bonus seq {b}"
    if check_topk and "topk_ids" in gpu and gpu["topk_ids"] is not None:
        k = orc["topk_ids"].shape[-1]
        for b in range(B):
            for i in range(gamma):
                if flag[b, i]:
                    continue
                # probabilities within tolerance; ids equal wherever neighbouring oracle
                # probabilities are separated by more than the tolerance
                op, oi = orc["topk_probs"][b, i], orc["topk_ids"][b, i]
                gp, gi = gpu["topk_probs"][b, i], gpu["topk_ids"][b, i]
                assert_scalars_close(gp, op, f"topk probs [{b},{i}]", tol=tol, floor=1e-6)
                for r in range(k):
                    sep_lo = r == 0 or (op[r - 1] - op[r]) > tol * op[r - 1]
                    sep_hi = r == k - 1 or (op[r] - op[r + 1]) > tol * op[r]
                    if sep_lo and sep_hi:
                        assert gi[r] == oi[r], f"topk id [{b},{i},{r}]"
    return dict(flagged_positions=int(flag.sum()), counted_sequences=counted,
                flagged_mismatch=int((~same & flag).sum()))


def to_np(outs):
    return {k: (v.detach().cpu().numpy() if v is not None else None) for k, v in outs.items()}
