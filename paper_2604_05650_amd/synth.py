"""Seeded synthetic inputs for the LVSpec verify step (no arithmetic of the method lives here).

The paper evaluates on video benchmarks with trained checkpoints; neither is available, so
these generators produce tensors with the *shapes and structure* of that workload: a long KV
cache dominated by one contiguous span of video tokens, a handful of chain-drafted tokens,
final-layer hidden rows, an lm_head matrix.  Values are i.i.d. normal, rounded to bf16 with
round-to-nearest-even; the bf16 *bit patterns* (uint16) are the ground truth handed to both the
GPU library and the CPU oracle.

Two generators produce the same kind of tensor:
  * ``normal_bf16``        numpy Philox, host memory, bit-reproducible everywhere (parity tests)
  * ``normal_bf16_torch``  torch generator on the given device (full-size benchmark inputs;
                           copied back to the host when the oracle needs them)
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20260405

# tensor ids used to key the counter-based generator
T_Q, T_K, T_V, T_HD, T_HV, T_W, T_IDS, T_COIN, T_MISC = range(9)


@dataclasses.dataclass(frozen=True)
class VerifyConfig:
    name: str
    B: int
    gamma: int
    Hq: int
    Hkv: int
    D: int
    kv_len: Tuple[int, ...]          # cached prefix length per sequence
    vis_begin: Tuple[int, ...]       # first cache position of the video span per sequence
    vis_len: int                     # number of video tokens (= l_v)
    d: int                           # hidden size
    V: int                           # vocabulary size
    top_n: int = 10                  # N of the relevance metric
    lam: float = 0.7                 # loose parameter lambda
    n_loose: int = 0                 # length of Eq. 9's slice for this lambda and chain length,
                                     # written out per configuration (an input: each side has
                                     # its own function for floor(lambda * K))
    pst_window: int = 0              # 0 = off; >= gamma-1 = the paper's whole-draft range
    layers: int = 1
    n_branches: int = 1              # chains of the draft tree; gamma counts the rows of all
    qkv_std: float = 1.0
    act_std: float = 1.0
    w_std: float = 0.02
    seed: int = BASE_SEED

    @property
    def cap(self) -> int:
        return max(self.kv_len) + self.gamma

    @property
    def chain_len(self) -> int:
        return self.gamma // self.n_branches


    def tree_mask(self) -> Optional[np.ndarray]:
        """Row-visibility bit masks of the draft rows (None for a plain chain)."""
        return None if self.n_branches == 1 else branch_mask(self.n_branches, self.chain_len)

    @property
    def kv_bytes_per_layer(self) -> int:
        return sum(2 * (L + self.gamma) * self.Hkv * self.D * 2 for L in self.kv_len)

    def with_(self, **kw) -> "VerifyConfig":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, VerifyConfig] = {
    # single-layer tiny verify
    "c1": VerifyConfig("c1-tiny", B=1, gamma=4, Hq=8, Hkv=2, D=128, kv_len=(2048,),
                       vis_begin=(16,), vis_len=1568, d=1024, V=8192, pst_window=2,
                       n_loose=2, qkv_std=0.5, seed=BASE_SEED + 1),
    # Qwen2.5-VL-32B-shaped single layer
    "c2": VerifyConfig("c2-qwen2.5-vl-32b-layer", B=1, gamma=5, Hq=40, Hkv=8, D=128,
                       kv_len=(16384,), vis_begin=(16,), vis_len=14336, d=5120, V=152064,
                       pst_window=5, n_loose=3, seed=BASE_SEED + 2),
    # LLaVA-OneVision-72B-shaped single layer
    "c3": VerifyConfig("c3-llava-ov-72b-layer", B=1, gamma=5, Hq=64, Hkv=8, D=128,
                       kv_len=(7296,), vis_begin=(16,), vis_len=6272, d=8192, V=152064,
                       pst_window=5, n_loose=3, seed=BASE_SEED + 3),
    # 64-layer stack of the 32B shape, then one relevance + one lm_head/accept
    "c4": VerifyConfig("c4-qwen2.5-vl-32b-64layer-step", B=1, gamma=5, Hq=40, Hkv=8, D=128,
                       kv_len=(16384,), vis_begin=(16,), vis_len=14336, d=5120, V=152064,
                       pst_window=5, n_loose=3, layers=64, seed=BASE_SEED + 4),
    # long-video stress at the 72B shape
    "c5": VerifyConfig("c5-llava-ov-72b-long-b4", B=4, gamma=8, Hq=64, Hkv=8, D=128,
                       kv_len=(65536,) * 4, vis_begin=(16, 256, 1024, 2048), vis_len=63488,
                       d=8192, V=152064, pst_window=8, n_loose=5, seed=BASE_SEED + 5),
}


# draft trees (appendix on draft token trees): two chains of K = 10 on the 32B shape, and a tiny one
CONFIGS["c2t"] = CONFIGS["c2"].with_(name="c2t-qwen2.5-vl-32b-layer-tree2x10", gamma=20,
                                     n_branches=2, pst_window=10, n_loose=7, seed=BASE_SEED + 12)
CONFIGS["c4t"] = CONFIGS["c4"].with_(name="c4t-qwen2.5-vl-32b-64layer-step-tree2x10", gamma=20,
                                     n_branches=2, pst_window=10, n_loose=7, seed=BASE_SEED + 14)
CONFIGS["c1t"] = CONFIGS["c1"].with_(name="c1t-tiny-tree2x4", gamma=8, n_branches=2, n_loose=2,
                                     seed=BASE_SEED + 11)


def branch_mask(n_branches: int, chain_len: int) -> np.ndarray:
    """Visibility among the draft rows of a static tree of independent chains stored one after
    the other: row a*chain_len + i sees rows a*chain_len .. a*chain_len + i (bit j = row j)."""
    m = np.zeros((n_branches * chain_len,), np.uint32)
    for a in range(n_branches):
        for i in range(chain_len):
            m[a * chain_len + i] = np.uint32(((1 << (i + 1)) - 1) << (a * chain_len))
    return m


# --------------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round binary32 to bf16 (round-to-nearest-even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(
        np.float32)


def to_torch_bf16(bits: np.ndarray, device=None):
    """uint16 bit patterns -> torch.bfloat16 tensor (same bits), optionally on ``device``."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16)
    return t if device is None else t.to(device)


def from_torch_bf16(t) -> np.ndarray:
    """torch.bfloat16 tensor (any device) -> uint16 bit patterns on the host."""
    import torch
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


# --------------------------------------------------------------------------- generators
def _rng(key: Sequence[int]) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(list(map(int, key)))))


def normal_bf16(key: Sequence[int], shape: Sequence[int], std: float) -> np.ndarray:
    """N(0, std^2) in binary32, rounded to bf16; returns uint16 bit patterns of ``shape``."""
    rng = _rng(key)
    n = int(np.prod(shape))
    out = np.empty((n,), np.uint16)
    step = 1 << 24
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = f32_to_bf16_bits(rng.standard_normal(e - s, dtype=np.float32)
                                    * np.float32(std))
    return out.reshape(tuple(shape))


def normal_bf16_torch(key: Sequence[int], shape: Sequence[int], std: float, device):
    """Same distribution, generated by torch on ``device`` (bfloat16 tensor)."""
    import torch
    seed = int(np.random.SeedSequence(list(map(int, key))).generate_state(1, np.uint64)[0]
               & np.uint64(0x7FFFFFFFFFFFFFFF))
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    n = int(np.prod(shape))
    out = torch.empty((n,), dtype=torch.bfloat16, device=device)
    step = 1 << 27
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = (torch.randn((e - s,), generator=g, device=device, dtype=torch.float32)
                    * std).to(torch.bfloat16)
    return out.view(tuple(shape))


# --------------------------------------------------------------------------- input builders
def attn_inputs(cfg: VerifyConfig, layer: int = 0, device=None) -> dict:
    """Q, K, V of one target layer.

    q [B,gamma,Hq,D]; k, v [B,Hkv,cap,D] with the gamma draft rows already stored at
    kv_len[b] .. kv_len[b]+gamma-1 (rows past that are generated too and must be ignored).
    Host numpy uint16 when ``device`` is None, torch bfloat16 on ``device`` otherwise.
    """
    gen = normal_bf16 if device is None else (
        lambda key, shape, std: normal_bf16_torch(key, shape, std, device))
    q = gen((cfg.seed, T_Q, layer), (cfg.B, cfg.gamma, cfg.Hq, cfg.D), cfg.qkv_std)
    k = gen((cfg.seed, T_K, layer), (cfg.B, cfg.Hkv, cfg.cap, cfg.D), cfg.qkv_std)
    v = gen((cfg.seed, T_V, layer), (cfg.B, cfg.Hkv, cfg.cap, cfg.D), cfg.qkv_std)
    kv_len = np.asarray(cfg.kv_len, np.int32)
    vis_begin = np.asarray(cfg.vis_begin, np.int32)
    vis_end = vis_begin + np.int32(cfg.vis_len)
    return dict(q=q, k=k, v=v, kv_len=kv_len, vis_begin=vis_begin, vis_end=vis_end, cap=cfg.cap)


def hidden_inputs(cfg: VerifyConfig, variant: str = "literal", device=None) -> dict:
    """Final-layer hidden rows: h_d [B,gamma,d] (drafts), h_v [B,l_v,d] (video tokens).

    ``literal``     every row i.i.d. N(0, act_std^2): relevance scores of the gamma rows are
                    near ties (the configuration as written).
    ``structured``  h_d[i] = g_i + beta_i * h_v[j_i] with beta a seeded permutation of a fixed
                    ladder and j_i a seeded visual row: some rows align sharply with a few
                    video tokens (anchors), others have a flat profile (fillers), which is the
                    structure the paper describes for its similarity matrix (Sec. 3.1).
    """
    gen = normal_bf16 if device is None else (
        lambda key, shape, std: normal_bf16_torch(key, shape, std, device))
    h_v = gen((cfg.seed, T_HV), (cfg.B, cfg.vis_len, cfg.d), cfg.act_std)
    h_d = gen((cfg.seed, T_HD), (cfg.B, cfg.gamma, cfg.d), cfg.act_std)
    l_v = np.full((cfg.B,), cfg.vis_len, np.int32)
    if variant == "structured":
        ladder = np.resize(np.array([0.0, 0.15, 0.3, 0.6, 1.0, 1.5, 0.05, 0.45, 0.8, 1.2, 0.1,
                                     0.2, 0.7, 0.9, 1.1, 1.3], np.float32), cfg.gamma)
        rng = _rng((cfg.seed, T_MISC, 1))
        if device is None:
            hd32 = bf16_bits_to_f32(h_d)
            for b in range(cfg.B):
                beta = ladder[rng.permutation(cfg.gamma)]
                rows = rng.integers(0, cfg.vis_len, cfg.gamma)
                hd32[b] += beta[:, None] * bf16_bits_to_f32(h_v[b, rows])
            h_d = f32_to_bf16_bits(hd32)
        else:
            import torch
            hd32 = h_d.float()
            for b in range(cfg.B):
                beta = torch.from_numpy(ladder[rng.permutation(cfg.gamma)]).to(device)
                rows = torch.from_numpy(rng.integers(0, cfg.vis_len, cfg.gamma)).to(device)
                hd32[b] += beta[:, None] * h_v[b, rows].float()
            h_d = hd32.to(torch.bfloat16)
    elif variant != "literal":
        raise ValueError(variant)
    return dict(h_d=h_d, h_v=h_v, l_v=l_v)


def lm_head(cfg: VerifyConfig, device=None):
    """lm_head weight [V, d], N(0, w_std^2), row-major, no bias."""
    if device is None:
        return normal_bf16((cfg.seed, T_W), (cfg.V, cfg.d), cfg.w_std)
    return normal_bf16_torch((cfg.seed, T_W), (cfg.V, cfg.d), cfg.w_std, device)


def plant_target_rows(h_d: np.ndarray, w: np.ndarray, gain: float, key: Sequence[int]):
    """Add gain * W[v_i] to hidden row i for seeded token ids v_i, so that row i's largest
    logit is v_i by a wide margin (decision tests must not hinge on near ties).

    Returns (new h_d bits, planted ids [B,gamma] int32)."""
    B, gamma, d = h_d.shape
    rng = _rng(key)
    ids = rng.integers(0, w.shape[0], (B, gamma)).astype(np.int32)
    h32 = bf16_bits_to_f32(h_d)
    h32 += np.float32(gain) * bf16_bits_to_f32(w[ids.reshape(-1)]).reshape(B, gamma, d)
    return f32_to_bf16_bits(h32), ids


def draft_ids_uniform(cfg: VerifyConfig) -> np.ndarray:
    """Draft token ids uniform over the vocabulary, [B, gamma] int32."""
    return _rng((cfg.seed, T_IDS)).integers(0, cfg.V, (cfg.B, cfg.gamma)).astype(np.int32)


def draft_ids_from_target(y: np.ndarray, key: Sequence[int], p_shift: float = 0.5,
                          p_wrong: float = 0.0, V: Optional[int] = None) -> np.ndarray:
    """Drafts derived from given target ids y [B,gamma]: per position a seeded coin picks a
    copy of y_i, or the neighbour y_{i-1} (y_1 at position 0) to exercise the position-shift
    rule; with probability ``p_wrong`` a uniform random id instead."""
    y = np.asarray(y, np.int32)
    B, gamma = y.shape
    rng = _rng(key)
    coin = rng.random((B, gamma))
    wrong = rng.random((B, gamma)) < p_wrong
    rnd = rng.integers(0, V if V else int(y.max()) + 1, (B, gamma)).astype(np.int32)
    shifted = np.empty_like(y)
    shifted[:, 1:] = y[:, :-1]
    shifted[:, 0] = y[:, 1] if gamma > 1 else y[:, 0]
    d = np.where(coin < p_shift, shifted, y)
    return np.where(wrong, rnd, d).astype(np.int32)
