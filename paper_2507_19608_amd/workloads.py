"""Seeded synthetic Q/K/V for the five benchmark configurations.

This module only draws random numbers.  It holds none of the method's
arithmetic (no delta, no threshold, no attention) so that both the GPU library's
callers and the CPU oracle's tests can take their inputs from it.

The paper measures on real activations of two language models over public
evaluation suites; neither is available offline, so these tensors stand in for
them: an AR(1) random walk per channel supplies the token-to-token correlation
that makes key deltas sparse, and occasional whole-vector jumps supply the dense
delta rows.  Recipe, per (tensor, batch, head) stream, all in float64:

    x_0 ~ N(0, sigma_s^2),  sigma_s = 0.1 / sqrt(1 - 0.95^2)   (stationary std)
    for t >= 1:  with probability p_jump (one draw per token, whole vector)
                     x_t ~ N(0, I)
                 else x_t = 0.95 x_{t-1} + N(0, 0.1^2 I)
    multi-head configs scale each stream by s ~ U(0.5, 2)

The stream is then rounded (nearest-even) to the configuration's dtype.
Random numbers come from numpy's counter-based Philox generator keyed by
(seed, tensor, batch, head, purpose), so any stream can be regenerated alone
and a longer sequence extends a shorter one.
"""
import json
import os
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

_TENSOR_ID = {"Q": 1, "K": 2, "V": 3}
_RHO = 0.95
_SIGMA = 0.1


def _gen(seed: int, tensor: str, b: int, h: int, purpose: int) -> np.random.Generator:
    key = np.array([np.uint64(seed), (np.uint64(_TENSOR_ID[tensor]) << np.uint64(56))
                    | (np.uint64(purpose) << np.uint64(48)) | (np.uint64(b) << np.uint64(24)) | np.uint64(h)],
                   dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def ar1_jump(seed: int, tensor: str, batch_ids, heads: int, n: int, d: int, p_jump: float,
             per_head_scale: bool) -> np.ndarray:
    """float64 array [len(batch_ids), heads, n, d] following the recipe above."""
    out = np.empty((len(batch_ids), heads, n, d))
    for bi, b in enumerate(batch_ids):
        noise = np.empty((heads, n, d))
        jumpv = np.empty((heads, n, d))
        jumpf = np.empty((heads, n), dtype=bool)
        scale = np.ones(heads)
        for h in range(heads):
            noise[h] = _gen(seed, tensor, b, h, 0).standard_normal((n, d))
            jumpv[h] = _gen(seed, tensor, b, h, 1).standard_normal((n, d))
            jumpf[h] = _gen(seed, tensor, b, h, 2).random(n) < p_jump
            if per_head_scale:
                scale[h] = 0.5 + 1.5 * _gen(seed, tensor, b, h, 3).random()
        x = out[bi]
        x[:, 0] = noise[:, 0] * (_SIGMA / np.sqrt(1.0 - _RHO * _RHO))
        for t in range(1, n):
            step = _RHO * x[:, t - 1] + _SIGMA * noise[:, t]
            x[:, t] = np.where(jumpf[:, t, None], jumpv[:, t], step)
        x *= scale[:, None, None]
    return out


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int            # prefill length (decode config: cached tokens)
    window: int             # prefill window W (decode config: W_d)
    dtype: str              # "f32" | "bf16"
    seed: int
    p_jump: float = 0.05
    decode_steps: int = 0
    theta: Optional[float] = None       # fixed threshold, or None -> looked up by target
    target_sparsity: Optional[float] = None
    per_head_scale: bool = True

    @property
    def total_len(self) -> int:
        return self.seq_len + self.decode_steps

    def key(self) -> str:
        t = "fixed" if self.target_sparsity is None else f"s{int(round(self.target_sparsity * 100)):02d}"
        return f"{self.name}/p{int(round(self.p_jump * 100)):02d}/{t}"


# The five configurations.  C5 is a family: theta in {0, s40, s60, s80} x p_jump in {1, 5, 20} %.
C1 = Workload("C1", 1, 1, 1, 64, 256, 32, "f32", seed=0, theta=0.05, per_head_scale=False)
C2 = Workload("C2", 1, 32, 8, 64, 2048, 128, "bf16", seed=2, target_sparsity=0.60)
C3 = Workload("C3", 1, 20, 5, 128, 4096, 256, "bf16", seed=3, target_sparsity=0.60)
C4 = Workload("C4", 32, 32, 8, 64, 2048, 128, "bf16", seed=4, decode_steps=256, target_sparsity=0.57)


def c5(target_sparsity: Optional[float] = 0.60, p_jump: float = 0.05) -> Workload:
    if target_sparsity is None or target_sparsity == 0.0:
        return Workload("C5", 4, 20, 5, 128, 8192, 512, "bf16", seed=5, p_jump=p_jump, theta=0.0)
    return Workload("C5", 4, 20, 5, 128, 8192, 512, "bf16", seed=5, p_jump=p_jump,
                    target_sparsity=target_sparsity)


C5 = c5()
C5_SWEEP = tuple(c5(s, p) for p in (0.01, 0.05, 0.20) for s in (0.0, 0.40, 0.60, 0.80))
ALL = {"C1": C1, "C2": C2, "C3": C3, "C4": C4, "C5": C5}

_THETA_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "workload_thetas.json")


def theta_for(w: Workload) -> float:
    """Threshold of a workload: its fixed value, or the stored value that was tuned (by the
    committed tuning script) to the workload's target delta-matrix sparsity."""
    if w.theta is not None:
        return float(w.theta)
    with open(_THETA_FILE) as f:
        table = json.load(f)
    return float.fromhex(table[w.key()]["theta_hex"])


def generate(w: Workload, tensors: Tuple[str, ...] = ("Q", "K", "V"), batch_ids=None) -> Dict[str, np.ndarray]:
    """float64 arrays (already rounded to w.dtype's grid) of length w.total_len.

    Q: [B, Hq, L, d], K/V: [B, Hkv, L, d].  `batch_ids` picks batch entries (streams are
    independent, so a subset equals the same entries of the full tensor)."""
    ids = list(range(w.batch)) if batch_ids is None else list(batch_ids)
    out = {}
    for name in tensors:
        H = w.n_q_heads if name == "Q" else w.n_kv_heads
        x = ar1_jump(w.seed, name, ids, H, w.total_len, w.head_dim, w.p_jump, w.per_head_scale)
        out[name] = round_to_dtype(x, w.dtype)
    return out


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the nearest (ties-to-even) value of dtype, returned as float64."""
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype == "bf16":
        f = np.ascontiguousarray(x.astype(np.float32))
        u = f.view(np.uint32).astype(np.uint64)
        u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
        return u.astype(np.uint32).view(np.float32).astype(np.float64)
    raise ValueError(dtype)
