"""Seeded synthetic inputs for the expert-group MoE layer.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests / benchmark.  It holds shapes and random-number recipes only:
no routing, no FFN arithmetic, nothing either implementation computes.

Shapes follow the public layer shapes of the two backbones the paper evaluates
(DeepSeek-V2 and Qwen3-MoE, Sec. 5.4); the values are synthetic because the
method's cost depends on shapes and on the routing histogram only.

Every tensor is drawn from its own PCG64 stream keyed by (seed, cfg_id,
tensor_id), so a tensor's values do not depend on which other tensors were
generated before it.

bf16 tensors are returned as uint16 bit patterns (round-to-nearest-even from
fp32); gate logits are fp32.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

__all__ = ["MoEWorkload", "CONFIGS", "make_inputs", "f32_to_bf16_bits",
           "bf16_bits_to_f32", "tiny_workload"]


@dataclass(frozen=True)
class MoEWorkload:
    """One synthetic MoE-layer problem (notation of Table 'Notations')."""
    name: str
    cfg_id: int
    n_tokens: int          # tokens handed to one forward
    hidden: int            # M
    inter: int             # H of a routed expert
    n_experts: int         # E, global
    local_begin: int       # first expert held by this GPU
    n_local: int           # E / eg
    top_k: int
    n_shared: int          # N_shared
    shared_inter: int      # H of a shared expert
    zipf_s: float = 0.0    # >0: add a Zipf(s) per-expert bias to the logits
    r_sweep: tuple = (1,)
    pinned_io: bool = False

    @property
    def routed_weight_elems(self) -> int:
        return self.n_local * 3 * self.inter * self.hidden

    @property
    def shared_weight_elems(self) -> int:
        return self.n_shared * 3 * self.shared_inter * self.hidden


CONFIGS: Dict[str, MoEWorkload] = {
    # 1. correctness anchor
    "tiny": MoEWorkload("tiny", 1, 128, 256, 512, 8, 0, 8, 2, 1, 512,
                        r_sweep=(1,)),
    # 2. DeepSeek-V2-Lite-shaped layer, all experts local, no skew
    "dsv2_lite": MoEWorkload("dsv2_lite", 2, 4096, 2048, 1408, 64, 0, 64, 6,
                             2, 1408, r_sweep=(1, 2, 4)),
    # 3. Qwen3-30B-A3B-shaped layer, Zipf-skewed expert load, no shared expert
    "qwen3_30b": MoEWorkload("qwen3_30b", 3, 8192, 2048, 768, 128, 0, 128, 8,
                             0, 0, zipf_s=1.1, r_sweep=(1, 2, 4, 8)),
    # 4. DeepSeek-V2-shaped expert-group share: 20 of 160 experts on this GPU
    "dsv2_eg": MoEWorkload("dsv2_eg", 4, 16384, 5120, 1536, 160, 0, 20, 6,
                           2, 1536, r_sweep=(1, 2, 4, 8)),
    # 5. Qwen3-235B-A22B-shaped expert-group share, decode-sized micro-batches
    "qwen3_235b_eg_256": MoEWorkload("qwen3_235b_eg_256", 5, 256, 4096, 1536,
                                     128, 0, 16, 8, 0, 0,
                                     r_sweep=(1, 2, 4, 8), pinned_io=True),
    "qwen3_235b_eg_1024": MoEWorkload("qwen3_235b_eg_1024", 5, 1024, 4096,
                                      1536, 128, 0, 16, 8, 0, 0,
                                      r_sweep=(1, 2, 4, 8), pinned_io=True),
    "qwen3_235b_eg_4096": MoEWorkload("qwen3_235b_eg_4096", 5, 4096, 4096,
                                      1536, 128, 0, 16, 8, 0, 0,
                                      r_sweep=(1, 2, 4, 8), pinned_io=True),
}


def tiny_workload(**overrides) -> MoEWorkload:
    """A small ad-hoc problem for unit tests (cfg_id 0)."""
    base = MoEWorkload("adhoc", 0, 16, 64, 64, 8, 0, 8, 2, 0, 0)
    return replace(base, **overrides)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


_TENSOR_IDS = {"tokens": 0, "gate_logits": 1, "routed_w": 2, "shared_w": 3,
               "zipf_perm": 4}


def _rng(seed: int, cfg_id: int, tensor: str) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(
        np.random.SeedSequence([seed, cfg_id, _TENSOR_IDS[tensor]])))


def _normal_bf16(rng: np.random.Generator, n: int, std: float) -> np.ndarray:
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24                      # bounded temporaries for the big layers
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        v = rng.standard_normal(hi - lo, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        out[lo:hi] = f32_to_bf16_bits(v)
    return out


def make_inputs(wl: MoEWorkload, seed: int = 0,
                n_tokens: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw the tensors of one forward call.

    tokens      uint16 [T, M]   bf16 bits of N(0, 1)
    gate_logits float32 [T, E]  N(0, 1) over the GLOBAL expert axis, plus the
                                per-expert bias b_e = -s * ln(rank_e) when
                                zipf_s > 0 (rank = seeded permutation of 1..E,
                                i.e. softmax prior proportional to rank^-s)
    routed_w    uint16 [E_l, 3, ...] per local expert: W_gate[H, M], W_up[H, M],
                                W_down[M, H], bf16 bits of N(0, 0.02^2); flat
    shared_w    uint16          same triple per shared expert, or None
    """
    T = wl.n_tokens if n_tokens is None else n_tokens
    M, H, E = wl.hidden, wl.inter, wl.n_experts
    tokens = _normal_bf16(_rng(seed, wl.cfg_id, "tokens"), T * M, 1.0)
    logits = _rng(seed, wl.cfg_id, "gate_logits").standard_normal(
        (T, E), dtype=np.float32)
    if wl.zipf_s > 0.0:
        rank = _rng(seed, wl.cfg_id, "zipf_perm").permutation(E) + 1
        bias = (-wl.zipf_s * np.log(rank.astype(np.float64))).astype(np.float32)
        logits = (logits + bias[None, :]).astype(np.float32)
    routed = _normal_bf16(_rng(seed, wl.cfg_id, "routed_w"),
                          wl.routed_weight_elems, 0.02)
    shared = None
    if wl.n_shared > 0:
        shared = _normal_bf16(_rng(seed, wl.cfg_id, "shared_w"),
                              wl.shared_weight_elems, 0.02)
    return {"tokens": tokens.reshape(T, M),
            "gate_logits": np.ascontiguousarray(logits),
            "routed_w": routed, "shared_w": shared}
