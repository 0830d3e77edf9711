"""CPU oracle for the expert-group MoE layer -- TEST INFRASTRUCTURE.

Thin ctypes access to ``moe_oracle.c`` (plain C, IEEE double).  Only tests,
the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the HIP library and its Python binding never do, and this package
imports nothing from them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (portable flags: the library travels to another host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.moe_oracle_threads.restype = ctypes.c_int
        for name in ("moe_oracle_router", "moe_oracle_dispatch", "moe_oracle_expert_ffn",
                     "moe_oracle_forward", "moe_oracle_forward_tokens"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def threads() -> int:
    return int(_load().moe_oracle_threads())


def router(logits: np.ndarray, k: int):
    """Sec. 2.1 gate. Returns (idx int32 [T,k], w float64 [T,k])."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    idx = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k), dtype=np.float64)
    rc = _load().moe_oracle_router(_p(logits), T, E, k, _p(idx), _p(w))
    if rc != 0:
        raise ValueError("moe_oracle_router: bad arguments")
    return idx, w


def dispatch(idx: np.ndarray, e0: int, n_local: int) -> Dict[str, np.ndarray]:
    """Partition of the kept assignments by local expert (stable)."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, k = idx.shape
    count = np.zeros(n_local, dtype=np.int32)
    offset = np.zeros(n_local + 1, dtype=np.int32)
    perm = np.full(T * k + 1, -1, dtype=np.int32)
    pos = np.full((T, k), -1, dtype=np.int32)
    rc = _load().moe_oracle_dispatch(_p(idx), T, k, e0, n_local, _p(count), _p(offset),
                                     _p(perm), _p(pos))
    if rc != 0:
        raise ValueError("moe_oracle_dispatch: bad arguments")
    return {"count": count, "offset": offset, "perm": perm[:offset[-1]].copy(), "pos": pos}


def expert_ffn(x_bits: np.ndarray, wexp_bits: np.ndarray, M: int, H: int,
               literal_swish: bool = False) -> np.ndarray:
    x_bits = np.ascontiguousarray(x_bits, dtype=np.uint16)
    wexp_bits = np.ascontiguousarray(wexp_bits, dtype=np.uint16)
    assert x_bits.size == M and wexp_bits.size == 3 * H * M
    y = np.zeros(M, dtype=np.float64)
    rc = _load().moe_oracle_expert_ffn(_p(x_bits), _p(wexp_bits), M, H, int(literal_swish), _p(y))
    if rc != 0:
        raise ValueError("moe_oracle_expert_ffn: bad arguments")
    return y


def forward(tokens: np.ndarray, logits: np.ndarray, routed_w: np.ndarray,
            shared_w: Optional[np.ndarray], *, hidden: int, inter: int, n_experts: int,
            local_begin: int, n_local: int, n_shared: int, shared_inter: int, top_k: int,
            r_chunks: int = 1, literal_swish: bool = False) -> Dict[str, np.ndarray]:
    """Whole path over r contiguous chunks. Returns out (float64), out_bf16 and routing."""
    tokens = np.ascontiguousarray(tokens, dtype=np.uint16)
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    routed_w = np.ascontiguousarray(routed_w, dtype=np.uint16)
    T = tokens.shape[0]
    M, H, E, k, r = hidden, inter, n_experts, top_k, r_chunks
    assert tokens.shape == (T, M) and logits.shape == (T, E)
    assert routed_w.size == n_local * 3 * H * M
    if n_shared > 0:
        shared_w = np.ascontiguousarray(shared_w, dtype=np.uint16)
        assert shared_w.size == n_shared * 3 * shared_inter * M
    Tc = (T + r - 1) // r if r > 0 else 0
    out = np.zeros((T, M), dtype=np.float64)
    out_bf16 = np.zeros((T, M), dtype=np.uint16)
    idx = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k), dtype=np.float64)
    pos = np.full((T, k), -1, dtype=np.int32)
    count = np.zeros((r, n_local), dtype=np.int32)
    offset = np.zeros((r, n_local + 1), dtype=np.int32)
    perm = np.full((r, max(Tc * k, 1)), -1, dtype=np.int32)
    rc = _load().moe_oracle_forward(
        _p(tokens), _p(logits), _p(routed_w), _p(shared_w), T, M, H, E, local_begin, n_local,
        n_shared, shared_inter, k, r, int(literal_swish), _p(out), _p(out_bf16),
        _p(idx), _p(w), _p(pos), _p(count), _p(offset), _p(perm))
    if rc != 0:
        raise ValueError("moe_oracle_forward: bad arguments")
    return {"out": out, "out_bf16": out_bf16, "idx": idx, "w": w, "pos": pos,
            "count": count, "offset": offset, "perm": perm}


def forward_tokens(tokens: np.ndarray, logits: np.ndarray, routed_w: np.ndarray,
                   shared_w: Optional[np.ndarray], ids: Sequence[int], *, hidden: int,
                   inter: int, n_experts: int, local_begin: int, n_local: int, n_shared: int,
                   shared_inter: int, top_k: int, literal_swish: bool = False) -> np.ndarray:
    """Layer output (float64 [len(ids), M]) of the listed tokens only."""
    tokens = np.ascontiguousarray(tokens, dtype=np.uint16)
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    routed_w = np.ascontiguousarray(routed_w, dtype=np.uint16)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T = tokens.shape[0]
    M, H, E = hidden, inter, n_experts
    assert tokens.shape == (T, M) and logits.shape == (T, E)
    assert routed_w.size == n_local * 3 * H * M
    if n_shared > 0:
        shared_w = np.ascontiguousarray(shared_w, dtype=np.uint16)
        assert shared_w.size == n_shared * 3 * shared_inter * M
    out = np.zeros((ids.size, M), dtype=np.float64)
    rc = _load().moe_oracle_forward_tokens(
        _p(tokens), _p(logits), _p(routed_w), _p(shared_w), T, M, H, E, local_begin, n_local,
        n_shared, shared_inter, top_k, int(literal_swish), _p(ids), int(ids.size), _p(out))
    if rc != 0:
        raise ValueError("moe_oracle_forward_tokens: bad arguments")
    return out
