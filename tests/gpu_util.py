"""Helpers for the GPU parity tests: move seeded inputs to the device and call the C ABI."""
from __future__ import annotations

import numpy as np
import torch

import paper_2512_21487_amd as pkg
from workloads import MoEWorkload


def to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_pinned(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    t = torch.empty(a.shape, dtype=torch.from_numpy(a[:0]).dtype, pin_memory=True)
    t.copy_(torch.from_numpy(np.ascontiguousarray(a)))
    return t


def make_ctx(wl: MoEWorkload, *, max_tokens=None, max_chunks=8, pinned=False) -> pkg.MoeEp:
    return pkg.MoeEp(hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts,
                     local_begin=wl.local_begin, n_local=wl.n_local, n_shared=wl.n_shared,
                     shared_inter=wl.shared_inter, max_tokens=max_tokens or max(wl.n_tokens, 1),
                     max_top_k=wl.top_k, max_chunks=max_chunks,
                     io_mode=pkg.IO_PINNED_HOST if pinned else pkg.IO_DEVICE)


class DeviceInputs:
    """Inputs of one workload resident where the context expects them."""

    def __init__(self, wl: MoEWorkload, inp, pinned=False):
        put = to_pinned if pinned else to_dev
        self.tokens = put(inp["tokens"])
        self.logits = put(inp["gate_logits"])
        self.routed = to_dev(inp["routed_w"])
        self.shared = to_dev(inp["shared_w"]) if inp["shared_w"] is not None else None
        T = inp["tokens"].shape[0]
        if pinned:
            self.out = torch.zeros((T, wl.hidden), dtype=torch.int16, pin_memory=True)
        else:
            self.out = torch.zeros((T, wl.hidden), dtype=torch.int16, device="cuda")
        self.T = T


def run_forward(ctx: pkg.MoeEp, wl: MoEWorkload, d: DeviceInputs, r=1, order=0, n_tokens=None):
    """One forward through the C ABI; returns the output as uint16 bf16 bits (host)."""
    T = d.T if n_tokens is None else n_tokens
    d.out.zero_()  # clear stale results
    torch.cuda.synchronize()
    ctx.forward(d.tokens, d.logits, d.routed, d.shared, wl.top_k, r, order, n_tokens=T, out=d.out)
    torch.cuda.synchronize()
    return d.out.cpu().numpy().view(np.uint16)[:T].copy()


def run_forward_dep(ctx: pkg.MoeEp, wl: MoEWorkload, d: DeviceInputs, r_1=1, r_2=1, dep_order=0, attn_us=0.0):
    """One moe_ep_forward_dep through the C ABI; returns the output as uint16 bf16 bits (host)."""
    d.out.zero_()
    torch.cuda.synchronize()
    ctx.forward_dep(d.tokens, d.logits, d.routed, d.shared, wl.top_k, r_1, r_2, dep_order, attn_us,
                    n_tokens=d.T, out=d.out)
    torch.cuda.synchronize()
    return d.out.cpu().numpy().view(np.uint16)[:d.T].copy()
