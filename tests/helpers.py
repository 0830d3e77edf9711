"""Test-side reference formulations that are independent of oracle/ (numpy, float64)."""
from __future__ import annotations

import numpy as np
from scipy.special import expit, softmax

from workloads import bf16_bits_to_f32


def f64(bits):
    return bf16_bits_to_f32(np.asarray(bits, dtype=np.uint16)).astype(np.float64)


def split_expert(w_bits, i, M, H):
    """(Wg [H,M], Wu [H,M], Wd [M,H]) of expert i as float64."""
    sz = 3 * H * M
    w = f64(np.asarray(w_bits).reshape(-1)[i * sz:(i + 1) * sz])
    return (w[:H * M].reshape(H, M), w[H * M:2 * H * M].reshape(H, M),
            w[2 * H * M:].reshape(M, H))


def dense_ffn(X, Wg, Wu, Wd):
    """Textbook SwiGLU feed-forward on all rows of X with library matmuls."""
    g = X @ Wg.T
    u = X @ Wu.T
    return (g * expit(g) * u) @ Wd.T


def topk_by_sort(logits_row, k):
    """Explicit full sort: larger score first, equal scores -> lower index first."""
    order = sorted(range(len(logits_row)), key=lambda e: (-float(logits_row[e]), e))
    return order[:k]


def brute_force_layer(tokens_bits, logits, routed_bits, shared_bits, *, M, H, E, e0, El,
                      Ns, Hs, k):
    """Dense-masked MoE layer: every local expert on every token, masked by the gate."""
    X = f64(tokens_bits)
    T = X.shape[0]
    P = softmax(np.asarray(logits, dtype=np.float64), axis=1)
    G = np.zeros((T, E))
    for t in range(T):
        sel = topk_by_sort(logits[t], k)
        G[t, sel] = P[t, sel] / P[t, sel].sum()
    out = np.zeros((T, M))
    for e in range(El):
        out += G[:, e0 + e, None] * dense_ffn(X, *split_expert(routed_bits, e, M, H))
    for i in range(Ns):
        out += dense_ffn(X, *split_expert(shared_bits, i, M, Hs))
    return out, G


def rel_err(got, ref):
    """max_i |got - ref| / max(|ref_i|, rms(ref)): the parity figure used everywhere."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), max(rms, 1e-30))
    return float(np.max(np.abs(got - ref) / den)) if ref.size else 0.0


def rel_err_rows(got, ref):
    """max over elements of |got - ref| / max(|ref_i|, rms of ref's own row): the GPU parity figure.

    A row is one token's output vector; tokens are independent (Sec. 2.3) and, on an expert-group
    share, their scales differ by an order of magnitude (the kept routing weights of a token sum to
    anything between 0 and 1), while every rounding error of the path scales with the row it is in.
    A floor taken over all rows would judge the rows of large norm by the scale of the small ones:
    with it, rounding the activation to bf16 alone, which a bf16 down projection cannot avoid, gives
    1.5-2.3e-2 on the decode-shaped shares.  Rows that are exactly zero in ref must be exactly zero."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    den = np.maximum(np.abs(ref), np.maximum(rms, 1e-30))
    return float(np.max(np.abs(got - ref) / den))


def load_tiny_golden(path):
    """Parse tests/golden/tiny_oracle_values.txt -> (count, routing rows, output samples, rms)."""
    sections, cur = [], None
    for line in open(path):
        line = line.strip()
        if not line:
            continue
        if line.startswith("#"):
            cur = []
            sections.append(cur)
            continue
        cur.append(line.split())
    _, count, routing, samples, rms = sections
    return ([int(v) for v in count[0]],
            [(int(r[0]), int(r[1]), int(r[2]), float(r[3]), float(r[4])) for r in routing],
            [(int(r[0]), int(r[1]), float(r[2])) for r in samples], float(rms[0][0]))
