#!/usr/bin/env python3
"""Writes tiny_oracle_values.txt from the CPU oracle (and nothing else) for the `tiny` workload."""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from workloads import CONFIGS, make_inputs  # noqa: E402


def main() -> None:
    wl = CONFIGS["tiny"]
    inp = make_inputs(wl, seed=0)
    res = oracle.forward(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"],
                         hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts, local_begin=0,
                         n_local=wl.n_local, n_shared=wl.n_shared, shared_inter=wl.shared_inter,
                         top_k=wl.top_k)
    lines = ["# tiny workload, seed 0, written by make_tiny_oracle_values.py from oracle/ only",
             "# count per expert", " ".join(str(int(c)) for c in res["count"][0]),
             "# token idx0 idx1 w0 w1 (first 16 tokens)"]
    for t in range(16):
        lines.append(f"{t} {res['idx'][t, 0]} {res['idx'][t, 1]} {res['w'][t, 0]:.12f} {res['w'][t, 1]:.12f}")
    lines.append("# token column value (output, float64)")
    rng = np.random.default_rng(7)
    for _ in range(64):
        t, c = int(rng.integers(0, wl.n_tokens)), int(rng.integers(0, wl.hidden))
        lines.append(f"{t} {c} {res['out'][t, c]:.12e}")
    lines.append(f"# rms of the whole output\n{float(np.sqrt(np.mean(res['out'] ** 2))):.12e}")
    with open(os.path.join(HERE, "tiny_oracle_values.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
