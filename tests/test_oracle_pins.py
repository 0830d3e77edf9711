"""Pins for the CPU oracle: it is checked against things other than itself.

The paper prints no worked numeric example of an MoE-layer forward, so the pins
are: a hand-derived closed form, a dense-masked brute force built from library
matmul / softmax / sort, special cases that collapse to a textbook dense FFN,
and invariants the definitions imply (Sec. 2.1, Sec. 3.1, Sec. 2.3, and the
token-conservation rule of Eq. 'limitation').
"""
import math
import os

import numpy as np
import pytest
from scipy.special import softmax

import oracle
from helpers import (brute_force_layer, dense_ffn, f64, load_tiny_golden, rel_err, split_expert,
                     topk_by_sort)
from workloads import CONFIGS, f32_to_bf16_bits, make_inputs, tiny_workload


def _fwd(inp, wl, **kw):
    args = dict(hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts,
                local_begin=wl.local_begin, n_local=wl.n_local, n_shared=wl.n_shared,
                shared_inter=wl.shared_inter, top_k=wl.top_k)
    args.update(kw)
    return oracle.forward(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"],
                          **args)


def silu(v):
    return v / (1.0 + math.exp(-v))


# ---------------------------------------------------------------- closed form
def test_hand_worked_example():
    """2 tokens, 3 experts, top-2, M = H = 2, integer weights: every output element is
    written out by hand from Sec. 2.1 (gate) and Sec. 3.1 (three projections + Swish gate)."""
    M = H = 2
    bits = lambda a: f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    experts = [  # (W_gate [H,M], W_up [H,M], W_down [M,H])
        ([[1, 0], [0, 1]], [[1, 1], [1, -1]], [[1, 0], [0, 2]]),
        ([[0, 1], [1, 0]], [[2, 0], [0, 2]], [[1, 1], [1, -1]]),
        ([[1, 1], [-1, 1]], [[1, 0], [0, 1]], [[0, 1], [1, 0]]),
    ]
    routed = np.concatenate([bits(m).reshape(-1) for e in experts for m in e])
    tokens = bits([[1.0, 2.0], [-1.0, 0.5]])
    logits = np.array([[0.0, math.log(2.0), math.log(3.0)],   # p = 1/6, 2/6, 3/6
                       [1.0, 1.0, 0.0]], dtype=np.float32)     # tie between experts 0 and 1
    res = oracle.forward(tokens, logits, routed, None, hidden=M, inter=H, n_experts=3,
                         local_begin=0, n_local=3, n_shared=0, shared_inter=0, top_k=2)
    assert res["idx"].tolist() == [[2, 1], [0, 1]]
    np.testing.assert_allclose(res["w"], [[0.6, 0.4], [0.5, 0.5]], rtol=0, atol=2e-7)
    # token 0 = (1, 2): 0.6 * expert2 + 0.4 * expert1
    e2 = [2 * silu(1), silu(3)]
    e1 = [2 * silu(2) + 4 * silu(1), 2 * silu(2) - 4 * silu(1)]
    # token 1 = (-1, 0.5): 0.5 * expert0 + 0.5 * expert1
    f0 = [-0.5 * silu(-1), -3 * silu(0.5)]
    f1 = [-2 * silu(0.5) + silu(-1), -2 * silu(0.5) - silu(-1)]
    want = [[0.6 * e2[0] + 0.4 * e1[0], 0.6 * e2[1] + 0.4 * e1[1]],
            [0.5 * (f0[0] + f1[0]), 0.5 * (f0[1] + f1[1])]]
    np.testing.assert_allclose(res["out"], want, rtol=0, atol=1e-6)
    # partition: expert 0 <- token 1; expert 1 <- tokens 0, 1; expert 2 <- token 0
    assert res["count"].tolist() == [[1, 2, 1]]
    assert res["offset"].tolist() == [[0, 1, 3, 4]]
    assert res["perm"][0, :4].tolist() == [2, 1, 3, 0]      # assignment id = t*k + slot
    assert res["pos"].tolist() == [[3, 1], [0, 2]]


def test_literal_swish_switch_differs_and_matches_its_formula():
    """The printed form Swish(z_gate * z_up) is kept as a switch; check it is that form."""
    M, H = 4, 3
    rng = np.random.default_rng(5)
    x = f32_to_bf16_bits(rng.standard_normal(M).astype(np.float32))
    w = f32_to_bf16_bits(rng.standard_normal(3 * H * M).astype(np.float32))
    Wg, Wu, Wd = split_expert(w, 0, M, H)
    g, u = Wg @ f64(x), Wu @ f64(x)
    lit = Wd @ np.array([silu(v) for v in g * u])
    std = Wd @ (np.array([silu(v) for v in g]) * u)
    np.testing.assert_allclose(oracle.expert_ffn(x, w, M, H, literal_swish=True), lit, atol=1e-12)
    np.testing.assert_allclose(oracle.expert_ffn(x, w, M, H), std, atol=1e-12)
    assert np.max(np.abs(lit - std)) > 1e-3


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("k", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("shared", [0, 2])
def test_brute_force_dense_masked(k, shared):
    wl = tiny_workload(n_tokens=13, hidden=24, inter=40, n_experts=8, n_local=8, top_k=k,
                       n_shared=shared, shared_inter=16 if shared else 0)
    inp = make_inputs(wl, seed=k + 10 * shared)
    res = _fwd(inp, wl)
    ref, G = brute_force_layer(inp["tokens"], inp["gate_logits"], inp["routed_w"],
                               inp["shared_w"], M=wl.hidden, H=wl.inter, E=8, e0=0, El=8,
                               Ns=wl.n_shared, Hs=wl.shared_inter, k=k)
    np.testing.assert_allclose(res["out"], ref, rtol=1e-10, atol=1e-12)
    for t in range(wl.n_tokens):
        assert res["idx"][t].tolist() == topk_by_sort(inp["gate_logits"][t], k)
        np.testing.assert_allclose(res["w"][t], G[t, res["idx"][t]], rtol=1e-12)


def test_brute_force_local_share_nonzero_begin():
    """Only experts [3, 6) of 8 are local: the other assignments drop out, weights are not
    renormalised after the filter."""
    wl = tiny_workload(n_tokens=16, hidden=16, inter=24, n_experts=8, local_begin=3, n_local=3,
                       top_k=3, n_shared=1, shared_inter=8)
    inp = make_inputs(wl, seed=3)
    res = _fwd(inp, wl)
    ref, _ = brute_force_layer(inp["tokens"], inp["gate_logits"], inp["routed_w"],
                               inp["shared_w"], M=16, H=24, E=8, e0=3, El=3, Ns=1, Hs=8, k=3)
    np.testing.assert_allclose(res["out"], ref, rtol=1e-10, atol=1e-12)


# ------------------------------------------------- special cases -> dense FFN
def test_single_expert_k1_is_dense_ffn():
    wl = tiny_workload(n_tokens=9, hidden=32, inter=48, n_experts=1, n_local=1, top_k=1)
    inp = make_inputs(wl, seed=1)
    res = _fwd(inp, wl)
    ref = dense_ffn(f64(inp["tokens"]), *split_expert(inp["routed_w"], 0, 32, 48))
    np.testing.assert_allclose(res["out"], ref, rtol=1e-10, atol=1e-12)
    assert np.all(res["idx"] == 0) and np.all(res["w"] == 1.0)


def test_identical_experts_give_dense_ffn_for_any_routing():
    """Weights sum to 1, so with all experts equal the routing cannot matter."""
    wl = tiny_workload(n_tokens=11, hidden=16, inter=32, n_experts=6, n_local=6, top_k=3)
    inp = make_inputs(wl, seed=2)
    one = inp["routed_w"][:3 * 32 * 16]
    inp["routed_w"] = np.tile(one, 6)
    res = _fwd(inp, wl)
    ref = dense_ffn(f64(inp["tokens"]), *split_expert(one, 0, 16, 32))
    np.testing.assert_allclose(res["out"], ref, rtol=1e-10, atol=1e-12)


def test_k_equals_E_is_full_softmax_mixture():
    wl = tiny_workload(n_tokens=7, hidden=16, inter=16, n_experts=5, n_local=5, top_k=5)
    inp = make_inputs(wl, seed=4)
    res = _fwd(inp, wl)
    P = softmax(inp["gate_logits"].astype(np.float64), axis=1)
    X = f64(inp["tokens"])
    ref = sum(P[:, e, None] * dense_ffn(X, *split_expert(inp["routed_w"], e, 16, 16))
              for e in range(5))
    np.testing.assert_allclose(res["out"], ref, rtol=1e-10, atol=1e-12)


def test_all_equal_logits_pick_first_k_with_uniform_weights():
    logits = np.full((5, 7), 0.25, dtype=np.float32)
    idx, w = oracle.router(logits, 4)
    assert idx.tolist() == [[0, 1, 2, 3]] * 5
    np.testing.assert_allclose(w, 0.25, rtol=0, atol=1e-15)


def test_zero_down_projection_gives_zeros():
    wl = tiny_workload(n_tokens=6, hidden=16, inter=16, n_experts=4, n_local=4, top_k=2)
    inp = make_inputs(wl, seed=6)
    w = inp["routed_w"].reshape(4, 3, 16 * 16).copy()
    w[:, 2, :] = 0
    inp["routed_w"] = w.reshape(-1)
    assert np.all(_fwd(inp, wl)["out"] == 0.0)


def test_shared_only_is_dense_ffn_of_concatenated_intermediate():
    """No token selects the (single) local expert -> output = sum of the shared experts."""
    wl = tiny_workload(n_tokens=10, hidden=16, inter=16, n_experts=4, local_begin=3, n_local=1,
                       top_k=2, n_shared=2, shared_inter=24)
    inp = make_inputs(wl, seed=7)
    inp["gate_logits"][:, 3] = -50.0
    res = _fwd(inp, wl)
    X = f64(inp["tokens"])
    ref = sum(dense_ffn(X, *split_expert(inp["shared_w"], i, 16, 24)) for i in range(2))
    np.testing.assert_allclose(res["out"], ref, rtol=1e-10, atol=1e-12)
    assert res["count"].sum() == 0 and np.all(res["pos"] == -1)


# ------------------------------------------------------------------ invariants
def test_router_weights_sum_to_one_and_are_sorted():
    inp = make_inputs(CONFIGS["tiny"])
    for k in (1, 2, 8):
        idx, w = oracle.router(inp["gate_logits"], k)
        np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-12)
        assert np.all(np.diff(w, axis=1) <= 1e-15)
        assert all(len(set(r)) == k for r in idx.tolist())


def test_router_ties_and_signed_zero():
    logits = np.array([[3.0, 1.0, 3.0, 3.0, -1.0],
                       [-0.0, 0.0, -2.0, 0.0, -0.0],
                       [-5.0, -7.0, -5.0, -6.0, -5.0]], dtype=np.float32)
    idx, w = oracle.router(logits, 3)
    assert idx.tolist() == [[0, 2, 3], [0, 1, 3], [0, 2, 4]]
    np.testing.assert_allclose(w, 1.0 / 3.0, atol=1e-15)


def test_router_quantised_logits_match_full_sort():
    rng = np.random.default_rng(11)
    logits = rng.integers(-2, 3, size=(200, 160)).astype(np.float32) * 0.5
    idx, _ = oracle.router(logits, 6)
    for t in range(200):
        assert idx[t].tolist() == topk_by_sort(logits[t], 6)


def test_dispatch_is_stable_counting_sort_and_conserves_assignments():
    """Token conservation (last rule of Eq. 'limitation'): every kept assignment is placed
    exactly once; rows are grouped by expert and ascend by token inside an expert."""
    rng = np.random.default_rng(12)
    T, k, E, e0, El = 300, 4, 20, 5, 9
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    d = oracle.dispatch(idx, e0, El)
    kept = [(t * k + s) for t in range(T) for s in range(k) if e0 <= idx[t, s] < e0 + El]
    assert d["offset"][-1] == len(kept) == d["count"].sum()
    assert sorted(d["perm"].tolist()) == kept                        # bijection
    ex = idx.reshape(-1)[d["perm"]] - e0
    assert np.all(np.diff(ex) >= 0)                                  # grouped by expert
    for e in range(El):
        rows = d["perm"][d["offset"][e]:d["offset"][e + 1]]
        assert np.all(np.diff(rows // k) > 0)                        # ascending token
        assert d["count"][e] == np.sum(idx == e0 + e)
    flat_pos = d["pos"].reshape(-1)
    assert np.all(flat_pos[d["perm"]] == np.arange(len(kept)))
    assert np.all(flat_pos[np.setdiff1d(np.arange(T * k), kept)] == -1)
    # library routine: a stable argsort of the kept assignments by expert is the same order
    kept = np.array(kept)
    assert d["perm"].tolist() == kept[np.argsort(idx.reshape(-1)[kept], kind="stable")].tolist()


def test_token_permutation_equivariance():
    wl = CONFIGS["tiny"]
    inp = make_inputs(wl)
    res = _fwd(inp, wl)
    P = np.random.default_rng(13).permutation(wl.n_tokens)
    inp2 = dict(inp, tokens=inp["tokens"][P], gate_logits=inp["gate_logits"][P])
    res2 = _fwd(inp2, wl)
    assert np.array_equal(res2["idx"], res["idx"][P])
    np.testing.assert_allclose(res2["out"], res["out"][P], rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("r", [2, 3, 4, 7, 200])
def test_chunked_equals_unchunked_bitwise(r):
    """The expert part is token-wise (Sec. 2.3): cutting the token range changes nothing.
    r = 200 > T leaves trailing chunks empty."""
    wl = CONFIGS["tiny"]
    inp = make_inputs(wl)
    a, b = _fwd(inp, wl), _fwd(inp, wl, r_chunks=r)
    assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["idx"], b["idx"])
    assert np.array_equal(a["w"], b["w"])
    assert b["count"].sum() == a["count"].sum() == wl.n_tokens * wl.top_k
    assert np.array_equal(b["count"].sum(axis=0), a["count"][0])


def test_expert_group_shares_sum_to_all_local():
    """Splitting the experts over eg devices and adding the per-device outputs gives the
    single-device layer (each expert lives on exactly one device, Sec. 2.2)."""
    wl = tiny_workload(n_tokens=24, hidden=32, inter=32, n_experts=8, n_local=8, top_k=3)
    inp = make_inputs(wl, seed=14)
    full = _fwd(inp, wl)["out"]
    sz = 3 * 32 * 32
    parts = np.zeros_like(full)
    for e0, El in ((0, 3), (3, 1), (4, 4)):
        sub = dict(inp, routed_w=inp["routed_w"][e0 * sz:(e0 + El) * sz])
        parts += _fwd(sub, wl, local_begin=e0, n_local=El)["out"]
    np.testing.assert_allclose(parts, full, rtol=1e-12, atol=1e-15)


def test_forward_tokens_matches_full_forward():
    wl = CONFIGS["tiny"]
    inp = make_inputs(wl)
    full = _fwd(inp, wl)["out"]
    ids = [0, 5, 127, 64, 5]
    sub = oracle.forward_tokens(inp["tokens"], inp["gate_logits"], inp["routed_w"],
                                inp["shared_w"], ids, hidden=wl.hidden, inter=wl.inter,
                                n_experts=wl.n_experts, local_begin=0, n_local=wl.n_local,
                                n_shared=wl.n_shared, shared_inter=wl.shared_inter,
                                top_k=wl.top_k)
    np.testing.assert_allclose(sub, full[ids], rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("n_shared", [0, 2])
@pytest.mark.parametrize("e0,El", [(3, 3), (0, 2), (5, 3), (7, 1)])
def test_forward_tokens_on_an_expert_group_share(e0, El, n_shared):
    """The per-token form on a device that holds experts [e0, e0 + El) of 8 (Sec. 3.1, "The MoE
    Part"): it must keep exactly the assignments to local experts, with the weights the gate gave
    them over all k selected experts (no second renormalisation), add the shared experts to every
    token, and give a token with nothing kept the shared part alone.  Checked against the
    dense-masked brute force (library matmul / softmax / sort) and against the whole-layer oracle."""
    M, H, Hs, E, k, T = 32, 48, 16, 8, 3, 40
    wl = tiny_workload(n_tokens=T, hidden=M, inter=H, n_experts=E, local_begin=e0, n_local=El, top_k=k,
                       n_shared=n_shared, shared_inter=Hs if n_shared else 0)
    inp = make_inputs(wl, seed=51)
    inp["gate_logits"][7, e0:e0 + El] = -50.0      # token 7 selects no local expert
    inp["gate_logits"][11, :] = 0.0                # token 11: all equal -> experts 0, 1, 2
    ref, G = brute_force_layer(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"],
                               M=M, H=H, E=E, e0=e0, El=El, Ns=n_shared, Hs=Hs, k=k)
    kept = (G[:, e0:e0 + El] > 0).sum(axis=1)
    assert kept[7] == 0 and 0 < kept.min(initial=9, where=kept > 0) < k   # partial selections exist
    # weights of the kept slots are the gate's own: they sum to less than 1 where a slot was dropped
    part = G[:, e0:e0 + El].sum(axis=1)
    assert np.any((part > 1e-3) & (part < 1.0 - 1e-3))
    ids = np.array([7, 0, 39, 11, 7, 20, 3], dtype=np.int32)
    args = dict(hidden=M, inter=H, n_experts=E, local_begin=e0, n_local=El, n_shared=n_shared,
                shared_inter=wl.shared_inter, top_k=k)
    sub = oracle.forward_tokens(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"],
                                ids, **args)
    assert rel_err(sub, ref[ids]) < 1e-9
    full = oracle.forward(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"], **args)
    np.testing.assert_allclose(sub, full["out"][ids], rtol=1e-12, atol=1e-15)
    assert rel_err(full["out"], ref) < 1e-9
    if n_shared == 0:
        assert not sub[0].any() and not sub[4].any()          # nothing kept, no shared expert: zeros
    else:
        X = f64(inp["tokens"][7:8])
        alone = sum(dense_ffn(X, *split_expert(inp["shared_w"], i, M, Hs)) for i in range(n_shared))
        assert rel_err(sub[0:1], alone) < 1e-9
    # all tokens, and the shares of a partition of the experts add up to the all-local layer
    every = oracle.forward_tokens(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"],
                                  np.arange(T, dtype=np.int32), **args)
    assert rel_err(every, ref) < 1e-9


def test_forward_tokens_filter_mistakes_are_caught():
    """What a wrong local filter would give differs measurably from the brute force: an off-by-one
    share, and weights renormalised over the kept slots."""
    M, H, E, k, T, e0, El = 32, 48, 8, 3, 40, 3, 3
    wl = tiny_workload(n_tokens=T, hidden=M, inter=H, n_experts=E, local_begin=e0, n_local=El, top_k=k)
    inp = make_inputs(wl, seed=51)
    ref, G = brute_force_layer(inp["tokens"], inp["gate_logits"], inp["routed_w"], None,
                               M=M, H=H, E=E, e0=e0, El=El, Ns=0, Hs=0, k=k)
    ids = np.arange(T, dtype=np.int32)
    args = dict(hidden=M, inter=H, n_experts=E, n_shared=0, shared_inter=0, top_k=k)
    good = oracle.forward_tokens(inp["tokens"], inp["gate_logits"], inp["routed_w"], None, ids,
                                 local_begin=e0, n_local=El, **args)
    assert rel_err(good, ref) < 1e-9
    shifted = oracle.forward_tokens(inp["tokens"], inp["gate_logits"], inp["routed_w"], None, ids,
                                    local_begin=e0 + 1, n_local=El, **args)
    assert rel_err(shifted, ref) > 1e-2
    Gl = G[:, e0:e0 + El]
    renorm = Gl / np.maximum(Gl.sum(axis=1, keepdims=True), 1e-300)
    X = f64(inp["tokens"])
    bad = sum(renorm[:, e, None] * dense_ffn(X, *split_expert(inp["routed_w"], e, M, H)) for e in range(El))
    assert rel_err(bad, ref) > 1e-2


def test_bf16_output_is_round_to_nearest():
    """out_bf16 of the whole-layer oracle is its double output rounded once to bf16 (through one fp32
    step): for every value the nearer of its two bf16 neighbours, chosen here in double arithmetic;
    where the two distances differ by less than an fp32 rounding error either neighbour is accepted."""
    wl = CONFIGS["tiny"]
    res = _fwd(make_inputs(wl), wl)
    out = res["out"]
    as_f32 = out.astype(np.float32)
    below = (as_f32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)   # a bf16 neighbour of out ...
    above = (below + np.uint16(1)).astype(np.uint16)                      # ... and the next one away from 0
    d0, d1 = np.abs(out - f64(below)), np.abs(out - f64(above))
    clear = np.abs(d0 - d1) > np.abs(out) * 2.0 ** -22
    assert clear.mean() > 0.99
    want = np.where(d1 < d0, above, below)
    assert np.array_equal(res["out_bf16"][clear], want[clear])
    assert np.all((res["out_bf16"] == below) | (res["out_bf16"] == above))
    exact = as_f32.astype(np.float64) == out          # no double rounding: the generator's own rule
    assert np.array_equal(res["out_bf16"][exact], f32_to_bf16_bits(as_f32)[exact])


def test_planted_mistakes_are_caught():
    """A transposed projection or a dropped renormalisation must fail the brute force."""
    wl = tiny_workload(n_tokens=8, hidden=16, inter=24, n_experts=4, n_local=4, top_k=2)
    inp = make_inputs(wl, seed=15)
    good = _fwd(inp, wl)["out"]
    ref, G = brute_force_layer(inp["tokens"], inp["gate_logits"], inp["routed_w"], None,
                               M=16, H=24, E=4, e0=0, El=4, Ns=0, Hs=0, k=2)
    assert rel_err(good, ref) < 1e-9
    # mistake 1: W_down read as [H, M] instead of [M, H]
    w = inp["routed_w"].reshape(4, -1).copy()
    for e in range(4):
        wd = w[e, 2 * 24 * 16:].reshape(16, 24)
        w[e, 2 * 24 * 16:] = np.ascontiguousarray(wd.T).reshape(-1)
    bad = _fwd(dict(inp, routed_w=w.reshape(-1)), wl)["out"]
    assert rel_err(bad, ref) > 1e-2
    # mistake 2: weights not renormalised over the selected k
    P = softmax(inp["gate_logits"].astype(np.float64), axis=1)
    unnorm = np.where(G > 0, P, 0.0)
    X = f64(inp["tokens"])
    bad2 = sum(unnorm[:, e, None] * dense_ffn(X, *split_expert(inp["routed_w"], e, 16, 24))
               for e in range(4))
    assert rel_err(bad2, good) > 1e-2


def test_bad_arguments_are_rejected():
    logits = np.zeros((2, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.router(logits, 0)
    with pytest.raises(ValueError):
        oracle.router(logits, 5)


def test_stored_tiny_values():
    """The committed oracle-written values of the tiny workload still come out of the oracle."""
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_oracle_values.txt")
    count, routing, samples, rms = load_tiny_golden(path)
    wl = CONFIGS["tiny"]
    res = _fwd(make_inputs(wl), wl)
    assert res["count"][0].tolist() == count
    for t, i0, i1, w0, w1 in routing:
        assert res["idx"][t].tolist() == [i0, i1]
        np.testing.assert_allclose(res["w"][t], [w0, w1], atol=1e-11)
    for t, c, v in samples:
        assert abs(res["out"][t, c] - v) <= 1e-10 * max(1.0, abs(v))
    assert abs(np.sqrt(np.mean(res["out"] ** 2)) - rms) <= 1e-10
