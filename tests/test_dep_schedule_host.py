"""The library's schedule model and configuration search (host code behind the C ABI) against the
oracle of oracle/dep_schedule.py, on seeded random task models.  No GPU is touched."""
import random

import numpy as np
import pytest

import paper_2512_21487_amd as P
from oracle import dep_schedule as D


def _pair(rng, max_layers=5):
    co = [rng.uniform(0.01, 1.0) if k % 2 == 0 else rng.uniform(0.001, 0.5) for k in range(8)]
    mod_o = D.TaskModels(D.Linear(co[0], co[1]), D.Linear(co[2], co[3]), D.Linear(co[4], co[5]), D.Linear(co[6], co[7]))
    mod_p = P.DepModels(*co)
    prob = dict(ag=rng.randint(1, 4), n_experts=rng.choice([8, 16, 64]), top_k=rng.randint(1, 4),
                seq_len=rng.choice([1, 16, 128]), n_layers=rng.randint(1, max_layers))
    return mod_o, mod_p, D.Problem(**prob), P.DepProblem(**prob)


def test_layer_models_match():
    kw = dict(alpha_gm=0.17, beta_gm=8.59e-11, alpha_attn=0.15, beta_attn=1.54e-11, alpha_c=0.10, beta_c=9.61e-7)
    shape = dict(seq_len=2048, hidden=5120, inter=1536, n_heads=128, d_k=192, d_v=128, n_shared=2, n_experts=160, eg=5)
    got = P.dep_layer_models(P.DepPrimitives(**kw, **shape))
    ref = D.layer_models(**kw, S=shape["seq_len"], M=shape["hidden"], H=shape["inter"], n_h=shape["n_heads"],
                         d_k=shape["d_k"], d_v=shape["d_v"], n_shared=shape["n_shared"], E=shape["n_experts"],
                         eg=shape["eg"])
    for name, lin in (("a", ref.a), ("s", ref.s), ("e", ref.e), ("c", ref.c)):
        assert getattr(got, "alpha_" + name) == pytest.approx(lin.alpha, rel=1e-14)
        assert getattr(got, "beta_" + name) == pytest.approx(lin.beta, rel=1e-14)


def test_replay_start_times_match_the_oracle():
    rng = random.Random(21)
    for _ in range(300):
        mod_o, mod_p, prob_o, prob_p = _pair(rng)
        m_a, r_1, r_2 = rng.randint(1, 8), rng.randint(1, 5), rng.randint(1, 6)
        assert P.dep_tokens_per_expert(prob_p, m_a, r_2) == pytest.approx(D.tokens_per_expert(prob_o, m_a, r_2), rel=1e-15)
        for order in (D.ASAS, D.AASS):
            ref = D.replay(mod_o, prob_o, m_a, r_1, r_2, order)
            span, tau = P.dep_replay(mod_p, prob_p, m_a, r_1, r_2, order)
            assert span == pytest.approx(ref["makespan"], rel=1e-12)
            for k in ("tau_a", "tau_s", "tau_a2e", "tau_e", "tau_e2a"):
                np.testing.assert_allclose(tau[k], np.asarray(ref[k]), rtol=1e-12, atol=1e-12)
            # and the library's schedule passes the oracle's rule checker
            sch = {k: tau[k].tolist() for k in tau}
            sch["t"] = ref["t"]
            assert D.check_schedule(sch, r_1, r_2, prob_o.n_layers) == []


def test_one_gpu_replay_matches_the_oracle():
    rng = random.Random(27)
    for _ in range(300):
        mod_o, mod_p, prob_o, prob_p = _pair(rng, max_layers=4)
        m_a, r_1, r_2 = rng.randint(1, 8), rng.randint(1, 5), rng.randint(1, 6)
        for order in (D.ASAS, D.AASS):
            ref = D.replay_one_gpu(mod_o, prob_o, m_a, r_1, r_2, order)
            span, tau = P.dep_replay(mod_p, prob_p, m_a, r_1, r_2, order, one_gpu=True)
            assert span == pytest.approx(ref["makespan"], rel=1e-12)
            for k in ("tau_a", "tau_s", "tau_a2e", "tau_e", "tau_e2a"):
                np.testing.assert_allclose(tau[k], np.asarray(ref[k]), rtol=1e-12, atol=1e-12)
            sch = {k: tau[k].tolist() for k in tau}
            sch["t"] = ref["t"]
            assert D.check_schedule(sch, r_1, r_2, prob_o.n_layers, one_gpu=True) == []


def test_makespan_model_matches():
    rng = random.Random(22)
    for _ in range(500):
        mod_o, mod_p, prob_o, prob_p = _pair(rng)
        m_a, r_1, r_2 = rng.randint(1, 8), rng.randint(1, 5), rng.randint(1, 6)
        assert P.dep_makespan(mod_p, prob_p, m_a, r_1, r_2) == pytest.approx(D.objective(mod_o, prob_o, m_a, r_1, r_2), rel=1e-13)


def test_solve_r2_matches_the_exhaustive_minimum():
    rng = random.Random(23)
    for _ in range(300):
        mod_o, mod_p, prob_o, prob_p = _pair(rng, max_layers=4)
        m_a, r_1, r2_max = rng.randint(1, 8), rng.randint(1, 5), rng.choice([1, 4, 16, 64])
        for order in (D.ASAS, D.AASS):
            r2_ref, span_ref = D.solve_r2(mod_o, prob_o, m_a, r_1, order, r2_max)
            r2, span = P.dep_solve_r2(mod_p, prob_p, m_a, r_1, order, r2_max)
            assert span == pytest.approx(span_ref, rel=1e-12)
            assert r2 == r2_ref


def test_search_matches_algorithm_1_of_the_oracle():
    rng = random.Random(24)
    n_same = 0
    for _ in range(150):
        mod_o, mod_p, prob_o, prob_p = _pair(rng, max_layers=4)
        cap, m_a_max, r1_cap, r2_max = rng.randint(1, 16), rng.randint(1, 12), rng.randint(1, 6), rng.choice([4, 8])
        ref = D.search(mod_o, prob_o, m_a_max, cap, r1_cap, r2_max)
        got = P.dep_search(mod_p, prob_p, m_a_max, cap, r1_cap, r2_max)
        assert got.throughput == pytest.approx(ref["throughput"], rel=1e-12)
        # the configuration is unique up to ties (the two orders often give the same makespan, and a
        # rounding error then decides): what the library returns must score the same in the oracle
        assert got.r_1 * got.m_a <= cap and got.r_1 == D.max_r1(got.m_a, cap, r1_cap) and 1 <= got.r_2 <= r2_max
        span = D.score(mod_o, prob_o, got.m_a, got.r_1, got.r_2, got.order)
        assert got.makespan == pytest.approx(span, rel=1e-12)
        assert got.r_1 * got.m_a * prob_o.ag / span == pytest.approx(ref["throughput"], rel=1e-12)
        assert got.m_e == pytest.approx(D.tokens_per_expert(prob_o, got.m_a, got.r_2), rel=1e-14)
        n_same += (got.m_a, got.r_1, got.r_2, got.order) == (ref["m_a"], ref["r_1"], ref["r_2"], ref["order"])
    assert n_same >= 140


def test_bad_arguments_and_empty_search():
    rng = random.Random(25)
    _, mod_p, _, prob_p = _pair(rng)
    assert P.dep_search(mod_p, prob_p, 4, 0, 4, 4) is None
    lib = P.load_library()
    import ctypes
    assert lib.moe_ep_dep_makespan(ctypes.byref(mod_p), ctypes.byref(prob_p), 0, 1, 1) < 0
    assert lib.moe_ep_dep_makespan(None, ctypes.byref(prob_p), 1, 1, 1) < 0
    assert lib.moe_ep_dep_replay(ctypes.byref(mod_p), ctypes.byref(prob_p), 1, 1, 1, 7, None, None, None, None, None, None) == -1
    assert lib.moe_ep_dep_solve_r2(ctypes.byref(mod_p), ctypes.byref(prob_p), 1, 1, 0, 0, None, None) == -1
    bad = P.DepProblem(ag=0, n_experts=8, top_k=1, seq_len=1, n_layers=1)
    assert lib.moe_ep_dep_tokens_per_expert(ctypes.byref(bad), 1, 1) < 0
