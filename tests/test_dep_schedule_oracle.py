"""Pins for oracle/dep_schedule.py (no GPU): the event replay of Eq. limitation, the layer-0 start
times and the T-layer makespan model of Sec. 4.2, Theorems 1, 3 and 4 as property tests, and
Algorithm 1 against an unpruned search.  The replay and the closed forms are written independently
(rules vs printed formulas), so their agreement pins both."""
import copy
import random

import pytest

from oracle import dep_schedule as D


def _models(rng):
    lin = lambda: D.Linear(rng.uniform(0.01, 1.0), rng.uniform(0.001, 0.5))
    return D.TaskModels(lin(), lin(), lin(), lin())


def _problem(rng, max_layers=5):
    return D.Problem(ag=rng.randint(1, 4), n_experts=rng.choice([8, 16, 64]), top_k=rng.randint(1, 4),
                     seq_len=rng.choice([1, 16, 128]), n_layers=rng.randint(1, max_layers))


def _cases(seed, n, max_layers=5):
    rng = random.Random(seed)
    for _ in range(n):
        yield _models(rng), _problem(rng, max_layers), rng.randint(1, 8), rng.randint(1, 5), rng.randint(1, 6)


def test_layer_models_hand_computed():
    # Sec. 4.1 with small integers, every coefficient worked out by hand
    m = D.layer_models(alpha_gm=1, beta_gm=1, alpha_attn=2, beta_attn=3, alpha_c=7, beta_c=1, S=2, M=3, H=5,
                       n_h=2, d_k=4, d_v=1, n_shared=2, E=8, eg=4)
    assert (m.a.alpha, m.a.beta) == (6, 240)      # 4*1+2 ; (96+24) + 3*(4*2*5)
    assert (m.s.alpha, m.s.beta) == (6, 180)      # 3*2*1 ; 3*2*(2*3*5)
    assert (m.e.alpha, m.e.beta) == (6, 90)       # 3*(8/4)*1 ; 3*(8/4)*(3*5)
    assert (m.c.alpha, m.c.beta) == (7, 6)        # alpha_c ; 1*8*3/4


def test_token_conservation():
    p = D.Problem(ag=3, n_experts=160, top_k=6, seq_len=2048, n_layers=2)
    for m_a in (1, 4):
        for r_2 in (1, 2, 8):
            m_e = D.tokens_per_expert(p, m_a, r_2)
            assert m_e * r_2 * p.n_experts == pytest.approx(m_a * p.ag * p.top_k * p.seq_len, rel=1e-15)


def test_replay_obeys_every_rule_and_never_idles_without_cause():
    for mod, p, m_a, r_1, r_2 in _cases(1, 400):
        for order in (D.ASAS, D.AASS):
            s = D.replay(mod, p, m_a, r_1, r_2, order)
            assert D.check_schedule(s, r_1, r_2, p.n_layers) == []
            t_a, t_s, t_e, t_c = s["t"]
            # earliest start: every start coincides with the end of something it had to wait for
            ends = {0.0}
            for t in range(p.n_layers):
                for i in range(r_1):
                    ends.add(round(s["tau_a"][t][i] + t_a, 9)); ends.add(round(s["tau_s"][t][i] + t_s, 9))
                    for j in range(r_2):
                        ends.add(round(s["tau_a2e"][t][i][j] + t_c, 9)); ends.add(round(s["tau_e"][t][i][j] + t_e, 9))
                        ends.add(round(s["tau_e2a"][t][i][j] + t_c, 9))
            for t in range(p.n_layers):
                for i in range(r_1):
                    assert round(s["tau_a"][t][i], 9) in ends and round(s["tau_s"][t][i], 9) in ends
                    for j in range(r_2):
                        for k in ("tau_a2e", "tau_e", "tau_e2a"):
                            assert round(s[k][t][i][j], 9) in ends


# ---------------------------------------------------------------- one GPU: shared experts and experts share the compute units
def test_one_gpu_replay_worked_example():
    """t_a = 1, t_s = 0.5, t_e = 0.7, t_c = 0.3, two micro-batches of two chunks, one layer, placed by hand
    with the procedure of the module header."""
    mod = D.TaskModels(D.Linear(1, 0), D.Linear(0.5, 0), D.Linear(0.7, 0), D.Linear(0.3, 0))
    p = D.Problem(ag=1, n_experts=8, top_k=1, seq_len=1, n_layers=1)
    s = D.replay_one_gpu(mod, p, 1, 2, 2, D.ASAS)
    # a0 0-1, s0 1-1.5 (the experts of chunk (0,0), ready at 1.3, wait for it), a1 1.5-2.5, e(0,0) 1.5-2.2,
    # e(0,1) 2.2-2.9, s1 waits for it: 2.9-3.4, e(1,0) 3.4-4.1, e(1,1) 4.1-4.8, its E2A ends at 5.1
    assert s["tau_a"] == [[0.0, 1.5]]
    assert s["tau_s"][0] == pytest.approx([1.0, 2.9])
    assert s["tau_a2e"][0] == [pytest.approx([1.0, 1.3]), pytest.approx([2.5, 2.8])]
    assert s["tau_e"][0] == [pytest.approx([1.5, 2.2]), pytest.approx([3.4, 4.1])]
    assert s["makespan"] == pytest.approx(5.1)
    assert D.replay(mod, p, 1, 2, 2, D.ASAS)["makespan"] == pytest.approx(4.5)     # two GPUs: 0.6 less
    s = D.replay_one_gpu(mod, p, 1, 2, 2, D.AASS)
    # a0 0-1, a1 1-2, e(0,0) 1.3-2.0, s0 2.0-2.5, s1 2.5-3.0 (the attention group wins ties), e(0,1) 3.0-3.7,
    # e(1,0) 3.7-4.4, e(1,1) 4.4-5.1, its E2A ends at 5.4
    assert s["tau_a"] == [[0.0, 1.0]]
    assert s["tau_s"][0] == pytest.approx([2.0, 2.5])
    assert s["tau_e"][0] == [pytest.approx([1.3, 3.0]), pytest.approx([3.7, 4.4])]
    assert s["makespan"] == pytest.approx(5.4)


def test_one_gpu_replay_is_valid_late_and_never_idles_without_cause():
    hit = same = 0
    for mod, p, m_a, r_1, r_2 in _cases(5, 300, max_layers=4):
        for order in (D.ASAS, D.AASS):
            two = D.replay(mod, p, m_a, r_1, r_2, order)
            one = D.replay_one_gpu(mod, p, m_a, r_1, r_2, order)
            T = p.n_layers
            assert D.check_schedule(one, r_1, r_2, T, one_gpu=True) == []
            # the same task orders under one rule more: nothing starts earlier than with two GPUs
            t_a, t_s, t_e, t_c = one["t"]
            ends = {0.0}
            for t in range(T):
                for i in range(r_1):
                    assert one["tau_a"][t][i] >= two["tau_a"][t][i] - 1e-9 and one["tau_s"][t][i] >= two["tau_s"][t][i] - 1e-9
                    ends.add(round(one["tau_a"][t][i] + t_a, 9)); ends.add(round(one["tau_s"][t][i] + t_s, 9))
                    for j in range(r_2):
                        for k in ("tau_a2e", "tau_e", "tau_e2a"):
                            assert one[k][t][i][j] >= two[k][t][i][j] - 1e-9
                        ends.add(round(one["tau_a2e"][t][i][j] + t_c, 9)); ends.add(round(one["tau_e"][t][i][j] + t_e, 9))
                        ends.add(round(one["tau_e2a"][t][i][j] + t_c, 9))
            for t in range(T):
                for i in range(r_1):
                    assert round(one["tau_a"][t][i], 9) in ends and round(one["tau_s"][t][i], 9) in ends
                    for j in range(r_2):
                        for k in ("tau_a2e", "tau_e", "tau_e2a"):
                            assert round(one[k][t][i][j], 9) in ends
            # all shared-expert and expert work on one set of compute units, after the first attention
            assert one["makespan"] >= t_a + T * r_1 * (t_s + r_2 * t_e) - 1e-9
            # where the two-GPU schedule never runs the two kinds at once, the extra rule changes nothing
            if D.check_schedule(two, r_1, r_2, T, one_gpu=True) == []:
                same += 1
                for k in ("tau_a", "tau_s", "tau_a2e", "tau_e", "tau_e2a"):
                    assert one[k] == two[k]
            else:
                hit += 1
    assert hit > 100 and same > 5


def test_one_gpu_single_micro_batch_closed_form():
    """One micro-batch, one layer: the shared experts start with the first transfer; the experts
    follow whichever of the two ends later, then run back to back when a chunk's transfer is the
    shorter task."""
    p = D.Problem(ag=1, n_experts=8, top_k=1, seq_len=1, n_layers=1)
    for t_a, t_s, t_e, t_c, r_2 in [(1.0, 0.5, 0.7, 0.3, 3), (1.0, 0.2, 0.7, 0.3, 3), (0.4, 0.9, 0.5, 0.5, 4), (0.0, 2.0, 0.1, 0.1, 2)]:
        mod = D.TaskModels(D.Linear(t_a, 0), D.Linear(t_s, 0), D.Linear(t_e, 0), D.Linear(t_c, 0))
        for order in (D.ASAS, D.AASS):
            s = D.replay_one_gpu(mod, p, 1, 1, r_2, order)
            assert t_e >= t_c
            assert s["makespan"] == pytest.approx(t_a + max(t_s, t_c) + r_2 * t_e + t_c)


def test_validator_catches_planted_violations():
    mod, p = D.TaskModels(D.Linear(1, 0), D.Linear(0.5, 0), D.Linear(0.7, 0), D.Linear(0.3, 0)), \
        D.Problem(ag=1, n_experts=8, top_k=1, seq_len=8, n_layers=2)
    good = D.replay(mod, p, 1, 2, 2, D.ASAS)
    assert D.check_schedule(good, 2, 2, 2) == []
    for key, where, delta, rule in (("tau_e", (0, 0, 1), -0.5, "rule"), ("tau_s", (0, 1), -0.6, "rule"),
                                    ("tau_a", (1, 0), -0.4, "rule 9"), ("tau_e2a", (1, 1, 1), -0.35, "rule")):
        bad = copy.deepcopy(good)
        ref = bad[key]
        for w in where[:-1]:
            ref = ref[w]
        ref[where[-1]] += delta
        found = D.check_schedule(bad, 2, 2, 2)
        assert found and any(rule in f for f in found), (key, found)


def test_order_of_the_attention_group():
    mod = D.TaskModels(D.Linear(1, 0), D.Linear(0.5, 0), D.Linear(0.1, 0), D.Linear(0.1, 0))
    p = D.Problem(ag=1, n_experts=8, top_k=1, seq_len=8, n_layers=1)
    asas = D.replay(mod, p, 1, 3, 1, D.ASAS)
    aass = D.replay(mod, p, 1, 3, 1, D.AASS)
    assert asas["tau_a"][0] == [0.0, 1.5, 3.0] and asas["tau_s"][0] == [1.0, 2.5, 4.0]
    assert aass["tau_a"][0] == [0.0, 1.0, 2.0] and aass["tau_s"][0] == [3.0, 3.5, 4.0]
    # AASS releases the transfers earlier: A2E of micro-batch 2 starts at 3.0 instead of 4.0
    assert aass["tau_a2e"][0][2][0] == 3.0 and asas["tau_a2e"][0][2][0] == 4.0


def test_single_microbatch_is_the_textbook_flow_shop():
    # r_1 = 1, one layer: r_2 identical jobs through link -> experts -> link; a permutation flow shop
    # with identical jobs ends at (sum of stage times) + (jobs - 1) * (slowest stage)
    for mod, p, m_a, _, r_2 in _cases(3, 300, max_layers=1):
        m_e = D.tokens_per_expert(p, m_a, r_2)
        t_a, t_s, t_e, t_c = mod.a(m_a), mod.s(m_a), mod.e(m_e), mod.c(m_e)
        expect = t_a + max(t_s, t_c + t_e + t_c + (r_2 - 1) * max(t_e, t_c))
        for order in (D.ASAS, D.AASS):
            assert D.replay(mod, p, m_a, 1, r_2, order)["makespan"] == pytest.approx(expect, rel=1e-12)


def test_printed_layer0_start_times_against_the_replay():
    for mod, p, m_a, r_1, r_2 in _cases(4, 500):
        s = D.replay(mod, p, m_a, r_1, r_2, D.ASAS)
        l0 = D.layer0_times(mod, p, m_a, r_1, r_2)
        for i in range(r_1):
            # attention / shared: the printed times are the replay's
            assert s["tau_a"][0][i] == pytest.approx(l0["tau_a"][i], abs=1e-9)
            assert s["tau_s"][0][i] == pytest.approx(l0["tau_s"][i], abs=1e-9)
            for j in range(r_2):
                # a transfer may leave earlier than printed (the link is free), never later
                assert s["tau_a2e"][0][i][j] <= l0["tau_a2e"][i][j] + 1e-9
                assert s["tau_e"][0][i][j] <= l0["tau_e"][i][j] + 1e-9
                # the return transfer starts exactly when printed
                assert s["tau_e2a"][0][i][j] == pytest.approx(l0["tau_e2a"][i][j], abs=1e-9)


def test_makespan_model_equals_the_replay_and_the_printed_form_double_counts():
    n_strict = 0
    for mod, p, m_a, r_1, r_2 in _cases(5, 800):
        span = D.replay(mod, p, m_a, r_1, r_2, D.ASAS)["makespan"]
        assert D.objective(mod, p, m_a, r_1, r_2) == pytest.approx(span, rel=1e-12)
        _, Y, _, _, _ = D._xyfg(mod, p, m_a, r_1, r_2)
        printed = D.objective_as_printed(mod, p, m_a, r_1, r_2)
        assert printed - span == pytest.approx((r_2 - 1) * Y, rel=1e-9, abs=1e-9 * span)
        n_strict += printed > span * (1 + 1e-9)
    assert n_strict > 400  # whenever r_2 > 1


def test_theorem_throughput_increases_with_m_a():
    for mod, p, _, r_1, r_2 in _cases(6, 300):
        prev = 0.0
        for m_a in range(1, 14):
            tps = r_1 * m_a / D.objective(mod, p, m_a, r_1, r_2)
            assert tps > prev
            prev = tps


def test_theorem_throughput_does_not_decrease_with_r_1():
    for mod, p, m_a, _, r_2 in _cases(7, 300):
        prev = 0.0
        for r_1 in range(1, 12):
            tps = r_1 * m_a / D.objective(mod, p, m_a, r_1, r_2)
            assert tps >= prev * (1 - 1e-13)
            prev = tps


def test_theorem_makespan_is_convex_in_one_over_r_2():
    for mod, p, m_a, r_1, _ in _cases(8, 300):
        us = [0.02 + 0.98 * k / 80 for k in range(81)]
        f = [D.objective(mod, p, m_a, r_1, 1.0 / u) for u in us]
        for k in range(1, 80):
            assert f[k - 1] - 2 * f[k] + f[k + 1] >= -1e-9 * max(1.0, abs(f[k]))


def test_algorithm_1_loses_nothing_by_skipping_non_pareto_pairs():
    rng = random.Random(9)
    for _ in range(120):
        mod, p = _models(rng), _problem(rng, max_layers=4)
        cap = rng.randint(1, 12)
        got = D.search(mod, p, 12, cap, 6, 6)
        ref = D.search_exhaustive(mod, p, 12, cap, 6, 6)
        assert got["throughput"] == pytest.approx(ref["throughput"], rel=1e-12)
        assert (got["m_a"], got["r_1"], got["r_2"], got["order"]) == (ref["m_a"], ref["r_1"], ref["r_2"], ref["order"])
        assert got["r_1"] * got["m_a"] <= cap


def test_search_returns_none_when_nothing_fits():
    rng = random.Random(10)
    assert D.search(_models(rng), _problem(rng), 4, 0, 4, 4) is None
