"""The library's timing-model routines (host code behind the C ABI) against the oracle: the fit,
the closed-form makespan, and the chosen r_2 (convex search vs the oracle's brute force)."""
import numpy as np
import pytest

import paper_2512_21487_amd as pkg
from oracle.pipeline_model import LinearModel, best_r, best_r_overlap, fit_linear, makespan, makespan_overlap


def _pm(mi, me, mo):
    return pkg.PipelineModel(mi.alpha, mi.beta, me.alpha, me.beta, mo.alpha, mo.beta)


def test_fit_matches_oracle():
    rng = np.random.default_rng(3)
    for n in (2, 5, 40):
        x = rng.uniform(1, 5000, n)
        t = 0.2 + 3e-4 * x + rng.normal(0, 0.01, n)
        a, b, r2 = pkg.fit_linear(x, t)
        a0, b0, r20 = fit_linear(x, t)
        assert a == pytest.approx(a0, rel=1e-9, abs=1e-12) and b == pytest.approx(b0, rel=1e-9)
        assert r2 == pytest.approx(r20, abs=1e-9)
    with pytest.raises(pkg.MoeEpError):
        pkg.fit_linear([3.0, 3.0, 3.0], [1.0, 2.0, 3.0])
    with pytest.raises(pkg.MoeEpError):
        pkg.fit_linear([3.0], [1.0])


def test_makespan_and_choice_match_oracle_brute_force():
    rng = np.random.default_rng(4)
    for case in range(2000):
        kind = case % 4
        mods = []
        for _ in range(3):
            alpha = float(rng.uniform(0.0, 0.5)) if kind != 1 else 0.0
            beta = float(rng.uniform(1e-6, 1e-3)) if kind != 2 else 0.0
            mods.append(LinearModel(alpha, beta))
        if kind == 3:                       # equal links, as the paper assumes
            mods[2] = mods[0]
        mi, me, mo = mods
        T = int(rng.integers(1, 70000))
        r_max = int(rng.choice([1, 2, 8, 64]))
        pm = _pm(mi, me, mo)
        for r in (1, 2, r_max):
            assert pkg.pipeline_makespan(pm, T, r) == pytest.approx(makespan(r, T, mi, me, mo), rel=1e-13)
        got, want = pkg.choose_chunks(pm, T, r_max), best_r(T, mi, me, mo, r_max)
        if got != want:                     # several r may tie: the spans must then be equal
            assert makespan(got, T, mi, me, mo) == pytest.approx(makespan(want, T, mi, me, mo), rel=1e-12)
        assert 1 <= got <= r_max


def test_choice_bad_arguments():
    pm = _pm(LinearModel(0.1, 1e-4), LinearModel(0.1, 1e-4), LinearModel(0.1, 1e-4))
    lib = pkg.load_library()
    assert lib.moe_ep_choose_chunks(None, 10, 4) < 0
    assert lib.moe_ep_choose_chunks(pm, 10, 0) < 0
    assert lib.moe_ep_pipeline_makespan(pm, 10, 0) < 0
    assert pkg.choose_chunks(pm, 0, 8) == 1


def test_overlap_models_match_oracle_brute_force():
    """A model with the second set of coefficients (tasks beside other tasks): makespan and chosen r_2
    against the oracle's two-set closed form and brute force, on random models whose second set is
    slower, equal, or (for the search's sake) faster than the first."""
    rng = np.random.default_rng(6)
    for case in range(1500):
        alone = tuple(LinearModel(float(rng.uniform(0.0, 0.5)), float(rng.uniform(1e-6, 1e-3))) for _ in range(3))
        lo, hi = ((1.0, 2.5), (1.0, 1.0), (0.6, 1.4))[case % 3]
        beside = tuple(LinearModel(m.alpha * float(rng.uniform(lo, hi)) + (1e-9 if case % 3 == 1 else 0.0),
                                   m.beta * float(rng.uniform(lo, hi))) for m in alone)
        T = int(rng.integers(1, 70000))
        r_max = int(rng.choice([1, 2, 3, 8, 64]))
        pm = pkg.PipelineModel(alone[0].alpha, alone[0].beta, alone[1].alpha, alone[1].beta, alone[2].alpha,
                               alone[2].beta, beside[0].alpha, beside[0].beta, beside[1].alpha, beside[1].beta,
                               beside[2].alpha, beside[2].beta)
        for r in (1, 2, r_max):
            assert pkg.pipeline_makespan(pm, T, r) == pytest.approx(makespan_overlap(r, T, alone, beside), rel=1e-13)
        got, want = pkg.choose_chunks(pm, T, r_max), best_r_overlap(T, alone, beside, r_max)
        if got != want:
            assert makespan_overlap(got, T, alone, beside) == pytest.approx(makespan_overlap(want, T, alone, beside), rel=1e-12)
        assert 1 <= got <= r_max
