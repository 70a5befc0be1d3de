"""Host-only tests of the step-composition entry points (Section 3.3.1): the oracle is pinned
to the paper's Eq. (3) and to special cases with known answers, then the library is compared
with the oracle."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import hfx_sched_oracle as so
from paper_2508_15919_amd import binding as hb


# ---------------------------------------------------------------- pins of the oracle
def eq3(ttft, tpot, a, b, e_d):
    """Eq. (3) as printed, in exact arithmetic."""
    F = Fraction
    return (F(tpot) - F(e_d)) * F(ttft) / ((2 * F(tpot) - F(e_d)) * F(b)) - F(a) / F(b)


def test_oracle_budget_is_the_floor_of_eq3():
    rng = np.random.default_rng(0)
    for _ in range(300):
        tpot = float(rng.uniform(0.02, 0.2))
        e_d = float(rng.uniform(0.0, 0.95) * tpot)
        ttft = float(rng.uniform(0.1, 5.0))
        a, b = float(rng.uniform(0, 0.02)), float(rng.uniform(1e-6, 1e-3))
        want = max(0, math.floor(eq3(ttft, tpot, a, b, e_d)))
        assert so.token_budget(ttft, tpot, a, b, e_d) == want


def test_oracle_special_cases():
    # no decode running (E_d = 0): the condition is just 2*E_p <= TTFT
    assert so.token_budget(4.0, 1.0, 1.0, 0.5, 0.0) == 2            # 2*(1 + 0.5*2) = 4
    assert so.token_budget(4.0, 123.0, 1.0, 0.5, 0.0) == 2          # TPOT is irrelevant then
    # E_d -> TPOT: slack vanishes, k explodes, nothing fits
    assert so.token_budget(10.0, 0.05, 0.0, 1e-4, 0.05) == 0
    assert so.token_budget(10.0, 0.05, 0.0, 1e-4, 0.06) == 0
    # a alone already breaks the bound
    assert so.token_budget(1.0, 0.1, 0.6, 1e-4, 0.0) == 0
    # at a budget that meets the bound exactly, maturity + E_p equals TTFT
    # TPOT 1, E_d 0.5: E_p <= TTFT*0.5/1.5; TTFT 6 -> E_p <= 2; a 0, b 0.25 -> n = 8
    assert so.token_budget(6.0, 1.0, 0.0, 0.25, 0.5) == 8
    k, m = so.maturity(so.e_p(0.0, 0.25, 8), 1.0, 0.5)
    assert k == 4 and m == 4 and m + so.e_p(0.0, 0.25, 8) == 6
    assert not so.admissible(9, 6.0, 1.0, 0.0, 0.25, 0.5)


def test_oracle_budget_monotone():
    base = dict(ttft=2.0, tpot=0.1, a=0.01, b=2e-4, e_d=0.03)
    n0 = so.token_budget(**base)
    assert so.token_budget(**{**base, "ttft": 2.5}) >= n0
    assert so.token_budget(**{**base, "e_d": 0.05}) <= n0
    assert so.token_budget(**{**base, "b": 4e-4}) <= n0
    assert so.token_budget(**{**base, "a": 0.05}) <= n0
    assert so.token_budget(**{**base, "tpot": 0.2}) >= n0


def test_oracle_compose_skips_what_does_not_fit():
    # budget 8 (see above); queue order by urgency: lengths 5, 6, 3, 1 -> take 5, pass over 6, take 3; the budget is then used up and 1 does not fit
    adm, kind, ql, cl, budget, n = so.compose(6.0, 1.0, 0.0, 0.25, 0.5, [10, 20], [3, 6, 5, 1], urgency=[2.0, 1.0, 0.0, 3.0])
    assert budget == 8 and n == 8 and adm == [1, 0, 1, 0]
    assert kind == [1, 1] and ql == [5, 3] and cl == [5, 3]
    adm, kind, ql, cl, _, _ = so.compose(6.0, 1.0, 0.0, 0.25, 0.5, [10, 20], [3, 6, 5, 1], urgency=[2.0, 1.0, 0.0, 3.0], mixed=True)
    assert kind == [0, 0, 1, 1] and ql == [1, 1, 5, 3] and cl == [11, 21, 5, 3]
    # nothing fits: the instance decodes on
    adm, kind, ql, cl, _, n = so.compose(6.0, 1.0, 0.0, 0.25, 0.5, [10, 20], [9, 12])
    assert adm == [0, 0] and n == 0 and kind == [0, 0] and cl == [11, 21]


# ---------------------------------------------------------------- library vs oracle
def model(a, b, e_d):
    return hb.hfx_latency_model(a, b, e_d)


def test_token_budget_matches_oracle():
    rng = np.random.default_rng(1)
    for _ in range(500):
        tpot = float(rng.uniform(0.02, 0.2))
        e_d = float(rng.uniform(0.0, 1.1) * tpot)
        ttft = float(rng.uniform(0.05, 5.0))
        a, b = float(rng.uniform(0, 0.05)), float(rng.uniform(1e-6, 1e-3))
        want = so.token_budget(ttft, tpot, a, b, e_d)
        got = hb.hfx_token_budget(ttft, tpot, model(a, b, e_d))
        if got != want:
            # only a bound that lands on an integer to within double rounding may differ, by one
            exact = eq3(ttft, tpot, a, b, e_d)
            assert abs(got - want) == 1 and abs(exact - round(exact)) < 1e-9, (ttft, tpot, a, b, e_d)
    assert hb.hfx_token_budget(4.0, 1.0, model(1.0, 0.5, 0.0)) == 2
    assert hb.hfx_token_budget(6.0, 1.0, model(0.0, 0.25, 0.5)) == 8
    assert hb.hfx_token_budget(10.0, 0.05, model(0.0, 1e-4, 0.05)) == 0


def test_maturity_matches_oracle():
    rng = np.random.default_rng(2)
    for _ in range(200):
        tpot = float(rng.uniform(0.02, 0.2))
        e_d = float(rng.uniform(0.0, 0.9) * tpot)
        ep = float(rng.uniform(0.0, 2.0))
        k, m = hb.hfx_maturity_time(ep, tpot, e_d)
        wk, wm = so.maturity(ep, tpot, e_d)
        assert k == pytest.approx(float(wk), rel=1e-12) and m == pytest.approx(float(wm), rel=1e-12)
    assert hb.hfx_maturity_time(2.0, 1.0, 0.5) == (4.0, 4.0)
    with pytest.raises(hb.HfxError) as e:
        hb.hfx_maturity_time(1.0, 0.05, 0.05)
    assert e.value.code == hb.HFX_ERR_MODEL


def test_model_validation():
    for bad in [(0.0, 0.1, 0.0, 1e-4, 0.0), (1.0, 0.0, 0.0, 1e-4, 0.0), (1.0, 0.1, -1.0, 1e-4, 0.0),
                (1.0, 0.1, 0.0, 0.0, 0.0), (1.0, 0.1, 0.0, 1e-4, -0.1), (float("nan"), 0.1, 0.0, 1e-4, 0.0),
                (1.0, 0.1, 0.0, float("inf"), 0.0)]:
        with pytest.raises(hb.HfxError) as e:
            hb.hfx_token_budget(bad[0], bad[1], model(*bad[2:]))
        assert e.value.code == hb.HFX_ERR_MODEL, bad


def test_fit_recovers_a_line_and_flags_curvature():
    n = np.array([128, 256, 512, 1024, 2048, 4096], np.int64)
    m, r2 = hb.hfx_fit_latency_model(n, 3e-3 + 2e-5 * n)
    assert m.a == pytest.approx(3e-3, rel=1e-9) and m.b == pytest.approx(2e-5, rel=1e-9) and r2 == pytest.approx(1.0)
    # against numpy's least squares on noisy data
    rng = np.random.default_rng(3)
    t = 1e-3 + 5e-6 * n + rng.normal(0, 2e-4, len(n))
    m, r2 = hb.hfx_fit_latency_model(n, t)
    b_ref, a_ref = np.polyfit(n.astype(np.float64), t, 1)
    assert m.b == pytest.approx(b_ref, rel=1e-9) and m.a == pytest.approx(max(a_ref, 0.0), rel=1e-9, abs=1e-15)
    _, r2_quad = hb.hfx_fit_latency_model(n, 1e-9 * n.astype(np.float64) ** 2)
    assert r2_quad < 0.97                            # a pure quadratic is visibly not a line
    with pytest.raises(hb.HfxError):
        hb.hfx_fit_latency_model(np.array([5, 5], np.int64), np.array([1.0, 2.0]))


def test_compose_matches_oracle_and_feeds_the_planner():
    rng = np.random.default_rng(4)
    for trial in range(60):
        tpot = float(rng.uniform(0.03, 0.2))
        e_d = float(rng.uniform(0.0, 0.8) * tpot)
        ttft = float(rng.uniform(0.2, 3.0))
        a, b = float(rng.uniform(0, 0.01)), float(rng.uniform(2e-5, 5e-4))
        running = rng.integers(1, 5000, rng.integers(0, 20)).astype(np.int32)
        prompts = np.maximum(1, rng.normal(400, 300, rng.integers(0, 30))).astype(np.int32)
        urg = rng.integers(0, 6, len(prompts)).astype(np.float64) if trial % 3 else None   # many ties
        mixed = bool(trial % 2)
        adm, kind, ql, cl, dec = hb.hfx_compose_step(ttft, tpot, model(a, b, e_d), running, prompts, urg, mixed)
        w = so.compose(ttft, tpot, a, b, e_d, running.tolist(), prompts.tolist(), None if urg is None else urg.tolist(), mixed)
        assert adm.tolist() == w[0] and kind.tolist() == w[1] and ql.tolist() == w[2] and cl.tolist() == w[3]
        assert dec.budget == w[4] and dec.n_token == w[5] <= dec.budget
        if dec.n_token:
            assert dec.e_p == pytest.approx(a + b * dec.n_token)
            wk, wm = so.maturity(dec.e_p, tpot, e_d)
            assert dec.k == pytest.approx(float(wk)) and dec.maturity == pytest.approx(float(wm))
            assert dec.maturity + dec.e_p <= ttft * (1 + 1e-12)
        else:
            assert dec.e_p == 0.0 and dec.maturity == 0.0
        if len(kind):
            shape = hb.make_shape(32, 8, 128, 1 << 20, 0.0)
            sizes = hb.hfx_batch_desc_sizes(shape, kind, ql, cl)        # the step is a valid planner input
            assert sizes[0] > 0


def test_compose_validation():
    m = model(0.0, 1e-4, 0.01)
    with pytest.raises(hb.HfxError) as e:
        hb.hfx_compose_step(1.0, 0.1, m, [0], [5])
    assert e.value.code == hb.HFX_ERR_LEN
    with pytest.raises(hb.HfxError) as e:
        hb.hfx_compose_step(1.0, 0.1, m, [5], [0])
    assert e.value.code == hb.HFX_ERR_LEN
    adm, kind, ql, cl, dec = hb.hfx_compose_step(1.0, 0.1, m, [], [])
    assert len(kind) == 0 and dec.n_token == 0
