"""Pins of the policy / state-update oracle (oracle/policy.py): hand-worked cases, closed forms, invariants."""
import os

import numpy as np
import pytest

from oracle import policy as P

GOLD = os.path.join(os.path.dirname(__file__), "golden", "stride_worked_cases.txt")


def _model(t_fixed_ms, t_marg_ms):
    # all of T_fixed in t_base, all of T_marginal in delta_cloud: the rate then plays no role
    return P.LatencyModel(0.0, 0.0, 0.0, 0.0, 0.0, t_fixed_ms * 1e-3, t_marg_ms * 1e-3, 0.0)


def _cases(kind):
    for line in open(GOLD):
        f = line.split()
        if f and f[0] == kind:
            yield [float(x) for x in f[1:]]


@pytest.mark.parametrize("c", list(_cases("stride")))
def test_stride_worked_cases(c):
    F, m, g, kmax, model, want = c
    k, obj = P.stride(_model(F, m), 1e6, g, int(kmax), int(model))
    assert k == int(want)
    assert obj == pytest.approx(P.expected_tokens(g, k, int(model)) / ((F + k * m) * 1e-3))


@pytest.mark.parametrize("c", list(_cases("ema")))
def test_ema_worked_cases(c):
    g, tau, k, mu, want = c
    assert P.ema(g, int(tau), int(k), mu) == pytest.approx(want, abs=1e-12)


def test_latency_model_grouping_matches_the_four_terms():
    # T_fixed + K * T_marginal must equal T_edge + T_up + T_cloud + T_down written out term by term
    m = P.LatencyModel(alpha_edge=0.012, beta=0.004, bits_per_token=17, header_bits=320, t_prop=0.02, t_base=0.03,
                       delta_cloud=0.0015, t_down=0.011)
    for rate in (2e4, 1e6, 3e8):
        for k in (1, 3, 8):
            t_edge = m.alpha_edge * k + m.beta
            t_up = m.t_prop + (k * m.bits_per_token + m.header_bits) / rate
            t_cloud = m.t_base + k * m.delta_cloud
            assert P.t_step(m, rate, k) == pytest.approx(t_edge + t_up + t_cloud + m.t_down, rel=1e-14)


def test_linear_numerator_is_monotone_so_the_optimum_is_an_endpoint():
    rng = np.random.default_rng(0)
    for _ in range(200):
        F, mm, g = rng.uniform(1, 200), rng.uniform(0.1, 200), rng.uniform(0.05, 0.99)
        k, _ = P.stride(_model(F, mm), 1.0, g, 12, P.LINEAR)
        assert k == (12 if g * F > mm * (1 + 1e-12) else 1) or abs(g * F - mm) < 1e-9


def test_geometric_model_closed_form_and_monotonicity_in_the_link():
    # 1 + sum gamma^i = (1 - gamma^(K+1)) / (1 - gamma)
    for g in (0.1, 0.5, 0.8, 0.95):
        for k in (1, 4, 9):
            assert P.expected_tokens(g, k, P.GEOMETRIC) == pytest.approx((1 - g ** (k + 1)) / (1 - g), rel=1e-13)
    # With no header the rate enters the marginal cost only: a faster link never shortens the stride (Sec. IV-B: a
    # reduced rate forces a smaller K).  A longer propagation delay never shortens it either (it is amortised).
    # (With a header the rate also sits in T_fixed through O_header / R, and a slower link can lengthen the stride.)
    m = P.LatencyModel(0.01, 0.002, 16, 0, 0.02, 0.03, 0.001, 0.01)
    ks = [P.stride(m, r, 0.8, 12, P.GEOMETRIC)[0] for r in (1e2, 3e2, 1e3, 1e4, 1e5, 1e6, 1e8)]
    assert ks == sorted(ks) and ks[0] < ks[-1], ks
    from dataclasses import replace
    kp = [P.stride(replace(m, t_prop=tp), 1e4, 0.8, 12, P.GEOMETRIC)[0] for tp in (0.0, 0.05, 0.2, 1.0)]
    assert kp == sorted(kp)
    # a better draft never shortens it
    kg = [P.stride(m, 1e4, g, 12, P.GEOMETRIC)[0] for g in (0.1, 0.3, 0.5, 0.7, 0.9)]
    assert kg == sorted(kg)


def test_ema_is_a_convex_combination_and_converges_to_the_observed_rate():
    g = P.GAMMA_INIT
    for _ in range(200):
        g2 = P.ema(g, 3, 6, 0.1)
        assert min(g, 0.5) - 1e-15 <= g2 <= max(g, 0.5) + 1e-15
        g = g2
    assert g == pytest.approx(0.5, abs=1e-8)


def test_pager_conserves_pages_and_never_shares_one():
    rng = np.random.default_rng(1)
    pg = P.Pager(64)
    lens = {}
    for step in range(2000):
        s = int(rng.integers(0, 6))
        op = rng.integers(0, 3)
        if op == 0:
            n = lens.get(s, 0) + int(rng.integers(1, 40))
            if pg.reserve(s, n):
                lens[s] = n
        elif op == 1 and lens.get(s, 0) > 0:
            n = int(rng.integers(0, lens[s] + 1))
            before = len(pg.owned[s])
            assert pg.trim(s, n) == before - (-(-n // 16))
            lens[s] = n
        else:
            pg.release(s)
            lens[s] = 0
        owned = [p for v in pg.owned.values() for p in v]
        assert len(owned) == len(set(owned)) and not set(owned) & set(pg.free)
        assert len(owned) + len(pg.free) == 64
        for t, v in pg.owned.items():
            assert len(v) == -(-lens.get(t, 0) // 16)
