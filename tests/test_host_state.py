"""The library's host-side state functions (stride selection, acceptance-rate average, page bookkeeping) against
the oracle in oracle/policy.py.  Host only: no GPU is touched."""
import numpy as np
import pytest

from oracle import policy as P
from paper_2601_00644_amd import flexverify as fv


@pytest.fixture(scope="module", autouse=True)
def _built_library():
    import os
    if not os.path.exists(fv.LIB_PATH):          # the host-side entry points need no GPU, only the built library
        from paper_2601_00644_amd import build
        build.build(verbose=False)


def _pair(rng):
    vals = dict(alpha_edge=rng.uniform(0, 0.03), beta=rng.uniform(0, 0.01), bits_per_token=rng.uniform(8, 32),
                header_bits=rng.uniform(0, 1024), t_prop=rng.uniform(0, 0.2), t_base=rng.uniform(0.001, 0.05),
                delta_cloud=rng.uniform(0, 0.005), t_down=rng.uniform(0, 0.05))
    return P.LatencyModel(**vals), fv.LatencyModel(**vals)


def test_stride_matches_oracle_on_a_seeded_grid():
    rng = np.random.default_rng(5)
    seen = set()
    for _ in range(3000):
        mo, ml = _pair(rng)
        rate = 10 ** rng.uniform(2, 9)
        g = rng.uniform(0.02, 0.99)
        kmax = int(rng.integers(1, 17))
        for model in (P.LINEAR, P.GEOMETRIC):
            k_ref, f_ref = P.stride(mo, rate, g, kmax, model)
            k, f = fv.policy_stride(ml, rate, g, kmax, model)
            assert f == pytest.approx(f_ref, rel=1e-13)
            if k != k_ref:   # only a tie to rounding may differ
                f_other = P.expected_tokens(g, k, model) / P.t_step(mo, rate, k)
                assert abs(f_other - f_ref) <= 1e-12 * f_ref
            seen.add(k)
    assert len(seen) >= 8     # the grid exercises short and long strides


def test_step_time_matches_oracle():
    rng = np.random.default_rng(8)
    for _ in range(300):
        mo, ml = _pair(rng)
        rate, k = 10 ** rng.uniform(2, 9), int(rng.integers(0, 17))
        assert fv.policy_step_time(ml, rate, k) == pytest.approx(P.t_step(mo, rate, k), rel=1e-13)
        assert fv.policy_step_time(ml, rate, k, 0.0123) == pytest.approx(
            P.t_step(mo, rate, k) - (mo.t_base + k * mo.delta_cloud) + 0.0123, rel=1e-12)
    assert fv.policy_step_time(_pair(rng)[1], 0.0, 3) == -1.0


def test_stride_rejects_bad_arguments():
    _, ml = _pair(np.random.default_rng(0))
    for args in ((0.0, 0.8, 8, 1), (1e6, 0.8, 0, 1), (1e6, -0.1, 8, 1), (1e6, 0.8, 8, 7)):
        with pytest.raises(fv.FsvError):
            fv.policy_stride(ml, *args)


def test_ema_matches_oracle():
    rng = np.random.default_rng(6)
    g_ref = g = P.GAMMA_INIT
    for _ in range(500):
        k = int(rng.integers(1, 13))
        tau = int(rng.integers(0, k + 1))
        mu = float(rng.uniform(0, 1))
        g_ref, g = P.ema(g_ref, tau, k, mu), fv.policy_ema(g, tau, k, mu)
        assert g == pytest.approx(g_ref, rel=1e-15, abs=1e-16)
    assert fv.policy_ema(0.6, 3, 0, 0.5) == 0.6     # no drafts: nothing to average


def test_pager_matches_oracle_page_for_page():
    rng = np.random.default_rng(7)
    NP, NS, MP = 96, 7, 24
    ref, lib = P.Pager(NP), fv.Pager(NP, NS, MP)
    lens = [0] * NS
    row = np.full(MP, -1, np.int32)
    for _ in range(3000):
        s = int(rng.integers(0, NS))
        op = int(rng.integers(0, 3))
        if op == 0:
            n = min(lens[s] + int(rng.integers(1, 60)), MP * 16)
            ok_ref = ref.reserve(s, n)
            if ok_ref:
                lib.reserve(s, n, row)
                assert row[: len(ref.owned[s])].tolist() == ref.owned[s]
                lens[s] = n
            else:
                with pytest.raises(fv.FsvError) as ei:
                    lib.reserve(s, n, row)
                assert ei.value.status == -2
        elif op == 1:
            n = int(rng.integers(0, lens[s] + 1))
            assert lib.trim(s, n) == ref.trim(s, n)
            lens[s] = n
        else:
            assert lib.trim(s, 0) == ref.release(s)
            lens[s] = 0
        assert lib.free_pages == len(ref.free)
        assert lib.session_pages(s) == len(ref.owned.get(s, []))
    with pytest.raises(fv.FsvError):
        lib.reserve(0, MP * 16 + 1, row)      # beyond max_pages_per_session
    lib.close()
