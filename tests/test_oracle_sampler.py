"""Pins for the oracle's acceptance / resampling step (CPU only).

The oracle is checked against what speculative sampling fixes, not against itself:
the emitted tokens follow the target law (brute force over a tiny vocabulary), every
draft is accepted when p == q, greedy mode is the longest argmax-matching prefix
(Alg. 2), and hand-worked cases from tests/golden/.
"""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

from oracle import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _driver():
    lib_path = os.path.join(HERE, "_brute_force.so")
    src = os.path.join(HERE, "brute_force_sampler.c")
    olib = oracle.build()
    if not os.path.exists(lib_path) or os.path.getmtime(lib_path) < max(os.path.getmtime(src), os.path.getmtime(olib)):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-o", lib_path, src, olib,
                               f"-Wl,-rpath,{os.path.dirname(olib)}", "-lm"])
    lib = C.CDLL(lib_path)
    lib.brute_force.restype = C.c_int
    return lib


def _level_offset(V, n):
    return sum(V ** k for k in range(n))


def _random_tables(V, gamma, seed, peaky):
    """Target / draft laws for every prefix of length 0..gamma (rows of a prefix-coded table)."""
    rng = np.random.default_rng(seed)
    rows = _level_offset(V, gamma + 1)
    p = rng.dirichlet(np.full(V, peaky), size=rows)
    q = rng.dirichlet(np.full(V, peaky), size=rows)
    q = np.maximum(q, 1e-3)
    q /= q.sum(1, keepdims=True)
    return p, q.astype(np.float32)


@pytest.mark.parametrize("V,gamma,N,T", [(5, 1, 400, 1.0), (4, 2, 128, 1.0), (3, 3, 40, 1.0), (4, 2, 96, 0.7),
                                         (6, 0, 4000, 1.3)])
def test_output_law_equals_target_bruteforce(V, gamma, N, T):
    p, q = _random_tables(V, gamma, seed=10 * V + gamma, peaky=2.0)
    # the sampler sees logits and a temperature: hand it T * log p so that softmax(logits / T) == p
    logits = T * np.log(p)
    hist = np.zeros(_level_offset(V, gamma + 2), np.float64)
    rc = _driver().brute_force(C.c_int(V), C.c_int(gamma), C.c_int(N), C.c_double(T),
                               C.c_void_p(logits.ctypes.data), C.c_void_p(q.ctypes.data), C.c_void_p(hist.ctypes.data))
    assert rc == 0
    assert abs(hist.sum() - 1.0) < 1e-6      # q is stored in fp32
    # a midpoint grid with N points misplaces at most 0.5/N of mass per uniform the step consumes
    tol = 0.5 * (gamma + 1) / N
    # mass[prefix] = P(the emitted sequence starts with prefix)
    def emitted_mass(prefix):
        n = len(prefix)
        total = 0.0
        for m in range(n, gamma + 2):      # sequences of length m that extend prefix
            ext = m - n
            base = 0
            for t in prefix:
                base = base * V + t
            for e in range(V ** ext):
                total += hist[_level_offset(V, m) + base * V ** ext + e]
        return total

    checked = 0
    for n in range(0, gamma + 1):          # position n+1 of the emitted sequence, given n emitted tokens
        for code in range(V ** n):
            prefix = []
            c = code
            for _ in range(n):
                prefix.insert(0, c % V)
                c //= V
            joint = np.array([emitted_mass(prefix + [b]) for b in range(V)])
            # only draft sequences that start with this prefix can emit it, so the grid error scales with
            # the draft chain's probability of the prefix
            wq, c2 = 1.0, 0
            for k, t in enumerate(prefix):
                wq *= float(q[_level_offset(V, k) + c2][t])
                c2 = c2 * V + t
            if joint.sum() < 8 * tol * wq:
                continue                  # prefix accepted too rarely for the grid to resolve
            cond = joint / joint.sum()
            want = p[_level_offset(V, n) + code]
            assert np.abs(cond - want).max() < 2 * tol * wq / joint.sum() + 1e-9, (prefix, cond, want)
            checked += 1
    print("prefixes checked:", checked)
    assert checked >= (1 if gamma == 0 else 1 + V)      # the root and most one-token prefixes at least


def test_first_token_law_when_draft_is_wrong_everywhere():
    # a draft law that puts almost everything on one token the target dislikes: output must still follow p
    V, gamma, N = 4, 1, 2000
    p = np.tile(np.array([0.05, 0.15, 0.3, 0.5]), (1 + V, 1))
    q = np.tile(np.array([0.97, 0.01, 0.01, 0.01], np.float32), (1 + V, 1))
    hist = np.zeros(_level_offset(V, 3), np.float64)
    lg = np.log(p)
    assert _driver().brute_force(C.c_int(V), C.c_int(gamma), C.c_int(N), C.c_double(1.0), C.c_void_p(lg.ctypes.data),
                                 C.c_void_p(q.ctypes.data), C.c_void_p(hist.ctypes.data)) == 0
    first = np.array([hist[1 + b] + hist[1 + V + b * V: 1 + V + (b + 1) * V].sum() for b in range(V)])
    assert np.abs(first - p[0]).max() < 3.0 / N


def test_all_accepted_when_p_equals_q():
    # equal logits over a power-of-two vocabulary give p = 1/V exactly, and q = 1/V is exact in fp32
    V, gamma = 64, 6
    logits = np.zeros((gamma + 1, V))
    q = np.full((gamma, V), 1.0 / V, np.float32)
    rng = np.random.default_rng(0)
    for trial in range(50):
        d = rng.integers(0, V, gamma)
        u = rng.integers(0, 1 << 24, gamma) / float(1 << 24)
        if trial == 0:
            u[:] = 1.0 - 2.0 ** -24        # the largest uniform the generator can emit
        if trial == 1:
            u[:] = 0.0
        r = oracle.sample(logits, d, q, u, 0.5, 1.0)
        assert r.tau == gamma and not r.used_residual
        assert r.next_token == 32             # bonus token from p: cumulative 33/64 is the first > 0.5
    # also when the draft law is a hair below the target everywhere it matters
    r = oracle.sample(logits, d, q * np.float32(0.999), u, 0.0, 1.0)
    assert r.tau == gamma and r.next_token == 0


def test_greedy_is_longest_argmax_prefix():
    V, gamma = 11, 5
    rng = np.random.default_rng(3)
    for trial in range(200):
        logits = rng.normal(size=(gamma + 1, V))
        am = logits.argmax(1)
        d = am[:gamma].copy()
        k = rng.integers(0, gamma + 1)      # first mismatch position (gamma = none)
        if k < gamma:
            d[k] = (am[k] + 1 + rng.integers(0, V - 1)) % V
            d[k + 1:] = rng.integers(0, V, gamma - k - 1)
        r = oracle.sample(logits, d, None, np.zeros(gamma), 0.3, 0.0)
        want_tau = k
        # drafts after the first mismatch may match by luck, they must not count
        assert r.tau == want_tau and r.next_token == am[want_tau]


def test_greedy_ties_take_lowest_index():
    logits = np.array([[0.0, 2.0, 2.0, 1.0], [3.0, 3.0, 3.0, 3.0]])
    r = oracle.sample(logits, [1], None, [0.0], 0.0, 0.0)
    assert r.tau == 1 and r.next_token == 0
    r = oracle.sample(logits, [2], None, [0.0], 0.0, 0.0)
    assert r.tau == 0 and r.next_token == 1


def test_small_temperature_with_one_hot_draft_reproduces_greedy():
    V, gamma = 9, 4
    rng = np.random.default_rng(5)
    for trial in range(100):
        logits = rng.normal(size=(gamma + 1, V)) * 3
        d = logits.argmax(1)[:gamma].copy()
        k = rng.integers(0, gamma + 1)
        if k < gamma:
            d[k] = (d[k] + 1) % V
        q = np.zeros((gamma, V), np.float32)
        q[np.arange(gamma), d] = 1.0
        u = rng.uniform(0.001, 0.999, gamma)
        g = oracle.sample(logits, d, None, u, 0.5, 0.0)
        s = oracle.sample(logits, d, q, u, rng.uniform(0.001, 0.999), 1e-3)
        assert (s.tau, s.next_token) == (g.tau, g.next_token)


def _golden_cases():
    path = os.path.join(HERE, "golden", "sampler_worked_cases.txt")
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, p, q, d, ua, us, tau, nxt = [f.strip() for f in line.split("|")]
        rows = lambda s: np.array([[float(x) for x in r.split(",")] for r in s.split(";")])
        yield name, rows(p), rows(q).astype(np.float32), [int(x) for x in d.split(",")], \
            [float(x) for x in ua.split(",")], float(us), int(tau), int(nxt)


@pytest.mark.parametrize("case", list(_golden_cases()), ids=lambda c: c[0])
def test_hand_worked_cases(case):
    name, p, q, d, ua, us, tau, nxt = case
    for T in (1.0, 0.5):
        r = oracle.sample(T * np.log(p), d, q, ua, us, T)
        assert (r.tau, r.next_token) == (tau, nxt), name


def test_zero_draft_request_is_plain_sampling():
    # gamma = 0: one row, the emitted token is an ordinary inverse-CDF draw from p
    p = np.array([[0.125, 0.125, 0.25, 0.5]])
    lg = np.log(p)
    for u, want in [(0.0, 0), (0.124, 0), (0.126, 1), (0.3, 2), (0.51, 3), (0.999, 3)]:
        r = oracle.sample(lg, [], None, [], u, 1.0)
        assert r.tau == 0 and r.next_token == want


def test_margins_report_distance_to_thresholds():
    p = np.array([[0.5, 0.3, 0.2], [0.25, 0.25, 0.5]])
    q = np.array([[0.2, 0.5, 0.3]], np.float32)
    r = oracle.sample(np.log(p), [1], q, [0.59], 0.60, 1.0)      # a = 0.6
    assert abs(r.accept_margin - 0.01) < 1e-6
    assert abs(r.cdf_margin - 0.10) < 1e-6                          # 0.60 sits 0.10 above the edge at 0.5
    assert abs(r.accept_prob[0] - 0.6) < 1e-6


def test_rollback_worked_cases():
    path = os.path.join(HERE, "golden", "rollback_worked_cases.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        L, g, tau, page, new_len, rel = [int(x) for x in line.split()]
        assert oracle.rollback(L, g, tau, page) == (new_len, rel), line
        n += 1
    assert n >= 10


def test_accept_test_is_strict():
    # equal logits over two tokens give p = 1/2 exactly; a draft law that is certain of its token gives
    # ratio exactly 1/2: the draft is accepted iff u < 1/2
    logits = np.zeros((2, 2))
    q = np.array([[1.0, 0.0]], np.float32)
    assert oracle.sample(logits, [0], q, [0.5], 0.1, 1.0).tau == 0
    assert oracle.sample(logits, [0], q, [0.5 - 2.0 ** -24], 0.1, 1.0).tau == 1
    # rejected: residual is max(0, p - q) = (0, 1/2) -> token 1 for every u_sample
    assert oracle.sample(logits, [0], q, [0.5], 0.0, 1.0).next_token == 1


# ---- nucleus (top-p) cut of the target law -------------------------------------------------------------

def _nucleus_cases():
    path = os.path.join(HERE, "golden", "nucleus_worked_cases.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, p, tp, kept, pp = [f.strip() for f in line.split("|")]
        yield name, np.array([float(x) for x in p.split(",")]), float(tp), [int(x) for x in kept.split(",")], \
            np.array([float(x) for x in pp.split(",")])


def _bonus_law_through_the_sampler(p, top_p, N=4000):
    """The law of the emitted token for a request without drafts, read off the oracle on a fine uniform grid."""
    V = len(p)
    lg = np.log(p)[None, :]
    counts = np.zeros(V)
    for k in range(N):
        s = oracle.sample(lg, np.zeros(0, np.int32), None, np.zeros(0, np.float32), (k + 0.5) / N, 1.0, top_p=top_p)
        counts[s.next_token] += 1
    return counts / N


@pytest.mark.parametrize("case", list(_nucleus_cases()), ids=lambda c: c[0])
def test_nucleus_hand_worked_cases(case):
    name, p, top_p, kept, want = case
    law = _bonus_law_through_the_sampler(p, top_p)
    assert sorted(np.nonzero(law)[0].tolist()) == kept
    assert np.abs(law - want).max() < 1.0 / 4000 + 1e-12


def test_nucleus_margin_reports_the_distance_to_the_cut():
    p = np.array([0.5, 0.3, 0.15, 0.05])
    s = oracle.sample(np.log(p)[None, :], np.zeros(0, np.int32), None, np.zeros(0, np.float32), 0.3, 1.0, top_p=0.9)
    assert s.nucleus_margin == pytest.approx(0.05, abs=1e-12)      # min(0.9 - 0.8, 0.95 - 0.9)
    s = oracle.sample(np.log(p)[None, :], np.zeros(0, np.int32), None, np.zeros(0, np.float32), 0.3, 1.0, top_p=1.0)
    assert s.nucleus_margin == float("inf")


@pytest.mark.parametrize("V,gamma,N,top_p", [(5, 1, 400, 0.8), (4, 2, 128, 0.7), (6, 0, 4000, 0.6)])
def test_output_law_equals_nucleus_cut_target_bruteforce(V, gamma, N, top_p):
    """Speculative sampling on the cut law: every emitted token, given the ones before it, follows the target law
    cut to its nucleus, whatever the draft law is (brute force over all drafts and a grid of uniforms)."""
    p, q = _random_tables(V, gamma, seed=100 * V + gamma, peaky=1.0)
    logits = np.log(p)
    hist = np.zeros(_level_offset(V, gamma + 2), np.float64)
    drv = _driver()
    drv.brute_force_warp.restype = C.c_int
    rc = drv.brute_force_warp(C.c_int(V), C.c_int(gamma), C.c_int(N), C.c_double(1.0), C.c_double(top_p),
                              C.c_void_p(logits.ctypes.data), C.c_void_p(q.ctypes.data), C.c_void_p(hist.ctypes.data))
    assert rc == 0

    def cut(row):   # the definition, written with numpy: sort, cumulate, keep ties of the last kept value
        order = np.argsort(-row, kind="stable")
        k = int(np.searchsorted(np.cumsum(row[order]), top_p, side="left"))
        thr = row[order[min(k, V - 1)]]
        out = np.where(row >= thr, row, 0.0)
        return out / out.sum()

    tol = 0.5 * (gamma + 1) / N
    first = np.zeros(V)
    for b in range(V):     # law of the first emitted token
        first[b] = hist[1 + b]
        for m in range(2, gamma + 2):
            ext = V ** (m - 1)
            first[b] += hist[_level_offset(V, m) + b * ext: _level_offset(V, m) + (b + 1) * ext].sum()
    want = cut(p[0])
    assert np.abs(first - want).max() < 2 * tol + 1e-9, (first, want)
    assert (first[want == 0] == 0).all()          # nothing outside the nucleus is ever emitted
    if gamma >= 1:         # second token given an accepted-or-corrected first token b
        for b in range(V):
            if first[b] < 16 * tol:
                continue
            joint = np.zeros(V)
            for c in range(V):
                joint[c] = hist[_level_offset(V, 2) + b * V + c]
                for m in range(3, gamma + 2):
                    ext = V ** (m - 2)
                    base = _level_offset(V, m) + (b * V + c) * ext
                    joint[c] += hist[base: base + ext].sum()
            # sequences that stop after the first token (a rejection at draft 1) carry no second token: condition
            # on those that continue
            if joint.sum() < 16 * tol * float(q[0][b]):
                continue
            cond = joint / joint.sum()
            want2 = cut(p[1 + b])
            assert np.abs(cond - want2).max() < 4 * tol / joint.sum() + 1e-9, (b, cond, want2)


def test_accepts_everything_when_draft_equals_the_cut_target():
    rng = np.random.default_rng(3)
    V, gamma, top_p = 50, 4, 0.85
    p = rng.dirichlet(np.full(V, 0.5), size=gamma + 1)
    lg = np.log(p)

    def cut(row):
        order = np.argsort(-row, kind="stable")
        k = int(np.searchsorted(np.cumsum(row[order]), top_p, side="left"))
        out = np.where(row >= row[order[min(k, V - 1)]], row, 0.0)
        return out / out.sum()

    q = np.stack([cut(p[i]) for i in range(gamma)]).astype(np.float32)
    for trial in range(50):
        d = np.array([rng.choice(V, p=q[i].astype(np.float64) / q[i].astype(np.float64).sum()) for i in range(gamma)], np.int32)
        u = rng.random(gamma).astype(np.float32) * 0.999
        s = oracle.sample(lg, d, q, u, 0.5, 1.0, top_p=top_p)
        assert s.tau == gamma      # fp32 storage of q can only make q slightly smaller or larger than p'; u < 0.999


# ---- top-k cut, alone and followed by top-p ------------------------------------------------------------------

def _topk_cases():
    path = os.path.join(HERE, "golden", "topk_worked_cases.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, p, tk, tp, kept, pp = [f.strip() for f in line.split("|")]
        yield name, np.array([float(x) for x in p.split(",")]), int(tk), float(tp), [int(x) for x in kept.split(",")], \
            np.array([float(x) for x in pp.split(",")])


@pytest.mark.parametrize("case", list(_topk_cases()), ids=lambda c: c[0])
def test_topk_hand_worked_cases(case):
    name, p, top_k, top_p, kept, want = case
    V, N = len(p), 4000
    lg = np.log(p)[None, :]
    counts = np.zeros(V)
    for k in range(N):    # the law of the emitted token of a request without drafts, read off a fine uniform grid
        s = oracle.sample(lg, np.zeros(0, np.int32), None, np.zeros(0, np.float32), (k + 0.5) / N, 1.0, top_p=top_p, top_k=top_k)
        counts[s.next_token] += 1
    law = counts / N
    assert sorted(np.nonzero(law)[0].tolist()) == kept
    assert np.abs(law - want).max() < 1.0 / N + 1e-12


def _cut_definition(row, top_k, top_p):
    """The cut written with numpy sorting (a library routine), independent of the oracle's code."""
    V = len(row)
    out = row.copy()
    if 0 < top_k < V:
        thr = np.sort(out)[::-1][top_k - 1]
        out = np.where(out >= thr, out, 0.0)
        out = out / out.sum()
    if top_p < 1.0:
        order = np.argsort(-out, kind="stable")
        k = int(np.searchsorted(np.cumsum(out[order]), top_p, side="left"))
        thr = out[order[min(k, V - 1)]]
        out = np.where(out >= thr, out, 0.0)
        out = out / out.sum()
    return out


@pytest.mark.parametrize("V,gamma,N,top_k,top_p", [(5, 1, 400, 3, 1.0), (4, 2, 128, 2, 1.0), (6, 1, 300, 4, 0.7), (6, 0, 4000, 3, 0.6)])
def test_output_law_equals_cut_target_bruteforce_topk(V, gamma, N, top_k, top_p):
    """Speculative sampling on the top-k (and top-p) cut law: the first emitted token follows the cut target law whatever
    the draft law is, and nothing outside the kept set is ever emitted (brute force over all drafts and uniforms)."""
    p, q = _random_tables(V, gamma, seed=200 * V + gamma, peaky=1.0)
    logits = np.log(p)
    hist = np.zeros(_level_offset(V, gamma + 2), np.float64)
    drv = _driver()
    drv.brute_force_cut.restype = C.c_int
    rc = drv.brute_force_cut(C.c_int(V), C.c_int(gamma), C.c_int(N), C.c_double(1.0), C.c_int(top_k), C.c_double(top_p),
                             C.c_void_p(logits.ctypes.data), C.c_void_p(q.ctypes.data), C.c_void_p(hist.ctypes.data))
    assert rc == 0
    tol = 0.5 * (gamma + 1) / N
    first = np.zeros(V)
    for b in range(V):
        first[b] = hist[1 + b]
        for m in range(2, gamma + 2):
            ext = V ** (m - 1)
            first[b] += hist[_level_offset(V, m) + b * ext: _level_offset(V, m) + (b + 1) * ext].sum()
    want = _cut_definition(p[0], top_k, top_p)
    assert np.abs(first - want).max() < 2 * tol + 1e-9, (first, want)
    assert (first[want == 0] == 0).all()
    assert int((want > 0).sum()) <= max(top_k, 1) or top_k == 0      # random tables have no ties: at most top_k tokens survive
