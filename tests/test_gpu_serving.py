"""Many rounds of draft -> verify -> state update on persistent paged sessions (Alg. 2), on the GPU.

Forty rounds on a small fp32 model with a pool too small to hold every session at its final length unless pages
are recycled: sessions are ended and reopened on the way.  Checked every round: the strides come from the
oracle's policy, the acceptance average follows the oracle's EMA, the page bookkeeping stays consistent with
the lengths; checked at the end: the KV of every live session equals what the oracle computes in ONE fresh pass
over the session's restored context and its whole accepted token history (so no stale or recycled slot was ever
read), and the library's next-token logits equal the oracle's.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from oracle import policy as P
from paper_2601_00644_amd import synth
from tests.helpers import logits_close

pytestmark = pytest.mark.gpu


def test_forty_rounds_with_page_reuse_f32():
    from paper_2601_00644_amd import flexverify as fv
    from paper_2601_00644_amd import serve
    cfg = synth.MODELS["minif32"]
    seed, S, rounds, kmax = 41, 5, 40, 6
    w = synth.make_weights(cfg, seed, std=0.06)
    wn = synth.weights_to_numpy(cfg, w)
    vals = dict(alpha_edge=0.010, beta=0.002, bits_per_token=16.0, header_bits=0.0, t_prop=0.030, t_base=0.020,
                delta_cloud=0.001, t_down=0.010)
    lm, lm_ref = fv.LatencyModel(**vals), P.LatencyModel(**vals)
    max_len = [60, 85, 110, 135, 160]            # a session is ended and reopened once it passes its length
    MP = (max(max_len) + kmax + 1 + 15) // 16 + 1
    num_pages = 40                               # enough for all sessions at their limits, far less than the test consumes
    srv = serve.Server(cfg, {k: v.cuda() for k, v in w.items()}, S, num_pages, kmax, MP, lm, mu=0.2, temperature=0.9,
                       sigma=0.6, seed=seed)
    contexts = {}
    opened = 0

    def open_new(s):
        nonlocal opened
        L = int(5 + 7 * ((opened * 3) % 5))
        k, v = synth.make_kv_context(cfg, L, seed, 100 + opened)
        contexts[s] = (k, v)
        srv.open_session(s, k, v, last_token=(17 * opened + 3) % cfg.vocab)
        opened += 1

    for s in range(S):
        open_new(s)
    gamma_ref = [P.GAMMA_INIT] * S
    strides, accepted, drafted, reopened = set(), 0, 0, 0
    for rnd in range(rounds):
        rates = serve.lognormal_rates(S, 2.0e3, 1.2, seed, rnd)
        want_K = [P.stride(lm_ref, float(rates[s]), gamma_ref[s], kmax, P.GEOMETRIC)[0] for s in range(S)]
        before = [srv.sessions[s].seq_len for s in range(S)]
        out = srv.round(rates, k_max=kmax)
        for j, s in enumerate(out["sessions"]):
            K, tau = int(out["K"][j]), int(out["tau"][j])
            assert K == want_K[s]                                   # the policy is the oracle's
            gamma_ref[s] = P.ema(gamma_ref[s], tau, K, 0.2)
            assert srv.sessions[s].gamma_hat == pytest.approx(gamma_ref[s], rel=1e-14)
            assert srv.sessions[s].seq_len == before[s] + 1 + tau   # Alg. 2 step 3: accepted drafts plus the pending token
            assert srv.pager.session_pages(s) == -(-srv.sessions[s].seq_len // 16)
            strides.add(K)
            accepted += tau
            drafted += K
        assert srv.pager.free_pages + sum(srv.pager.session_pages(s) for s in range(S)) == num_pages
        for s in range(S):
            if srv.sessions[s].seq_len > max_len[s]:
                srv.end_session(s)
                open_new(s)
                gamma_ref[s] = P.GAMMA_INIT
                reopened += 1
    assert reopened >= 2 and len(strides) >= 3 and 0 < accepted < drafted
    print(f"rounds {rounds}: strides seen {sorted(strides)}, accepted {accepted}/{drafted}, sessions reopened {reopened}")

    # the sessions as they stand: one fresh oracle pass over context + accepted history must reproduce them
    probe_batch = None
    for s in range(S):
        ss = srv.sessions[s]
        k, v = contexts[s]
        L0, n = ss.start_len, len(ss.history)
        assert ss.seq_len == L0 + n
        kc, vc = oracle.new_cache(cfg, L0 + n + 1)
        kc[:, :L0] = synth.kv_to_f64(k)
        vc[:, :L0] = synth.kv_to_f64(v)
        if n > 0:
            oracle.forward(cfg, wn, kc, vc, L0, np.array(ss.history, np.int32))
        gk, gv = srv.ctx.kv_export(srv.k_pool, srv.v_pool, num_pages, torch.as_tensor(srv.page_table[s]).cuda(), 0, ss.seq_len)
        for got, ref in ((gk, kc[:, :ss.seq_len]), (gv, vc[:, :ss.seq_len])):
            assert np.abs(got.cpu().numpy() - ref).max() <= 1e-4 * max(1.0, float(np.abs(ref).max())), s
        # and the next pending token scores the same on both sides
        lg_ref = oracle.forward(cfg, wn, kc, vc, ss.seq_len, np.array([ss.last_token], np.int32))[0]
        srv.pager.reserve(s, ss.seq_len + 1, srv.page_table[s])
        t = lambda a: torch.as_tensor(np.ascontiguousarray(a)).cuda()
        z = np.zeros(1, np.float32)
        b = fv.DeviceBatch(t(np.array([ss.seq_len], np.int32)), t(np.array([ss.last_token], np.int32)),
                           t(np.zeros(2, np.int32)), None, None, None, t(z), t(z), t(srv.page_table[s:s + 1]),
                           srv.k_pool, srv.v_pool, num_pages, np.array([ss.seq_len], np.int32), np.zeros(2, np.int32), z)
        res = fv.DeviceResult.alloc(1, 1, cfg.vocab, want_logits=True)
        srv.ctx.verify(b, res)
        torch.cuda.synchronize()
        ok, ratio = logits_close(res.logits_out.cpu().numpy().astype(np.float64), lg_ref[None, :], 1e-4)
        assert ok, (s, ratio)
    srv.close()
