"""GPU parity of the whole verification step in fp32 (the tiny CPU-finishable configuration).

Inputs: seeded weights, a context the oracle prefilled, drafts uniform over the vocabulary with a
random draft law (configuration 1), plus ragged GQA batches on a second small fp32 model.  Bar:
logits within 1e-4 (relative to max(|ref|, row rms)), accepted lengths / tokens / rollback exact
except flagged draws, appended KV equal to the oracle's cache.
"""
import numpy as np
import pytest
import torch

from paper_2601_00644_amd import synth
from tests.helpers import build_case, compare_decisions, logits_close

pytestmark = pytest.mark.gpu


def run_library(case, ctx=None, page_kind=None, want_logits=True):
    from paper_2601_00644_amd import flexverify as fv
    cfg, req = case.cfg, case.req
    dev = "cuda"
    own = ctx is None
    if own:
        ctx = fv.Context(cfg, {k: v.to(dev) for k, v in case.weights.items()}, max_batch=req.batch,
                         max_gamma=16, max_pages_per_req=req.page_table.shape[1])
    kp, vp = fv.alloc_pools(cfg, req.num_pages, dev)
    pt = torch.as_tensor(req.page_table, device=dev)
    for b in range(req.batch):
        if case.ctx_k[b].shape[1] > 0:
            ctx.kv_import(kp, vp, req.num_pages, pt[b], 0, case.ctx_k[b].to(dev), case.ctx_v[b].to(dev))
    batch = fv.device_batch(req, case.draft_tokens, case.draft_probs.to(dev), kp, vp, dev)
    res = fv.DeviceResult.alloc(req.batch, batch.rows, cfg.vocab, want_logits=want_logits)
    ctx.verify(batch, res)
    torch.cuda.synchronize()
    return ctx, batch, res, kp, vp, pt


def check_against_oracle(case, ctx, res, kp, vp, pt, tol):
    cfg, req = case.cfg, case.req
    lg = res.logits_out.cpu().numpy().astype(np.float64)
    worst = 0.0
    for b, e in enumerate(case.expected):
        if e is None:
            continue
        rs = int(req.draft_offsets[b]) + b
        ok, ratio = logits_close(lg[rs: rs + int(req.gammas[b]) + 1], e.logits, tol)
        worst = max(worst, ratio)
        assert ok, (b, ratio)
    tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
    bad, excused, flagged = compare_decisions(case.expected, tau, nxt)
    assert not bad, bad
    nl, pr = res.new_seq_lens.cpu().numpy(), res.pages_released.cpu().numpy()
    for b, e in enumerate(case.expected):
        if e is None or int(tau[b]) != e.sample.tau:
            continue
        assert (int(nl[b]), int(pr[b])) == (e.new_len, e.pages_released)
        # the session after the call: appended KV of the valid prefix equals the oracle's cache
        L = int(req.seq_lens[b])
        gk, gv = ctx.kv_export(kp, vp, req.num_pages, pt[b], 0, e.new_len)
        kc, vc = case.caches[b]
        kref, vref = kc[:, : e.new_len], vc[:, : e.new_len]
        ktol = tol * max(1.0, float(np.abs(kref).max()))
        assert np.abs(gk.float().cpu().numpy() - kref).max() <= ktol
        assert np.abs(gv.float().cpu().numpy() - vref).max() <= ktol
    return worst, excused, flagged


def test_config1_tiny_end_to_end():
    cfg = synth.MODELS["tiny"]
    case = build_case(cfg, synth.WORKLOADS["c1_tiny"], seed=1, prefill_context=True, independent_draft_law=True)
    ctx, batch, res, kp, vp, pt = run_library(case)
    worst, excused, flagged = check_against_oracle(case, ctx, res, kp, vp, pt, 1e-4)
    print(f"tiny: worst logit ratio {worst:.2e}, tau {res.accepted_len.cpu().tolist()}, excused {excused}")
    ctx.close()


@pytest.mark.parametrize("seed,pages", [(2, "interleaved"), (3, "permuted")])
def test_ragged_gqa_batch_f32(seed, pages):
    cfg = synth.MODELS["minif32"]
    wl = synth.Workload("t", "minif32", 6, 3, 90, "uniform", 0, 7, "uniform", 0.7, 0.9, pages)
    case = build_case(cfg, wl, seed=seed, weight_std=0.06)
    ctx, batch, res, kp, vp, pt = run_library(case)
    worst, excused, flagged = check_against_oracle(case, ctx, res, kp, vp, pt, 1e-4)
    acc = int(res.accepted_len.sum())
    print(f"minif32/{pages}: worst {worst:.2e}, accepted {acc}/{int(case.req.draft_offsets[-1])}, flagged {flagged}")
    ctx.close()


def test_greedy_mode_f32():
    cfg = synth.MODELS["minif32"]
    wl = synth.Workload("t", "minif32", 4, 5, 40, "uniform", 1, 5, "uniform", 0.0, 0.0)
    # sigma 0 and temperature 0: drafts come from the target's own law at T=1 (draft_law divides by 1)
    case = build_case(cfg, wl, seed=5, weight_std=0.3)
    ctx, batch, res, kp, vp, pt = run_library(case)
    tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
    for b, e in enumerate(case.expected):
        # argmax decisions are integer work: exact, unless the two best logits are closer than the tolerance
        top2 = np.sort(e.logits, axis=1)[:, -2:]
        if (top2[:, 1] - top2[:, 0]).min() > 1e-3:
            assert (int(tau[b]), int(nxt[b])) == (e.sample.tau, e.sample.next_token)
    ctx.close()


def test_batch_invariance_and_paging_invariance():
    # a request alone gives the same logits as inside a ragged batch, whatever the page placement
    cfg = synth.MODELS["minif32"]
    wl = synth.Workload("t", "minif32", 5, 3, 70, "uniform", 1, 6, "uniform", 0.7, 1.0, "interleaved")
    case = build_case(cfg, wl, seed=7, weight_std=0.06, run_oracle=False)
    ctx, batch, res, kp, vp, pt = run_library(case)
    full = res.logits_out.cpu().numpy()
    import copy
    perm = copy.deepcopy(case)
    perm.req.page_table, _ = synth.make_page_table(case.req.seq_lens, case.req.gammas, cfg.page_size, "permuted", 99)
    _, _, res2, *_ = run_library(perm, ctx=ctx)
    assert np.array_equal(res2.logits_out.cpu().numpy(), full)
    assert np.array_equal(res2.next_token.cpu().numpy(), res.next_token.cpu().numpy())
    ctx.close()


def test_sessions_over_several_rounds_f32():
    """Verify -> roll back -> verify again on the same paged sessions, five rounds, ragged gamma per round.

    Every round the oracle and the library verify the same drafts on their own copy of the session; the
    accepted prefix and the emitted token carry over (Alg. 2 step 3), rejected positions are overwritten
    by the next round's appends (Sec. IV-C: the KV pairs from the first rejected draft onward are invalid).
    Logits within 1e-4, decisions exact, and at the end the whole valid KV prefix equals the oracle's cache.
    """
    from oracle import oracle
    from paper_2601_00644_amd import flexverify as fv
    cfg = synth.MODELS["minif32"]
    seed, B, rounds, gmax = 31, 3, 5, 6
    w = synth.make_weights(cfg, seed, std=0.06)
    wn = synth.weights_to_numpy(cfg, w)
    L = np.array([5, 20, 33], np.int32)
    cap = int(L.max()) + rounds * (gmax + 1) + 1
    max_pages = (cap + 15) // 16
    pt_np, num_pages = synth.make_page_table(np.full(B, cap - 1, np.int32), np.zeros(B, np.int32), 16, "permuted", seed)
    ctx = fv.Context(cfg, {k: v.cuda() for k, v in w.items()}, max_batch=B, max_gamma=gmax, max_pages_per_req=pt_np.shape[1])
    kp, vp = fv.alloc_pools(cfg, num_pages)
    pt = torch.as_tensor(pt_np).cuda()
    caches = []
    for b in range(B):
        k, v = synth.make_kv_context(cfg, int(L[b]), seed, b)
        kc, vc = oracle.new_cache(cfg, cap)
        kc[:, :L[b]] = synth.kv_to_f64(k)
        vc[:, :L[b]] = synth.kv_to_f64(v)
        caches.append((kc, vc))
        ctx.kv_import(kp, vp, num_pages, pt[b], 0, k.cuda(), v.cuda())
    last = np.array([3, 500, 999], np.int32)
    T = np.array([0.9, 1.0, 0.7], np.float32)
    rng = np.random.default_rng(seed)
    accepted_total = 0
    for rnd in range(rounds):
        g = rng.integers(0, gmax + 1, B).astype(np.int32)
        off = np.zeros(B + 1, np.int32)
        off[1:] = np.cumsum(g)
        G = int(off[-1])
        u_acc, u_smp = synth.uniforms24(G, seed, 100 + rnd), synth.uniforms24(B, seed, 200 + rnd)
        u_d = synth.uniforms24(G, seed, 300 + rnd)
        d = np.zeros(G, np.int32)
        q = torch.zeros((G, cfg.vocab), dtype=torch.float32)
        for b in range(B):   # the synthetic edge model drafts from the target's noised law (oracle stepping on a copy)
            k2, v2 = caches[b][0].copy(), caches[b][1].copy()
            tok = int(last[b])
            for i in range(int(g[b])):
                lg = oracle.forward(cfg, wn, k2, v2, int(L[b]) + i, np.array([tok], np.int32))[0]
                q[off[b] + i] = synth.draft_law(torch.from_numpy(lg), float(T[b]), 0.5, seed, 1000 * rnd + int(off[b]) + i)
                tok = synth.draw_from(q[off[b] + i], float(u_d[off[b] + i]))
                d[off[b] + i] = tok
        exp = [oracle.verify(cfg, wn, caches[b][0], caches[b][1], int(L[b]), int(last[b]), d[off[b]:off[b + 1]],
                             q[off[b]:off[b + 1]].numpy(), u_acc[off[b]:off[b + 1]], float(u_smp[b]), float(T[b]))
               for b in range(B)]
        t = lambda a: torch.as_tensor(np.ascontiguousarray(a)).cuda()
        batch = fv.DeviceBatch(t(L), t(last), t(off), t(d), q.cuda(), t(u_acc), t(u_smp), t(T), pt, kp, vp, num_pages,
                               L.copy(), off, T.copy())
        res = fv.DeviceResult.alloc(B, G + B, cfg.vocab, want_logits=True)
        ctx.verify(batch, res)
        torch.cuda.synchronize()
        lg = res.logits_out.cpu().numpy().astype(np.float64)
        for b, e in enumerate(exp):
            ok, ratio = logits_close(lg[off[b] + b: off[b + 1] + b + 1], e.logits, 1e-4)
            assert ok, (rnd, b, ratio)
        tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
        bad, excused, flagged = compare_decisions(exp, tau, nxt)
        assert not bad, (rnd, bad)
        if excused:
            pytest.skip("a draw fell inside the flag margin; the sessions would diverge")
        nl = res.new_seq_lens.cpu().numpy()
        for b, e in enumerate(exp):
            assert int(nl[b]) == e.new_len == int(L[b]) + 1 + e.sample.tau
            assert int(res.pages_released.cpu()[b]) == e.pages_released
        accepted_total += int(tau.sum())
        L = nl.astype(np.int32)
        last = nxt.astype(np.int32)
    assert accepted_total > 0
    for b in range(B):   # the sessions as they stand after the last rollback
        gk, gv = ctx.kv_export(kp, vp, num_pages, pt[b], 0, int(L[b]))
        kc, vc = caches[b]
        assert np.abs(gk.cpu().numpy() - kc[:, :L[b]]).max() <= 1e-4 * max(1.0, float(np.abs(kc[:, :L[b]]).max()))
        assert np.abs(gv.cpu().numpy() - vc[:, :L[b]]).max() <= 1e-4 * max(1.0, float(np.abs(vc[:, :L[b]]).max()))
    ctx.close()


def test_regime_b_top_p_end_to_end_f32():
    """The whole step with the sampling set-up of Regime B (Sec. V): temperature 1, top-p 0.9 on the target law."""
    from oracle import oracle
    from paper_2601_00644_amd import flexverify as fv
    cfg = synth.MODELS["minif32"]
    wl = synth.Workload("t", "minif32", 6, 3, 90, "uniform", 0, 7, "uniform", 0.7, 1.0, "permuted")
    case = build_case(cfg, wl, seed=12, weight_std=0.3, run_oracle=False)     # wide logits: the nucleus is a real subset
    req = case.req
    top_p = np.full(req.batch, 0.9, np.float32)
    ctx = fv.Context(cfg, {k: v.cuda() for k, v in case.weights.items()}, max_batch=req.batch, max_gamma=16,
                     max_pages_per_req=req.page_table.shape[1])
    kp, vp = fv.alloc_pools(cfg, req.num_pages)
    pt = torch.as_tensor(req.page_table).cuda()
    for b in range(req.batch):
        ctx.kv_import(kp, vp, req.num_pages, pt[b], 0, case.ctx_k[b].cuda(), case.ctx_v[b].cuda())
    batch = fv.device_batch(req, case.draft_tokens, case.draft_probs.cuda(), kp, vp)
    batch.top_p, batch.top_p_host = torch.as_tensor(top_p).cuda(), top_p
    res = fv.DeviceResult.alloc(req.batch, batch.rows, cfg.vocab, want_logits=True)
    ctx.verify(batch, res)
    torch.cuda.synchronize()
    tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
    lg = res.logits_out.cpu().numpy().astype(np.float64)
    exp, exp_off, cut_matters = [], [], 0
    for b in range(req.batch):
        L, g, o = int(req.seq_lens[b]), int(req.gammas[b]), int(req.draft_offsets[b])
        kc, vc = oracle.new_cache(cfg, L + g + 1)
        kc[:, :L], vc[:, :L] = synth.kv_to_f64(case.ctx_k[b]), synth.kv_to_f64(case.ctx_v[b])
        toks = np.concatenate([[req.last_token[b]], case.draft_tokens[o:o + g]]).astype(np.int32)
        ref = oracle.forward(cfg, case.weights_np, kc, vc, L, toks)
        ok, ratio = logits_close(lg[o + b: o + b + g + 1], ref, 1e-4)
        assert ok, (b, ratio)
        args = (ref, case.draft_tokens[o:o + g], case.draft_probs[o:o + g].numpy(), req.u_accept[o:o + g],
                float(req.u_sample[b]), 1.0)
        s = oracle.sample(*args, top_p=0.9)
        s0 = oracle.sample(*args)
        cut_matters += int((s.tau, s.next_token) != (s0.tau, s0.next_token))
        exp.append(None if s.nucleus_margin < 1e-5 else type("R", (), {"sample": s})())
    bad, excused, flagged = compare_decisions(exp, tau, nxt)
    print(f"regime B: accepted {int(tau.sum())}/{int(req.draft_offsets[-1])}, requests the cut changes {cut_matters}")
    assert not bad, bad
    assert (res.new_seq_lens.cpu().numpy() == req.seq_lens + 1 + tau).all()
    ctx.close()
