"""GPU parity at the full sizes of the configurations, in the launch configuration bench.py times.

The oracle cannot score a whole 8B-shape batch in test time, but requests are independent in every
step of the verification path, so a subset is exact: a few sampled requests are given drafts the
ORACLE stepped (nothing the oracle consumes comes from the library), the library verifies the full
batch, and for the sampled requests logits, decisions, rollback and appended KV are compared with
the oracle.  The logit bar is helpers.check_bf16_logits: a flat 2e-2 against the plain fp64 oracle at
every size (what 16-bit storage alone costs on the same request is computed beside it, by the oracle
in its storage mode, and printed); the appended cache rows of layer 0 equal the storage-mode oracle's
bit for bit, deeper layers within the same bar.
For every request of the batch the accept / resample arithmetic is compared exactly on identical
logits: the oracle's sampler is run on the logits the library produced (flagged draws counted), and
the rollback outputs against their closed form.  The sampling configuration (logits are inputs) is
compared in full at all five noise levels.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2601_00644_amd import synth
from tests.helpers import (STORED_BF16, check_bf16_kv, check_bf16_logits, compare_decisions, decision_margins,
                           fmt_bf16_report)

pytestmark = pytest.mark.gpu



def _oracle_drafts(cfg, wn, wl, req, seed, b):
    """Step the oracle through request b's drafts; returns (tokens, laws, cache) with the cache at length L."""
    L, g, o = int(req.seq_lens[b]), int(req.gammas[b]), int(req.draft_offsets[b])
    k, v = synth.make_kv_context(cfg, L, seed, b, device="cuda")     # the bits workload.build imports for b
    kc, vc = oracle.new_cache(cfg, L + g + 1)
    kc[:, :L] = synth.kv_to_f64(k)
    vc[:, :L] = synth.kv_to_f64(v)
    del k, v
    k2, v2 = kc.copy(), vc.copy()
    tok, T = int(req.last_token[b]), float(req.temperature[b])
    q = torch.zeros((g, cfg.vocab), dtype=torch.float32)
    d = np.zeros(g, np.int32)
    for i in range(g):
        lg = oracle.forward(cfg, wn, k2, v2, L + i, np.array([tok], np.int32))[0]
        q[i] = synth.draft_law(torch.from_numpy(lg), T, wl.sigma, seed, o + i)
        tok = synth.draw_from(q[i], float(req.u_draft[o + i]))
        d[i] = tok
    return d, q, (kc, vc)


def _check_workload(wl_name, weights, wn, seed, pick, flat):
    from paper_2601_00644_amd import flexverify as fv
    from paper_2601_00644_amd import workload
    wl = synth.WORKLOADS[wl_name]
    cfg = synth.MODELS[wl.model]
    req = synth.make_requests(wl, cfg, seed)
    sampled = pick(req)
    host_drafts, caches = {}, {}
    for b in sampled:
        d, q, cache = _oracle_drafts(cfg, wn, wl, req, seed, b)
        host_drafts[b] = (d, q)
        caches[b] = cache
    w = workload.build(wl, seed, weights=weights, host_drafts=host_drafts)
    B, G = req.batch, w.drafts
    res = fv.DeviceResult.alloc(B, G + B, cfg.vocab, want_logits=True)
    w.ctx.verify(w.batch, res)
    torch.cuda.synchronize()
    tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
    nl, pr, flags = res.new_seq_lens.cpu().numpy(), res.pages_released.cpu().numpy(), res.flags.cpu().numpy()
    d_all, q_all = w.draft_tokens.cpu().numpy(), w.draft_probs

    # every request: the library's decisions against the oracle's sampler on the library's own logits
    stage_b = []
    for b in range(B):
        o, g = int(req.draft_offsets[b]), int(req.gammas[b])
        rows = res.logits_out[o + b: o + b + g + 1].cpu().numpy().astype(np.float64)
        s = oracle.sample(rows, d_all[o:o + g], q_all[o:o + g].cpu().numpy(), req.u_accept[o:o + g],
                          float(req.u_sample[b]), float(req.temperature[b]))
        stage_b.append(type("R", (), {"sample": s})())
        L = int(req.seq_lens[b])
        assert 0 <= tau[b] <= g
        assert nl[b] == L + 1 + tau[b]
        assert pr[b] == (L + 1 + g + 15) // 16 - (int(nl[b]) + 15) // 16
    bad, excused, flagged = compare_decisions(stage_b, tau, nxt)
    print(f"{wl_name}: B={B} G={G} accepted {int(tau.sum())}; sampler on identical logits: flagged {flagged}, excused {excused}")
    assert not bad, bad

    # sampled requests: everything against the oracle's own forward, in its two modes
    for b in sampled:
        L, g, o = int(req.seq_lens[b]), int(req.gammas[b]), int(req.draft_offsets[b])
        kc, vc = caches[b]
        ks, vs = kc.copy(), vc.copy()
        d, q = host_drafts[b]
        args = (L, int(req.last_token[b]), d, q.numpy(), req.u_accept[o:o + g], float(req.u_sample[b]), float(req.temperature[b]))
        e = oracle.verify(cfg, wn, kc, vc, *args)
        es = oracle.verify(cfg, wn, ks, vs, *args, stored=STORED_BF16)
        got = res.logits_out[o + b: o + b + g + 1].cpu().numpy().astype(np.float64)
        rep = check_bf16_logits(got, e.logits, es.logits, f"{wl_name} request {b}", flat)
        print(f"  request {b} (L={L}, gamma={g}): {fmt_bf16_report(rep)}; tau {int(tau[b])} vs {es.sample.tau} "
              f"(fp64 oracle {e.sample.tau})")
        exp = [None] * B
        exp[b] = es
        exp[b] = e
        acc_m, cdf_m = decision_margins(rep["vs_fp64"]["abs"], float(req.temperature[b]))
        bad, _, _ = compare_decisions(exp, tau, nxt, acc_m, cdf_m)
        assert not bad, (bad, acc_m, cdf_m)
        n_new = int(min(nl[b], es.new_len)) - L
        gk, gv = w.ctx.kv_export(w.k_pool, w.v_pool, req.num_pages, w.page_table[b], L, n_new)
        for name, gotkv, ref in (("k", gk, ks[:, L:L + n_new]), ("v", gv, vs[:, L:L + n_new])):
            g2 = gotkv.float().cpu().numpy().astype(np.float64).reshape(cfg.n_layers, n_new, -1)
            check_bf16_kv(g2, ref.reshape(cfg.n_layers, n_new, -1), True, (b, name), rep["bar_fp64"])
    w.ctx.close()
    del w, res
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def llama8b():
    cfg = synth.MODELS["llama8b"]
    weights = synth.make_weights(cfg, 1, device="cuda")
    wn = synth.weights_to_numpy(cfg, weights)
    yield weights, wn
    del weights, wn
    torch.cuda.empty_cache()


def test_c3_8b_batch16_sampled_requests(llama8b):
    weights, wn = llama8b
    # the shortest and the longest session, the one with the most drafts and the one with the fewest (at least four)
    def pick(req):
        want = {int(np.argmin(req.seq_lens)), int(np.argmax(req.seq_lens)), int(np.argmax(req.gammas)), int(np.argmin(req.gammas))}
        for b in range(req.batch):
            if len(want) >= 4:
                break
            want.add(b)
        return sorted(want)
    _check_workload("c3_8b_b16", weights, wn, 1, pick, flat=True)


def test_c5_8b_batch128_sampled_requests(llama8b):
    weights, wn = llama8b
    # the shortest session and one of the longest among those with few drafts (the oracle's cost grows with rows)
    def pick(req):
        few = np.nonzero(req.gammas <= 4)[0]
        return sorted({int(np.argmin(req.seq_lens)), int(few[np.argmax(req.seq_lens[few])]), int(np.argmax(req.gammas))})
    _check_workload("c5_8b_b128", weights, wn, 1, pick, flat=True)


@pytest.fixture(scope="module")
def llama1b():
    cfg = synth.MODELS["llama1b"]
    weights = synth.make_weights(cfg, 2, device="cuda")
    wn = synth.weights_to_numpy(cfg, weights)
    yield weights, wn
    del weights, wn
    torch.cuda.empty_cache()


@pytest.mark.parametrize("gamma", [2, 3, 4, 5, 6, 7, 8])
def test_c2_1b_single_request_gamma_sweep(llama1b, gamma):
    from dataclasses import replace
    weights, wn = llama1b
    name = f"c2_1b_g{gamma}"
    synth.WORKLOADS[name] = replace(synth.WORKLOADS["c2_1b"], name=name, gamma_lo=gamma, gamma_hi=gamma)
    try:
        _check_workload(name, weights, wn, 2, lambda req: [0], flat=True)
    finally:
        del synth.WORKLOADS[name]


@pytest.mark.parametrize("sigma,lo,hi", [(0.3, 0.75, 0.99), (0.5, 0.65, 0.95), (0.7, 0.50, 0.90), (1.0, 0.35, 0.80),
                                         (1.5, 0.20, 0.70)])
def test_c4_sampler_full_size(sigma, lo, hi):
    """Batch 64, ragged gamma 1..16, vocabulary 152064, bf16 logits ~ N(0,3), temperature 0.7: every request."""
    from paper_2601_00644_amd import flexverify as fv
    V, B = 152064, 64
    case = synth.make_sampler_case(B, 1, 16, V, sigma, 0.7, 7, logits_dtype="bf16", device="cuda")
    cfg = synth.ModelCfg("sampler", 0, 0, 0, 0, 0, 0, V, "bf16")
    ctx = fv.Context(cfg, None, B, 16, sampler_only=True)
    t = lambda a: torch.as_tensor(np.ascontiguousarray(a), device="cuda")
    batch = fv.DeviceBatch(None, None, t(case.draft_offsets), t(case.draft_tokens), case.draft_probs, t(case.u_accept),
                           t(case.u_sample), t(case.temperature), None, None, None, 0, None,
                           np.ascontiguousarray(case.draft_offsets), np.ascontiguousarray(case.temperature))
    res = fv.DeviceResult.alloc(B)
    ctx.sample(case.logits, batch, res)
    torch.cuda.synchronize()
    tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
    lg = case.logits.float().cpu().numpy().astype(np.float64)
    q = case.draft_probs.cpu().numpy()
    exp = []
    for b in range(B):
        o, e = int(case.draft_offsets[b]), int(case.draft_offsets[b + 1])
        s = oracle.sample(lg[o + b: e + b + 1], case.draft_tokens[o:e], q[o:e], case.u_accept[o:e],
                          float(case.u_sample[b]), 0.7)
        exp.append(type("R", (), {"sample": s})())
    bad, excused, flagged = compare_decisions(exp, tau, nxt)
    # per-draft acceptance rate over the drafts that were tested (those up to and including the first rejection)
    tested = sum(min(int(x.sample.tau) + 1, int(case.draft_offsets[b + 1] - case.draft_offsets[b])) for b, x in enumerate(exp))
    rate = float(sum(x.sample.tau for x in exp)) / tested
    print(f"sigma {sigma}: acceptance per tested draft {rate:.3f}, flagged {flagged}, excused {excused}")
    assert not bad, bad
    assert lo <= rate <= hi, rate      # the closed form 2*Phi(-sigma/2) for a diffuse target: 0.88, 0.80, 0.73, 0.62, 0.45
    ctx.close()
