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
