"""GPU parity of the whole bf16 verification step on reduced Llama-shaped models the oracle finishes
in seconds (GQA, head sizes 64 and 128, ragged vocabulary, ragged gamma, several key ranges).

Bar (helpers.check_bf16_logits): every logits row within a flat 2e-2 of the fp64 oracle (in L2, and
each element against the row's scale); the appended cache rows of layer 0 bit for bit equal to the
oracle's forward with the bf16 storage points rounded (helpers.check_bf16_kv).  Accept / reject
decisions must equal the oracle's except where its own margin to the threshold is inside what the
measured logit difference can move (counted and printed); the accept / resample arithmetic itself
is compared draw by draw on identical logits in test_gpu_sampler.py.
"""
import numpy as np
import pytest
import torch

from paper_2601_00644_amd import synth
from tests.helpers import build_case, check_bf16_kv, check_bf16_requests, fmt_bf16_report
from tests.test_gpu_verify_f32 import run_library

pytestmark = pytest.mark.gpu


def _kv_check(case, ctx, kp, vp, pt, nl):
    cfg, req = case.cfg, case.req
    for b, e in enumerate(case.expected_st):
        L = int(req.seq_lens[b])
        n_new = int(min(nl[b], e.new_len)) - L     # appended rows of the valid prefix
        gk, gv = ctx.kv_export(kp, vp, req.num_pages, pt[b], L, n_new)
        kc, vc = case.caches_st[b]
        for name, got, ref in (("k", gk, kc[:, L:L + n_new]), ("v", gv, vc[:, L:L + n_new])):
            g2 = got.float().cpu().numpy().astype(np.float64).reshape(cfg.n_layers, n_new, -1)
            check_bf16_kv(g2, ref.reshape(cfg.n_layers, n_new, -1), True, (b, name))


@pytest.mark.parametrize("name,batch,ctx_hi,gmax,seed", [
    ("mini128", 5, 700, 8, 1),
    ("mini64", 4, 1100, 16, 2),
    ("mini128", 9, 90, 3, 3),
])
def test_bf16_end_to_end(name, batch, ctx_hi, gmax, seed):
    cfg = synth.MODELS[name]
    wl = synth.Workload("t", name, batch, 1, ctx_hi, "uniform", 0, gmax, "uniform", 0.7, 0.8, "permuted")
    case = build_case(cfg, wl, seed=seed, weight_std=0.04)
    ctx, batch_d, res, kp, vp, pt = run_library(case)
    req = case.req
    lg = res.logits_out.cpu().numpy().astype(np.float64)
    tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
    reports, excused, flagged = check_bf16_requests(cfg, req, case.expected, case.expected_st, lg, tau, nxt, True, name)
    worst = max(reports.values(), key=lambda r: r["vs_fp64"]["l2"])
    print(f"{name}: worst request: {fmt_bf16_report(worst)}; accepted {int(tau.sum())}/{int(req.draft_offsets[-1])}; "
          f"decisions differing inside the margin: {excused}")
    nl, pr = res.new_seq_lens.cpu().numpy(), res.pages_released.cpu().numpy()
    for b in range(req.batch):
        L, g = int(req.seq_lens[b]), int(req.gammas[b])
        assert nl[b] == L + 1 + tau[b]
        assert pr[b] == (L + 1 + g + 15) // 16 - (int(nl[b]) + 15) // 16
    _kv_check(case, ctx, kp, vp, pt, nl)
    # determinism: the same call again gives bit-identical logits
    _, _, res2, *_ = run_library(case, ctx=ctx)
    assert torch.equal(res2.logits_out, res.logits_out)
    ctx.close()


def test_bf16_fused_step_uses_the_same_sampler_as_fsv_sample():
    # self-consistency inside the library: decisions of fsv_verify equal fsv_sample run on its own logits
    from paper_2601_00644_amd import flexverify as fv
    cfg = synth.MODELS["mini64"]
    wl = synth.Workload("t", "mini64", 6, 1, 300, "uniform", 1, 8, "uniform", 0.7, 0.8)
    case = build_case(cfg, wl, seed=4, weight_std=0.04, run_oracle=False)
    ctx, batch_d, res, kp, vp, pt = run_library(case)
    res2 = fv.DeviceResult.alloc(case.req.batch)
    ctx.sample(res.logits_out, batch_d, res2)
    torch.cuda.synchronize()
    assert torch.equal(res.accepted_len, res2.accepted_len) and torch.equal(res.next_token, res2.next_token)
    ctx.close()


def test_bf16_seeded_shape_sweep():
    """Eight seeded shapes of the whole bf16 step (both head sizes, batch 1..12, contexts from empty to 1500, gamma up
    to 16, every page layout): logits against the oracle, rollback outputs against their closed form."""
    rng = np.random.default_rng(77)
    for case_no in range(8):
        name = ("mini128", "mini64")[case_no % 2]
        cfg = synth.MODELS[name]
        batch = int(rng.integers(1, 13))
        ctx_hi = int(rng.choice([0, 40, 300, 900, 1500]))
        gmax = int(rng.choice([1, 4, 9, 16]))
        pages = ("interleaved", "permuted", "contiguous")[case_no % 3]
        wl = synth.Workload("t", name, batch, 0, ctx_hi, "uniform", 0, gmax, "uniform", 0.7, 0.8, pages)
        case = build_case(cfg, wl, seed=200 + case_no, weight_std=0.04)
        ctx, batch_d, res, kp, vp, pt = run_library(case)
        req = case.req
        lg = res.logits_out.cpu().numpy().astype(np.float64)
        tau = res.accepted_len.cpu().numpy()
        reports, excused, flagged = check_bf16_requests(cfg, req, case.expected, case.expected_st, lg, tau,
                                                        res.next_token.cpu().numpy(), True, f"case {case_no} {name}")
        worst = max(max(r["vs_fp64"]["l2"], r["vs_fp64"]["row"]) for r in reports.values())
        worst_st = max(r["vs_stored"]["l2"] for r in reports.values())
        nl, pr = res.new_seq_lens.cpu().numpy(), res.pages_released.cpu().numpy()
        for b in range(req.batch):
            L, g = int(req.seq_lens[b]), int(req.gammas[b])
            assert nl[b] == L + 1 + tau[b] and pr[b] == (L + 1 + g + 15) // 16 - (int(nl[b]) + 15) // 16
        print(f"case {case_no}: {name} B={batch} ctx<={ctx_hi} gamma<={gmax} {pages}: worst vs fp64 {worst:.3e}, "
              f"worst row L2 vs bf16-storage oracle {worst_st:.3e}")
        ctx.close()
