"""GPU edge cases of fsv_verify on a reduced bf16 model: degenerate batches the method allows
(no drafts at all, empty sessions, greedy mode), and the error paths of the boundary (nothing is
launched on an error; the status says why).
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2601_00644_amd import synth
from tests.helpers import build_case, check_bf16_logits, compare_decisions
from tests.test_gpu_verify_f32 import run_library

pytestmark = pytest.mark.gpu


def _stage_b(case, res):
    """The oracle's sampler on the library's own logits, per request."""
    req = case.req
    out = []
    for b in range(req.batch):
        o, g = int(req.draft_offsets[b]), int(req.gammas[b])
        rows = res.logits_out[o + b: o + b + g + 1].cpu().numpy().astype(np.float64)
        s = oracle.sample(rows, case.draft_tokens[o:o + g], case.draft_probs[o:o + g].numpy(), req.u_accept[o:o + g],
                          float(req.u_sample[b]), float(req.temperature[b]))
        out.append(type("R", (), {"sample": s})())
    return out


def test_no_drafts_is_plain_decoding():
    # gamma = 0 for every request: one row per request, tau = 0, the token is drawn from p_0
    cfg = synth.MODELS["mini64"]
    wl = synth.Workload("t", "mini64", 5, 1, 200, "uniform", 0, 0, "fixed", 0.7, 0.9, "permuted")
    case = build_case(cfg, wl, seed=21, weight_std=0.04)
    ctx, batch, res, kp, vp, pt = run_library(case)
    assert int(case.req.draft_offsets[-1]) == 0
    tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
    assert (tau == 0).all()
    assert (res.new_seq_lens.cpu().numpy() == case.req.seq_lens + 1).all()
    assert (res.pages_released.cpu().numpy() == 0).all()
    bad, _, _ = compare_decisions(_stage_b(case, res), tau, nxt)
    assert not bad, bad
    lg = res.logits_out.cpu().numpy().astype(np.float64)
    for b, e in enumerate(case.expected):
        check_bf16_logits(lg[b: b + 1], e.logits, case.expected_st[b].logits, f"request {b}")
    ctx.close()


def test_empty_sessions():
    # L = 0: nothing cached, the pending token sits at position 0 and the drafts see only the block itself
    cfg = synth.MODELS["mini128"]
    wl = synth.Workload("t", "mini128", 4, 0, 0, "fixed", 1, 7, "uniform", 0.7, 0.8, "interleaved")
    case = build_case(cfg, wl, seed=22, weight_std=0.04)
    assert (case.req.seq_lens == 0).all()
    ctx, batch, res, kp, vp, pt = run_library(case)
    lg = res.logits_out.cpu().numpy().astype(np.float64)
    for b, e in enumerate(case.expected):
        rs = int(case.req.draft_offsets[b]) + b
        check_bf16_logits(lg[rs: rs + int(case.req.gammas[b]) + 1], e.logits, case.expected_st[b].logits, f"request {b}")
    tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
    bad, _, _ = compare_decisions(_stage_b(case, res), tau, nxt)
    assert not bad, bad
    assert (res.new_seq_lens.cpu().numpy() == 1 + tau).all()
    ctx.close()


def test_greedy_mode_bf16():
    # T = 0 (the acceptance loop as printed in Alg. 2): longest prefix with draft == argmax, then the argmax
    cfg = synth.MODELS["mini64"]
    wl = synth.Workload("t", "mini64", 6, 1, 300, "uniform", 1, 8, "uniform", 0.7, 0.8, "permuted")
    case = build_case(cfg, wl, seed=23, weight_std=0.04, run_oracle=False)
    # make some drafts certain to match: replace the first draft of even requests by the oracle-free trick of
    # running the library once and reading its own argmax (the check below is against the oracle's sampler on
    # the logits of the SECOND run, so nothing is compared with itself)
    case.req.temperature[:] = 0.0
    ctx, batch, res, kp, vp, pt = run_library(case)
    lg = res.logits_out.cpu().numpy()
    for b in range(0, case.req.batch, 2):
        o = int(case.req.draft_offsets[b])
        case.draft_tokens[o] = int(lg[o + b].argmax())
    ctx.close()
    ctx, batch, res, kp, vp, pt = run_library(case)
    tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
    exp = _stage_b(case, res)
    bad, _, _ = compare_decisions(exp, tau, nxt)
    assert not bad, bad
    assert any(int(t) >= 1 for t in tau[0::2])
    assert (res.flags.cpu().numpy() == 0).all()
    ctx.close()


def test_never_written_slots_may_hold_anything():
    # KV pools that were never zeroed: every slot that holds no valid position (the tail of each session's last page, and
    # every unused page) is filled with NaN / Inf / huge bit patterns.  Such slots are masked out of the softmax and must
    # not reach the output through the matrix cores either (0 * NaN): logits stay within the bar and hold no NaN.
    from paper_2601_00644_amd import flexverify as fv
    cfg = synth.MODELS["mini128"]
    wl = synth.Workload("t", "mini128", 5, 1, 300, "uniform", 0, 7, "uniform", 0.7, 0.8, "permuted")
    case = build_case(cfg, wl, seed=25, weight_std=0.04)
    req = case.req
    ctx = fv.Context(cfg, {k: v.cuda() for k, v in case.weights.items()}, max_batch=req.batch, max_gamma=16,
                     max_pages_per_req=req.page_table.shape[1])
    junk = np.array([0x7FC0, 0xFFC0, 0x7F80, 0xFF80, 0x7F7F, 0xFF7F, 0x7FFF, 0x0001], np.uint16)   # NaNs, infinities, huge
    shape = fv.pool_shape(cfg, req.num_pages)
    n = int(np.prod(shape))
    bits = junk[np.arange(n) % junk.size]
    kp = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).reshape(shape).cuda()
    vp = torch.from_numpy(bits[::-1].view(np.int16).copy()).view(torch.bfloat16).reshape(shape).cuda()
    pt = torch.as_tensor(req.page_table, device="cuda")
    for b in range(req.batch):
        if case.ctx_k[b].shape[1] > 0:
            ctx.kv_import(kp, vp, req.num_pages, pt[b], 0, case.ctx_k[b].cuda(), case.ctx_v[b].cuda())
    batch = fv.device_batch(req, case.draft_tokens, case.draft_probs.cuda(), kp, vp)
    res = fv.DeviceResult.alloc(req.batch, batch.rows, cfg.vocab, want_logits=True)
    ctx.verify(batch, res)
    torch.cuda.synchronize()
    lg = res.logits_out.cpu().numpy().astype(np.float64)
    assert np.isfinite(lg).all()
    for b, e in enumerate(case.expected):
        rs = int(req.draft_offsets[b]) + b
        check_bf16_logits(lg[rs: rs + int(req.gammas[b]) + 1], e.logits, case.expected_st[b].logits, f"request {b}")
    ctx.close()


def test_late_validation_failures_launch_nothing():
    # failures that are only found while the launches are being planned (a KV pool layer of 4 GiB or more on the bf16
    # path; more keys than the fp32 path keeps in LDS) are reported before the first launch, as the header promises
    from paper_2601_00644_amd import flexverify as fv
    cfg = synth.MODELS["mini64"]
    wl = synth.Workload("t", "mini64", 2, 10, 60, "uniform", 1, 4, "uniform", 0.7, 0.8, "interleaved")
    case = build_case(cfg, wl, seed=26, weight_std=0.04, run_oracle=False)
    req = case.req
    ctx = fv.Context(cfg, {k: v.cuda() for k, v in case.weights.items()}, max_batch=2, max_gamma=4,
                     max_pages_per_req=req.page_table.shape[1])
    kp, vp = fv.alloc_pools(cfg, req.num_pages)
    batch = fv.device_batch(req, case.draft_tokens, case.draft_probs.cuda(), kp, vp)
    res = fv.DeviceResult.alloc(req.batch)
    sentinel = torch.full_like(res.next_token, -7)
    res.next_token.copy_(sentinel)
    # (the pools are not touched: the call must fail on the claimed page count alone)
    batch.num_pages = (1 << 32) // (cfg.n_kv_heads * 16 * cfg.head_dim * 2) + 1
    with pytest.raises(fv.FsvError) as ei:
        ctx.verify(batch, res)
    assert ei.value.status == -3
    torch.cuda.synchronize()
    assert torch.equal(res.next_token, sentinel)
    ctx.close()
    # fp32 path: a session longer than the 16384 keys its attention kernel keeps in LDS
    cfg32 = synth.MODELS["minif32"]
    w32 = synth.make_weights(cfg32, 27)
    ctx = fv.Context(cfg32, {k: v.cuda() for k, v in w32.items()}, max_batch=1, max_gamma=2, max_pages_per_req=1100)
    L = np.array([17000], np.int32)
    off = np.array([0, 1], np.int32)
    kp, vp = fv.alloc_pools(cfg32, 4)
    t = lambda a: torch.as_tensor(a, device="cuda")
    b32 = fv.DeviceBatch(t(L), t(np.zeros(1, np.int32)), t(off), t(np.zeros(1, np.int32)),
                         torch.zeros((1, cfg32.vocab), device="cuda"), t(np.zeros(1, np.float32)), t(np.zeros(1, np.float32)),
                         t(np.ones(1, np.float32)), torch.zeros((1, 1100), dtype=torch.int32, device="cuda"), kp, vp, 4, L, off,
                         np.ones(1, np.float32))
    res = fv.DeviceResult.alloc(1)
    res.next_token.fill_(-7)
    with pytest.raises(fv.FsvError) as ei:
        ctx.verify(b32, res)
    assert ei.value.status == -3
    torch.cuda.synchronize()
    assert int(res.next_token[0]) == -7
    ctx.close()


def test_error_paths_launch_nothing():
    from paper_2601_00644_amd import flexverify as fv
    cfg = synth.MODELS["mini64"]
    wl = synth.Workload("t", "mini64", 3, 10, 60, "uniform", 1, 4, "uniform", 0.7, 0.8, "interleaved")
    case = build_case(cfg, wl, seed=24, weight_std=0.04, run_oracle=False)
    req = case.req
    ctx = fv.Context(cfg, {k: v.cuda() for k, v in case.weights.items()}, max_batch=3, max_gamma=4,
                     max_pages_per_req=req.page_table.shape[1])
    kp, vp = fv.alloc_pools(cfg, req.num_pages)
    batch = fv.device_batch(req, case.draft_tokens, case.draft_probs.cuda(), kp, vp)
    res = fv.DeviceResult.alloc(req.batch)
    sentinel = torch.full_like(res.next_token, -7)
    res.next_token.copy_(sentinel)

    def expect(status, mutate):
        import copy
        b2 = copy.copy(batch)
        mutate(b2)
        with pytest.raises(fv.FsvError) as ei:
            ctx.verify(b2, res)
        assert ei.value.status == status, (ei.value.status, status)
        torch.cuda.synchronize()
        assert torch.equal(res.next_token, sentinel)      # nothing ran

    # more drafts than the context was created for
    off_big = req.draft_offsets.copy()
    off_big[1:] += 5
    expect(-2, lambda b: (setattr(b, "draft_offsets_host", off_big.astype(np.int32))))
    # a session longer than the page table covers
    L_big = req.seq_lens.copy()
    L_big[0] = req.page_table.shape[1] * 16
    expect(-2, lambda b: setattr(b, "seq_lens_host", L_big.astype(np.int32)))
    # inconsistent CSR
    off_bad = req.draft_offsets.copy()
    off_bad[0] = 1
    expect(-1, lambda b: setattr(b, "draft_offsets_host", off_bad.astype(np.int32)))
    # a required pointer missing
    expect(-1, lambda b: setattr(b, "page_table", None))
    expect(-1, lambda b: setattr(b, "draft_probs", None))
    # negative temperature
    expect(-1, lambda b: setattr(b, "temperature_host", np.array([0.8, -1.0, 0.8], np.float32)))
    # an empty batch is not an error and touches nothing
    empty = fv.DeviceBatch(batch.seq_lens, batch.last_token, torch.zeros(1, dtype=torch.int32, device="cuda"), None, None,
                           None, batch.u_sample, batch.temperature, batch.page_table, kp, vp, req.num_pages,
                           np.zeros(0, np.int32), np.zeros(1, np.int32), np.zeros(0, np.float32))
    ctx.verify(empty, res)
    torch.cuda.synchronize()
    assert torch.equal(res.next_token, sentinel)
    # and the context still works afterwards
    ctx.verify(batch, res)
    torch.cuda.synchronize()
    assert (res.next_token >= 0).all() and (res.next_token < cfg.vocab).all()
    ctx.close()
