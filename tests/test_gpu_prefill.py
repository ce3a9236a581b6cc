"""GPU parity of fsv_prefill, the target forward without the accept / reject step: a session's context restored from
tokens, taken in pieces of at most max_gamma + 1 rows that continue each other inside one call.

The oracle side is its plain forward over the whole chunk at once (pinned in test_oracle_forward.py: a block of tokens
equals the same tokens one by one).  Bars as for the verification step: fp32 model 1e-4; bf16 models a flat 2e-2
against the fp64 oracle, layer-0 cache rows against the oracle with the bf16 storage points rounded.
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2601_00644_amd import synth
from tests.helpers import STORED_BF16, check_bf16_kv, check_bf16_logits, fmt_bf16_report, logits_close, oracle_cache_from_context

pytestmark = pytest.mark.gpu


def _setup(name, sessions, seed, max_gamma):
    from paper_2601_00644_amd import flexverify as fv
    cfg = synth.MODELS[name]
    w = synth.make_weights(cfg, seed, std=0.04 if cfg.dtype == "bf16" else 0.02)
    wn = synth.weights_to_numpy(cfg, w)
    rng = np.random.default_rng(seed)
    chunks, ctxs = [], []
    for s_, (L0, n) in enumerate(sessions):
        k, v = synth.make_kv_context(cfg, L0, seed, s_)
        ctxs.append((k.contiguous(), v.contiguous()))
        chunks.append((s_, L0, rng.integers(0, cfg.vocab, n).astype(np.int32)))
    mp = max((L0 + n + cfg.page_size - 1) // cfg.page_size for L0, n in sessions) + 1
    S = len(sessions)
    # pages of the sessions interleaved (page j of session s = j * S + s), as the serving workloads lay them out
    page_rows = np.array([[j * S + s_ for j in range(mp)] for s_ in range(S)], np.int32)
    num_pages = S * mp
    pieces = sum((n + max_gamma) // (max_gamma + 1) for _, n in sessions)
    ctx = fv.Context(cfg, {k_: v_.to("cuda") for k_, v_ in w.items()}, max_batch=pieces, max_gamma=max_gamma, max_pages_per_req=mp)
    kp, vp = fv.alloc_pools(cfg, num_pages, "cuda")
    pt = torch.as_tensor(page_rows, device="cuda")
    for s_, (k, v) in enumerate(ctxs):
        if k.shape[1] > 0:
            ctx.kv_import(kp, vp, num_pages, pt[s_], 0, k.to("cuda"), v.to("cuda"))
    return fv, cfg, wn, chunks, ctxs, ctx, kp, vp, pt, page_rows, num_pages


def _oracle(cfg, wn, ctxs, chunks, stored):
    out = []
    for (s_, L0, tokens), (k, v) in zip(chunks, ctxs):
        kc, vc = oracle_cache_from_context(cfg, k, v, L0 + len(tokens))
        lg = oracle.forward(cfg, wn, kc, vc, L0, tokens, stored=stored)
        out.append((lg, kc, vc))
    return out


@pytest.mark.parametrize("name,sessions,max_gamma,seed", [
    ("mini128", [(37, 45), (0, 9), (300, 1)], 8, 1),      # five pieces + one piece from an empty session + a single row
    ("mini64", [(513, 70), (64, 33)], 15, 2),              # pieces of 16 rows; a chunk that starts on a page boundary
])
def test_prefill_in_pieces_matches_the_oracle_bf16(name, sessions, max_gamma, seed):
    fv, cfg, wn, chunks, ctxs, ctx, kp, vp, pt, page_rows, num_pages = _setup(name, sessions, seed, max_gamma)
    batch = fv.prefill_pieces(chunks, page_rows, kp, vp, num_pages, max_gamma + 1)
    lg = ctx.prefill(batch, want_logits=True)
    torch.cuda.synchronize()
    lg = lg.cpu().numpy().astype(np.float64)
    ref, ref_st = _oracle(cfg, wn, ctxs, chunks, 0), _oracle(cfg, wn, ctxs, chunks, STORED_BF16)
    row = 0
    for (s_, L0, tokens), (r64, _, _), (rst, kst, vst) in zip(chunks, ref, ref_st):
        n = len(tokens)
        rep = check_bf16_logits(lg[row:row + n], r64, rst, f"{name} session {s_}", flat=True)
        print(f"{name} session {s_} ({n} rows on {L0}): {fmt_bf16_report(rep)}")
        row += n
        gk, gv = ctx.kv_export(kp, vp, num_pages, pt[s_], L0, n)
        for nm, got, want in (("k", gk, kst[:, L0:L0 + n]), ("v", gv, vst[:, L0:L0 + n])):
            check_bf16_kv(got.float().cpu().numpy().astype(np.float64).reshape(cfg.n_layers, n, -1),
                          want.reshape(cfg.n_layers, n, -1), True, (s_, nm))
    assert row == lg.shape[0]
    # the same chunks again, cache only: identical cache rows, and no logits buffer needed
    before = [ctx.kv_export(kp, vp, num_pages, pt[s_], L0, len(t)) for s_, L0, t in chunks]
    assert ctx.prefill(batch) is None
    torch.cuda.synchronize()
    for (s_, L0, t), (k0, v0) in zip(chunks, before):
        k1, v1 = ctx.kv_export(kp, vp, num_pages, pt[s_], L0, len(t))
        assert torch.equal(k0, k1) and torch.equal(v0, v1)
    ctx.close()


def test_prefill_in_pieces_matches_the_oracle_f32():
    fv, cfg, wn, chunks, ctxs, ctx, kp, vp, pt, page_rows, num_pages = _setup("minif32", [(21, 30), (0, 5)], 3, 6)
    batch = fv.prefill_pieces(chunks, page_rows, kp, vp, num_pages, 7)
    lg = ctx.prefill(batch, want_logits=True).cpu().numpy().astype(np.float64)
    row = 0
    for (s_, L0, tokens), (r64, kc, vc) in zip(chunks, _oracle(cfg, wn, ctxs, chunks, 0)):
        n = len(tokens)
        ok, ratio = logits_close(lg[row:row + n], r64, 1e-4)
        assert ok, (s_, ratio)
        row += n
        gk, gv = ctx.kv_export(kp, vp, num_pages, pt[s_], 0, L0 + n)
        tol = 1e-4 * max(1.0, float(np.abs(kc[:, :L0 + n]).max()))
        assert np.abs(gk.float().cpu().numpy() - kc[:, :L0 + n]).max() <= tol
        assert np.abs(gv.float().cpu().numpy() - vc[:, :L0 + n]).max() <= tol
    ctx.close()


def test_prefill_then_verify_continues_the_session():
    """A context restored from tokens by fsv_prefill serves the next verification call like one restored from a saved
    cache: the logits of a verification step on top of it match the oracle run on the oracle's own prefilled cache."""
    fv, cfg, wn, chunks, ctxs, ctx, kp, vp, pt, page_rows, num_pages = _setup("mini128", [(5, 40)], 4, 8)
    ctx.prefill(fv.prefill_pieces(chunks, page_rows, kp, vp, num_pages, 9))
    s_, L0, tokens = chunks[0]
    L = L0 + len(tokens)
    rng = np.random.default_rng(9)
    nxt = rng.integers(0, cfg.vocab, 6).astype(np.int32)       # pending token + five drafts, greedy verification
    b = fv.DeviceBatch(torch.tensor([L], dtype=torch.int32, device="cuda"), torch.tensor([int(nxt[0])], dtype=torch.int32, device="cuda"),
                       torch.tensor([0, 5], dtype=torch.int32, device="cuda"), torch.as_tensor(nxt[1:], device="cuda"), None, None,
                       torch.zeros(1, device="cuda"), torch.zeros(1, device="cuda"), pt[:1].contiguous(), kp, vp, num_pages,
                       np.array([L], np.int32), np.array([0, 5], np.int32), np.zeros(1, np.float32))
    res = fv.DeviceResult.alloc(1, 6, cfg.vocab, want_logits=True)
    ctx.verify(b, res)
    torch.cuda.synchronize()
    k, v = ctxs[0]
    kc, vc = oracle_cache_from_context(cfg, k, v, L + 6)
    oracle.forward(cfg, wn, kc, vc, L0, tokens)
    ref = oracle.forward(cfg, wn, kc, vc, L, nxt)
    k2, v2 = oracle_cache_from_context(cfg, k, v, L + 6)
    oracle.forward(cfg, wn, k2, v2, L0, tokens, stored=STORED_BF16)
    ref_st = oracle.forward(cfg, wn, k2, v2, L, nxt, stored=STORED_BF16)
    rep = check_bf16_logits(res.logits_out.cpu().numpy().astype(np.float64), ref, ref_st, "verify after prefill", flat=True)
    print("verify after prefill:", fmt_bf16_report(rep))
    ctx.close()


def test_prefill_refusals():
    fv, cfg, wn, chunks, ctxs, ctx, kp, vp, pt, page_rows, num_pages = _setup("mini64", [(10, 12)], 5, 15)
    batch = fv.prefill_pieces(chunks, page_rows, kp, vp, num_pages, 16)
    for field in ("last_token", "page_table", "seq_lens"):
        saved = getattr(batch, field)
        setattr(batch, field, None)
        with pytest.raises(fv.FsvError) as ei:
            ctx.prefill(batch)
        assert ei.value.status == -1
        setattr(batch, field, saved)
    too_long = fv.prefill_pieces([(0, 10, np.zeros(40, np.int32))], page_rows, kp, vp, num_pages, 40)   # one piece of 40 rows
    with pytest.raises(fv.FsvError) as ei:
        ctx.prefill(too_long)
    assert ei.value.status == -2
    ctx.close()
