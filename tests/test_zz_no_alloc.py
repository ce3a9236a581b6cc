"""fsv_sample_static (the entry point that allocates nothing) against fsv_sample, through the C ABI.

Two calls in a row on the same GPU, the second with a smaller input (fewer requests, fewer rows, a smaller vocabulary):
the library's fixed device array still holds the first call's contents then, and the results must not depend on them.
Bar: integer outputs (accepted lengths, emitted tokens, flags) bit for bit equal to fsv_sample's on the same inputs,
which the other sampler tests hold to the oracle.  Also: inputs beyond the fixed limits are refused and launch nothing.
"""
import numpy as np
import pytest
import torch

from paper_2601_00644_amd import synth

pytestmark = pytest.mark.gpu


def _batch(fv, case, top_p=None):
    t = lambda a: torch.as_tensor(np.ascontiguousarray(a), device="cuda")
    b = fv.DeviceBatch(None, None, t(case.draft_offsets), t(case.draft_tokens), case.draft_probs.cuda(), t(case.u_accept),
                       t(case.u_sample), t(case.temperature), None, None, None, 0, None,
                       np.ascontiguousarray(case.draft_offsets), np.ascontiguousarray(case.temperature))
    if top_p is not None:
        b.top_p_host = np.ascontiguousarray(top_p, np.float32)
        b.top_p = t(b.top_p_host)
    return b


def _both(fv, case, top_p=None):
    B = len(case.draft_offsets) - 1
    V = int(case.logits.shape[1])
    cfg = synth.ModelCfg("sampler", 0, 0, 0, 0, 0, 0, V, "bf16")
    ctx = fv.Context(cfg, None, B, 16, sampler_only=True)
    batch = _batch(fv, case, top_p)
    logits = case.logits.cuda()
    want = fv.DeviceResult.alloc(B)
    ctx.sample(logits, batch, want)
    got = fv.DeviceResult.alloc(B)
    for t_ in (got.accepted_len, got.next_token, got.flags):
        t_.fill_(-3)
    fv.sample_static(V, logits, batch, got)
    torch.cuda.synchronize()
    ctx.close()
    return got, want


def test_static_entry_point_matches_fsv_sample_on_two_calls_in_a_row():
    from paper_2601_00644_amd import flexverify as fv
    big = synth.make_sampler_case(48, 1, 16, 152064, 0.7, 0.7, 31, logits_dtype="bf16", device="cuda")
    small = synth.make_sampler_case(5, 0, 6, 5003, 1.0, 0.9, 32, logits_dtype="f32")
    mixed_t = small.temperature.copy()
    mixed_t[1] = 0.0                       # one greedy request among the sampled ones
    small.temperature = mixed_t
    calls = [(big, None), (small, None), (small, np.array([0.9, 1.0, 0.5, 1.0, 0.8], np.float32))]
    for case, top_p in calls:
        got, want = _both(fv, case, top_p)
        assert torch.equal(got.accepted_len, want.accepted_len)
        assert torch.equal(got.next_token, want.next_token)
        assert torch.equal(got.flags, want.flags)
        B = len(case.draft_offsets) - 1
        assert int(got.accepted_len.min()) >= 0 and int(got.next_token.min()) >= 0 and B > 0


def test_static_entry_point_refuses_what_exceeds_its_fixed_workspace():
    from paper_2601_00644_amd import flexverify as fv
    case = synth.make_sampler_case(4, 1, 3, 4096, 0.5, 0.8, 33, logits_dtype="bf16")
    batch = _batch(fv, case)
    res = fv.DeviceResult.alloc(4)
    res.next_token.fill_(-7)
    logits = case.logits.cuda()
    # more requests than the workspace holds (only the host copy of the offsets is read before the refusal)
    too_many = np.arange(130, dtype=np.int32)
    b2 = fv.DeviceBatch(None, None, batch.draft_offsets, batch.draft_tokens, batch.draft_probs, batch.u_accept,
                        batch.u_sample, batch.temperature, None, None, None, 0, None, too_many, None)
    with pytest.raises(fv.FsvError) as ei:
        fv.sample_static(4096, logits, b2, res)
    assert ei.value.status == -2
    # more rows than the workspace holds: 100 requests with 16 drafts each
    off = (np.arange(101, dtype=np.int32) * 16).astype(np.int32)
    b3 = fv.DeviceBatch(None, None, batch.draft_offsets, batch.draft_tokens, batch.draft_probs, batch.u_accept,
                        batch.u_sample, batch.temperature, None, None, None, 0, None, off, None)
    with pytest.raises(fv.FsvError) as ei:
        fv.sample_static(4096, logits, b3, res)
    assert ei.value.status == -2
    # a vocabulary beyond 327680
    with pytest.raises(fv.FsvError) as ei:
        fv.sample_static(400000, logits, batch, res)
    assert ei.value.status == -2
    torch.cuda.synchronize()
    assert (res.next_token == -7).all()
    # and a call within the limits still works afterwards
    fv.sample_static(4096, logits, batch, res)
    torch.cuda.synchronize()
    assert (res.next_token >= 0).all()
