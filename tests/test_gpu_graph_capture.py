"""fsv_verify under HIP graph capture: a serving loop may record the call once and replay it.  The call allocates
nothing, reads nothing back and clears its workspace in kernels, so it can be captured; this test records it with
torch's graph object, replays it several times with the program's own eager work and synchronisations in between,
changes the device-side inputs (drafts, uniforms) between replays, and checks every replay bit for bit against an
eager call on the same inputs."""
import numpy as np
import pytest
import torch

from paper_2601_00644_amd import synth
from tests.helpers import build_case
from tests.test_gpu_verify_f32 import run_library

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("top_p", [1.0, 0.9])
def test_verify_replays_match_eager_calls(top_p):
    from paper_2601_00644_amd import flexverify as fv
    cfg = synth.MODELS["mini128"]
    wl = synth.Workload("t", "mini128", 6, 1, 400, "uniform", 1, 8, "uniform", 0.7, 0.8, "permuted")
    case = build_case(cfg, wl, seed=12, weight_std=0.04, run_oracle=False)
    ctx, batch, res_eager, kp, vp, pt = run_library(case)
    B, M = case.req.batch, batch.rows
    if top_p < 1.0:
        batch.top_p_host = np.full(B, top_p, np.float32)
        batch.top_p = torch.as_tensor(batch.top_p_host, device="cuda")
        ctx.verify(batch, res_eager)
    res_graph = fv.DeviceResult.alloc(B, M, cfg.vocab, want_logits=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ctx.verify(batch, res_graph)              # warm-up on the capture stream
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            ctx.verify(batch, res_graph)
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda").manual_seed(5)
    for replay in range(4):
        if replay:   # new uniforms and a changed draft token: inputs the recorded call reads from the same buffers
            batch.u_accept.copy_(torch.randint(0, 1 << 24, batch.u_accept.shape, generator=gen, device="cuda").float() / (1 << 24))
            batch.u_sample.copy_(torch.randint(0, 1 << 24, batch.u_sample.shape, generator=gen, device="cuda").float() / (1 << 24))
            batch.draft_tokens[replay % batch.draft_tokens.numel()] = (7 * replay) % cfg.vocab
        for f in ("accepted_len", "next_token", "new_seq_lens", "pages_released", "flags"):
            getattr(res_graph, f).fill_(-1)
        res_graph.logits_out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ctx.verify(batch, res_eager)              # the same inputs, eagerly
        torch.cuda.synchronize()
        assert torch.equal(res_graph.logits_out, res_eager.logits_out), replay
        for f in ("accepted_len", "next_token", "new_seq_lens", "pages_released", "flags"):
            assert torch.equal(getattr(res_graph, f), getattr(res_eager, f)), (replay, f)
        # eager work of the program between replays: another call that uses the same workspace
        ctx.sample(res_eager.logits_out, batch, fv.DeviceResult.alloc(B))
        torch.cuda.synchronize()
    ctx.close()
