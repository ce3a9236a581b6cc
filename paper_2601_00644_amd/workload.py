"""Device-side construction of a full-size synthetic verification workload.

Builds weights, paged KV sessions and request shapes with the seeded generators of `synth`, and lets
a synthetic edge model produce the drafts: draft i of a request is drawn from
q_i = softmax(target logits / T + sigma * noise), where the target logits after the previous drafts
come from the library's own forward (one untimed single-row pass per draft position).  Requests
listed in `host_drafts` take their drafts and draft laws from the caller instead (tests and the CPU
baseline pass values the oracle produced, so that nothing the oracle consumes depends on the library).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from . import flexverify as fv
from . import synth


@dataclass
class DeviceWorkload:
    cfg: synth.ModelCfg
    wl: synth.Workload
    ctx: fv.Context
    req: synth.Requests
    batch: fv.DeviceBatch
    k_pool: torch.Tensor
    v_pool: torch.Tensor
    page_table: torch.Tensor
    draft_tokens: torch.Tensor
    draft_probs: torch.Tensor

    @property
    def drafts(self) -> int:
        return int(self.req.draft_offsets[-1])


def build(wl: synth.Workload, seed: int, weights: dict | None = None, host_drafts: dict | None = None,
          host_kv: dict | None = None, device="cuda", log=lambda s: None) -> DeviceWorkload:
    cfg = synth.MODELS[wl.model]
    if weights is None:
        weights = synth.make_weights(cfg, seed, device=device)
    req = synth.make_requests(wl, cfg, seed)
    B, G = req.batch, int(req.draft_offsets[-1])
    gmax = int(req.gammas.max())
    ctx = fv.Context(cfg, weights, max_batch=B, max_gamma=max(gmax, 1), max_pages_per_req=req.page_table.shape[1],
                     max_rows=G + B)
    log(f"context created: B={B} G={G} pages/request={req.page_table.shape[1]}")
    kp, vp = fv.alloc_pools(cfg, req.num_pages, device)
    pt = torch.as_tensor(req.page_table, device=device)
    for b in range(B):
        if host_kv and b in host_kv:
            k, v = host_kv[b]
            k, v = k.to(device), v.to(device)
        else:
            k, v = synth.make_kv_context(cfg, int(req.seq_lens[b]), seed, b, device=device)
        ctx.kv_import(kp, vp, req.num_pages, pt[b], 0, k, v)
        del k, v
    torch.cuda.synchronize()
    log("KV sessions imported")

    d_tok = torch.zeros(max(G, 1), dtype=torch.int32, device=device)
    q = torch.zeros((max(G, 1), cfg.vocab), dtype=torch.float32, device=device)
    host_drafts = host_drafts or {}
    for b, (toks, probs) in host_drafts.items():
        o, g = int(req.draft_offsets[b]), int(req.gammas[b])
        d_tok[o:o + g] = torch.as_tensor(np.asarray(toks, np.int32), device=device)
        q[o:o + g] = probs.to(device)
    # the synthetic edge model drafts autoregressively; step i scores one pending token per still-active request
    cur = torch.as_tensor(req.last_token.copy(), device=device)
    for i in range(gmax):
        act = [b for b in range(B) if int(req.gammas[b]) > i and b not in host_drafts]
        if not act:
            break
        idx = torch.as_tensor(act, device=device)
        n = len(act)
        L_host = (req.seq_lens[act] + i).astype(np.int32)
        off_host = np.zeros(n + 1, np.int32)
        sub = fv.DeviceBatch(torch.as_tensor(L_host, device=device), cur[idx].contiguous(),
                             torch.zeros(n + 1, dtype=torch.int32, device=device), None, None, None,
                             torch.zeros(n, dtype=torch.float32, device=device),
                             torch.zeros(n, dtype=torch.float32, device=device), pt[idx].contiguous(), kp, vp,
                             req.num_pages, L_host, off_host, np.zeros(n, np.float32))
        res = fv.DeviceResult.alloc(n, n, cfg.vocab, want_logits=True, device=device)
        ctx.verify(sub, res)             # greedy, gamma 0: only the logits are used
        torch.cuda.synchronize()
        for j, b in enumerate(act):
            gi = int(req.draft_offsets[b]) + i
            q[gi] = synth.draft_law(res.logits_out[j], float(req.temperature[b]), wl.sigma, seed, gi)
            tok = synth.draw_from(q[gi], float(req.u_draft[gi]))
            d_tok[gi] = tok
            cur[b] = tok
    log("drafts generated")
    batch = fv.device_batch(req, None, q, kp, vp, device)
    batch.draft_tokens = d_tok
    return DeviceWorkload(cfg, wl, ctx, req, batch, kp, vp, pt, d_tok, q)
