"""Many rounds of draft -> verify -> state update on persistent paged sessions (Alg. 2, all three steps).

The cloud side is the library: fsv_verify on the sessions' pages, page bookkeeping through fsv_pager, stride
selection and acceptance-rate average through fsv_policy_* (Alg. 2 steps 1 and 3).  The edge side does not exist
here; a synthetic edge model stands in for it: draft i of a session is drawn from softmax(target logits / T +
sigma * noise), the target logits coming from the library's own single-row passes (as in workload.py), and the
link rate of every session follows a seeded lognormal trace.  Nothing in this module does arithmetic of the
method itself; it only moves the outputs of one call into the inputs of the next.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

from . import flexverify as fv
from . import synth


@dataclass
class Session:
    seq_len: int = 0
    last_token: int = 0
    gamma_hat: float = 0.8           # Alg. 2: the average starts at 0.8
    history: list = field(default_factory=list)   # tokens whose KV is valid, in position order from the session's start
    start_len: int = 0               # cached positions the session was opened with (restored context)
    emitted: int = 0
    open: bool = False


class Server:
    def __init__(self, cfg: synth.ModelCfg, weights: dict, n_sessions: int, num_pages: int, max_gamma: int,
                 max_pages_per_session: int, model: fv.LatencyModel, mu: float = 0.1, tau_model: int = fv.TAU_GEOMETRIC,
                 temperature: float = 1.0, sigma: float = 0.5, seed: int = 0, device: str = "cuda"):
        self.cfg, self.dev, self.seed = cfg, device, seed
        self.S, self.num_pages, self.max_gamma, self.MP = n_sessions, num_pages, max_gamma, max_pages_per_session
        self.model, self.mu, self.tau_model, self.T, self.sigma = model, mu, tau_model, temperature, sigma
        self.ctx = fv.Context(cfg, weights, max_batch=n_sessions, max_gamma=max(max_gamma, 1),
                              max_pages_per_req=max_pages_per_session)
        self.k_pool, self.v_pool = fv.alloc_pools(cfg, num_pages, device)
        self.pager = fv.Pager(num_pages, n_sessions, max_pages_per_session)
        self.page_table = np.zeros((n_sessions, max_pages_per_session), np.int32)
        self.sessions = [Session() for _ in range(n_sessions)]
        self.round_no = 0

    def close(self):
        self.ctx.close()
        self.pager.close()

    # -- session life cycle ------------------------------------------------------------------------------------
    def open_session(self, s: int, k_ctx: torch.Tensor, v_ctx: torch.Tensor, last_token: int):
        """Restore a user's KV context ([n_layers][L][kv heads][head_dim]) into freshly reserved pages."""
        L = int(k_ctx.shape[1])
        self.pager.trim(s, 0)
        self.pager.reserve(s, L + 1, self.page_table[s])
        if L > 0:
            self.ctx.kv_import(self.k_pool, self.v_pool, self.num_pages, torch.as_tensor(self.page_table[s], device=self.dev),
                               0, k_ctx.to(self.dev), v_ctx.to(self.dev))
        self.sessions[s] = Session(seq_len=L, last_token=int(last_token), start_len=L, open=True)

    def end_session(self, s: int):
        self.pager.trim(s, 0)
        self.sessions[s].open = False

    # -- one round ---------------------------------------------------------------------------------------------
    def _device_batch(self, act, L, last, off, d_tok, q, u_acc, u_smp, temp):
        t = lambda a: torch.as_tensor(np.ascontiguousarray(a), device=self.dev)
        return fv.DeviceBatch(t(L), t(last), t(off), d_tok, q, t(u_acc), t(u_smp), t(temp),
                              t(self.page_table[act]), self.k_pool, self.v_pool, self.num_pages,
                              np.ascontiguousarray(L, np.int32), np.ascontiguousarray(off, np.int32),
                              np.ascontiguousarray(temp, np.float32))

    def _draft(self, act, L, last, K):
        """The synthetic edge model: K[j] tokens for active session j, and the laws they were drawn from."""
        n, V = len(act), self.cfg.vocab
        off = np.zeros(n + 1, np.int32)
        off[1:] = np.cumsum(K)
        G = int(off[-1])
        d_tok = torch.zeros(max(G, 1), dtype=torch.int32, device=self.dev)
        q = torch.zeros((max(G, 1), V), dtype=torch.float32, device=self.dev)
        cur = np.array(last, np.int32)
        u_d = synth.uniforms24(max(G, 1), self.seed, 50_000 + self.round_no)
        for i in range(int(K.max()) if n else 0):
            sub = [j for j in range(n) if K[j] > i]
            Ls = np.array([L[j] + i for j in sub], np.int32)
            zero = np.zeros(len(sub), np.float32)
            b = self._device_batch([act[j] for j in sub], Ls, cur[sub], np.zeros(len(sub) + 1, np.int32), None, None,
                                   np.zeros(0, np.float32), zero, zero)
            res = fv.DeviceResult.alloc(len(sub), len(sub), V, want_logits=True, device=self.dev)
            self.ctx.verify(b, res)             # greedy, no drafts: only the logits are used
            torch.cuda.synchronize()
            for r, j in enumerate(sub):
                gi = int(off[j]) + i
                q[gi] = synth.draft_law(res.logits_out[r], self.T, self.sigma, self.seed, 1_000_000 * self.round_no + gi)
                tok = synth.draw_from(q[gi], float(u_d[gi]))
                d_tok[gi] = tok
                cur[j] = tok
        return off, d_tok, q

    def round(self, rates: np.ndarray, k_max: int | None = None, want_logits: bool = False) -> dict:
        """Alg. 2 once for every open session: pick K from the session's link rate and acceptance average, draft,
        verify, move the outcome into the session state.  rates[s] in bit/s."""
        k_max = self.max_gamma if k_max is None else min(k_max, self.max_gamma)
        act = [s for s in range(self.S) if self.sessions[s].open]
        n = len(act)
        K = np.zeros(n, np.int32)
        for j, s in enumerate(act):
            K[j], _ = fv.policy_stride(self.model, float(rates[s]), self.sessions[s].gamma_hat, k_max, self.tau_model)
        L = np.array([self.sessions[s].seq_len for s in act], np.int32)
        last = np.array([self.sessions[s].last_token for s in act], np.int32)
        for j, s in enumerate(act):             # pages for the rows this call appends
            self.pager.reserve(s, int(L[j]) + int(K[j]) + 1, self.page_table[s])
        off, d_tok, q = self._draft(act, L, last, K)
        G = int(off[-1])
        u_acc = synth.uniforms24(max(G, 1), self.seed, 60_000 + self.round_no)[:G]
        u_smp = synth.uniforms24(n, self.seed, 70_000 + self.round_no)
        temp = np.full(n, self.T, np.float32)
        batch = self._device_batch(act, L, last, off, d_tok, q, u_acc, u_smp, temp)
        res = fv.DeviceResult.alloc(n, G + n, self.cfg.vocab, want_logits=want_logits, device=self.dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        self.ctx.verify(batch, res)
        e1.record()
        torch.cuda.synchronize()
        tau, nxt = res.accepted_len.cpu().numpy(), res.next_token.cpu().numpy()
        new_len, released = res.new_seq_lens.cpu().numpy(), res.pages_released.cpu().numpy()
        d_host = d_tok.cpu().numpy()
        for j, s in enumerate(act):
            ss = self.sessions[s]
            ss.history += [int(last[j])] + [int(x) for x in d_host[off[j]: off[j] + int(tau[j])]]
            ss.seq_len, ss.last_token = int(new_len[j]), int(nxt[j])
            ss.emitted += int(tau[j]) + 1
            if K[j] > 0:
                ss.gamma_hat = fv.policy_ema(ss.gamma_hat, int(tau[j]), int(K[j]), self.mu)
            freed = self.pager.trim(s, ss.seq_len)
            assert freed == int(released[j]), (s, freed, int(released[j]))
        self.round_no += 1
        return {"sessions": act, "K": K, "tau": tau, "next": nxt, "cloud_ms": e0.elapsed_time(e1), "result": res,
                "offsets": off, "drafts": d_host}


def lognormal_rates(n: int, median_bps: float, sigma: float, seed: int, stream: int) -> np.ndarray:
    """A link rate per session for one round: median * exp(sigma * N(0,1))."""
    g = torch.Generator()
    g.manual_seed((int(seed) * 1000003 + int(stream)) & 0x7FFFFFFFFFFFFFFF)
    z = torch.randn(n, generator=g, dtype=torch.float64).numpy()
    return median_bps * np.exp(sigma * z)
