"""Shared test plumbing: build a seeded verification case, run the oracle on it, compare results."""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

from oracle import oracle
from paper_2601_00644_amd import synth

ACCEPT_FLAG = 1e-4     # draws this close to an acceptance threshold may legitimately differ (counted, not failed)
CDF_FLAG = 1e-6        # same for the emitted token's inverse-CDF edges (normalised mass)


@dataclass
class Case:
    cfg: synth.ModelCfg
    weights: dict                 # torch tensors (host), model dtype
    weights_np: dict              # what the oracle takes
    req: synth.Requests
    ctx_k: list                   # per request [n_layers, L_b, Hkv, hd] torch (host, model dtype)
    ctx_v: list
    draft_tokens: np.ndarray      # [G]
    draft_probs: torch.Tensor     # [G, V] fp32 host
    expected: list = field(default_factory=list)   # oracle.VerifyResult per request
    caches: list = field(default_factory=list)     # oracle caches after the call


def oracle_cache_from_context(cfg, k, v, cap):
    kc, vc = oracle.new_cache(cfg, cap)
    L = k.shape[1]
    kc[:, :L] = synth.kv_to_f64(k)
    vc[:, :L] = synth.kv_to_f64(v)
    return kc, vc


def build_case(cfg, wl: synth.Workload, seed: int, batch=None, ctx_hi=None, weight_std=0.02, prefill_context=False,
               independent_draft_law=False, temperature=None, run_oracle=True) -> Case:
    """Everything comes from seeded generators and the oracle; nothing from the GPU library.

    Drafts are what a synthetic edge model would send: token i is drawn from q_i = softmax(target logits / T
    + sigma * noise), which needs the target logits after the previous drafts, so the oracle is stepped
    autoregressively (or, with independent_draft_law, q_i is a random law unrelated to the target and the
    drafts are uniform over the vocabulary).
    """
    w = synth.make_weights(cfg, seed, std=weight_std)
    wn = synth.weights_to_numpy(cfg, w)
    req = synth.make_requests(wl, cfg, seed, batch=batch, ctx_hi=ctx_hi)
    if temperature is not None:
        req.temperature[:] = np.asarray(temperature, np.float32)
    B = req.batch
    G = int(req.draft_offsets[-1])
    ctx_k, ctx_v = [], []
    d_all = np.zeros(G, np.int32)
    q_all = torch.zeros((G, cfg.vocab), dtype=torch.float32)
    rng_tok = np.random.default_rng(seed + 77)
    for b in range(B):
        L, g, o = int(req.seq_lens[b]), int(req.gammas[b]), int(req.draft_offsets[b])
        cap = L + g + 1
        if prefill_context:
            kc, vc = oracle.new_cache(cfg, cap)
            if L > 0:
                oracle.forward(cfg, wn, kc, vc, 0, rng_tok.integers(0, cfg.vocab, L).astype(np.int32))
            tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
            k = torch.from_numpy(kc[:, :L]).to(tdt)
            v = torch.from_numpy(vc[:, :L]).to(tdt)
        else:
            k, v = synth.make_kv_context(cfg, L, seed, b)
        ctx_k.append(k.contiguous())
        ctx_v.append(v.contiguous())
        if independent_draft_law:
            for i in range(g):
                q_all[o + i] = synth.random_law(cfg.vocab, 2.0, seed, o + i)
                d_all[o + i] = int(req.u_draft[o + i] * cfg.vocab)
        else:
            kc, vc = oracle_cache_from_context(cfg, k, v, cap)
            tok = int(req.last_token[b])
            T = float(req.temperature[b])
            for i in range(g):
                lg = oracle.forward(cfg, wn, kc, vc, L + i, np.array([tok], np.int32))[0]
                q_all[o + i] = synth.draft_law(torch.from_numpy(lg), T, wl.sigma, seed, o + i)
                tok = synth.draw_from(q_all[o + i], float(req.u_draft[o + i]))
                d_all[o + i] = tok
    case = Case(cfg, w, wn, req, ctx_k, ctx_v, d_all, q_all)
    if run_oracle:
        run_oracle_on(case)
    return case


def run_oracle_on(case: Case, only=None):
    cfg, req = case.cfg, case.req
    case.expected, case.caches = [], []
    for b in range(req.batch):
        if only is not None and b not in only:
            case.expected.append(None)
            case.caches.append(None)
            continue
        L, g, o = int(req.seq_lens[b]), int(req.gammas[b]), int(req.draft_offsets[b])
        kc, vc = oracle_cache_from_context(cfg, case.ctx_k[b], case.ctx_v[b], L + g + 1)
        r = oracle.verify(cfg, case.weights_np, kc, vc, L, int(req.last_token[b]), case.draft_tokens[o:o + g],
                          case.draft_probs[o:o + g].numpy(), req.u_accept[o:o + g], float(req.u_sample[b]),
                          float(req.temperature[b]))
        case.expected.append(r)
        case.caches.append((kc, vc))


def logits_close(got: np.ndarray, ref: np.ndarray, tol: float):
    """|got - ref| <= tol * max(|ref|, rms(ref row)) element-wise; returns (ok, worst ratio)."""
    rms = np.sqrt((ref * ref).mean(axis=-1, keepdims=True))
    scale = np.maximum(np.abs(ref), rms)
    ratio = np.abs(got - ref) / scale
    return bool((ratio <= tol).all()), float(ratio.max())


def logits_close_bf16(got: np.ndarray, ref: np.ndarray, tol: float = 2e-2):
    """The bf16 bar: every element within tol of the row's scale max|ref|, and every row within tol in L2.

    Storing activations in bf16 between kernels (what the bf16 configuration means) by itself leaves an
    rms logit error of 0.6 % (2 layers) to 1.3 % (24 layers) against an fp64 forward, whatever the
    kernels do, so single elements cannot be held to tol of their own magnitude; the row scale can.
    Returns (ok, worst element ratio, worst row L2 ratio).
    """
    scale = np.abs(ref).max(axis=-1, keepdims=True)
    elem = float((np.abs(got - ref) / scale).max())
    l2 = float((np.linalg.norm(got - ref, axis=-1) / np.linalg.norm(ref, axis=-1)).max())
    return (elem <= tol and l2 <= tol), elem, l2


def bf16_logit_tol(n_layers: int) -> float:
    """The bf16 logit bar as a function of depth: 2e-2 up to 4 layers, then 9.6e-3 * sqrt(n_layers).

    An exact (fp64) forward that merely STORES bf16 where the bf16 configuration does (GEMM inputs, q/k/v,
    probabilities, attention output, SwiGLU output) differs from the fp64 forward by a worst-row L2 error of
    0.64 % after 1 layer, 1.6 % after 8, 2.3 % after 16 and 3.3 % after 32 at the 8B shapes (measured with
    plain torch fp64, independent of the library): about 6.4e-3 * sqrt(n_layers).  No kernel can do better
    than that against the fp64 oracle, so beyond a few layers the bar is 1.5 times this inherent figure.
    """
    return max(2e-2, 9.6e-3 * float(np.sqrt(n_layers)))


def compare_decisions(exp_list, tau, nxt, accept_flag=ACCEPT_FLAG, cdf_flag=CDF_FLAG):
    """Exact match of (tau, next token) except draws the oracle itself places within the flag margins.

    Returns (mismatches that are not excused, number of excused mismatches, number of flagged requests).
    """
    bad, excused, flagged = [], 0, 0
    for b, e in enumerate(exp_list):
        if e is None:
            continue
        s = e.sample
        near_acc = s.accept_margin < accept_flag
        near_cdf = s.cdf_margin < cdf_flag
        flagged += int(near_acc or near_cdf)
        if int(tau[b]) != s.tau:
            if near_acc:
                excused += 1
            else:
                bad.append((b, "tau", int(tau[b]), s.tau, s.accept_margin))
            continue
        if int(nxt[b]) != s.next_token:
            if near_cdf or near_acc:
                excused += 1
            else:
                bad.append((b, "next", int(nxt[b]), s.next_token, s.cdf_margin))
    return bad, excused, flagged
