"""A second, independent statement of "the forward with bf16 storage points", in plain torch fp64.

Used only to pin the oracle's storage mode (tests/test_oracle_forward.py): the same Llama-style block forward over a
restored KV context (Alg. 2 step 2; Sec. IV-C), written with torch tensor operations instead of the oracle's loops,
with the same named tensors rounded to bf16 by torch's own conversion.  It shares no code with the oracle or the
library.
"""
from __future__ import annotations

import numpy as np
import torch
import torch.nn.functional as F

POINTS = ("a", "q", "kv", "p", "o", "act")
POINTS_F16 = ("a16", "o16")     # the tensors of "a" and "o" rounded to fp16 instead (numpy's conversion: it rounds a
                                # double once, where torch's goes through fp32 and can round twice)


def _rb(t: torch.Tensor, on: bool, f16: bool = False) -> torch.Tensor:
    if on:
        return t.to(torch.bfloat16).double()
    if f16:
        return torch.from_numpy(t.clamp(-65504.0, 65504.0).numpy().astype(np.float16).astype(np.float64))
    return t


def forward_stored(cfg, w: dict, k_ctx: torch.Tensor, v_ctx: torch.Tensor, toks: torch.Tensor, points=()):
    """Logits [n][vocab] (fp64) of tokens `toks` placed after a context of L positions.

    w: torch tensors as synth.make_weights returns them; k_ctx / v_ctx: [layers][L][Hkv][hd]; points: which of POINTS
    are rounded to bf16, which of POINTS_F16 to fp16 (bf16 wins where both are named)."""
    pts = set(points)
    assert pts <= set(POINTS) | set(POINTS_F16)
    H, Hkv, hd, n, L = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, int(toks.shape[0]), int(k_ctx.shape[1])
    x = w["embed"][toks.long()].double()
    pos = torch.arange(L, L + n, dtype=torch.float64)
    inv = float(cfg.rope_theta) ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(n, hd // 2, dtype=torch.float64), pos[:, None] * inv[None])

    def rope(t):   # half-split pairing (i, i + hd/2) as one complex rotation
        c = torch.complex(t[..., : hd // 2], t[..., hd // 2:]) * rot[:, None]
        return torch.cat([c.real, c.imag], -1)

    def norm(t, g):
        return t / torch.sqrt((t * t).mean(-1, keepdim=True) + cfg.rms_eps) * g.double()

    mask = torch.arange(L + n)[None, :] <= (L + torch.arange(n))[:, None]
    for l in range(cfg.n_layers):
        a = _rb(norm(x, w[f"attn_norm.{l}"]), "a" in pts, "a16" in pts)
        q, k, v = (a @ w[f"w_qkv.{l}"].double().T).split([H * hd, Hkv * hd, Hkv * hd], -1)
        q = _rb(rope(q.reshape(n, H, hd)), "q" in pts)
        k = _rb(rope(k.reshape(n, Hkv, hd)), "kv" in pts)
        v = _rb(v.reshape(n, Hkv, hd), "kv" in pts)
        K = torch.cat([k_ctx[l].double(), k], 0).repeat_interleave(H // Hkv, 1)
        V = torch.cat([v_ctx[l].double(), v], 0).repeat_interleave(H // Hkv, 1)
        s = torch.einsum("nhd,mhd->hnm", q, K) / hd ** 0.5
        s = s.masked_fill(~mask[None], float("-inf"))
        p = torch.exp(s - s.max(-1, keepdim=True).values)
        den = p.sum(-1, keepdim=True)
        o = torch.einsum("hnm,mhd->nhd", _rb(p, "p" in pts) / den, V)
        o = _rb(o.reshape(n, H * hd), "o" in pts, "o16" in pts)
        x = x + o @ w[f"w_o.{l}"].double().T
        m = _rb(norm(x, w[f"mlp_norm.{l}"]), "a" in pts, "a16" in pts)
        g, u = (m @ w[f"w_gate_up.{l}"].double().T).split([cfg.d_ffn, cfg.d_ffn], -1)
        act = _rb(F.silu(g) * u, "act" in pts)
        x = x + act @ w[f"w_down.{l}"].double().T
    return _rb(norm(x, w["final_norm"]), "a" in pts, "a16" in pts) @ w["lm_head"].double().T
