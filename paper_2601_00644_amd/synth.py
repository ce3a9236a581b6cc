"""Seeded synthetic inputs for the verification step (model shapes, sessions, drafts).

This module serves both the GPU library's callers and the CPU oracle's tests and
holds none of the verification arithmetic: it only draws weights, KV contexts,
request shapes, uniforms and draft distributions from seeded generators.  The
paper's evaluation uses trained Llama-family targets and public benchmarks
(Sec. V); neither exists here, so random-initialised models of the same shapes
and random sessions stand in.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np
import torch


@dataclass(frozen=True)
class ModelCfg:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str              # "f32" or "bf16": storage type of weights, activations and KV
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5
    page_size: int = 16

    @property
    def qkv_dim(self) -> int:
        return (self.n_heads + 2 * self.n_kv_heads) * self.head_dim


MODELS = {
    # tiny fp32 decoder, the CPU-finishable correctness configuration
    "tiny": ModelCfg("tiny", 2, 256, 4, 4, 64, 1024, 4096, "f32", 10000.0),
    # 1B-class and 8B-class Llama shapes
    "llama1b": ModelCfg("llama1b", 16, 2048, 32, 8, 64, 8192, 128256, "bf16", 500000.0),
    "llama8b": ModelCfg("llama8b", 32, 4096, 32, 8, 128, 14336, 128256, "bf16", 500000.0),
    # reduced bf16 shapes the oracle finishes in seconds; they keep GQA, both head sizes and a ragged vocab
    "mini128": ModelCfg("mini128", 2, 512, 8, 2, 128, 1536, 5024, "bf16", 500000.0),
    "mini64": ModelCfg("mini64", 3, 256, 8, 2, 64, 768, 3104, "bf16", 500000.0),
    "minif32": ModelCfg("minif32", 2, 128, 4, 2, 32, 320, 1000, "f32", 10000.0),
}


@dataclass(frozen=True)
class Workload:
    name: str
    model: str
    batch: int
    ctx_lo: int
    ctx_hi: int
    ctx_dist: str           # "fixed" | "uniform" | "loguniform"
    gamma_lo: int
    gamma_hi: int
    gamma_dist: str         # "fixed" | "uniform" | "channel"
    sigma: float            # std of the noise added to the target logits to form the draft law
    temperature: float
    pages: str = "interleaved"   # "interleaved" | "permuted"


WORKLOADS = {
    "c1_tiny": Workload("c1_tiny", "tiny", 1, 128, 128, "fixed", 4, 4, "fixed", 0.0, 1.0),
    "c2_1b": Workload("c2_1b", "llama1b", 1, 2048, 2048, "fixed", 4, 4, "fixed", 0.5, 1.0),
    "c3_8b_b16": Workload("c3_8b_b16", "llama8b", 16, 512, 4096, "uniform", 1, 8, "uniform", 0.7, 0.8),
    "c5_8b_b128": Workload("c5_8b_b128", "llama8b", 128, 256, 8192, "loguniform", 1, 12, "channel", 0.7, 1.0),
}


# ----------------------------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------------------------

def _gen(seed: int, stream: int, device="cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(stream)) & 0x7FFFFFFFFFFFFFFF)
    return g


def uniforms24(n: int, seed: int, stream: int) -> np.ndarray:
    """n uniforms k / 2^24, k integer in [0, 2^24): exactly representable in fp32, always < 1."""
    k = torch.randint(0, 1 << 24, (n,), generator=_gen(seed, stream), dtype=torch.int64)
    return (k.double() / float(1 << 24)).float().numpy()


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Round an fp32 tensor to bf16 (nearest even) and return the bit patterns as uint16."""
    return t.to(torch.bfloat16).view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_f32(a: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns exactly to fp32."""
    return (a.astype(np.uint32) << 16).view(np.float32)


def weight_names(cfg: ModelCfg):
    """(name, shape, kind) of every parameter; matrices are [out_features, in_features]."""
    d, qd = cfg.d_model, cfg.n_heads * cfg.head_dim
    out = [("embed", (cfg.vocab, d), "mat"), ("final_norm", (d,), "gain"), ("lm_head", (cfg.vocab, d), "mat")]
    for l in range(cfg.n_layers):
        out += [(f"attn_norm.{l}", (d,), "gain"), (f"w_qkv.{l}", (cfg.qkv_dim, d), "mat"),
                (f"w_o.{l}", (d, qd), "mat"), (f"mlp_norm.{l}", (d,), "gain"),
                (f"w_gate_up.{l}", (2 * cfg.d_ffn, d), "mat"), (f"w_down.{l}", (d, cfg.d_ffn), "mat")]
    return out


def make_weights(cfg: ModelCfg, seed: int, device="cpu", std: float = 0.02) -> dict:
    """Random-initialised parameters: matrices ~ N(0, std), norm gains 1 + N(0, std).

    Returns torch tensors on `device` in the model's storage dtype.  The stream of a tensor is
    fixed by its position in weight_names(), so a given (seed, device type) always gives the
    same bits.
    """
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    w = {}
    for i, (name, shape, kind) in enumerate(weight_names(cfg)):
        x = torch.randn(shape, generator=_gen(seed, 100 + i, device), device=device, dtype=torch.float32) * std
        if kind == "gain":
            x = x + 1.0
        w[name] = x.to(tdt)
    return w


def make_lora(cfg: ModelCfg, rank: int, seed: int, adapter: int, device="cpu", std_a: float = 0.05, std_b: float = 0.05) -> dict:
    """A seeded LoRA adapter for every layer but the last (the paper's evolving target keeps its last block and LM head
    frozen): random A ~ N(0, std_a) and B ~ N(0, std_b) on the fused q|k|v projection and the output projection, in the
    model's storage dtype.  Trained adapters start from B = 0; random B stands in for a fine-tuned one."""
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    qd = cfg.n_heads * cfg.head_dim
    shapes = {"a_qkv": (rank, cfg.d_model), "b_qkv": (cfg.qkv_dim, rank), "a_o": (rank, qd), "b_o": (cfg.d_model, rank)}
    out = {"rank": rank, "scale": 2.0}
    for j, (name, shape) in enumerate(shapes.items()):
        std = std_a if name.startswith("a_") else std_b
        out[name] = [(torch.randn(shape, generator=_gen(seed, 50_000 + 1000 * adapter + 10 * l + j, device), device=device,
                                  dtype=torch.float32) * std).to(tdt) for l in range(cfg.n_layers - 1)]
    return out


def lora_to_numpy(cfg: ModelCfg, lora: dict) -> dict:
    """Host copy of an adapter in the layout the oracle takes."""
    conv = (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)) if cfg.dtype == "bf16" else (lambda t: t.cpu().numpy())
    return {k: ([conv(t) for t in v] if isinstance(v, list) else v) for k, v in lora.items()}


def make_draft_head(cfg: ModelCfg, d_hidden: int, d_proj: int, seed: int, device="cpu", std: float = 0.05) -> dict:
    """A seeded head of the edge draft model (two-layer MLP + vocabulary projection); a trained one is distilled from
    the base target (Alg. 1), random matrices stand in for it."""
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    shapes = {"w1": (d_hidden, cfg.d_model), "w2": (d_proj, d_hidden), "wv": (cfg.vocab, d_proj)}
    return {k: (torch.randn(sh, generator=_gen(seed, 60_000 + j, device), device=device, dtype=torch.float32) * std).to(tdt)
            for j, (k, sh) in enumerate(shapes.items())}


def weights_to_numpy(cfg: ModelCfg, w: dict) -> dict:
    """Host copies in the layout the oracle takes: float32, or uint16 bf16 bit patterns."""
    if cfg.dtype == "bf16":
        return {k: v.view(torch.int16).cpu().numpy().view(np.uint16) for k, v in w.items()}
    return {k: v.cpu().numpy() for k, v in w.items()}


def make_kv_context(cfg: ModelCfg, L: int, seed: int, req: int, device="cpu"):
    """A session's restored KV context as N(0,1) values: two tensors [n_layers, L, n_kv_heads, head_dim]."""
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    shape = (cfg.n_layers, L, cfg.n_kv_heads, cfg.head_dim)
    k = torch.randn(shape, generator=_gen(seed, 10_000 + 2 * req, device), device=device, dtype=torch.float32)
    v = torch.randn(shape, generator=_gen(seed, 10_001 + 2 * req, device), device=device, dtype=torch.float32)
    return k.to(tdt), v.to(tdt)


def kv_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


@dataclass
class Requests:
    seq_lens: np.ndarray       # [B] int32, cached positions before the call
    gammas: np.ndarray         # [B] int32, drafts per request
    draft_offsets: np.ndarray  # [B+1] int32, CSR over drafts
    last_token: np.ndarray     # [B] int32, pending token at position seq_lens[b]
    temperature: np.ndarray    # [B] float32
    u_accept: np.ndarray       # [G] float32
    u_sample: np.ndarray       # [B] float32
    u_draft: np.ndarray        # [G] float32, uniforms the synthetic edge device draws its drafts with
    page_table: np.ndarray     # [B, max_pages] int32
    num_pages: int

    @property
    def batch(self) -> int:
        return int(self.seq_lens.shape[0])


def channel_gammas(n: int, seed: int, lo: int = 1, hi: int = 12, sigma: float = 0.5) -> np.ndarray:
    """Draft lengths an edge policy would pick under a lognormal link rate: clip(round(rate/E[rate]*6), lo, hi)."""
    z = torch.randn(n, generator=_gen(seed, 3), dtype=torch.float64).numpy()
    rate = np.exp(sigma * z)
    mean = math.exp(sigma * sigma / 2.0)
    return np.clip(np.rint(rate / mean * 6.0), lo, hi).astype(np.int32)


def make_page_table(seq_lens, gammas, page_size: int, kind: str, seed: int):
    """Physical page ids for every request's logical pages.

    "interleaved": logical page j of request b is physical page j*B + b (round-robin over requests);
    "permuted": a seeded random permutation of the same set of pages;
    "contiguous": request b owns physical pages b*max_pages .. (b+1)*max_pages - 1 in order.
    """
    B = len(seq_lens)
    need = [(int(seq_lens[b]) + int(gammas[b]) + 1 + page_size - 1) // page_size for b in range(B)]
    max_pages = max(need)
    num_pages = max_pages * B
    pt = np.empty((B, max_pages), np.int32)
    for j in range(max_pages):
        pt[:, j] = j * B + np.arange(B)
    if kind == "permuted":
        perm = torch.randperm(num_pages, generator=_gen(seed, 4)).numpy().astype(np.int32)
        pt = perm[pt]
    elif kind == "contiguous":
        pt = (np.arange(B, dtype=np.int32)[:, None] * max_pages + np.arange(max_pages, dtype=np.int32)[None, :]).astype(np.int32)
    elif kind != "interleaved":
        raise ValueError(kind)
    return pt, num_pages


def make_requests(wl: Workload, cfg: ModelCfg, seed: int, batch: int | None = None, ctx_hi: int | None = None) -> Requests:
    B = batch if batch is not None else wl.batch
    hi = ctx_hi if ctx_hi is not None else wl.ctx_hi
    lo = min(wl.ctx_lo, hi)
    if wl.ctx_dist == "fixed":
        L = np.full(B, hi, np.int32)
    elif wl.ctx_dist == "uniform":
        L = torch.randint(lo, hi + 1, (B,), generator=_gen(seed, 1)).numpy().astype(np.int32)
    elif wl.ctx_dist == "loguniform":
        u = torch.rand(B, generator=_gen(seed, 1), dtype=torch.float64).numpy()
        L = np.floor(np.exp(math.log(lo) + u * (math.log(hi + 1) - math.log(lo)))).astype(np.int32)
        L = np.clip(L, lo, hi)
    else:
        raise ValueError(wl.ctx_dist)
    if wl.gamma_dist == "fixed":
        g = np.full(B, wl.gamma_hi, np.int32)
    elif wl.gamma_dist == "uniform":
        g = torch.randint(wl.gamma_lo, wl.gamma_hi + 1, (B,), generator=_gen(seed, 2)).numpy().astype(np.int32)
    elif wl.gamma_dist == "channel":
        g = channel_gammas(B, seed, wl.gamma_lo, wl.gamma_hi)
    else:
        raise ValueError(wl.gamma_dist)
    off = np.zeros(B + 1, np.int32)
    off[1:] = np.cumsum(g)
    G = int(off[-1])
    last = torch.randint(0, cfg.vocab, (B,), generator=_gen(seed, 5)).numpy().astype(np.int32)
    pt, npages = make_page_table(L, g, cfg.page_size, wl.pages, seed)
    return Requests(L, g, off, last, np.full(B, wl.temperature, np.float32),
                    uniforms24(G, seed, 6), uniforms24(B, seed, 7), uniforms24(G, seed, 8), pt, npages)


def draft_law(logits_row: torch.Tensor, temperature: float, sigma: float, seed: int, stream: int) -> torch.Tensor:
    """The synthetic edge model's law for one position: softmax(target_logits / T + sigma * N(0,1)), fp32.

    logits_row may live on any device; the noise comes from a generator on that device.
    """
    dev = logits_row.device
    z = logits_row.double() / (temperature if temperature > 0 else 1.0)
    if sigma > 0:
        z = z + sigma * torch.randn(z.shape, generator=_gen(seed, 20_000 + stream, dev), device=dev, dtype=torch.float64)
    return torch.softmax(z, dim=-1).float()


def draw_from(q_row: torch.Tensor, u: float) -> int:
    """Inverse-CDF draw of one token id from a probability row with a given uniform."""
    cdf = torch.cumsum(q_row.double(), dim=-1)
    idx = int(torch.searchsorted(cdf, torch.tensor([u * float(cdf[-1])], dtype=torch.float64, device=cdf.device),
                                 right=True)[0])
    return min(idx, q_row.shape[-1] - 1)


def random_law(vocab: int, std: float, seed: int, stream: int) -> torch.Tensor:
    """A draft law unrelated to the target: softmax of N(0, std) logits (the tiny configuration's recipe)."""
    z = torch.randn(vocab, generator=_gen(seed, 30_000 + stream), dtype=torch.float64) * std
    return torch.softmax(z, dim=-1).float()


@dataclass
class SamplerCase:
    """The rejection-sampling step in isolation: logits are inputs."""
    logits: torch.Tensor       # [M, V] bf16 or fp32, M = sum(gamma_b + 1)
    draft_probs: torch.Tensor  # [G, V] fp32
    draft_tokens: np.ndarray   # [G] int32
    draft_offsets: np.ndarray  # [B+1] int32
    u_accept: np.ndarray
    u_sample: np.ndarray
    temperature: np.ndarray


def make_sampler_case(batch: int, gamma_lo: int, gamma_hi: int, vocab: int, sigma: float, temperature: float,
                      seed: int, logit_std: float = 3.0, logits_dtype: str = "bf16", device="cpu") -> SamplerCase:
    """Target logits ~ N(0, logit_std); draft law softmax(l/T + sigma*xi); drafts drawn from their own law."""
    g = torch.randint(gamma_lo, gamma_hi + 1, (batch,), generator=_gen(seed, 2)).numpy().astype(np.int32)
    off = np.zeros(batch + 1, np.int32)
    off[1:] = np.cumsum(g)
    G, M = int(off[-1]), int(off[-1]) + batch
    tdt = torch.bfloat16 if logits_dtype == "bf16" else torch.float32
    logits = (torch.randn((M, vocab), generator=_gen(seed, 40, device), device=device, dtype=torch.float32)
              * logit_std).to(tdt)
    u_d = uniforms24(G, seed, 8)
    q = torch.empty((G, vocab), dtype=torch.float32, device=device)
    d = np.empty(G, np.int32)
    for b in range(batch):
        for i in range(int(g[b])):
            row = int(off[b]) + b + i           # logits row that scores draft i+1 of request b
            gi = int(off[b]) + i
            q[gi] = draft_law(logits[row].float(), temperature, sigma, seed, gi)
            d[gi] = draw_from(q[gi], float(u_d[gi]))
    return SamplerCase(logits, q, d, off, uniforms24(G, seed, 6), uniforms24(batch, seed, 7),
                       np.full(batch, temperature, np.float32))


def with_dtype(cfg: ModelCfg, dtype: str) -> ModelCfg:
    return replace(cfg, dtype=dtype, name=f"{cfg.name}_{dtype}")
