"""GPU parity of the two bandwidth-bound bf16 kernels against the oracle's own steps.

fsv_linear (the weight-streaming MFMA GEMM) vs the oracle's dense projection, and fsv_attention
(multi-query paged attention) vs the oracle's block attention, on seeded bf16 inputs both sides
read bit-identically.  Sizes span several row tiles, K splits, key ranges and ragged tails.
Tolerances: the GEMM accumulates exact bf16 products in fp32 (1e-3 of max(|ref|, row rms));
attention rounds probabilities and its output to bf16 (2e-2, the bf16 bar).
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2601_00644_amd import synth
from tests.helpers import logits_close

pytestmark = pytest.mark.gpu


def _ctx(cfg, seed, max_batch=8, max_gamma=16, max_pages=96, std=0.05, max_rows=0):
    from paper_2601_00644_amd import flexverify as fv
    w = synth.make_weights(cfg, seed, std=std)
    ctx = fv.Context(cfg, {k: v.cuda() for k, v in w.items()}, max_batch, max_gamma, max_pages, max_rows=max_rows)
    return fv, ctx, w, synth.weights_to_numpy(cfg, w)


@pytest.mark.parametrize("name", ["mini128", "mini64"])
@pytest.mark.parametrize("M", [1, 5, 33, 88, 136, 224, 225, 257, 512, 883])   # up to the row counts of the batch-128 workload (several row blocks per weight strip)
def test_linear_matches_oracle(name, M):
    cfg = synth.MODELS[name]
    fv, ctx, w, wn = _ctx(cfg, 3, max_batch=8, max_gamma=16, max_rows=max(M, 136))
    g = torch.Generator().manual_seed(M)
    which = [(fv.W_QKV, "w_qkv.1", cfg.d_model), (fv.W_O, "w_o.0", cfg.n_heads * cfg.head_dim),
             (fv.W_GATE_UP, "w_gate_up.1", cfg.d_model), (fv.W_DOWN, "w_down.0", cfg.d_ffn),
             (fv.W_LM_HEAD, "lm_head", cfg.d_model)]
    for wh, key, K in which:
        layer = int(key.split(".")[1]) if "." in key else 0
        x = torch.randn((M, K), generator=g).to(torch.bfloat16)
        n_out = wn[key].shape[0]
        y = ctx.linear(wh, layer, x.cuda(), n_out).cpu().numpy().astype(np.float64)
        ref = oracle.linear(wn[key], x.float().numpy().astype(np.float64), True)
        ok, ratio = logits_close(y, ref, 1e-3)
        assert ok, (key, M, ratio)
    ctx.close()


@pytest.mark.parametrize("ncw", [2, 3, 4])
@pytest.mark.parametrize("M", [7, 97, 128, 300])
def test_linear_with_every_block_shape(ncw, M, monkeypatch):
    """The projections choose two, three or four weight strips per block by what fills the machine; here each shape is
    forced (FSV_GEMM_NCW) on matrices whose strip count is and is not a multiple of it (the last block then has waves
    without a strip), one row block and several."""
    monkeypatch.setenv("FSV_GEMM_NCW", str(ncw))
    cfg = synth.MODELS["mini128"]
    fv, ctx, w, wn = _ctx(cfg, 11, max_batch=8, max_gamma=16, max_rows=max(M, 136))
    g = torch.Generator().manual_seed(100 * ncw + M)
    for wh, key, K in [(fv.W_QKV, "w_qkv.0", cfg.d_model), (fv.W_O, "w_o.1", cfg.n_heads * cfg.head_dim),
                       (fv.W_GATE_UP, "w_gate_up.0", cfg.d_model), (fv.W_DOWN, "w_down.1", cfg.d_ffn),
                       (fv.W_LM_HEAD, "lm_head", cfg.d_model)]:
        layer = int(key.split(".")[1]) if "." in key else 0
        x = torch.randn((M, K), generator=g).to(torch.bfloat16)
        y = ctx.linear(wh, layer, x.cuda(), wn[key].shape[0]).cpu().numpy().astype(np.float64)
        ref = oracle.linear(wn[key], x.float().numpy().astype(np.float64), True)
        ok, ratio = logits_close(y, ref, 1e-3)
        assert ok, (key, ncw, M, ratio)
    ctx.close()


@pytest.mark.parametrize("scale", [1e-7, 1.0, 2.0e4])
def test_linear_over_the_range_of_weight_magnitudes(scale):
    """The projections that keep their operands in fp16 convert their bf16 weights once, times a power of two per matrix:
    matrices whose largest weight is far below or far above the fp16 range, with entries spread over twelve decades inside
    one matrix, and an all-zero matrix, against the oracle's definition on the bf16 weights."""
    from paper_2601_00644_amd import flexverify as fv
    cfg = synth.MODELS["mini64"]
    w = synth.make_weights(cfg, 5, std=0.05)
    g = torch.Generator().manual_seed(17)
    keys = [(fv.W_QKV, "w_qkv.0", cfg.d_model), (fv.W_O, "w_o.1", cfg.n_heads * cfg.head_dim),
            (fv.W_GATE_UP, "w_gate_up.0", cfg.d_model), (fv.W_LM_HEAD, "lm_head", cfg.d_model)]
    for _, key, _ in keys:
        decades = torch.rand(w[key].shape, generator=g) * 12.0                 # each entry 10^-u of its size, u in [0, 12)
        w[key] = (w[key].float() * scale * 20.0 * torch.pow(10.0, -decades)).to(torch.bfloat16)
    w["w_o.0"] = torch.zeros_like(w["w_o.0"])
    wn = synth.weights_to_numpy(cfg, w)
    ctx = fv.Context(cfg, {k: v.cuda() for k, v in w.items()}, 4, 8, 8, max_rows=40)
    for wh, key, K in keys + [(fv.W_O, "w_o.0", cfg.n_heads * cfg.head_dim)]:
        layer = int(key.split(".")[1]) if "." in key else 0
        x = torch.randn((37, K), generator=g).to(torch.bfloat16)
        y = ctx.linear(wh, layer, x.cuda(), wn[key].shape[0]).cpu().numpy().astype(np.float64)
        ref = oracle.linear(wn[key], x.float().numpy().astype(np.float64), True)
        if key == "w_o.0":
            assert not y.any() and not ref.any()
            continue
        assert np.isfinite(y).all() and np.abs(ref).max() > 0
        ok, ratio = logits_close(y, ref, 1e-3)
        assert ok, (key, scale, ratio)
    ctx.close()


def test_fp16_operand_conversion_saturates_and_keeps_nan():
    """An operand beyond the fp16 range is held at +-65504 (never turned into an infinity), a NaN stays a NaN, and values
    on the fp16 subnormal grid survive: the q|k|v projection of hand-placed rows against the oracle's definition applied to
    the oracle's own fp16 rounding of the same rows."""
    cfg = synth.MODELS["mini64"]
    fv, ctx, w, wn = _ctx(cfg, 9, max_batch=4, max_gamma=8, max_rows=40)
    K = cfg.d_model
    g = torch.Generator().manual_seed(23)
    x = torch.randn((6, K), generator=g)
    x[1, ::7] = 1.0e6
    x[1, 3::7] = -3.0e5
    x[2] *= 2.0e-6                       # most of the row below the smallest normal fp16 number
    x[3, 5] = float("nan")
    x[4] *= 3.0e4                        # some entries beyond the range, some inside
    xb = x.to(torch.bfloat16)
    y = ctx.linear(fv.W_QKV, 0, xb.cuda(), wn["w_qkv.0"].shape[0]).cpu().numpy().astype(np.float64)
    x16 = np.vectorize(oracle.round_f16)(xb.float().numpy().astype(np.float64))
    assert np.abs(x16[np.isfinite(x16)]).max() == 65504.0
    ref = oracle.linear(wn["w_qkv.0"], np.nan_to_num(x16, nan=0.0), True)
    rows = [0, 1, 2, 4, 5]
    assert np.isfinite(y[rows]).all()
    ok, ratio = logits_close(y[rows], ref[rows], 1e-3)
    assert ok, ratio
    assert np.isnan(y[3]).all()          # every feature of the row sums over the NaN
    ctx.close()


def _attention_case(cfg, seed, seq_lens, gammas, pages):
    B = len(seq_lens)
    seq_lens, gammas = np.asarray(seq_lens, np.int32), np.asarray(gammas, np.int32)
    off = np.zeros(B + 1, np.int32)
    off[1:] = np.cumsum(gammas)
    pt, npages = synth.make_page_table(seq_lens, gammas, cfg.page_size, pages, seed)
    M = int(off[-1]) + B
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((M, cfg.n_heads, cfg.head_dim), generator=g).to(torch.bfloat16)
    ks, vs = [], []
    for b in range(B):
        n = int(seq_lens[b] + gammas[b] + 1)     # context plus the block's own keys, all given
        k1 = torch.randn((1, n, cfg.n_kv_heads, cfg.head_dim), generator=g).to(torch.bfloat16)
        v1 = torch.randn((1, n, cfg.n_kv_heads, cfg.head_dim), generator=g).to(torch.bfloat16)
        ks.append(k1)
        vs.append(v1)
    return seq_lens, gammas, off, pt, npages, q, ks, vs


@pytest.mark.parametrize("name,seq_lens,gammas,pages", [
    ("mini128", [0, 5, 31, 200], [0, 3, 7, 1], "interleaved"),          # empty context, one key range
    ("mini128", [511, 512, 1290, 40, 700], [4, 8, 16, 15, 2], "permuted"),   # several key ranges, 3 row tiles
    ("mini64", [17, 1023, 530], [16, 6, 0], "permuted"),
])
def test_attention_matches_oracle(name, seq_lens, gammas, pages):
    cfg = synth.MODELS[name]
    L, gm, off, pt, npages, q, ks, vs = _attention_case(cfg, 5, seq_lens, gammas, pages)
    fv, ctx, w, wn = _ctx(cfg, 4, max_batch=8, max_gamma=16, max_pages=pt.shape[1])   # page-table row stride
    B = len(L)
    kp, vp = fv.alloc_pools(cfg, npages)
    ptd = torch.as_tensor(pt).cuda()
    layer = 1
    for b in range(B):
        n = ks[b].shape[1]
        kfull = torch.zeros((cfg.n_layers, n, cfg.n_kv_heads, cfg.head_dim), dtype=torch.bfloat16)
        vfull = torch.zeros_like(kfull)
        kfull[layer], vfull[layer] = ks[b][0], vs[b][0]
        ctx.kv_import(kp, vp, npages, ptd[b], 0, kfull.cuda(), vfull.cuda())
    batch = fv.DeviceBatch(torch.as_tensor(L).cuda(), None, torch.as_tensor(off).cuda(), None, None, None, None, None,
                           ptd, kp, vp, npages, L, off)
    out = ctx.attention(layer, q.cuda(), batch).cpu().numpy().astype(np.float64)
    worst = 0.0
    for b in range(B):
        rs, n = int(off[b]) + b, int(gm[b]) + 1
        ref = oracle.attention(q[rs:rs + n].float().numpy(), ks[b][0].float().numpy(), vs[b][0].float().numpy(), int(L[b]))
        ok, ratio = logits_close(out[rs:rs + n], ref, 2e-2)
        worst = max(worst, ratio)
        assert ok, (b, ratio)
    print(f"attention {name}: worst ratio {worst:.3e}")
    ctx.close()


def test_kv_import_export_roundtrip():
    cfg = synth.MODELS["mini128"]
    fv, ctx, w, wn = _ctx(cfg, 6, max_pages=8)
    k, v = synth.make_kv_context(cfg, 77, 1, 0)
    pt = torch.tensor([5, 0, 3, 7, 1, 2, 4, 6], dtype=torch.int32).cuda()
    kp, vp = fv.alloc_pools(cfg, 8)
    ctx.kv_import(kp, vp, 8, pt, 10, k.cuda(), v.cuda())
    gk, gv = ctx.kv_export(kp, vp, 8, pt, 10, 77)
    assert torch.equal(gk.cpu(), k) and torch.equal(gv.cpu(), v)
    ctx.close()
