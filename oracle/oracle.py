"""ctypes front end of the CPU oracle (flexspec_oracle.c).

TEST INFRASTRUCTURE ONLY: the oracle defines what the verification step of
Alg. 2 (step 2) and the KV rollback of Sec. IV-C must compute.  Only tests,
the smoke check and the benchmark's cpu_baseline leg may import this module;
the GPU library never does, and this module imports nothing from it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flexspec_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over output features only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Model(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn",
                                       "vocab", "weights_bf16")] + [("rms_eps", C.c_double), ("rope_theta", C.c_double)]


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + [
        (n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "w_qkv", "w_o", "mlp_norm", "w_gate_up", "w_down")]


class _Lora(C.Structure):
    _fields_ = [("rank", C.c_int), ("scale", C.c_double)] + [
        (n, C.POINTER(C.c_void_p)) for n in ("a_qkv", "b_qkv", "a_o", "b_o")]


class _DraftHead(C.Structure):
    _fields_ = [("d_hidden", C.c_int), ("d_proj", C.c_int), ("w1", C.c_void_p), ("w2", C.c_void_p), ("wv", C.c_void_p)]


class _SampleOut(C.Structure):
    _fields_ = [("tau", C.c_int32), ("next_token", C.c_int32), ("used_residual", C.c_int32), ("pad_", C.c_int32),
                ("accept_margin", C.c_double), ("cdf_margin", C.c_double), ("nucleus_margin", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_forward.restype = C.c_int
        _lib.orc_forward_stored.restype = C.c_int
        _lib.orc_forward_lora.restype = C.c_int
        _lib.orc_draft_forward.restype = C.c_int
        _lib.orc_round_bf16.restype = C.c_double
        _lib.orc_round_bf16.argtypes = [C.c_double]
        _lib.orc_round_f16.restype = C.c_double
        _lib.orc_round_f16.argtypes = [C.c_double]
        _lib.orc_sample.restype = C.c_int
        _lib.orc_sample_warp.restype = C.c_int
        _lib.orc_sample_cut.restype = C.c_int
        _lib.orc_rollback.restype = C.c_int
        _lib.orc_linear.restype = None
        _lib.orc_attention.restype = None
    return _lib


@dataclass
class SampleResult:
    tau: int
    next_token: int
    used_residual: bool
    accept_margin: float
    cdf_margin: float
    accept_prob: np.ndarray
    nucleus_margin: float = float("inf")


def _model_struct(cfg) -> _Model:
    return _Model(cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab,
                  1 if cfg.dtype == "bf16" else 0, float(cfg.rms_eps), float(cfg.rope_theta))


def _weights_struct(cfg, w):
    """w: dict of numpy arrays (float32, or uint16 holding bf16 bits), [out][in] row-major."""
    want = np.uint16 if cfg.dtype == "bf16" else np.float32
    keep = []

    def ptr(a):
        a = np.ascontiguousarray(a)
        assert a.dtype == want, (a.dtype, want)
        keep.append(a)
        return a.ctypes.data

    def per_layer(name):
        arr = (C.c_void_p * cfg.n_layers)(*[ptr(w[f"{name}.{l}"]) for l in range(cfg.n_layers)])
        keep.append(arr)
        return C.cast(arr, C.POINTER(C.c_void_p))

    ws = _Weights(ptr(w["embed"]), ptr(w["final_norm"]), ptr(w["lm_head"]),
                  per_layer("attn_norm"), per_layer("w_qkv"), per_layer("w_o"),
                  per_layer("mlp_norm"), per_layer("w_gate_up"), per_layer("w_down"))
    return ws, keep


def new_cache(cfg, cap: int):
    """Empty per-session KV cache: two [n_layers][cap][n_kv_heads][head_dim] fp64 arrays."""
    shape = (cfg.n_layers, cap, cfg.n_kv_heads, cfg.head_dim)
    return np.zeros(shape, np.float64), np.zeros(shape, np.float64)


# Tensors a bf16 deployment stores between steps (bit mask for forward(..., stored=)): normalised activations entering
# a projection, rotated queries, the new rows' keys / values, probabilities relative to the row maximum, the attention
# output, the SwiGLU output.  ST_BF16 is what "the model runs in bf16" means for the configurations: every tensor that
# one step hands to the next through memory; the probabilities never leave the attention step and are not part of it.
ST_A, ST_Q, ST_KV, ST_P, ST_O, ST_ACT = 1, 2, 4, 8, 16, 32
ST_BF16 = ST_A | ST_Q | ST_KV | ST_O | ST_ACT
ST_NAMES = {"a": ST_A, "q": ST_Q, "kv": ST_KV, "p": ST_P, "o": ST_O, "act": ST_ACT}
# The two tensors that are bounded whatever the model (normalised activations, attention outputs) kept in fp16 instead:
# the same 16 bits with 11 significant ones.  The bf16 bit of a tensor wins over its fp16 bit.
ST_A16, ST_O16 = 64, 128


def round_bf16(x: float) -> float:
    """Nearest bf16 value (ties to even) of a double."""
    return float(lib().orc_round_bf16(float(x)))


def round_f16(x: float) -> float:
    """Nearest fp16 value (ties to even, held at +-65504 beyond the range) of a double."""
    return float(lib().orc_round_f16(float(x)))


def _lora_struct(cfg, lora):
    """lora: dict(rank, scale, a_qkv=[...], b_qkv=[...], a_o=[...], b_o=[...]) with n_layers - 1 arrays per list, in the
    model's weight storage type (float32, or uint16 bf16 bits)."""
    want = np.uint16 if cfg.dtype == "bf16" else np.float32
    keep = []

    def per_layer(name):
        arrs = [np.ascontiguousarray(a) for a in lora[name]]
        assert len(arrs) == cfg.n_layers - 1 and all(a.dtype == want for a in arrs), name
        keep.extend(arrs)
        tab = (C.c_void_p * max(len(arrs), 1))(*[a.ctypes.data for a in arrs])
        keep.append(tab)
        return C.cast(tab, C.POINTER(C.c_void_p))

    ls = _Lora(int(lora["rank"]), float(lora["scale"]), per_layer("a_qkv"), per_layer("b_qkv"), per_layer("a_o"),
               per_layer("b_o"))
    return ls, keep


def forward(cfg, w, kc, vc, L: int, tokens, want_hidden: bool = False, stored: int = 0, lora=None):
    """Target forward over tokens placed at positions L.. on top of cache (kc, vc); appends their KV.

    Returns logits [n][vocab] fp64 (and the pre-norm hidden state if asked).  Alg. 2 step 2.
    stored: mask of ST_* tensors rounded to bf16 (ST_A16 / ST_O16: to fp16), fp64 arithmetic otherwise; 0 = the plain fp64
    definition.
    lora: this request's adapter of the evolved target (Sec. IV-A), see _lora_struct; None = the base target.
    """
    tokens = np.ascontiguousarray(tokens, np.int32)
    n = int(tokens.shape[0])
    assert kc.dtype == np.float64 and vc.dtype == np.float64 and kc.flags.c_contiguous and vc.flags.c_contiguous
    cap = kc.shape[1]
    logits = np.empty((n, cfg.vocab), np.float64)
    hidden = np.empty((n, cfg.d_model), np.float64) if want_hidden else None
    ms = _model_struct(cfg)
    ws, keep = _weights_struct(cfg, w)
    lp, keep2 = (None, None)
    if lora is not None:
        ls, keep2 = _lora_struct(cfg, lora)
        lp = C.byref(ls)
    rc = lib().orc_forward_lora(C.byref(ms), C.byref(ws), lp, C.c_void_p(kc.ctypes.data), C.c_void_p(vc.ctypes.data),
                                C.c_int(cap), C.c_int(L), C.c_void_p(tokens.ctypes.data), C.c_int(n),
                                C.c_void_p(logits.ctypes.data),
                                C.c_void_p(hidden.ctypes.data) if want_hidden else C.c_void_p(0), C.c_int(int(stored)))
    del keep, keep2
    if rc != 0:
        raise ValueError("orc_forward rejected its arguments")
    return (logits, hidden) if want_hidden else logits


def draft_forward(cfg, w, head, kc, vc, L: int, tokens, stored: int = 0):
    """The edge draft model of Sec. IV-A over tokens placed at positions L.. of ITS one-layer KV session (kc, vc:
    [1][cap][n_kv_heads][head_dim]): anchor block (the target's last block, from w) + two-layer MLP + vocabulary projection.

    head: dict(w1 [d_hidden][d_model], w2 [d_proj][d_hidden], wv [vocab][d_proj]) in the model's weight storage type.
    Returns the draft's logits [n][vocab] fp64; its law is softmax(logits / T)."""
    tokens = np.ascontiguousarray(tokens, np.int32)
    n = int(tokens.shape[0])
    assert kc.shape[0] == 1 and kc.dtype == np.float64 and kc.flags.c_contiguous and vc.flags.c_contiguous
    want = np.uint16 if cfg.dtype == "bf16" else np.float32
    mats = [np.ascontiguousarray(head[k]) for k in ("w1", "w2", "wv")]
    assert all(m.dtype == want for m in mats)
    hs = _DraftHead(int(mats[0].shape[0]), int(mats[1].shape[0]), mats[0].ctypes.data, mats[1].ctypes.data, mats[2].ctypes.data)
    logits = np.empty((n, cfg.vocab), np.float64)
    ms = _model_struct(cfg)
    ws, keep = _weights_struct(cfg, w)
    rc = lib().orc_draft_forward(C.byref(ms), C.byref(ws), C.byref(hs), C.c_void_p(kc.ctypes.data), C.c_void_p(vc.ctypes.data),
                                 C.c_int(kc.shape[1]), C.c_int(L), C.c_void_p(tokens.ctypes.data), C.c_int(n),
                                 C.c_void_p(logits.ctypes.data), C.c_int(int(stored)))
    del keep, mats
    if rc != 0:
        raise ValueError("orc_draft_forward rejected its arguments")
    return logits


def linear(W, x, bf16: bool):
    """y = x W^T for W [out][in] (float32, or uint16 bf16 bits) and x [n][in] fp64: the dense step of the forward."""
    W = np.ascontiguousarray(W)
    x = np.ascontiguousarray(x, np.float64)
    out, inn = W.shape
    y = np.empty((x.shape[0], out), np.float64)
    lib().orc_linear(C.c_void_p(W.ctypes.data), C.c_int(1 if bf16 else 0), C.c_int(out), C.c_int(inn),
                     C.c_void_p(x.ctypes.data), C.c_int(x.shape[0]), C.c_void_p(y.ctypes.data))
    return y


def attention(q, kl, vl, L: int):
    """Block attention over one layer of a session cache: q [n][H][hd] (rotated), kl/vl [>=L+n][Hkv][hd], fp64."""
    q = np.ascontiguousarray(q, np.float64)
    kl = np.ascontiguousarray(kl, np.float64)
    vl = np.ascontiguousarray(vl, np.float64)
    n, H, hd = q.shape
    Hkv = kl.shape[1]
    assert kl.shape[0] >= L + n and vl.shape == kl.shape
    out = np.empty((n, H * hd), np.float64)
    lib().orc_attention(C.c_void_p(q.ctypes.data), C.c_int(H * hd), C.c_void_p(kl.ctypes.data),
                        C.c_void_p(vl.ctypes.data), C.c_int(L), C.c_int(n), C.c_int(H), C.c_int(Hkv), C.c_int(hd),
                        C.c_void_p(out.ctypes.data))
    return out


def sample(logits, draft, q, u_acc, u_smp: float, T: float, top_p: float = 1.0, top_k: int = 0) -> SampleResult:
    """Acceptance loop + correction/bonus token for one request (Alg. 2 step 2; speculative sampling for T>0).

    top_k > 0 and / or top_p < 1 cut the target law of every row to its most probable tokens first (Regime B of Sec. V
    samples with top-p): top-k, then top-p on what is left, ties kept together."""
    logits = np.ascontiguousarray(logits, np.float64)
    gamma = int(len(draft))
    V = int(logits.shape[1])
    assert logits.shape[0] == gamma + 1
    draft = np.ascontiguousarray(draft, np.int32)
    u_acc = np.ascontiguousarray(u_acc, np.float32)
    if T > 0 and gamma > 0:
        q = np.ascontiguousarray(q, np.float32)
        assert q.shape == (gamma, V)
        qp = C.c_void_p(q.ctypes.data)
    else:
        qp = C.c_void_p(0)
    out = _SampleOut()
    a = np.full(gamma, np.nan, np.float64)
    rc = lib().orc_sample_cut(C.c_void_p(logits.ctypes.data), C.c_int(V), C.c_int(gamma), C.c_void_p(draft.ctypes.data),
                              qp, C.c_void_p(u_acc.ctypes.data), C.c_float(float(u_smp)), C.c_double(float(T)),
                              C.c_int(int(top_k)), C.c_double(float(top_p)), C.byref(out), C.c_void_p(a.ctypes.data))
    if rc != 0:
        raise ValueError("orc_sample_cut rejected its arguments")
    return SampleResult(out.tau, out.next_token, bool(out.used_residual), out.accept_margin, out.cdf_margin, a,
                        out.nucleus_margin)


def rollback(L: int, gamma: int, tau: int, page_size: int):
    """KV rollback of Sec. IV-C: returns (new valid length, pages released)."""
    nl, pr = C.c_int32(), C.c_int32()
    rc = lib().orc_rollback(C.c_int(L), C.c_int(gamma), C.c_int(tau), C.c_int(page_size), C.byref(nl), C.byref(pr))
    if rc != 0:
        raise ValueError("orc_rollback rejected its arguments")
    return nl.value, pr.value


@dataclass
class VerifyResult:
    logits: np.ndarray
    sample: SampleResult
    new_len: int
    pages_released: int


def verify(cfg, w, kc, vc, L: int, last_token: int, draft, q, u_acc, u_smp: float, T: float,
           stored: int = 0, lora=None) -> VerifyResult:
    """One request of the verification step: score [last_token, drafts], accept/reject, roll back."""
    toks = np.concatenate([[last_token], np.asarray(draft, np.int64)]).astype(np.int32)
    logits = forward(cfg, w, kc, vc, L, toks, stored=stored, lora=lora)
    s = sample(logits, draft, q, u_acc, u_smp, T)
    nl, pr = rollback(L, len(draft), s.tau, cfg.page_size)
    return VerifyResult(logits, s, nl, pr)
