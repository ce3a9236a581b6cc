"""ctypes binding of libflexverify.so: argument marshalling only.

Every step of the verification path (Alg. 2 step 2, Sec. IV-C) runs inside the library's HIP
kernels; torch is used here for device memory and for the current stream.  There is no CPU
fallback: importing this module without the built library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, os.environ.get("FSV_LIB_NAME", "libflexverify.so"))

F32, BF16 = 0, 1
W_QKV, W_O, W_GATE_UP, W_DOWN, W_LM_HEAD = range(5)

EXPORTS = ["fsv_create", "fsv_destroy", "fsv_lora_load", "fsv_draft_attach", "fsv_draft_probs", "fsv_draft_kv_import", "fsv_draft_kv_export", "fsv_verify", "fsv_prefill", "fsv_sample", "fsv_sample_static", "fsv_rollback", "fsv_kv_import", "fsv_kv_export",
           "fsv_linear", "fsv_attention", "fsv_profile_enable", "fsv_profile_sample", "fsv_profile_read", "fsv_kernel_class_name",
           "fsv_strerror", "fsv_last_error", "fsv_policy_stride", "fsv_policy_ema", "fsv_policy_step_time", "fsv_pager_create",
           "fsv_pager_destroy", "fsv_pager_reserve", "fsv_pager_trim", "fsv_pager_free_pages", "fsv_pager_session_pages"]


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab",
                                         "dtype")] + [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("page_size", "max_batch", "max_gamma", "max_pages_per_req", "max_rows")]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("attn_norm", "w_qkv", "w_o", "mlp_norm", "w_gate_up", "w_down")]


class Batch(C.Structure):
    _fields_ = [("batch", C.c_int32), ("num_pages", C.c_int32)] + [(n, C.c_void_p) for n in (
        "seq_lens", "seq_lens_host", "last_token", "draft_offsets", "draft_offsets_host", "draft_tokens", "draft_probs",
        "u_accept", "u_sample", "temperature", "temperature_host", "page_table", "k_pool", "v_pool", "top_p",
        "top_p_host", "top_k", "top_k_host", "adapter")]


class Lora(C.Structure):
    _fields_ = [("n_adapters", C.c_int32), ("rank", C.c_int32), ("scale", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("a_qkv", "b_qkv", "a_o", "b_o")]


class DraftHead(C.Structure):
    _fields_ = [("d_hidden", C.c_int32), ("d_proj", C.c_int32), ("w1", C.c_void_p), ("w2", C.c_void_p), ("w_vocab", C.c_void_p)]


DRAFT_Q_VERIFY, DRAFT_Q_ALL = 0, 1


class Result(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("accepted_len", "next_token", "new_seq_lens", "pages_released", "flags",
                                          "logits_out")]


class KernelTime(C.Structure):
    _fields_ = [("kernel_class", C.c_int32), ("launches", C.c_int32), ("total_ms", C.c_double), ("bytes", C.c_double)]


class LatencyModel(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("alpha_edge", "beta", "bits_per_token", "header_bits", "t_prop", "t_base",
                                          "delta_cloud", "t_down")]


TAU_LINEAR, TAU_GEOMETRIC = 0, 1


class FsvError(RuntimeError):
    def __init__(self, status, what, detail=""):
        super().__init__(f"{what}: {status} ({detail})")
        self.status = status


_lib = None


def lib():
    """Load the built library; fail loudly when it is missing (there is no other implementation)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2601_00644_amd.build` "
                              "(or __graft_entry__.build()) first")
        _lib = C.CDLL(LIB_PATH)
        for n in EXPORTS:
            getattr(_lib, n)
        _lib.fsv_strerror.restype = C.c_char_p
        _lib.fsv_last_error.restype = C.c_char_p
        _lib.fsv_last_error.argtypes = [C.c_void_p]
        _lib.fsv_kernel_class_name.restype = C.c_char_p
        _lib.fsv_destroy.argtypes = [C.c_void_p]
        _lib.fsv_destroy.restype = None
        _lib.fsv_policy_stride.argtypes = [C.POINTER(LatencyModel), C.c_double, C.c_double, C.c_int32, C.c_int32,
                                           C.POINTER(C.c_double)]
        _lib.fsv_policy_ema.argtypes = [C.c_double, C.c_int32, C.c_int32, C.c_double]
        _lib.fsv_policy_ema.restype = C.c_double
        _lib.fsv_policy_step_time.argtypes = [C.POINTER(LatencyModel), C.c_double, C.c_int32, C.c_double]
        _lib.fsv_policy_step_time.restype = C.c_double
        _lib.fsv_pager_create.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
        _lib.fsv_pager_destroy.argtypes = [C.c_void_p]
        _lib.fsv_pager_destroy.restype = None
        _lib.fsv_pager_reserve.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        _lib.fsv_pager_trim.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        _lib.fsv_pager_free_pages.argtypes = [C.c_void_p]
        _lib.fsv_pager_session_pages.argtypes = [C.c_void_p, C.c_int32]
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return t.data_ptr()
    if isinstance(t, np.ndarray):
        assert t.flags.c_contiguous
        return t.ctypes.data
    return int(t)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


@dataclass
class DeviceBatch:
    """Device tensors of one batch plus the host copies the library needs to size its launches."""
    seq_lens: torch.Tensor | None
    last_token: torch.Tensor | None
    draft_offsets: torch.Tensor
    draft_tokens: torch.Tensor | None
    draft_probs: torch.Tensor | None
    u_accept: torch.Tensor | None
    u_sample: torch.Tensor | None
    temperature: torch.Tensor | None
    page_table: torch.Tensor | None
    k_pool: torch.Tensor | None
    v_pool: torch.Tensor | None
    num_pages: int
    seq_lens_host: np.ndarray | None
    draft_offsets_host: np.ndarray
    temperature_host: np.ndarray | None = None
    top_p: torch.Tensor | None = None          # [B] nucleus mass per request (None = no cut)
    top_p_host: np.ndarray | None = None
    top_k: torch.Tensor | None = None          # [B] int32 top-k cut per request (0 = off)
    top_k_host: np.ndarray | None = None
    adapter: torch.Tensor | None = None        # [B] int32 adapter id of the request's target version (-1 = base)

    @property
    def batch(self):
        return int(self.draft_offsets_host.shape[0]) - 1

    @property
    def rows(self):
        return int(self.draft_offsets_host[-1]) + self.batch

    def struct(self) -> Batch:
        return Batch(self.batch, int(self.num_pages), _ptr(self.seq_lens), _ptr(self.seq_lens_host),
                     _ptr(self.last_token), _ptr(self.draft_offsets), _ptr(self.draft_offsets_host),
                     _ptr(self.draft_tokens), _ptr(self.draft_probs), _ptr(self.u_accept), _ptr(self.u_sample),
                     _ptr(self.temperature), _ptr(self.temperature_host), _ptr(self.page_table), _ptr(self.k_pool),
                     _ptr(self.v_pool), _ptr(self.top_p), _ptr(self.top_p_host), _ptr(self.top_k), _ptr(self.top_k_host), _ptr(self.adapter))


@dataclass
class DeviceResult:
    accepted_len: torch.Tensor
    next_token: torch.Tensor
    new_seq_lens: torch.Tensor
    pages_released: torch.Tensor
    flags: torch.Tensor
    logits_out: torch.Tensor | None = None

    @staticmethod
    def alloc(batch: int, rows: int = 0, vocab: int = 0, want_logits: bool = False, device="cuda"):
        i32 = lambda: torch.zeros(batch, dtype=torch.int32, device=device)
        lg = torch.empty((rows, vocab), dtype=torch.float32, device=device) if want_logits else None
        return DeviceResult(i32(), i32(), i32(), i32(), i32(), lg)

    def struct(self) -> Result:
        return Result(_ptr(self.accepted_len), _ptr(self.next_token), _ptr(self.new_seq_lens),
                      _ptr(self.pages_released), _ptr(self.flags), _ptr(self.logits_out))


class Context:
    """Owns one fsv_ctx.  Method names follow the C entry points."""

    def __init__(self, cfg, weights: dict | None, max_batch: int, max_gamma: int, max_pages_per_req: int = 1,
                 max_rows: int = 0, sampler_only: bool = False):
        self._h = C.c_void_p(0)
        self.cfg = cfg
        dt = BF16 if cfg.dtype == "bf16" else F32
        n_layers = 0 if sampler_only else cfg.n_layers
        desc = ModelDesc(n_layers, cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab, dt,
                         cfg.rms_eps, cfg.rope_theta, cfg.page_size, max_batch, max_gamma, max_pages_per_req, max_rows)
        wp = None
        if not sampler_only:
            keep = []

            def per_layer(name):
                arr = (C.c_void_p * cfg.n_layers)(*[weights[f"{name}.{l}"].data_ptr() for l in range(cfg.n_layers)])
                keep.append(arr)
                return C.cast(arr, C.POINTER(C.c_void_p))

            ws = Weights(weights["embed"].data_ptr(), weights["final_norm"].data_ptr(), weights["lm_head"].data_ptr(),
                         per_layer("attn_norm"), per_layer("w_qkv"), per_layer("w_o"), per_layer("mlp_norm"),
                         per_layer("w_gate_up"), per_layer("w_down"))
            wp = C.byref(ws)
        rc = lib().fsv_create(C.byref(desc), wp, C.byref(self._h))
        if rc != 0:
            raise FsvError(rc, "fsv_create", lib().fsv_strerror(rc).decode())

    def _check(self, rc, what):
        if rc != 0:
            raise FsvError(rc, what, lib().fsv_strerror(rc).decode() + ": " + lib().fsv_last_error(self._h).decode())

    def close(self):
        if self._h:
            lib().fsv_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def lora_load(self, adapters: list | None):
        """adapters: list of dicts as synth.make_lora returns them (device tensors), all of one rank; None removes them."""
        if not adapters:
            self._check(lib().fsv_lora_load(self._h, None), "fsv_lora_load")
            return
        n, nl = len(adapters), self.cfg.n_layers - 1
        scale = np.ascontiguousarray([a["scale"] for a in adapters], np.float32)
        keep = []

        def table(name):
            arr = (C.c_void_p * max(nl * n, 1))(*[adapters[a][name][l].data_ptr() for l in range(nl) for a in range(n)])
            keep.append(arr)
            return C.cast(arr, C.POINTER(C.c_void_p))

        lo = Lora(n, int(adapters[0]["rank"]), scale.ctypes.data, table("a_qkv"), table("b_qkv"), table("a_o"), table("b_o"))
        self._check(lib().fsv_lora_load(self._h, C.byref(lo)), "fsv_lora_load")

    def draft_attach(self, head: dict | None):
        """head: dict(w1, w2, wv) of device tensors as synth.make_draft_head returns them; None removes the head."""
        if head is None:
            self._check(lib().fsv_draft_attach(self._h, None), "fsv_draft_attach")
            return
        for t in head.values():
            assert t.is_contiguous()
        h = DraftHead(int(head["w1"].shape[0]), int(head["w2"].shape[0]), head["w1"].data_ptr(), head["w2"].data_ptr(),
                      head["wv"].data_ptr())
        self._check(lib().fsv_draft_attach(self._h, C.byref(h)), "fsv_draft_attach")

    def draft_kv_import(self, k_pool, v_pool, num_pages, page_table_row, pos0, src_k, src_v):
        """src_k / src_v: [n_pos][n_kv_heads][head_dim] of the draft's one-layer session."""
        assert src_k.is_contiguous() and src_v.is_contiguous() and src_k.dim() == 3
        self._check(lib().fsv_draft_kv_import(self._h, C.c_void_p(k_pool.data_ptr()), C.c_void_p(v_pool.data_ptr()),
                                              int(num_pages), C.c_void_p(page_table_row.data_ptr()), int(pos0),
                                              int(src_k.shape[0]), C.c_void_p(src_k.data_ptr()), C.c_void_p(src_v.data_ptr()),
                                              _stream()), "fsv_draft_kv_import")

    def draft_kv_export(self, k_pool, v_pool, num_pages, page_table_row, pos0, n_pos):
        cfg = self.cfg
        shape = (n_pos, cfg.n_kv_heads, cfg.head_dim)
        dk = torch.empty(shape, dtype=torch.bfloat16, device=k_pool.device)
        dv = torch.empty(shape, dtype=torch.bfloat16, device=k_pool.device)
        self._check(lib().fsv_draft_kv_export(self._h, C.c_void_p(k_pool.data_ptr()), C.c_void_p(v_pool.data_ptr()),
                                              int(num_pages), C.c_void_p(page_table_row.data_ptr()), int(pos0), int(n_pos),
                                              C.c_void_p(dk.data_ptr()), C.c_void_p(dv.data_ptr()), _stream()),
                    "fsv_draft_kv_export")
        return dk, dv

    def draft_probs(self, batch: DeviceBatch, rows_mode: int = DRAFT_Q_VERIFY, want_logits: bool = False):
        """(q, logits or None): the draft model's laws for the rows of `batch` on the draft's one-layer KV pools."""
        B, G = batch.batch, batch.rows - batch.batch
        n = batch.rows if rows_mode == DRAFT_Q_ALL else G
        q = torch.zeros((max(n, 1), self.cfg.vocab), dtype=torch.float32, device="cuda")
        lg = torch.empty((batch.rows, self.cfg.vocab), dtype=torch.float32, device="cuda") if want_logits else None
        b = batch.struct()
        self._check(lib().fsv_draft_probs(self._h, C.byref(b), int(rows_mode), C.c_void_p(q.data_ptr()),
                                          C.c_void_p(lg.data_ptr()) if want_logits else None, _stream()), "fsv_draft_probs")
        return q, lg

    def verify(self, batch: DeviceBatch, result: DeviceResult):
        b, r = batch.struct(), result.struct()
        self._check(lib().fsv_verify(self._h, C.byref(b), C.byref(r), _stream()), "fsv_verify")

    def prefill(self, batch: DeviceBatch, want_logits: bool = False):
        """The forward alone (fsv_prefill): appends the K / V rows of the batch's rows; returns the [M][vocab] fp32
        logits when asked for."""
        b = batch.struct()
        lg = None
        if want_logits:
            rows = batch.rows
            lg = torch.empty((rows, self.cfg.vocab), dtype=torch.float32, device="cuda")
        self._check(lib().fsv_prefill(self._h, C.byref(b), C.c_void_p(lg.data_ptr()) if want_logits else None, _stream()),
                    "fsv_prefill")
        return lg

    def sample(self, logits: torch.Tensor, batch: DeviceBatch, result: DeviceResult):
        dt = BF16 if logits.dtype == torch.bfloat16 else F32
        assert logits.dtype in (torch.bfloat16, torch.float32) and logits.is_contiguous()
        b, r = batch.struct(), result.struct()
        self._check(lib().fsv_sample(self._h, C.c_void_p(logits.data_ptr()), dt, C.byref(b), C.byref(r), _stream()),
                    "fsv_sample")

    def rollback(self, batch: DeviceBatch, accepted_len: torch.Tensor, result: DeviceResult):
        b, r = batch.struct(), result.struct()
        self._check(lib().fsv_rollback(self._h, C.byref(b), C.c_void_p(accepted_len.data_ptr()), C.byref(r), _stream()),
                    "fsv_rollback")

    def kv_import(self, k_pool, v_pool, num_pages, page_table_row, pos0, src_k, src_v):
        n = int(src_k.shape[1])
        assert src_k.is_contiguous() and src_v.is_contiguous()
        self._check(lib().fsv_kv_import(self._h, C.c_void_p(k_pool.data_ptr()), C.c_void_p(v_pool.data_ptr()),
                                        int(num_pages), C.c_void_p(page_table_row.data_ptr()), int(pos0), n,
                                        C.c_void_p(src_k.data_ptr()), C.c_void_p(src_v.data_ptr()), _stream()),
                    "fsv_kv_import")

    def kv_export(self, k_pool, v_pool, num_pages, page_table_row, pos0, n_pos):
        cfg = self.cfg
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        shape = (cfg.n_layers, n_pos, cfg.n_kv_heads, cfg.head_dim)
        dk = torch.empty(shape, dtype=tdt, device=k_pool.device)
        dv = torch.empty(shape, dtype=tdt, device=k_pool.device)
        self._check(lib().fsv_kv_export(self._h, C.c_void_p(k_pool.data_ptr()), C.c_void_p(v_pool.data_ptr()),
                                        int(num_pages), C.c_void_p(page_table_row.data_ptr()), int(pos0), int(n_pos),
                                        C.c_void_p(dk.data_ptr()), C.c_void_p(dv.data_ptr()), _stream()),
                    "fsv_kv_export")
        return dk, dv

    def linear(self, which: int, layer: int, x: torch.Tensor, n_out: int) -> torch.Tensor:
        assert x.is_contiguous()
        y = torch.empty((x.shape[0], n_out), dtype=torch.float32, device=x.device)
        self._check(lib().fsv_linear(self._h, int(which), int(layer), C.c_void_p(x.data_ptr()), int(x.shape[0]),
                                     C.c_void_p(y.data_ptr()), _stream()), "fsv_linear")
        return y

    def attention(self, layer: int, q: torch.Tensor, batch: DeviceBatch) -> torch.Tensor:
        assert q.is_contiguous()
        out = torch.empty((q.shape[0], self.cfg.n_heads * self.cfg.head_dim), dtype=torch.float32, device=q.device)
        b = batch.struct()
        self._check(lib().fsv_attention(self._h, int(layer), C.c_void_p(q.data_ptr()), C.byref(b),
                                        C.c_void_p(out.data_ptr()), _stream()), "fsv_attention")
        return out

    def profile_enable(self, classes=True, every: int = 1):
        """classes: True = all kernel classes, False = off, or an iterable of class names; every: record only every
        n-th launch of each enabled class."""
        self._check(lib().fsv_profile_sample(self._h, C.c_int32(max(1, int(every)))), "fsv_profile_sample")
        if classes is True:
            mask = 0xFFFFFFFF
        elif not classes:
            mask = 0
        else:
            names = [lib().fsv_kernel_class_name(i).decode() for i in range(32)]
            mask = 0
            for n in classes:
                mask |= 1 << names.index(n)
        self._check(lib().fsv_profile_enable(self._h, C.c_uint32(mask)), "fsv_profile_enable")

    def profile_read(self) -> dict:
        buf = (KernelTime * 32)()
        n = lib().fsv_profile_read(self._h, buf, 32)
        if n < 0:
            self._check(n, "fsv_profile_read")
        return {lib().fsv_kernel_class_name(buf[i].kernel_class).decode():
                dict(launches=buf[i].launches, total_ms=buf[i].total_ms, bytes=buf[i].bytes) for i in range(n)}


def sample_static(vocab: int, logits: torch.Tensor, batch: DeviceBatch, result: DeviceResult):
    """fsv_sample_static: the accept / resample step without a context and without any allocation."""
    dt = BF16 if logits.dtype == torch.bfloat16 else F32
    assert logits.dtype in (torch.bfloat16, torch.float32) and logits.is_contiguous()
    b, r = batch.struct(), result.struct()
    rc = lib().fsv_sample_static(int(vocab), C.c_void_p(logits.data_ptr()), dt, C.byref(b), C.byref(r), _stream())
    if rc != 0:
        raise FsvError(rc, "fsv_sample_static", lib().fsv_strerror(rc).decode())


def policy_stride(model: LatencyModel, rate: float, gamma_hat: float, k_max: int, tau_model: int = TAU_GEOMETRIC):
    """(K*, objective) of fsv_policy_stride."""
    obj = C.c_double(0.0)
    k = lib().fsv_policy_stride(C.byref(model), float(rate), float(gamma_hat), int(k_max), int(tau_model), C.byref(obj))
    if k < 1:
        raise FsvError(k, "fsv_policy_stride", lib().fsv_strerror(k).decode())
    return k, obj.value


def policy_ema(gamma_hat: float, tau: int, k: int, mu: float) -> float:
    return lib().fsv_policy_ema(float(gamma_hat), int(tau), int(k), float(mu))


def policy_step_time(model: LatencyModel, rate: float, k: int, cloud_seconds: float = -1.0) -> float:
    return lib().fsv_policy_step_time(C.byref(model), float(rate), int(k), float(cloud_seconds))


class Pager:
    """Owns one fsv_pager; page-table rows are numpy int32 arrays the caller uploads."""

    def __init__(self, num_pages: int, max_sessions: int, max_pages_per_session: int):
        self._h = C.c_void_p(0)
        self.max_pages_per_session = max_pages_per_session
        rc = lib().fsv_pager_create(num_pages, max_sessions, max_pages_per_session, C.byref(self._h))
        if rc != 0:
            raise FsvError(rc, "fsv_pager_create", lib().fsv_strerror(rc).decode())

    def reserve(self, session: int, n_positions: int, row: np.ndarray | None = None) -> None:
        ptr = None
        if row is not None:
            assert row.dtype == np.int32 and row.flags.c_contiguous and row.shape[0] >= self.max_pages_per_session
            ptr = row.ctypes.data
        rc = lib().fsv_pager_reserve(self._h, int(session), int(n_positions), ptr)
        if rc != 0:
            raise FsvError(rc, "fsv_pager_reserve", lib().fsv_strerror(rc).decode())

    def trim(self, session: int, n_positions: int) -> int:
        rc = lib().fsv_pager_trim(self._h, int(session), int(n_positions))
        if rc < 0:
            raise FsvError(rc, "fsv_pager_trim", lib().fsv_strerror(rc).decode())
        return rc

    @property
    def free_pages(self) -> int:
        return lib().fsv_pager_free_pages(self._h)

    def session_pages(self, session: int) -> int:
        return lib().fsv_pager_session_pages(self._h, int(session))

    def close(self):
        if self._h:
            lib().fsv_pager_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pool_shape(cfg, num_pages: int):
    """Elements of one KV pool: [n_layers][num_pages][n_kv_heads][page_size * head_dim]."""
    return (cfg.n_layers, num_pages, cfg.n_kv_heads, cfg.page_size * cfg.head_dim)


def alloc_draft_pools(cfg, num_pages: int, device="cuda"):
    """KV pools of the draft model's one-layer session."""
    shape = (1, num_pages, cfg.n_kv_heads, cfg.page_size * cfg.head_dim)
    return (torch.zeros(shape, dtype=torch.bfloat16, device=device), torch.zeros(shape, dtype=torch.bfloat16, device=device))


def alloc_pools(cfg, num_pages: int, device="cuda"):
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    return (torch.zeros(pool_shape(cfg, num_pages), dtype=tdt, device=device),
            torch.zeros(pool_shape(cfg, num_pages), dtype=tdt, device=device))


def prefill_pieces(chunks, page_rows, k_pool, v_pool, num_pages: int, rows_per_piece: int, device="cuda") -> DeviceBatch:
    """A DeviceBatch for fsv_prefill from token chunks: chunks = [(session index into page_rows, L0, tokens)], every chunk
    cut into pieces of at most rows_per_piece rows; the pieces of one chunk are requests that share the session's
    page-table row and continue each other.  page_rows: host int32 [sessions][max_pages_per_req]."""
    L, last, off, toks, rows = [], [], [0], [], []
    for sess, L0, tokens in chunks:
        tokens = np.asarray(tokens, np.int32)
        for p0 in range(0, len(tokens), rows_per_piece):
            piece = tokens[p0:p0 + rows_per_piece]
            L.append(int(L0) + p0)
            last.append(int(piece[0]))
            toks.extend(int(x) for x in piece[1:])
            off.append(off[-1] + len(piece) - 1)
            rows.append(np.asarray(page_rows[sess], np.int32))
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(np.asarray(a, dt)), device=device)
    Lh, offh = np.asarray(L, np.int32), np.asarray(off, np.int32)
    return DeviceBatch(t(Lh, np.int32), t(last, np.int32), t(offh, np.int32), t(toks if toks else [0], np.int32), None, None,
                       None, None, t(np.stack(rows), np.int32), k_pool, v_pool, num_pages, Lh, offh)


def device_batch(req, draft_tokens=None, draft_probs=None, k_pool=None, v_pool=None, device="cuda") -> DeviceBatch:
    """Upload a synth.Requests (numpy) as a DeviceBatch."""
    t = lambda a, dt=None: None if a is None else torch.as_tensor(np.ascontiguousarray(a), device=device)
    return DeviceBatch(t(req.seq_lens), t(req.last_token), t(req.draft_offsets),
                       t(np.asarray(draft_tokens, np.int32)) if draft_tokens is not None else None,
                       draft_probs, t(req.u_accept), t(req.u_sample), t(req.temperature), t(req.page_table),
                       k_pool, v_pool, req.num_pages, np.ascontiguousarray(req.seq_lens, np.int32),
                       np.ascontiguousarray(req.draft_offsets, np.int32), np.ascontiguousarray(req.temperature, np.float32))
