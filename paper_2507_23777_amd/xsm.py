"""ctypes binding of libxsm.so: the same names as include/xsm.h, argument
marshalling only.  ``Engine`` owns the torch-allocated device buffers the C ABI
asks the caller to provide."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

XSM_F32, XSM_BF16 = 0, 1
XSM_HEAD_MLP, XSM_HEAD_CA = 0, 1
XSM_OPT_SINGLE_LAUNCH = 1
XSM_OPT_TIMELINE = 2
XSM_OPT_ATTN_SPLITS = 3
XSM_OPT_PREFILL_ROWS = 4
_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libxsm.so")
API = ["xsm_create", "xsm_destroy", "xsm_last_error", "xsm_weights_bytes", "xsm_kv_bytes",
       "xsm_workspace_bytes", "xsm_canonical_weight_elems", "xsm_bind", "xsm_load_weights",
       "xsm_prefill", "xsm_spec_step", "xsm_plain_step", "xsm_debug_kv_export",
       "xsm_debug_kv_import", "xsm_debug_trace_enable", "xsm_debug_trace_report", "xsm_set_option",
       "xsm_check_device", "xsm_debug_timeline", "xsm_debug_kv_clone", "xsm_debug_inject_device_error",
       "xsm_spec_step_static"]
XSM_FLAG_NEAR_TIE, XSM_FLAG_BAD_LEN, XSM_FLAG_BAD_TOKEN, XSM_FLAG_BAD_SLOT, XSM_FLAG_DEVICE_TIMEOUT = 1, 2, 4, 8, 16


class XsmError(RuntimeError):
    pass


class xsm_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn",
                                         "vocab", "n_draft", "max_batch", "max_ctx", "n_cond",
                                         "dtype")] + [("rope_theta", C.c_float), ("rms_eps", C.c_float),
                                                      ("head_kind", C.c_int32)]


class xsm_verify_params(C.Structure):
    _fields_ = [("mode", C.c_int32), ("top_ka", C.c_int32), ("delta", C.c_float),
                ("temperature", C.c_float), ("sample", C.c_int32), ("seed", C.c_uint64),
                ("top_ks", C.c_int32), ("pts_prune", C.c_float)]


class xsm_batch(C.Structure):
    _fields_ = [("n_seq", C.c_int32), ("kv_len_bound", C.c_int32), ("slot", C.c_void_p),
                ("kv_len", C.c_void_p), ("block", C.c_void_p), ("out_tokens", C.c_void_p),
                ("n_accepted", C.c_void_p), ("flags", C.c_void_p), ("logits_dbg", C.c_void_p),
                ("head_logits_dbg", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Load libxsm.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise XsmError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_23777_amd.build`")
    # torch first: its bundled HIP runtime must be the one already in the process, so that
    # libxsm.so binds to the same runtime that owns the tensors' device memory and streams
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int32
    L.xsm_create.argtypes, L.xsm_create.restype = [C.POINTER(xsm_config), C.POINTER(vp)], C.c_int
    L.xsm_destroy.argtypes, L.xsm_destroy.restype = [vp], None
    L.xsm_last_error.argtypes, L.xsm_last_error.restype = [vp], C.c_char_p
    for f in ("xsm_weights_bytes", "xsm_kv_bytes", "xsm_workspace_bytes", "xsm_canonical_weight_elems"):
        getattr(L, f).argtypes, getattr(L, f).restype = [vp], sz
    L.xsm_bind.argtypes, L.xsm_bind.restype = [vp, vp, vp, vp], C.c_int
    L.xsm_load_weights.argtypes, L.xsm_load_weights.restype = [vp, vp, sz, vp], C.c_int
    L.xsm_prefill.argtypes, L.xsm_prefill.restype = [vp, i32, C.POINTER(i32), vp, i32, vp, vp], C.c_int
    for f in ("xsm_spec_step", "xsm_plain_step", "xsm_spec_step_static"):
        getattr(L, f).argtypes = [vp, C.POINTER(xsm_batch), C.POINTER(xsm_verify_params), vp]
        getattr(L, f).restype = C.c_int
    for f in ("xsm_debug_kv_export", "xsm_debug_kv_import"):
        getattr(L, f).argtypes, getattr(L, f).restype = [vp, i32, i32, i32, i32, i32, vp], C.c_int
    L.xsm_set_option.argtypes, L.xsm_set_option.restype = [vp, i32, i32], C.c_int
    L.xsm_debug_kv_clone.argtypes, L.xsm_debug_kv_clone.restype = [vp, i32, i32], C.c_int
    L.xsm_debug_timeline.argtypes, L.xsm_debug_timeline.restype = [vp, vp, sz], C.c_int
    L.xsm_check_device.argtypes, L.xsm_check_device.restype = [vp], C.c_int
    L.xsm_debug_inject_device_error.argtypes, L.xsm_debug_inject_device_error.restype = [vp, C.c_uint32], C.c_int
    L.xsm_debug_trace_enable.argtypes, L.xsm_debug_trace_enable.restype = [C.c_int], None
    L.xsm_debug_trace_report.argtypes, L.xsm_debug_trace_report.restype = [C.c_char_p, sz], C.c_int
    _lib = L
    return L


def xsm_debug_trace_enable(on: bool) -> None:
    lib().xsm_debug_trace_enable(1 if on else 0)


def xsm_debug_trace_report() -> dict:
    """{kernel_class: (count, total_ms)} since the last report."""
    buf = C.create_string_buffer(1 << 16)
    n = lib().xsm_debug_trace_report(buf, len(buf))
    if n < 0:
        raise XsmError("xsm_debug_trace_report failed")
    out = {}
    for line in buf.value.decode().splitlines():
        name, cnt, ms = line.split()
        out[name] = (int(cnt), float(ms))
    return out


def make_config(cfg: dict, max_batch: int | None = None, max_ctx: int | None = None) -> xsm_config:
    return xsm_config(cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ffn"],
                      cfg["vocab"], cfg["n_draft"], max_batch or cfg["batch"], max_ctx or cfg["max_ctx"],
                      cfg["n_cond"], XSM_BF16 if cfg["dtype"] == "bf16" else XSM_F32,
                      cfg["rope_theta"], cfg["rms_eps"], XSM_HEAD_CA if cfg.get("head_kind", "mlp") == "ca" else XSM_HEAD_MLP)


class StepBuffers:
    """Device arrays of one xsm_batch (torch int32/float32 tensors)."""

    def __init__(self, torch, device, n_seq: int, R: int, vocab: int, K: int, debug: bool):
        i32 = dict(dtype=torch.int32, device=device)
        self.n_seq, self.R = n_seq, R
        self.slot = torch.arange(n_seq, **i32)
        self.kv_len = torch.zeros(n_seq, **i32)
        self.block = torch.zeros((n_seq, R), **i32)
        self.out_tokens = torch.zeros((n_seq, R), **i32)
        self.n_accepted = torch.zeros(n_seq, **i32)
        self.flags = torch.zeros(n_seq, **i32)
        self.logits = torch.zeros((n_seq, R, vocab), dtype=torch.float32, device=device) if debug else None
        self.head_logits = (torch.zeros((n_seq, max(K, 1), vocab), dtype=torch.float32, device=device)
                            if debug and R > 1 else None)

    def struct(self, kv_len_bound: int) -> xsm_batch:
        p = lambda t: None if t is None else t.data_ptr()
        return xsm_batch(self.n_seq, int(kv_len_bound), p(self.slot), p(self.kv_len), p(self.block),
                         p(self.out_tokens), p(self.n_accepted), p(self.flags), p(self.logits),
                         p(self.head_logits))


class Engine:
    """One xsm context with its torch-allocated weights / cache / workspace buffers."""

    def __init__(self, cfg: dict, max_batch: int | None = None, max_ctx: int | None = None,
                 device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise XsmError("no GPU: the xsm hot path has no CPU fallback")
        self.torch, self.device, self.cfg = torch, torch.device(device), dict(cfg)
        self.L = lib()
        self.c_cfg = make_config(cfg, max_batch, max_ctx)
        self.max_batch, self.max_ctx = self.c_cfg.max_batch, self.c_cfg.max_ctx
        h = C.c_void_p()
        rc = self.L.xsm_create(C.byref(self.c_cfg), C.byref(h))
        if rc != 0:
            raise XsmError(f"xsm_create: {self.L.xsm_last_error(None).decode()} ({rc})")
        self.h = h
        mk = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device=self.device)
        self.d_weights = mk(self.L.xsm_weights_bytes(h))
        self.d_kv = mk(self.L.xsm_kv_bytes(h))
        self.d_ws = mk(self.L.xsm_workspace_bytes(h))
        self._check(self.L.xsm_bind(h, self.d_weights.data_ptr(), self.d_kv.data_ptr(), self.d_ws.data_ptr()),
                    "xsm_bind")

    def _check(self, rc: int, what: str):
        if rc != 0:
            raise XsmError(f"{what}: {self.L.xsm_last_error(self.h).decode()} ({rc})")

    def stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def close(self):
        if getattr(self, "h", None):
            self.torch.cuda.synchronize(self.device)
            self.L.xsm_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- entry points, same names as the C ABI -----------------------------------
    def xsm_load_weights(self, packed: np.ndarray):
        packed = np.ascontiguousarray(packed)
        want = np.uint16 if self.c_cfg.dtype == XSM_BF16 else np.float32
        if packed.dtype != want:
            raise XsmError(f"weights must be {want.__name__}")
        self._check(self.L.xsm_load_weights(self.h, packed.ctypes.data, packed.size, self.stream()),
                    "xsm_load_weights")
        self.torch.cuda.synchronize(self.device)

    def to_device(self, x: np.ndarray):
        """float32 host values -> device tensor in the storage dtype."""
        t = self.torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.device)
        return t.to(self.torch.bfloat16) if self.c_cfg.dtype == XSM_BF16 else t

    def xsm_prefill(self, slots, prefix=None, cond=None):
        slots = [int(s) for s in slots]
        arr = (C.c_int32 * len(slots))(*slots)
        P = 0 if prefix is None else int(prefix.shape[1])
        self._check(self.L.xsm_prefill(self.h, len(slots), arr,
                                       None if prefix is None else prefix.data_ptr(), P,
                                       None if cond is None else cond.data_ptr(), self.stream()),
                    "xsm_prefill")

    def buffers(self, n_seq: int, spec: bool = True, debug: bool = False) -> StepBuffers:
        K = self.c_cfg.n_draft
        return StepBuffers(self.torch, self.device, n_seq, K + 1 if spec else 1, self.c_cfg.vocab, K, debug)

    def xsm_spec_step(self, buf: StepBuffers, vp: xsm_verify_params, kv_len_bound: int):
        bt = buf.struct(kv_len_bound)
        self._check(self.L.xsm_spec_step(self.h, C.byref(bt), C.byref(vp), self.stream()), "xsm_spec_step")

    def xsm_spec_step_static(self, buf: StepBuffers, vp: xsm_verify_params, kv_len_bound: int):
        bt = buf.struct(kv_len_bound)
        self._check(self.L.xsm_spec_step_static(self.h, C.byref(bt), C.byref(vp), self.stream()),
                    "xsm_spec_step_static")

    def xsm_plain_step(self, buf: StepBuffers, vp: xsm_verify_params, kv_len_bound: int):
        bt = buf.struct(kv_len_bound)
        self._check(self.L.xsm_plain_step(self.h, C.byref(bt), C.byref(vp), self.stream()), "xsm_plain_step")

    def xsm_set_option(self, option: int, value: int):
        self._check(self.L.xsm_set_option(self.h, option, value), "xsm_set_option")

    def xsm_debug_kv_clone(self, src_slot: int, dst_slot: int):
        self._check(self.L.xsm_debug_kv_clone(self.h, src_slot, dst_slot), "xsm_debug_kv_clone")

    def xsm_debug_timeline(self) -> np.ndarray:
        out = np.zeros((256, self.c_cfg.n_layers * 16 + 8), np.uint64)
        self._check(self.L.xsm_debug_timeline(self.h, out.ctypes.data, out.size), "xsm_debug_timeline")
        return out

    def xsm_check_device(self):
        self._check(self.L.xsm_check_device(self.h), "xsm_check_device")

    def xsm_debug_inject_device_error(self, code: int):
        self._check(self.L.xsm_debug_inject_device_error(self.h, code), "xsm_debug_inject_device_error")

    def xsm_debug_kv_export(self, layer: int, which: int, slot: int, pos0: int, n_pos: int) -> np.ndarray:
        out = np.empty((self.c_cfg.n_heads, n_pos, self.c_cfg.head_dim), np.float32)
        self._check(self.L.xsm_debug_kv_export(self.h, layer, which, slot, pos0, n_pos, out.ctypes.data),
                    "xsm_debug_kv_export")
        return out

    def xsm_debug_kv_import(self, layer: int, which: int, slot: int, pos0: int, rows: np.ndarray):
        rows = np.ascontiguousarray(rows, dtype=np.float32)
        assert rows.shape[0] == self.c_cfg.n_heads and rows.shape[2] == self.c_cfg.head_dim
        self._check(self.L.xsm_debug_kv_import(self.h, layer, which, slot, pos0, rows.shape[1],
                                               rows.ctypes.data), "xsm_debug_kv_import")
