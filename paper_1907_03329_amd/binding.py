"""Thin ctypes binding of the HIP library (C ABI in include/esrnn.h).

Argument marshalling only: every step of the training step runs in the
library's kernels.  PyTorch is used for device memory and the current stream.
There is no CPU fallback: if the shared library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libesrnn_hip.so")

ESRNN_OK = 0
PARAMS_DIRECT, PARAMS_LOGIT = 0, 1
LAYOUT_TIME_MAJOR, LAYOUT_TILE, LAYOUT_GATE_TILE = 0, 1, 2
BUFFERS = {name: i for i, name in enumerate([
    "level", "S1", "S2", "u", "v", "X", "Z", "gates", "c", "hid", "block_out", "O",
    "grad_O", "grad_top", "grad_X", "grad_u", "grad_v"])}


class EsrnnConfig(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("T", C.c_int32),
        ("n_seas", C.c_int32), ("m1", C.c_int32), ("m2", C.c_int32),
        ("I", C.c_int32), ("H", C.c_int32),
        ("hidden", C.c_int32),
        ("n_blocks", C.c_int32),
        ("layers_in_block", C.c_int32 * 4),
        ("dilation", (C.c_int32 * 4) * 4),
        ("tau", C.c_float), ("lambda_lv", C.c_float),
        ("param_space", C.c_int32),
        ("n_categories", C.c_int32),
        ("lambda_cs", C.c_float),
    ]


class AdamConfig(C.Structure):
    _fields_ = [("lr_weights", C.c_float), ("lr_es", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("clip_norm", C.c_float)]


class BufferView(C.Structure):
    _fields_ = [("offset_bytes", C.c_size_t), ("layout", C.c_int32), ("dims", C.c_int32 * 4)]


class EsrnnError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({status_string(status)})")
        self.status = status


_lib = None


def load_library():
    """Load libesrnn_hip.so (built in-tree by build.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_1907_03329_amd.build` "
            "(there is no fallback implementation)")
    lib = C.CDLL(LIB_PATH)
    vp, i32p, fp = C.c_void_p, C.c_void_p, C.c_void_p
    lib.esrnn_create.argtypes = [C.POINTER(EsrnnConfig), C.POINTER(vp)]
    lib.esrnn_destroy.argtypes = [vp]
    lib.esrnn_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
    lib.esrnn_check_workspace.argtypes = [vp, vp, C.c_size_t, C.c_int32]
    lib.esrnn_check_workspace.restype = C.c_int
    lib.esrnn_es_param_rows.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.esrnn_weight_count.argtypes = [vp, C.POINTER(C.c_size_t)]
    lib.esrnn_status_string.argtypes = [C.c_int]
    lib.esrnn_status_string.restype = C.c_char_p
    lib.esrnn_forward.argtypes = [vp, fp, i32p, fp, fp, vp, fp, fp, vp]
    lib.esrnn_backward.argtypes = [vp, fp, i32p, fp, fp, vp, fp, fp, vp]
    lib.esrnn_workspace_buffer.argtypes = [vp, C.c_int32, C.c_int32, C.POINTER(BufferView)]
    lib.esrnn_es_window_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
    lib.esrnn_es_window_forward.argtypes = [vp, fp, i32p, fp, vp, vp]
    lib.esrnn_es_window_backward.argtypes = [vp, fp, i32p, fp, vp, fp, vp]
    for fn in ("esrnn_es_window_workspace_bytes", "esrnn_es_window_forward", "esrnn_es_window_backward"):
        getattr(lib, fn).restype = C.c_int
    lib.esrnn_set_forward_only.argtypes = [vp, C.c_int32]
    lib.esrnn_set_forward_only.restype = C.c_int
    lib.esrnn_set_categories.argtypes = [vp, i32p]
    lib.esrnn_set_categories.restype = C.c_int
    lib.esrnn_adam_update.argtypes = [vp, C.POINTER(AdamConfig), C.c_int32, fp, fp, fp, fp, fp, fp, fp, fp, vp, vp]
    lib.esrnn_adam_update.restype = C.c_int
    lib.esrnn_gather_batch.argtypes = [vp, fp, i32p, fp, i32p, C.c_int32, fp, i32p, fp, vp]
    lib.esrnn_gather_batch.restype = C.c_int
    lib.esrnn_adam_update_indexed.argtypes = [vp, C.POINTER(AdamConfig), C.c_int32, fp, fp, fp, fp, fp, fp, fp, fp,
                                              i32p, i32p, C.c_int32, vp, vp]
    lib.esrnn_adam_update_indexed.restype = C.c_int
    lib.esrnn_predict.argtypes = [vp, fp, i32p, fp, fp, vp, fp, vp]
    lib.esrnn_predict_static.argtypes = [vp, fp, i32p, fp, fp, fp, vp]
    lib.esrnn_forecast_metrics.argtypes = [vp, fp, fp, fp, i32p, C.c_int32, fp, fp, vp]
    for fn in ("esrnn_predict", "esrnn_predict_static", "esrnn_forecast_metrics"):
        getattr(lib, fn).restype = C.c_int
    lib.esrnn_profile_enable.argtypes = [vp, C.c_int32]
    lib.esrnn_profile_stage_count.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.esrnn_profile_stage_name.argtypes = [vp, C.c_int32, C.POINTER(C.c_char_p)]
    lib.esrnn_profile_collect.argtypes = [vp]
    lib.esrnn_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int32)]
    lib.esrnn_probe_issue_overlap.argtypes = [C.c_int32, C.c_int32, C.c_int32, fp, vp]
    lib.esrnn_probe_issue_overlap.restype = C.c_int
    for fn in ("esrnn_profile_enable", "esrnn_profile_stage_count", "esrnn_profile_stage_name",
               "esrnn_profile_collect", "esrnn_profile_read"):
        getattr(lib, fn).restype = C.c_int
    for fn in ("esrnn_create", "esrnn_destroy", "esrnn_workspace_bytes", "esrnn_es_param_rows",
               "esrnn_weight_count", "esrnn_forward", "esrnn_backward", "esrnn_workspace_buffer"):
        getattr(lib, fn).restype = C.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().esrnn_status_string(int(status)).decode()


def make_config(cfg) -> EsrnnConfig:
    """Build the C struct from any object with fields B, T, n_seas, m1, m2, I, H,
    hidden, blocks, tau, lambda_lv, param_space and, optionally, n_cat."""
    c = EsrnnConfig()
    c.B, c.T = int(cfg.B), int(cfg.T)
    c.n_seas, c.m1, c.m2 = int(cfg.n_seas), int(cfg.m1), int(cfg.m2)
    c.I, c.H, c.hidden = int(cfg.I), int(cfg.H), int(cfg.hidden)
    if len(cfg.blocks) > 4 or any(len(b) > 4 for b in cfg.blocks):
        raise EsrnnError(2, "make_config")
    c.n_blocks = len(cfg.blocks)
    for k, blk in enumerate(cfg.blocks):
        c.layers_in_block[k] = len(blk)
        for j, d in enumerate(blk):
            c.dilation[k][j] = int(d)
    c.tau, c.lambda_lv = float(cfg.tau), float(cfg.lambda_lv)
    c.param_space = int(cfg.param_space)
    c.n_categories = int(getattr(cfg, "n_cat", 0))
    c.lambda_cs = float(getattr(cfg, "lambda_c", 0.0))
    return c


def esrnn_create(cfg) -> C.c_void_p:
    lib = load_library()
    h = C.c_void_p()
    cc = cfg if isinstance(cfg, EsrnnConfig) else make_config(cfg)
    st = lib.esrnn_create(C.byref(cc), C.byref(h))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_create")
    return h


def esrnn_destroy(handle) -> None:
    st = load_library().esrnn_destroy(handle)
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_destroy")


def esrnn_workspace_bytes(handle) -> int:
    n = C.c_size_t()
    st = load_library().esrnn_workspace_bytes(handle, C.byref(n))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_workspace_bytes")
    return int(n.value)


def esrnn_check_workspace(handle, workspace, es_window_only: bool = False) -> None:
    """Raises EsrnnError unless the tensor is large enough and aligned for this handle (host-side check)."""
    st = load_library().esrnn_check_workspace(handle, C.c_void_p(workspace.data_ptr()),
                                              workspace.numel() * workspace.element_size(), 1 if es_window_only else 0)
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_check_workspace")


def esrnn_es_param_rows(handle) -> int:
    k = C.c_int32()
    st = load_library().esrnn_es_param_rows(handle, C.byref(k))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_es_param_rows")
    return int(k.value)


def esrnn_weight_count(handle) -> int:
    n = C.c_size_t()
    st = load_library().esrnn_weight_count(handle, C.byref(n))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_weight_count")
    return int(n.value)


def esrnn_workspace_buffer(handle, which, index: int = 0) -> BufferView:
    v = BufferView()
    w = BUFFERS[which] if isinstance(which, str) else int(which)
    st = load_library().esrnn_workspace_buffer(handle, w, int(index), C.byref(v))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_workspace_buffer")
    return v


def esrnn_profile_enable(handle, on: bool) -> None:
    st = load_library().esrnn_profile_enable(handle, 1 if on else 0)
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_profile_enable")


def esrnn_profile_collect(handle) -> None:
    st = load_library().esrnn_profile_collect(handle)
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_profile_collect")


def esrnn_profile_read(handle):
    """Returns [(stage name, total milliseconds, collected launches)]."""
    lib = load_library()
    n = C.c_int32()
    st = lib.esrnn_profile_stage_count(handle, C.byref(n))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_profile_stage_count")
    ms = (C.c_double * n.value)()
    cnt = (C.c_int32 * n.value)()
    st = lib.esrnn_profile_read(handle, ms, cnt)
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_profile_read")
    out = []
    for i in range(n.value):
        name = C.c_char_p()
        st = lib.esrnn_profile_stage_name(handle, i, C.byref(name))
        if st != ESRNN_OK:
            raise EsrnnError(st, "esrnn_profile_stage_name")
        out.append((name.value.decode(), float(ms[i]), int(cnt[i])))
    return out


def _ptr(t, dtype=None, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise EsrnnError(1, "null tensor")
    import torch
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors passed to the library must be contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def esrnn_forward(handle, y, lengths, es_params, weights, workspace, loss, forecasts=None, stream=None) -> None:
    import torch
    st = load_library().esrnn_forward(handle, _ptr(y, torch.float32), _ptr(lengths, torch.int32),
                                      _ptr(es_params, torch.float32), _ptr(weights, torch.float32),
                                      _ptr(workspace), _ptr(loss, torch.float32),
                                      _ptr(forecasts, torch.float32, allow_none=True), _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_forward")


def esrnn_backward(handle, y, lengths, es_params, weights, workspace, grad_es_params, grad_weights,
                   stream=None) -> None:
    import torch
    st = load_library().esrnn_backward(handle, _ptr(y, torch.float32), _ptr(lengths, torch.int32),
                                       _ptr(es_params, torch.float32), _ptr(weights, torch.float32),
                                       _ptr(workspace), _ptr(grad_es_params, torch.float32),
                                       _ptr(grad_weights, torch.float32), _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_backward")


def esrnn_es_window_workspace_bytes(handle) -> int:
    n = C.c_size_t()
    st = load_library().esrnn_es_window_workspace_bytes(handle, C.byref(n))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_es_window_workspace_bytes")
    return int(n.value)


def esrnn_es_window_forward(handle, y, lengths, es_params, workspace, stream=None) -> None:
    import torch
    st = load_library().esrnn_es_window_forward(handle, _ptr(y, torch.float32), _ptr(lengths, torch.int32),
                                                _ptr(es_params, torch.float32), _ptr(workspace), _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_es_window_forward")


def esrnn_es_window_backward(handle, y, lengths, es_params, workspace, grad_es_params, stream=None) -> None:
    import torch
    st = load_library().esrnn_es_window_backward(handle, _ptr(y, torch.float32), _ptr(lengths, torch.int32),
                                                 _ptr(es_params, torch.float32), _ptr(workspace),
                                                 _ptr(grad_es_params, torch.float32), _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_es_window_backward")


def esrnn_set_forward_only(handle, on: bool) -> None:
    st = load_library().esrnn_set_forward_only(handle, 1 if on else 0)
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_set_forward_only")


def esrnn_set_categories(handle, categories) -> None:
    import torch
    st = load_library().esrnn_set_categories(handle, _ptr(categories, torch.int32, allow_none=True))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_set_categories")


def esrnn_adam_update(handle, opt: "AdamConfig", step, weights, grad_weights, m_weights, v_weights,
                      es_params, grad_es_params, m_es, v_es, workspace, stream=None) -> None:
    import torch
    f = torch.float32
    st = load_library().esrnn_adam_update(handle, C.byref(opt), int(step), _ptr(weights, f), _ptr(grad_weights, f),
                                          _ptr(m_weights, f), _ptr(v_weights, f), _ptr(es_params, f),
                                          _ptr(grad_es_params, f), _ptr(m_es, f), _ptr(v_es, f), _ptr(workspace),
                                          _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_adam_update")


def esrnn_gather_batch(handle, y_store, lengths_store, es_store, index, y, lengths, es_params, stream=None) -> None:
    import torch
    f, i = torch.float32, torch.int32
    st = load_library().esrnn_gather_batch(handle, _ptr(y_store, f), _ptr(lengths_store, i), _ptr(es_store, f),
                                           _ptr(index, i), int(lengths_store.numel()), _ptr(y, f), _ptr(lengths, i),
                                           _ptr(es_params, f), _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_gather_batch")


def esrnn_adam_update_indexed(handle, opt: "AdamConfig", step, weights, grad_weights, m_weights, v_weights,
                              es_store, grad_es_params, m_es_store, v_es_store, counts_store, index, workspace,
                              stream=None) -> None:
    import torch
    f, i = torch.float32, torch.int32
    st = load_library().esrnn_adam_update_indexed(
        handle, C.byref(opt), int(step), _ptr(weights, f), _ptr(grad_weights, f), _ptr(m_weights, f),
        _ptr(v_weights, f), _ptr(es_store, f), _ptr(grad_es_params, f), _ptr(m_es_store, f), _ptr(v_es_store, f),
        _ptr(counts_store, i), _ptr(index, i), int(counts_store.numel()), _ptr(workspace), _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_adam_update_indexed")


def esrnn_predict(handle, y, lengths, es_params, weights, workspace, forecasts, stream=None) -> None:
    import torch
    st = load_library().esrnn_predict(handle, _ptr(y, torch.float32), _ptr(lengths, torch.int32),
                                      _ptr(es_params, torch.float32), _ptr(weights, torch.float32), _ptr(workspace),
                                      _ptr(forecasts, torch.float32), _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_predict")


def esrnn_predict_static(handle, y, lengths, es_params, weights, forecasts, stream=None) -> None:
    import torch
    st = load_library().esrnn_predict_static(handle, _ptr(y, torch.float32), _ptr(lengths, torch.int32),
                                             _ptr(es_params, torch.float32), _ptr(weights, torch.float32),
                                             _ptr(forecasts, torch.float32), _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_predict_static")


def esrnn_forecast_metrics(handle, forecasts, actuals, y, lengths, m, smape, mase, stream=None) -> None:
    import torch
    st = load_library().esrnn_forecast_metrics(handle, _ptr(forecasts, torch.float32), _ptr(actuals, torch.float32),
                                               _ptr(y, torch.float32), _ptr(lengths, torch.int32), int(m),
                                               _ptr(smape, torch.float32), _ptr(mase, torch.float32), _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_forecast_metrics")


def esrnn_probe_issue_overlap(mode: int, iterations: int, per_cu: int, out, stream=None) -> None:
    """Diagnostic launch (see include/esrnn.h); `out` is a device float32 tensor of 256 * per_cu * 256 elements."""
    import torch
    if out.numel() < 256 * per_cu * 256:
        raise ValueError("out is too small")
    st = load_library().esrnn_probe_issue_overlap(int(mode), int(iterations), int(per_cu), _ptr(out, torch.float32),
                                                  _stream(stream))
    if st != ESRNN_OK:
        raise EsrnnError(st, "esrnn_probe_issue_overlap")


class TrainingStep:
    """Owns a handle plus the device buffers of one forward/backward pair."""

    def __init__(self, cfg, device="cuda:0", want_forecasts: bool = True):
        import torch
        self.cfg = cfg
        self.device = torch.device(device)
        self.handle = esrnn_create(cfg)
        self.K = esrnn_es_param_rows(self.handle)
        self.n_weights = esrnn_weight_count(self.handle)
        self.workspace_bytes = esrnn_workspace_bytes(self.handle)
        self.P = cfg.T - cfg.I - cfg.H + 1
        self.workspace = torch.empty(self.workspace_bytes // 4, dtype=torch.float32, device=self.device)
        assert self.workspace.data_ptr() % 256 == 0
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.device)
        self.forecasts = (torch.empty((self.P, cfg.B, cfg.H), dtype=torch.float32, device=self.device)
                          if want_forecasts else None)
        self.grad_es_params = torch.empty((self.K, cfg.B), dtype=torch.float32, device=self.device)
        self.grad_weights = torch.empty(self.n_weights, dtype=torch.float32, device=self.device)

    def set_categories(self, categories):
        """Device int32 tensor [B]; kept referenced here so that it outlives the calls that read it."""
        self._categories = categories
        esrnn_set_categories(self.handle, categories)

    def forward(self, y, lengths, es_params, weights, stream=None):
        esrnn_forward(self.handle, y, lengths, es_params, weights, self.workspace, self.loss, self.forecasts, stream)

    def backward(self, y, lengths, es_params, weights, stream=None):
        esrnn_backward(self.handle, y, lengths, es_params, weights, self.workspace, self.grad_es_params,
                       self.grad_weights, stream)

    def predict(self, y, lengths, es_params, weights, stream=None):
        """Out-of-sample forecasts [B, H] (new tensor).  A later backward() needs a new forward()."""
        import torch
        out = torch.empty((self.cfg.B, self.cfg.H), dtype=torch.float32, device=self.device)
        esrnn_predict(self.handle, y, lengths, es_params, weights, self.workspace, out, stream)
        return out

    def buffer(self, which, index: int = 0):
        """Logical view of a workspace intermediate as a new tensor:
        time-major -> [T, B]; tile -> [P, B, rows]; gate tile -> [P, B, rows, 4]."""
        v = esrnn_workspace_buffer(self.handle, which, index)
        lead, Bp, R, logical = (int(x) for x in v.dims)
        off = v.offset_bytes // 4
        B = self.cfg.B
        if v.layout == LAYOUT_TIME_MAJOR:
            return self.workspace[off: off + lead * Bp].view(lead, Bp)[:, :B].clone()
        inner = 4 if v.layout == LAYOUT_GATE_TILE else 1
        n = lead * Bp * R * inner
        t = self.workspace[off: off + n].view(lead, Bp // 16, R, 16, inner)
        t = t.permute(0, 1, 3, 2, 4).reshape(lead, Bp, R, inner)[:, :B, :logical]
        return t.clone() if inner == 4 else t[..., 0].clone()

    def close(self):
        if self.handle is not None:
            esrnn_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
