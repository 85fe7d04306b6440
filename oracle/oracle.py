"""ctypes front end of the float64 CPU oracle (oracle/esrnn_oracle.c).

TEST INFRASTRUCTURE ONLY: argument marshalling around the C oracle, which is
the statement of the method (see esrnn_oracle.h for the passages of the paper
it follows).  Nothing here imports the HIP package.  The configuration is any
object with the fields B, T, n_seas, m1, m2, I, H, hidden, blocks (tuple of
tuples of dilations), tau, lambda_lv, param_space.
"""
from __future__ import annotations

import ctypes as C
import os
from types import SimpleNamespace

import numpy as np

from . import build as _build

_dp = C.POINTER(C.c_double)


class _Config(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("T", C.c_int32),
        ("n_seas", C.c_int32), ("m1", C.c_int32), ("m2", C.c_int32),
        ("I", C.c_int32), ("H", C.c_int32),
        ("hidden", C.c_int32),
        ("n_blocks", C.c_int32),
        ("layers_in_block", C.c_int32 * 4),
        ("dilation", (C.c_int32 * 4) * 4),
        ("param_space", C.c_int32),
        ("tau", C.c_double), ("lambda_lv", C.c_double),
        ("n_pin", C.c_double), ("n_lv", C.c_double),
        ("n_cat", C.c_int32), ("categories", C.POINTER(C.c_int32)),
        ("lambda_c", C.c_double),
        ("pin_side", C.POINTER(C.c_int8)),
    ]


class _Tape(C.Structure):
    _fields_ = [(n, _dp) for n in ("alpha", "gamma1", "gamma2", "l", "S1", "S2", "u", "v",
                                   "X", "Z", "gates", "c", "h", "blk", "a", "o")] + \
               [(n, C.c_double) for n in ("sum_pin", "sum_lv", "n_pin", "n_lv", "sum_cs", "n_cs")]


class _Adjoint(C.Structure):
    _fields_ = [(n, _dp) for n in ("gO", "gR", "gX", "gu", "gv")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        _lib = C.CDLL(path)
        _lib.eso_es_param_rows.restype = C.c_int
        _lib.eso_weight_count.restype = C.c_int64
        _lib.eso_num_layers.restype = C.c_int
        _lib.eso_max_threads.restype = C.c_int
        _lib.eso_forward.restype = C.c_int
        _lib.eso_backward.restype = C.c_int
        _lib.eso_predict.restype = C.c_int
    return _lib


def max_threads() -> int:
    return int(lib().eso_max_threads())


def set_num_threads(n: int) -> None:
    """Host threads of later oracle calls (for timing the baseline on one core)."""
    lib().eso_set_num_threads(C.c_int(int(n)))


def _c_config(cfg, n_pin=0.0, n_lv=0.0, B=None, categories=None) -> _Config:
    c = _Config()
    c.n_cat = int(getattr(cfg, "n_cat", 0))
    c.lambda_c = float(getattr(cfg, "lambda_c", 0.0))
    if c.n_cat > 0:
        if categories is None:
            raise ValueError("oracle: this configuration needs the categories of the series")
        cat = np.ascontiguousarray(categories, dtype=np.int32)
        assert cat.min() >= 0 and cat.max() < c.n_cat
        c._keep = cat                                   # keeps the array alive as long as the struct
        c.categories = cat.ctypes.data_as(C.POINTER(C.c_int32))
    c.B, c.T = int(cfg.B if B is None else B), int(cfg.T)
    c.n_seas, c.m1, c.m2 = int(cfg.n_seas), int(cfg.m1), int(cfg.m2)
    c.I, c.H, c.hidden = int(cfg.I), int(cfg.H), int(cfg.hidden)
    c.n_blocks = len(cfg.blocks)
    for k, blk in enumerate(cfg.blocks):
        c.layers_in_block[k] = len(blk)
        for j, d in enumerate(blk):
            c.dilation[k][j] = int(d)
    c.param_space = int(cfg.param_space)
    c.tau, c.lambda_lv = float(cfg.tau), float(cfg.lambda_lv)
    c.n_pin, c.n_lv = float(n_pin), float(n_lv)
    return c


def _ptr(a):
    return a.ctypes.data_as(_dp)


def forward(cfg, y, lengths, es_params, weights, n_pin=0.0, n_lv=0.0, want_forecasts=True, categories=None):
    """Run the oracle forward.  Inputs are converted to float64; returns a
    namespace with loss, forecasts [P,B,H] and every intermediate (series-major
    arrays, see esrnn_oracle.h)."""
    L_ = lib()
    y = np.ascontiguousarray(y, dtype=np.float64)
    es_params = np.ascontiguousarray(es_params, dtype=np.float64)
    weights = np.ascontiguousarray(weights, dtype=np.float64)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    T, B = y.shape
    cc = _c_config(cfg, n_pin, n_lv, B=B, categories=categories)
    assert T == cfg.T
    K = L_.eso_es_param_rows(C.byref(cc))
    nw = L_.eso_weight_count(C.byref(cc))
    nl = L_.eso_num_layers(C.byref(cc))
    if K < 0:
        raise ValueError("oracle: invalid configuration")
    assert es_params.shape == (K, B), (es_params.shape, K, B)
    assert weights.shape == (nw,), (weights.shape, nw)
    h, I, H = cfg.hidden, cfg.I, cfg.H
    P = T - I - H + 1
    nb = len(cfg.blocks)
    r = SimpleNamespace()
    r.alpha, r.gamma1, r.gamma2 = (np.zeros(B) for _ in range(3))
    r.l, r.S1, r.S2, r.u, r.v = (np.zeros((B, T)) for _ in range(5))
    Iw = I + int(getattr(cfg, "n_cat", 0))
    r.X = np.zeros((B, P, Iw))
    r.Z = np.zeros((B, P, H))
    r.gates = np.zeros((nl, B, P, 4, h))
    r.c = np.zeros((nl, B, P, h))
    r.h = np.zeros((nl, B, P, h))
    r.blk = np.zeros((nb, B, P, h))
    r.a = np.zeros((B, P, h))
    r.o = np.zeros((B, P, H))
    r.forecasts = np.zeros((P, B, H)) if want_forecasts else None
    tape = _Tape()
    for name in ("alpha", "gamma1", "gamma2", "l", "S1", "S2", "u", "v", "X", "Z", "gates", "c", "h",
                 "blk", "a", "o"):
        setattr(tape, name, _ptr(getattr(r, name)))
    loss = C.c_double(0.0)
    rc = L_.eso_forward(C.byref(cc), _ptr(y), lengths.ctypes.data_as(C.POINTER(C.c_int32)),
                        _ptr(es_params), _ptr(weights), C.byref(tape), C.byref(loss),
                        _ptr(r.forecasts) if want_forecasts else None)
    if rc != 0:
        raise ValueError(f"oracle forward failed with code {rc}")
    r.loss = loss.value
    r.sum_pin, r.sum_lv, r.n_pin, r.n_lv = tape.sum_pin, tape.sum_lv, tape.n_pin, tape.n_lv
    r.sum_cs, r.n_cs = tape.sum_cs, tape.n_cs
    r._tape, r._cc = tape, cc
    r._inputs = (y, lengths, es_params, weights)
    r.P, r.K, r.n_layers = P, K, nl
    return r


def backward(cfg, fwd, want_adjoints=True, pin_side=None):
    """Reverse mode for the forward result ``fwd``; returns grad_es_params
    [K,B], grad_weights (flat) and, optionally, the adjoint intermediates.

    ``pin_side`` (int8 [B,P,H], optional) names the one-sided derivative of the
    pinball loss to take at outputs that sit on its kink (+1: the target >=
    output side, -1: the other, 0: decided by the sign as usual)."""
    L_ = lib()
    y, lengths, es_params, weights = fwd._inputs
    if pin_side is not None:
        side = np.ascontiguousarray(pin_side, dtype=np.int8)
        assert side.shape == (y.shape[1], fwd.P, cfg.H), side.shape
        fwd._cc.pin_side = side.ctypes.data_as(C.POINTER(C.c_int8))
    else:
        fwd._cc.pin_side = None
    T, B = y.shape
    h, I, H, P = cfg.hidden, cfg.I, cfg.H, fwd.P
    g = SimpleNamespace()
    g.grad_es_params = np.zeros_like(es_params)
    g.grad_weights = np.zeros_like(weights)
    adj = _Adjoint()
    if want_adjoints:
        g.gO = np.zeros((B, P, H))
        g.gR = np.zeros((B, P, h))
        g.gX = np.zeros((B, P, I + int(getattr(cfg, "n_cat", 0))))
        g.gu = np.zeros((B, T))
        g.gv = np.zeros((B, T))
        for name in ("gO", "gR", "gX", "gu", "gv"):
            setattr(adj, name, _ptr(getattr(g, name)))
    rc = L_.eso_backward(C.byref(fwd._cc), _ptr(y), lengths.ctypes.data_as(C.POINTER(C.c_int32)),
                         _ptr(es_params), _ptr(weights), C.byref(fwd._tape),
                         C.byref(adj) if want_adjoints else None,
                         _ptr(g.grad_es_params), _ptr(g.grad_weights))
    fwd._cc.pin_side = None      # the array above goes out of scope with this call
    if rc != 0:
        raise ValueError(f"oracle backward failed with code {rc}")
    return g


def loss_only(cfg, y, lengths, es_params, weights, **kw) -> float:
    return forward(cfg, y, lengths, es_params, weights, want_forecasts=False, **kw).loss


def predict(cfg, y, lengths, es_params, weights, categories=None):
    """Out-of-sample forecasts [B, H] of the H steps after each series' last
    observation (Section 3.4, Eq. (4), (5)); rows of y past a length are not read."""
    L_ = lib()
    y = np.ascontiguousarray(y, dtype=np.float64)
    es_params = np.ascontiguousarray(es_params, dtype=np.float64)
    weights = np.ascontiguousarray(weights, dtype=np.float64)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    T, B = y.shape
    assert T == cfg.T
    cc = _c_config(cfg, B=B, categories=categories)
    out = np.zeros((B, cfg.H))
    rc = L_.eso_predict(C.byref(cc), _ptr(y), lengths.ctypes.data_as(C.POINTER(C.c_int32)),
                        _ptr(es_params), _ptr(weights), _ptr(out))
    if rc != 0:
        raise ValueError(f"oracle predict failed with code {rc}")
    return out


def smape(forecasts, actuals):
    """Symmetric mean absolute percentage error per series, in percent, as used
    in the M4 competition (Section 3.5 names the metric): mean over the horizon
    of 200 |a - f| / (|a| + |f|).  forecasts, actuals: [B, H]."""
    f = np.asarray(forecasts, dtype=np.float64)
    a = np.asarray(actuals, dtype=np.float64)
    return np.mean(200.0 * np.abs(a - f) / (np.abs(a) + np.abs(f)), axis=1)


def mase(forecasts, actuals, y, lengths, m):
    """Mean absolute scaled error per series (M4 definition): mean absolute
    forecast error divided by the in-sample mean absolute error of the seasonal
    naive forecast with period m, mean over t = m .. len-1 of |y_t - y_{t-m}|.
    y: [T, B] time-major, only rows below lengths[b] are read."""
    f = np.asarray(forecasts, dtype=np.float64)
    a = np.asarray(actuals, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    out = np.zeros(f.shape[0])
    for b in range(f.shape[0]):
        s = y[:int(lengths[b]), b]
        scale = np.mean(np.abs(s[m:] - s[:-m]))
        out[b] = np.mean(np.abs(a[b] - f[b])) / scale
    return out


def adam_update(params, grads, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, clip_norm=0.0):
    """One Adam step (Kingma & Ba 2015, Algorithm 1 with bias correction) on a list of float64 arrays,
    after clipping the gradients by their global L2 norm: g <- g * min(1, clip_norm / (||g|| + 1e-6)).
    ``lr`` is one rate or one per array.  Returns new (params, m, v) lists; inputs are not modified.
    The paper names no optimiser (Section 3.3 only says the two parameter sets are trained jointly);
    this is the published rule."""
    grads = [np.asarray(g, dtype=np.float64) for g in grads]
    lrs = list(lr) if isinstance(lr, (list, tuple)) else [lr] * len(grads)
    scale = 1.0
    if clip_norm > 0.0:
        norm = np.sqrt(sum(float(np.sum(g * g)) for g in grads))
        scale = min(1.0, clip_norm / (norm + 1e-6))
    new_p, new_m, new_v = [], [], []
    for p, g, m_, v_, a in zip(params, grads, m, v, lrs):
        g = g * scale
        m2 = beta1 * np.asarray(m_, dtype=np.float64) + (1.0 - beta1) * g
        v2 = beta2 * np.asarray(v_, dtype=np.float64) + (1.0 - beta2) * g * g
        mhat = m2 / (1.0 - beta1 ** step)
        vhat = v2 / (1.0 - beta2 ** step)
        new_p.append(np.asarray(p, dtype=np.float64) - a * mhat / (np.sqrt(vhat) + eps))
        new_m.append(m2)
        new_v.append(v2)
    return new_p, new_m, new_v



def adam_update_indexed(weights, grad_weights, m_w, v_w, step, es_store, grad_es, m_es, v_es, counts, index,
                        lr, beta1=0.9, beta2=0.999, eps=1e-8, clip_norm=0.0):
    """One training-loop update when the batch is a subset of a store of N series (Section 3.3: every series
    has its own smoothing parameters, N (2 + S) in all, trained jointly with the shared weights; Table 5:
    training runs over epochs of batches).

    The shared weights take a plain Adam step with step counter ``step``.  The per-series parameters live in
    ``es_store`` [K, N] with moments ``m_es``, ``v_es`` [K, N] and one update counter per series ``counts``
    [N]; only the columns named by ``index`` [B] (distinct) are touched: column index[b] takes an Adam step
    with gradient grad_es[:, b] and its own counter counts[index[b]] + 1 in the bias correction, as if that
    series were optimised on its own and simply had no step when it is not in the batch.  The gradient is
    clipped by its global L2 norm over the weights and the batch's per-series gradients, as in adam_update.
    Reading: the paper names neither the optimiser nor how per-series state is handled between batches.
    Returns new (weights, m_w, v_w, es_store, m_es, v_es, counts); inputs are not modified."""
    gw = np.asarray(grad_weights, dtype=np.float64)
    ge = np.asarray(grad_es, dtype=np.float64)
    index = np.asarray(index, dtype=np.int64)
    assert len(np.unique(index)) == len(index), "a series may appear once per batch"
    lr_w, lr_e = lr
    scale = 1.0
    if clip_norm > 0.0:
        norm = np.sqrt(float(np.sum(gw * gw)) + float(np.sum(ge * ge)))
        scale = min(1.0, clip_norm / (norm + 1e-6))
    # shared weights
    g = gw * scale
    m_w2 = beta1 * np.asarray(m_w, dtype=np.float64) + (1.0 - beta1) * g
    v_w2 = beta2 * np.asarray(v_w, dtype=np.float64) + (1.0 - beta2) * g * g
    w2 = np.asarray(weights, dtype=np.float64) - lr_w * (m_w2 / (1.0 - beta1 ** step)) / (
        np.sqrt(v_w2 / (1.0 - beta2 ** step)) + eps)
    # per-series parameters, one series at a time
    es2 = np.array(es_store, dtype=np.float64)
    m_e2 = np.array(m_es, dtype=np.float64)
    v_e2 = np.array(v_es, dtype=np.float64)
    counts2 = np.array(counts, dtype=np.int64)
    for b, n in enumerate(index):
        t = int(counts2[n]) + 1
        g = ge[:, b] * scale
        m_e2[:, n] = beta1 * m_e2[:, n] + (1.0 - beta1) * g
        v_e2[:, n] = beta2 * v_e2[:, n] + (1.0 - beta2) * g * g
        es2[:, n] -= lr_e * (m_e2[:, n] / (1.0 - beta1 ** t)) / (np.sqrt(v_e2[:, n] / (1.0 - beta2 ** t)) + eps)
        counts2[n] = t
    return w2, m_w2, v_w2, es2, m_e2, v_e2, counts2
