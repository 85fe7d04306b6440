"""Pins of the oracle's out-of-sample forecast (Section 3.4, Eq. (4), (5)) and of the
two accuracy metrics the paper names (Section 3.5), all on the CPU."""
import numpy as np
import pytest

from oracle import oracle
from paper_1907_03329_amd import synth


def cfg_small(**kw):
    base = dict(name="p", B=5, T=48, n_seas=1, m1=4, m2=0, I=4, H=6, hidden=6, blocks=((1, 2), (3,)),
                tau=0.48, lambda_lv=50.0, param_space=0)
    base.update(kw)
    return synth.Config(**base)


def test_matches_training_forecast_at_the_same_position():
    """A forecast made from the first n observations is the training pass's forecast for the window
    ending at n-1 of the longer series, for the steps whose seasonal factor the recursion had already
    produced at time n-1 (h <= m): same level, same network state (causal), same factors."""
    cfg = cfg_small()
    inp = synth.make_inputs(cfg, seed=3)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], inp["weights"])
    for n in (cfg.I, 17, cfg.T - cfg.H):
        short = np.full(cfg.B, n, dtype=np.int32)
        got = oracle.predict(cfg, inp["y"], short, inp["es_params"], inp["weights"])
        p = n - cfg.I
        want = f.forecasts[p]                      # [B, H]
        hmax = min(cfg.m1, cfg.H)
        np.testing.assert_allclose(got[:, :hmax], want[:, :hmax], rtol=1e-12)


def test_rows_past_the_length_are_not_read():
    cfg = cfg_small()
    inp = synth.make_inputs(cfg, seed=4)
    n = np.array([10, 20, 30, 40, 44], dtype=np.int32)
    a = oracle.predict(cfg, inp["y"], n, inp["es_params"], inp["weights"])
    y2 = inp["y"].copy()
    for b in range(cfg.B):
        y2[n[b]:, b] = np.nan
    b_ = oracle.predict(cfg, y2, n, inp["es_params"], inp["weights"])
    np.testing.assert_array_equal(a, b_)


def test_seasonal_factors_repeat_with_their_period():
    """Eq. (4): with a head that outputs zero the forecast is level x factor, and the factor of step
    h + m is that of step h."""
    cfg = cfg_small(H=11)
    inp = synth.make_inputs(cfg, seed=5)
    w = inp["weights"].astype(np.float64)
    lay = {name: (off, shape) for name, off, shape in synth.weight_layout(cfg)}
    for name in ("Wo", "bo"):
        off, shape = lay[name]
        w[off:off + int(np.prod(shape))] = 0.0
    n = np.full(cfg.B, 30, dtype=np.int32)
    got = oracle.predict(cfg, inp["y"], n, inp["es_params"], w)
    np.testing.assert_allclose(got[:, cfg.m1:], got[:, :-cfg.m1], rtol=1e-13)
    # and the first m steps are level x the last m factors of the recursion on the first 30 observations
    f = oracle.forward(cfg.with_(T=30 + cfg.m1 + 1, H=1, I=4), inp["y"][:30 + cfg.m1 + 1],
                       np.full(cfg.B, 30 + cfg.m1 + 1, dtype=np.int32), inp["es_params"],
                       synth.make_inputs(cfg.with_(T=30 + cfg.m1 + 1, H=1, I=4), seed=5)["weights"])
    for h in range(1, cfg.m1 + 1):
        np.testing.assert_allclose(got[:, h - 1], f.l[:, 29] * f.S1[:, 29 + h], rtol=1e-12)


def test_exactly_seasonal_series_is_continued():
    """A series level x periodic factors with the true factors as initial seasonality is a fixed point
    of the smoothing; a zero head then forecasts its continuation exactly, also beyond one period."""
    cfg = cfg_small(H=9, B=3)
    inp = synth.make_inputs(cfg, seed=6)
    prof = np.array([[0.8, 1.1, 1.3, 0.8], [1.2, 0.9, 0.7, 1.2], [1.0, 1.0, 1.0, 1.0]])
    prof = prof / prof.mean(axis=1, keepdims=True)
    level = np.array([100.0, 7.0, 3000.0])
    t = np.arange(cfg.T + cfg.H)
    full = level[None, :] * prof[np.arange(3)[None, :], (t % 4)[:, None]]
    es = inp["es_params"].astype(np.float64)      # float64 so that the profile is exact
    rows = synth.es_param_rows(cfg)
    es[rows["s1_init"]] = prof.T
    w = inp["weights"].astype(np.float64)
    lay = {name: (off, shape) for name, off, shape in synth.weight_layout(cfg)}
    for name in ("Wo", "bo"):
        off, shape = lay[name]
        w[off:off + int(np.prod(shape))] = 0.0
    n = np.array([21, 34, 48], dtype=np.int32)
    got = oracle.predict(cfg, full[:cfg.T].astype(np.float64), n, es, w)
    for b in range(3):
        np.testing.assert_allclose(got[b], full[n[b]:n[b] + cfg.H, b], rtol=1e-12)


def test_level_only_forecast_is_flat_level_times_exp_output():
    cfg = cfg_small(n_seas=0, m1=0, H=5)
    inp = synth.make_inputs(cfg, seed=7)
    w = inp["weights"].astype(np.float64)
    lay = {name: (off, shape) for name, off, shape in synth.weight_layout(cfg)}
    off, shape = lay["Wo"]
    w[off:off + int(np.prod(shape))] = 0.0
    off, shape = lay["bo"]
    bo = np.linspace(-0.2, 0.3, cfg.H)
    w[off:off + cfg.H] = bo
    n = np.full(cfg.B, 25, dtype=np.int32)
    got = oracle.predict(cfg, inp["y"], n, inp["es_params"], w)
    # simple exponential smoothing in closed form
    alpha = inp["es_params"][0].astype(np.float64)
    y = inp["y"].astype(np.float64)
    l = y[0].copy()
    for t in range(1, 25):
        l = alpha * y[t] + (1 - alpha) * l
    np.testing.assert_allclose(got, l[:, None] * np.exp(bo)[None, :], rtol=1e-12)


def test_double_seasonality_uses_both_periods():
    cfg = cfg_small(n_seas=2, m1=3, m2=5, H=12, T=60)
    inp = synth.make_inputs(cfg, seed=8)
    w = inp["weights"].astype(np.float64)
    lay = {name: (off, shape) for name, off, shape in synth.weight_layout(cfg)}
    for name in ("Wo", "bo"):
        off, shape = lay[name]
        w[off:off + int(np.prod(shape))] = 0.0
    n = np.full(cfg.B, 41, dtype=np.int32)
    got = oracle.predict(cfg, inp["y"], n, inp["es_params"], w)
    # period of the product pattern is lcm(3, 5) = 15 > H, but the pattern factorises: f[h] = L a[h mod 3] b[h mod 5]
    r = got / got[:, :1]
    # ratios f[h+3]/f[h] depend on h mod 5 only through b, f[h+5]/f[h] on a only: check the cross identity
    for h in range(cfg.H - 8):
        np.testing.assert_allclose(r[:, h + 8] * r[:, h], r[:, h + 3] * r[:, h + 5], rtol=1e-12)


def test_metrics_closed_forms():
    a = np.array([[100.0, 200.0, 50.0]])
    np.testing.assert_allclose(oracle.smape(a, a), [0.0])
    np.testing.assert_allclose(oracle.smape(np.zeros_like(a) + 1e-300, a), [200.0])
    np.testing.assert_allclose(oracle.smape(3.0 * a, a), [100.0])           # 200 * 2a / 4a
    # a forecast that repeats the last period of a series that grows by c per period has MASE 1, 2, ... per period
    m, c = 4, 5.0
    t = np.arange(40)
    y = (10.0 + c * (t // m) + (t % m))[:, None]
    n = np.array([32], dtype=np.int32)
    actual = y[32:40, 0][None, :]
    naive = np.concatenate([y[28:32, 0], y[28:32, 0]])[None, :]
    np.testing.assert_allclose(oracle.mase(naive, actual, y, n, m), [1.5])  # errors c, c, c, c, 2c, 2c, 2c, 2c over scale c
    np.testing.assert_allclose(oracle.mase(actual, actual, y, n, m), [0.0])
