"""Pins of the CPU oracle's smoothing recursions, windows and forecasts against
closed forms and invariants (Section 3.1 Eq. (1), (3), (5), (6); Section 5.3;
Section 8.2).  No GPU."""
import numpy as np
import pytest

from oracle import oracle
from paper_1907_03329_amd import synth
from paper_1907_03329_amd.synth import Config, es_param_rows, make_inputs


def cfg_single(**kw):
    base = dict(name="t", B=5, T=30, n_seas=1, m1=4, m2=0, I=3, H=5, hidden=6, blocks=((1, 2), (3,)),
                tau=0.48, lambda_lv=50.0)
    base.update(kw)
    return Config(**base)


def cfg_none(**kw):
    return cfg_single(n_seas=0, m1=0, **kw)


def cfg_double(**kw):
    base = dict(n_seas=2, m1=3, m2=7, T=40, seas_sd2=0.1)
    base.update(kw)
    return cfg_single(**base)


def run(cfg, inp, **kw):
    return oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], inp["weights"], **kw)


def test_alpha_one_level_is_deseasonalised_observation():
    cfg = cfg_single()
    inp = make_inputs(cfg, seed=1)
    inp["es_params"][es_param_rows(cfg)["alpha"]] = 1.0
    f = run(cfg, inp)
    y = inp["y"].astype(np.float64).T
    np.testing.assert_allclose(f.l, y / f.S1, rtol=1e-14)


def test_gamma_zero_freezes_seasonality():
    cfg = cfg_single()
    inp = make_inputs(cfg, seed=2)
    rows = es_param_rows(cfg)
    inp["es_params"][rows["gamma1"]] = 0.0
    f = run(cfg, inp)
    s_init = inp["es_params"][rows["s1_init"]].astype(np.float64).T  # [B, m]
    t = np.arange(cfg.T)
    np.testing.assert_allclose(f.S1, s_init[:, t % cfg.m1], rtol=1e-15)


def test_constant_series_unit_seasonality_keeps_level():
    cfg = cfg_single()
    inp = make_inputs(cfg, seed=3)
    rows = es_param_rows(cfg)
    inp["y"][:] = 123.5
    inp["es_params"][rows["s1_init"]] = 1.0
    f = run(cfg, inp)
    np.testing.assert_allclose(f.l, 123.5, rtol=1e-14)
    np.testing.assert_allclose(f.S1, 1.0, rtol=1e-14)


def test_exact_seasonal_series_is_a_fixed_point():
    """y_t = c * f[t mod m] with s_init = f: level stays c, factors stay f, for
    any alpha and gamma; windows are all zero and a zero head forecasts y."""
    cfg = cfg_single()
    inp = make_inputs(cfg, seed=4)
    rows = es_param_rows(cfg)
    f_true = inp["es_params"][rows["s1_init"]].astype(np.float64)  # [m, B]
    c = np.linspace(50.0, 900.0, cfg.B)
    t = np.arange(cfg.T)
    y = (c[None, :] * f_true[t % cfg.m1, :]).astype(np.float32)
    inp["y"] = y
    # zero head: o = 0
    for name, off, shape in synth.weight_layout(cfg):
        if name in ("Wo", "bo"):
            inp["weights"][off:off + int(np.prod(shape))] = 0.0
    f = run(cfg, inp)
    y64 = y.astype(np.float64).T
    # y was rounded to float32, so the fixed point holds to float32 rounding
    np.testing.assert_allclose(f.l, np.broadcast_to(c[:, None], f.l.shape), rtol=3e-7)
    np.testing.assert_allclose(f.S1, f_true.T[:, t % cfg.m1], rtol=3e-7)
    assert np.abs(f.X).max() < 1e-6 and np.abs(f.Z).max() < 1e-6
    P, I, H = f.P, cfg.I, cfg.H
    for p in (0, 3, P - 1):
        tt = p + I - 1
        np.testing.assert_allclose(f.forecasts[p], y64[:, tt + 1: tt + 1 + H], rtol=1e-6)


def test_level_only_is_simple_exponential_smoothing():
    cfg = cfg_none()
    inp = make_inputs(cfg, seed=5)
    f = run(cfg, inp)
    y = inp["y"].astype(np.float64)
    alpha = inp["es_params"][0].astype(np.float64)
    for t in (0, 1, 7, cfg.T - 1):
        k = np.arange(t)
        closed = (1 - alpha) ** t * y[0] + alpha * sum((1 - alpha) ** kk * y[t - kk] for kk in k)
        np.testing.assert_allclose(f.l[:, t], closed, rtol=1e-13)
    np.testing.assert_array_equal(f.S1, 1.0)
    np.testing.assert_allclose(f.v, np.log(y.T), rtol=1e-15)


def test_geometric_series_windows_and_zero_penalty():
    """Level-only, alpha = 1, y_t = c g^t: u is linear in t, so the windows are
    x[p,i] = (i - I + 1) ln g and z[p,j] = j ln g, and the level penalty is 0."""
    cfg = cfg_none(lambda_lv=7.0)
    inp = make_inputs(cfg, seed=6)
    g = 1.01
    c = np.linspace(10.0, 20.0, cfg.B)
    inp["y"] = (c[None, :] * g ** np.arange(cfg.T)[:, None]).astype(np.float32)
    inp["es_params"][0] = 1.0
    f = run(cfg, inp)
    I, H = cfg.I, cfg.H
    lg = np.log(g)
    np.testing.assert_allclose(f.X, np.broadcast_to((np.arange(I) - I + 1) * lg, f.X.shape), atol=2e-6)
    np.testing.assert_allclose(f.Z, np.broadcast_to(np.arange(1, H + 1) * lg, f.Z.shape), atol=2e-6)
    assert f.sum_lv / f.n_lv < 1e-12  # float32 rounding of y only


def test_scale_equivariance():
    cfg = cfg_double()
    inp = make_inputs(cfg, seed=7)
    f1 = run(cfg, inp)
    inp2 = dict(inp)
    inp2["y"] = inp["y"] * np.float32(8.0)  # exact in float32
    f2 = run(cfg, inp2)
    np.testing.assert_allclose(f2.l, 8.0 * f1.l, rtol=1e-13)
    np.testing.assert_allclose(f2.S1, f1.S1, rtol=1e-13)
    np.testing.assert_allclose(f2.S2, f1.S2, rtol=1e-13)
    np.testing.assert_allclose(f2.X, f1.X, atol=1e-12)
    np.testing.assert_allclose(f2.Z, f1.Z, atol=1e-12)
    np.testing.assert_allclose(f2.loss, f1.loss, rtol=1e-11)
    np.testing.assert_allclose(f2.forecasts, 8.0 * f1.forecasts, rtol=1e-10)


@pytest.mark.parametrize("which", ["s1_init", "s2_init"])
def test_regauging_initial_seasonality_leaves_loss_unchanged(which):
    cfg = cfg_double()
    inp = make_inputs(cfg, seed=8)
    f1 = run(cfg, inp)
    inp2 = {k: v.copy() for k, v in inp.items()}
    inp2["es_params"][es_param_rows(cfg)[which]] *= np.float32(2.0)
    f2 = run(cfg, inp2)
    np.testing.assert_allclose(f2.l, f1.l / 2.0, rtol=1e-13)
    np.testing.assert_allclose(f2.loss, f1.loss, rtol=1e-11)
    np.testing.assert_allclose(f2.forecasts, f1.forecasts, rtol=1e-10)


def test_double_seasonal_reduces_to_single_and_to_ses():
    cfg2 = cfg_double()
    inp2 = make_inputs(cfg2, seed=9)
    rows2 = es_param_rows(cfg2)
    inp2["es_params"][rows2["gamma2"]] = 0.0
    inp2["es_params"][rows2["s2_init"]] = 1.0
    f2 = run(cfg2, inp2)
    cfg1 = cfg2.with_(n_seas=1, m2=0)
    rows1 = es_param_rows(cfg1)
    es1 = np.zeros((cfg1.K, cfg1.B), dtype=np.float32)
    es1[rows1["alpha"]] = inp2["es_params"][rows2["alpha"]]
    es1[rows1["gamma1"]] = inp2["es_params"][rows2["gamma1"]]
    es1[rows1["s1_init"]] = inp2["es_params"][rows2["s1_init"]]
    f1 = oracle.forward(cfg1, inp2["y"], inp2["lengths"], es1, inp2["weights"])
    np.testing.assert_allclose(f2.l, f1.l, rtol=1e-14)
    np.testing.assert_allclose(f2.S1, f1.S1, rtol=1e-14)
    np.testing.assert_array_equal(f2.S2, 1.0)
    np.testing.assert_allclose(f2.loss, f1.loss, rtol=1e-13)
    # both seasonalities trivial -> simple exponential smoothing
    inp2["es_params"][rows2["gamma1"]] = 0.0
    inp2["es_params"][rows2["s1_init"]] = 1.0
    f3 = run(cfg2, inp2)
    cfg0 = cfg2.with_(n_seas=0, m1=0, m2=0)
    f0 = oracle.forward(cfg0, inp2["y"], inp2["lengths"], inp2["es_params"][:1], inp2["weights"])
    np.testing.assert_allclose(f3.l, f0.l, rtol=1e-14)
    np.testing.assert_allclose(f3.loss, f0.loss, rtol=1e-13)


def test_double_seasonal_symmetric_under_swapping_the_two_seasonalities():
    """Swapping (m1, gamma1, s1_init) with (m2, gamma2, s2_init) is the same model."""
    cfg = cfg_double()
    inp = make_inputs(cfg, seed=10)
    rows = es_param_rows(cfg)
    f = run(cfg, inp)
    cfg_s = cfg.with_(m1=cfg.m2, m2=cfg.m1)
    rows_s = es_param_rows(cfg_s)
    es = np.zeros_like(inp["es_params"])
    es[rows_s["alpha"]] = inp["es_params"][rows["alpha"]]
    es[rows_s["gamma1"]] = inp["es_params"][rows["gamma2"]]
    es[rows_s["gamma2"]] = inp["es_params"][rows["gamma1"]]
    es[rows_s["s1_init"]] = inp["es_params"][rows["s2_init"]]
    es[rows_s["s2_init"]] = inp["es_params"][rows["s1_init"]]
    fs = oracle.forward(cfg_s, inp["y"], inp["lengths"], es, inp["weights"])
    np.testing.assert_allclose(fs.l, f.l, rtol=1e-13)
    np.testing.assert_allclose(fs.S1, f.S2, rtol=1e-13)
    np.testing.assert_allclose(fs.S2, f.S1, rtol=1e-13)
    np.testing.assert_allclose(fs.loss, f.loss, rtol=1e-12)


def test_logit_space_matches_direct_space_forward():
    cfg_d = cfg_double()
    cfg_l = cfg_d.with_(param_space=synth.PARAMS_LOGIT)
    inp_d = make_inputs(cfg_d, seed=11)
    inp_l = make_inputs(cfg_l, seed=11)
    fd, fl = run(cfg_d, inp_d), run(cfg_l, inp_l)
    # the float32 rounding of the parameters differs between the two spaces
    np.testing.assert_allclose(fl.alpha, fd.alpha, rtol=1e-6)
    np.testing.assert_allclose(fl.l, fd.l, rtol=1e-4)
    np.testing.assert_allclose(fl.loss, fd.loss, rtol=1e-3)
    a = inp_l["es_params"][0].astype(np.float64)
    np.testing.assert_allclose(fl.alpha, 1.0 / (1.0 + np.exp(-a)), rtol=1e-15)
    s = inp_l["es_params"][es_param_rows(cfg_l)["s2_init"]].astype(np.float64)
    np.testing.assert_allclose(fl.S2[:, :cfg_l.m2], np.exp(s).T, rtol=1e-15)


def test_padding_is_ignored_and_short_series_equal_truncated_run():
    cfg = cfg_single(B=4)
    inp = make_inputs(cfg, seed=12, ragged=True)
    f = run(cfg, inp)
    g = oracle.backward(cfg, f)
    # garbage in the padding changes nothing
    inp2 = {k: v.copy() for k, v in inp.items()}
    pad = np.arange(cfg.T)[:, None] >= inp["lengths"][None, :]
    assert pad.any()
    inp2["y"][pad] = 77.0
    f2 = run(cfg, inp2)
    g2 = oracle.backward(cfg, f2)
    assert f2.loss == f.loss
    np.testing.assert_array_equal(g2.grad_es_params, g.grad_es_params)
    # (weight gradients are summed over threads in a run-dependent order)
    np.testing.assert_allclose(g2.grad_weights, g.grad_weights, rtol=1e-12, atol=1e-18)
    # the shortest series alone, run at T := its length, with the batch's normalisers
    b = int(np.argmin(inp["lengths"]))
    n = int(inp["lengths"][b])
    assert n < cfg.T
    one = synth.take_series(inp, [b])
    one["y"] = np.ascontiguousarray(one["y"][:n])
    cfg1 = cfg.with_(B=1, T=n)
    f1 = oracle.forward(cfg1, one["y"], one["lengths"], one["es_params"], one["weights"],
                        n_pin=f.n_pin, n_lv=f.n_lv)
    g1 = oracle.backward(cfg1, f1)
    np.testing.assert_allclose(g1.grad_es_params[:, 0], g.grad_es_params[:, b], rtol=1e-12, atol=1e-18)
    Pb = n - cfg.I - cfg.H + 1
    np.testing.assert_allclose(f1.forecasts[:, 0], f.forecasts[:Pb, b], rtol=1e-13)
    assert np.all(f.forecasts[Pb:, b] == 0.0)
    # loss of the batch = sum over single-series runs with the batch's normalisers
    total = 0.0
    for bb in range(cfg.B):
        o1 = synth.take_series(inp, [bb])
        total += oracle.forward(cfg.with_(B=1), o1["y"], o1["lengths"], o1["es_params"], o1["weights"],
                                n_pin=f.n_pin, n_lv=f.n_lv).loss
    np.testing.assert_allclose(total, f.loss, rtol=1e-13)
