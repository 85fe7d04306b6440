"""The oracle's hand-written reverse mode against central finite differences of
its own forward (float64), plus gradient invariants.  Covers the joint training
of per-series smoothing parameters and network weights (Section 3.3).  No GPU."""
import numpy as np
import pytest

from oracle import oracle
from paper_1907_03329_amd import synth
from paper_1907_03329_amd.synth import Config, es_param_rows, make_inputs, weight_layout


def cfg_for(kind, **kw):
    base = dict(name=kind, B=3, T=40, n_seas=1, m1=4, m2=0, I=3, H=5, hidden=5, blocks=((1, 2), (3, 5)),
                tau=0.48, lambda_lv=50.0)
    if kind == "none":
        base.update(n_seas=0, m1=0)
    elif kind == "double":
        base.update(n_seas=2, m1=3, m2=7, seas_sd2=0.1)
    elif kind == "long_season":           # period longer than some of the ragged series' usable range
        base.update(m1=12, T=44)
    base.update(kw)
    return Config(**base)


def loss_at(cfg, inp, es, w):
    return oracle.loss_only(cfg, inp["y"], inp["lengths"], es, w)


def fd_check(cfg, inp, n_samples=48, seed=0, rel=1e-6):
    es = inp["es_params"].astype(np.float64)
    w = inp["weights"].astype(np.float64)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], es, w)
    g = oracle.backward(cfg, f)
    rng = np.random.default_rng(seed)
    worst = {}
    # per-series parameter rows
    for name, sl in es_param_rows(cfg).items():
        rows = np.arange(sl.start, sl.stop)
        cand = [(r, b) for r in rows for b in range(cfg.B)]
        pick = [cand[i] for i in rng.permutation(len(cand))[:n_samples]]
        num = np.zeros(len(pick))
        ana = np.zeros(len(pick))
        for i, (r, b) in enumerate(pick):
            step = 1e-6 * max(1.0, abs(es[r, b]))
            ep, em = es.copy(), es.copy()
            ep[r, b] += step
            em[r, b] -= step
            num[i] = (loss_at(cfg, inp, ep, w) - loss_at(cfg, inp, em, w)) / (2 * step)
            ana[i] = g.grad_es_params[r, b]
        scale = max(np.abs(g.grad_es_params[sl]).max(), 1e-30)
        worst[name] = np.abs(num - ana).max() / scale
    for name, off, shape in weight_layout(cfg):
        n = int(np.prod(shape))
        pick = off + rng.permutation(n)[:n_samples]
        num = np.zeros(len(pick))
        for i, q in enumerate(pick):
            step = 1e-6 * max(1.0, abs(w[q]))
            wp, wm = w.copy(), w.copy()
            wp[q] += step
            wm[q] -= step
            num[i] = (loss_at(cfg, inp, es, wp) - loss_at(cfg, inp, es, wm)) / (2 * step)
        scale = max(np.abs(g.grad_weights[off:off + n]).max(), 1e-30)
        worst[name] = np.abs(num - g.grad_weights[pick]).max() / scale
    bad = {k: v for k, v in worst.items() if not v <= rel}
    assert not bad, f"finite-difference mismatch (relative to the group's largest gradient): {bad}"
    return g


@pytest.mark.parametrize("kind,space,ragged", [
    ("single", synth.PARAMS_DIRECT, False),
    ("single", synth.PARAMS_LOGIT, True),
    ("none", synth.PARAMS_DIRECT, True),
    ("none", synth.PARAMS_LOGIT, False),
    ("double", synth.PARAMS_DIRECT, True),
    ("double", synth.PARAMS_LOGIT, False),
    ("long_season", synth.PARAMS_DIRECT, True),
])
def test_gradients_match_central_differences(kind, space, ragged):
    cfg = cfg_for(kind, param_space=space)
    inp = make_inputs(cfg, seed=40, ragged=ragged)
    fd_check(cfg, inp)


def test_gradients_without_penalty_and_single_block():
    cfg = cfg_for("single", lambda_lv=0.0, blocks=((2,),))
    fd_check(cfg, make_inputs(cfg, seed=41))


@pytest.mark.parametrize("kind", ["single", "double"])
def test_gauge_invariant_of_initial_seasonality_gradient(kind):
    """Scaling all initial factors of one seasonality by k divides the level by
    k and changes nothing else, so sum_k s_init[k] * dL/ds_init[k] = 0."""
    cfg = cfg_for(kind)
    inp = make_inputs(cfg, seed=42, ragged=True)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], inp["weights"])
    g = oracle.backward(cfg, f)
    rows = es_param_rows(cfg)
    for name in ("s1_init", "s2_init"):
        if name in rows:
            s = inp["es_params"][rows[name]].astype(np.float64)
            gs = g.grad_es_params[rows[name]]
            inv = np.sum(s * gs, axis=0)
            assert np.abs(inv).max() <= 1e-13 * np.abs(s * gs).sum(axis=0).max()


def test_logit_gradient_is_direct_gradient_times_transform_derivative():
    cfg_d = cfg_for("double")
    inp = make_inputs(cfg_d, seed=43)
    es_d = inp["es_params"].astype(np.float64)
    f_d = oracle.forward(cfg_d, inp["y"], inp["lengths"], es_d, inp["weights"])
    g_d = oracle.backward(cfg_d, f_d)
    cfg_l = cfg_d.with_(param_space=synth.PARAMS_LOGIT)
    es_l = es_d.copy()
    es_l[:3] = np.log(es_d[:3]) - np.log1p(-es_d[:3])
    es_l[3:] = np.log(es_d[3:])
    f_l = oracle.forward(cfg_l, inp["y"], inp["lengths"], es_l, inp["weights"])
    g_l = oracle.backward(cfg_l, f_l)
    np.testing.assert_allclose(f_l.loss, f_d.loss, rtol=1e-12)
    np.testing.assert_allclose(g_l.grad_es_params[:3], g_d.grad_es_params[:3] * es_d[:3] * (1 - es_d[:3]),
                               rtol=1e-9, atol=1e-16)
    np.testing.assert_allclose(g_l.grad_es_params[3:], g_d.grad_es_params[3:] * es_d[3:], rtol=1e-9, atol=1e-16)
    np.testing.assert_allclose(g_l.grad_weights, g_d.grad_weights, rtol=1e-8, atol=1e-16)


def test_weight_gradient_is_sum_over_series_and_es_gradient_is_per_series():
    cfg = cfg_for("single", B=4)
    inp = make_inputs(cfg, seed=44, ragged=True)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], inp["weights"])
    g = oracle.backward(cfg, f)
    gw = np.zeros_like(g.grad_weights)
    for b in range(cfg.B):
        one = synth.take_series(inp, [b])
        f1 = oracle.forward(cfg.with_(B=1), one["y"], one["lengths"], one["es_params"], one["weights"],
                            n_pin=f.n_pin, n_lv=f.n_lv)
        g1 = oracle.backward(cfg.with_(B=1), f1)
        gw += g1.grad_weights
        np.testing.assert_allclose(g1.grad_es_params[:, 0], g.grad_es_params[:, b], rtol=1e-12, atol=1e-18)
    np.testing.assert_allclose(gw, g.grad_weights, rtol=1e-11, atol=1e-17)


def test_adjoint_intermediates_are_consistent():
    """gZ = -gO sums to the stated values; window adjoints conserve mass:
    sum_t gu + sum_t gv = 0 without the penalty (every window entry is v - u)."""
    cfg = cfg_for("single", lambda_lv=0.0)
    inp = make_inputs(cfg, seed=45)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], inp["weights"])
    g = oracle.backward(cfg, f)
    np.testing.assert_allclose(g.gu.sum(axis=1) + g.gv.sum(axis=1), 0.0, atol=1e-15)
    d = f.Z - f.o
    expect = np.where(d >= 0, -cfg.tau, 1 - cfg.tau) / f.n_pin
    np.testing.assert_allclose(g.gO, expect, rtol=1e-15)
