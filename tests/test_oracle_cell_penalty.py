"""Pins of the cell-state penalty (Section 8.4: the mean of the squared cell states of the first layer of
every block enters the loss).  No GPU."""
import numpy as np

from oracle import oracle
from paper_1907_03329_amd import synth


def cfg_pen(**kw):
    base = dict(name="cpen", B=4, T=36, n_seas=1, m1=4, m2=0, I=3, H=5, hidden=5, blocks=((1, 2), (3, 1), (2,)),
                tau=0.48, lambda_lv=50.0, lambda_c=0.3)
    base.update(kw)
    return synth.Config(**base)


def test_penalty_is_the_plain_mean_of_squares_of_the_first_layers():
    cfg = cfg_pen()
    inp = synth.make_inputs(cfg, seed=1, ragged=True)
    f1 = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], inp["weights"])
    f0 = oracle.forward(cfg.with_(lambda_c=0.0), inp["y"], inp["lengths"], inp["es_params"], inp["weights"])
    first_layers = [0, 2, 4]                              # blocks (1,2), (3,1), (2,)
    Pb = inp["lengths"].astype(int) - cfg.I - cfg.H + 1
    vals = np.concatenate([f0.c[l][b, :Pb[b], :].ravel() for l in first_layers for b in range(cfg.B)])
    np.testing.assert_allclose(f1.loss - f0.loss, cfg.lambda_c * np.mean(vals ** 2), rtol=1e-10)
    assert f1.n_cs == vals.size
    np.testing.assert_array_equal(f1.forecasts, f0.forecasts)        # the forward values themselves do not change


def test_gradients_by_finite_differences_with_the_penalty():
    cfg = cfg_pen(B=3, lambda_c=5.0)                    # large weight so that the term matters in the gradient
    inp = synth.make_inputs(cfg, seed=2, ragged=True)
    es, w = inp["es_params"].astype(np.float64), inp["weights"].astype(np.float64)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], es, w)
    g = oracle.backward(cfg, f)
    g0 = oracle.backward(cfg.with_(lambda_c=0.0), oracle.forward(cfg.with_(lambda_c=0.0), inp["y"], inp["lengths"], es, w))
    assert np.abs(g.grad_weights - g0.grad_weights).max() > 1e-3 * np.abs(g0.grad_weights).max()
    rng = np.random.default_rng(0)
    for name, off, shape in synth.weight_layout(cfg):
        n = int(np.prod(shape))
        scale = max(np.abs(g.grad_weights[off:off + n]).max(), 1e-12)
        for q in off + rng.permutation(n)[:8]:
            step = 1e-6 * max(1.0, abs(w[q]))
            wp, wm = w.copy(), w.copy()
            wp[q] += step
            wm[q] -= step
            num = (oracle.loss_only(cfg, inp["y"], inp["lengths"], es, wp)
                   - oracle.loss_only(cfg, inp["y"], inp["lengths"], es, wm)) / (2 * step)
            assert abs(num - g.grad_weights[q]) <= 2e-6 * scale, (name, q)
    for r in range(es.shape[0]):
        for b in range(cfg.B):
            step = 1e-6 * max(1.0, abs(es[r, b]))
            ep, em = es.copy(), es.copy()
            ep[r, b] += step
            em[r, b] -= step
            num = (oracle.loss_only(cfg, inp["y"], inp["lengths"], ep, w)
                   - oracle.loss_only(cfg, inp["y"], inp["lengths"], em, w)) / (2 * step)
            assert abs(num - g.grad_es_params[r, b]) <= 2e-6 * np.abs(g.grad_es_params[r]).max(), (r, b)


def test_layers_after_the_first_of_a_block_are_not_penalised():
    """Scaling the output gate of a block's second layer changes that layer's hidden state but no
    first-layer cell state of its own block or of earlier blocks; with one block of two layers the
    penalty term must not move when only the second layer's weights change."""
    cfg = cfg_pen(blocks=((1, 2),), lambda_c=1.0)
    inp = synth.make_inputs(cfg, seed=3)
    w = inp["weights"].astype(np.float64)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], w)
    lay = {name: (off, shape) for name, off, shape in synth.weight_layout(cfg)}
    off, shape = lay["W1"]
    w2 = w.copy()
    w2[off:off + int(np.prod(shape))] *= 1.7
    f2 = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], w2)
    np.testing.assert_allclose(f.sum_cs, f2.sum_cs, rtol=1e-14)
    assert f.loss != f2.loss
