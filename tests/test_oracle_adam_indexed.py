"""Pins of the oracle's update for batches drawn from a store of N series (oracle.adam_update_indexed).

Two epochs of random batches over N series must give, for every series, exactly what the dense update
(oracle.adam_update, itself pinned against the library optimiser of PyTorch) gives when it is applied to that
series alone at the steps where the series was in the batch; series that never appear keep parameters,
moments and counter bit for bit; with clipping the scale is the one of the whole batch.  No GPU."""
import numpy as np
import torch

from oracle import oracle


def run_epochs(N, B, K, nw, epochs, clip, seed, skip=()):
    rng = np.random.default_rng(seed)
    w = rng.normal(size=nw)
    es = rng.normal(size=(K, N))
    state = dict(w=w, m_w=np.zeros(nw), v_w=np.zeros(nw), es=es, m_e=np.zeros((K, N)), v_e=np.zeros((K, N)),
                 counts=np.zeros(N, dtype=np.int64))
    history = []      # (step, index, gw, ge, scale)
    step = 0
    pool = np.array([n for n in range(N) if n not in skip])
    for _ in range(epochs):
        perm = rng.permutation(pool)
        for s in range(0, len(perm) - B + 1, B):
            index = perm[s:s + B]
            step += 1
            gw = rng.normal(size=nw) * (4.0 if step % 2 else 0.1)
            ge = rng.normal(size=(K, B)) * (4.0 if step % 2 else 0.1)
            out = oracle.adam_update_indexed(state["w"], gw, state["m_w"], state["v_w"], step, state["es"], ge,
                                             state["m_e"], state["v_e"], state["counts"], index, (3e-3, 2e-2),
                                             0.9, 0.999, 1e-8, clip)
            state = dict(zip(("w", "m_w", "v_w", "es", "m_e", "v_e", "counts"), out))
            norm = np.sqrt((gw ** 2).sum() + (ge ** 2).sum())
            history.append((step, index.copy(), gw, ge, min(1.0, clip / (norm + 1e-6)) if clip > 0 else 1.0))
    return es, state, history


def test_two_epochs_equal_the_dense_update_series_by_series():
    N, B, K, nw = 12, 4, 5, 9
    for clip in (0.0, 3.0):
        es0, state, history = run_epochs(N, B, K, nw, epochs=2, clip=clip, seed=1)
        for n in range(N):
            # the dense update on this series alone, fed the (already scaled) gradients of its own steps
            p, m, v = [es0[:, n].copy()], [np.zeros(K)], [np.zeros(K)]
            t = 0
            for step, index, gw, ge, scale in history:
                hit = np.nonzero(index == n)[0]
                if len(hit):
                    t += 1
                    p, m, v = oracle.adam_update(p, [ge[:, hit[0]] * scale], m, v, t, 2e-2, 0.9, 0.999, 1e-8, 0.0)
            assert t == 2 and state["counts"][n] == 2
            np.testing.assert_allclose(state["es"][:, n], p[0], rtol=1e-13, atol=1e-15)
            np.testing.assert_allclose(state["m_e"][:, n], m[0], rtol=1e-13, atol=1e-15)
            np.testing.assert_allclose(state["v_e"][:, n], v[0], rtol=1e-13, atol=1e-15)


def test_shared_weights_take_the_library_adam_step_with_the_batch_scale():
    N, B, K, nw = 12, 4, 5, 9
    es0, state, history = run_epochs(N, B, K, nw, epochs=2, clip=3.0, seed=2)
    rng = np.random.default_rng(2)
    w0 = rng.normal(size=nw)
    tw = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tw], lr=3e-3, betas=(0.9, 0.999), eps=1e-8)
    for step, index, gw, ge, scale in history:
        tw.grad = torch.tensor(gw * scale, dtype=torch.float64)
        opt.step()
    np.testing.assert_allclose(state["w"], tw.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_series_outside_every_batch_are_untouched_bit_for_bit():
    N, B, K, nw = 14, 4, 3, 5
    es0, state, _ = run_epochs(N, B, K, nw, epochs=2, clip=3.0, seed=3, skip=(2, 9))
    for n in (2, 9):
        assert np.array_equal(state["es"][:, n], es0[:, n])
        assert not state["m_e"][:, n].any() and not state["v_e"][:, n].any() and state["counts"][n] == 0
    assert state["counts"].sum() == 2 * 12


def test_full_batch_reduces_to_the_dense_update():
    rng = np.random.default_rng(4)
    K, N, nw = 4, 6, 7
    w, es = rng.normal(size=nw), rng.normal(size=(K, N))
    gw, ge = rng.normal(size=nw), rng.normal(size=(K, N))
    mw, vw, me, ve = rng.normal(size=nw) * .1, rng.random(nw) * .1, rng.normal(size=(K, N)) * .1, rng.random((K, N)) * .1
    out = oracle.adam_update_indexed(w, gw, mw, vw, 3, es, ge, me, ve, np.full(N, 2), np.arange(N), (1e-3, 1e-2),
                                     0.9, 0.999, 1e-8, 1.5)
    p, m, v = oracle.adam_update([w, es], [gw, ge], [mw, me], [vw, ve], 3, [1e-3, 1e-2], 0.9, 0.999, 1e-8, 1.5)
    np.testing.assert_allclose(out[0], p[0], rtol=1e-14)
    np.testing.assert_allclose(out[3], p[1], rtol=1e-14)
    np.testing.assert_allclose(out[4], m[1], rtol=1e-14)
    np.testing.assert_allclose(out[5], v[1], rtol=1e-14)
