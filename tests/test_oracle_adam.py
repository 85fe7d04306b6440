"""Pins of the oracle's parameter update against the library optimiser of PyTorch (CPU, float64, used
as a black box) and against closed forms."""
import numpy as np
import torch

from oracle import oracle


def test_matches_library_adam_and_clipping_over_several_steps():
    rng = np.random.default_rng(0)
    shapes = [(7, 5), (11,)]
    p0 = [rng.normal(size=s) for s in shapes]
    tp = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in p0]
    lrs = [3e-3, 2e-2]
    opt = torch.optim.Adam([{"params": [tp[0]], "lr": lrs[0]}, {"params": [tp[1]], "lr": lrs[1]}],
                           betas=(0.9, 0.999), eps=1e-8)
    p = [x.copy() for x in p0]
    m = [np.zeros(s) for s in shapes]
    v = [np.zeros(s) for s in shapes]
    for step in range(1, 7):
        g = [rng.normal(size=s) * (5.0 if step % 2 else 0.05) for s in shapes]   # clipped and unclipped steps
        for t, gi in zip(tp, g):
            t.grad = torch.tensor(gi, dtype=torch.float64)
        torch.nn.utils.clip_grad_norm_(tp, max_norm=1.5)
        opt.step()
        p, m, v = oracle.adam_update(p, g, m, v, step, lrs, 0.9, 0.999, 1e-8, clip_norm=1.5)
        for a, b in zip(p, tp):
            np.testing.assert_allclose(a, b.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_first_step_moves_by_the_learning_rate_against_the_gradient_sign():
    g = np.array([3.0, -0.2, 1e-3])
    p, m, v = oracle.adam_update([np.zeros(3)], [g], [np.zeros(3)], [np.zeros(3)], 1, 0.01, eps=1e-12)
    np.testing.assert_allclose(p[0], -0.01 * np.sign(g), rtol=1e-8)
    np.testing.assert_allclose(m[0], 0.1 * g)
    np.testing.assert_allclose(v[0], 0.001 * g * g)


def test_clipping_scales_to_the_norm():
    g = [np.array([3.0, 4.0]), np.array([12.0])]          # global norm 13
    _, m, _ = oracle.adam_update([np.zeros(2), np.zeros(1)], g, [np.zeros(2), np.zeros(1)],
                                 [np.zeros(2), np.zeros(1)], 1, 0.1, beta1=0.0, clip_norm=6.5)
    np.testing.assert_allclose(np.concatenate(m), np.array([3.0, 4.0, 12.0]) * 6.5 / (13.0 + 1e-6), rtol=1e-12)
    _, m, _ = oracle.adam_update([np.zeros(2), np.zeros(1)], g, [np.zeros(2), np.zeros(1)],
                                 [np.zeros(2), np.zeros(1)], 1, 0.1, beta1=0.0, clip_norm=20.0)
    np.testing.assert_allclose(np.concatenate(m), [3.0, 4.0, 12.0])
