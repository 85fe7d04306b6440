"""Training over a store of N series in batches of B (esrnn_gather_batch, esrnn_adam_update_indexed) against
the float64 oracle: two epochs of random batches over N = 4 B ragged series, every call through the C ABI.
Per-series parameters, moments and counters of the store are compared after every step; series outside a
batch must stay bit-identical."""
import numpy as np
import pytest

from oracle import oracle
from paper_1907_03329_amd import binding, synth
from paper_1907_03329_amd.synth import CONFIGS

pytestmark = pytest.mark.gpu

B1, B2, EPS = (float(np.float32(x)) for x in (0.9, 0.999, 1e-8))


def f32(x):
    return float(np.float32(x))


def rel(a, b):
    return float(np.abs(np.asarray(a, dtype=np.float64) - b).max() / np.abs(b).max())


def test_gather_copies_the_batch_out_of_the_store():
    import torch
    cfg = CONFIGS["tiny_quarterly"].with_(B=19)
    N = 70
    store = synth.make_inputs(cfg.with_(B=N), seed=3, ragged=True)
    idx = np.random.default_rng(0).permutation(N)[:cfg.B].astype(np.int32)
    h = binding.esrnn_create(cfg)
    d = {k: torch.from_numpy(v).cuda() for k, v in store.items()}
    y = torch.empty((cfg.T, cfg.B), dtype=torch.float32, device="cuda")
    n = torch.empty(cfg.B, dtype=torch.int32, device="cuda")
    es = torch.empty((cfg.K, cfg.B), dtype=torch.float32, device="cuda")
    binding.esrnn_gather_batch(h, d["y"], d["lengths"], d["es_params"], torch.from_numpy(idx).cuda(), y, n, es)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy(), store["y"][:, idx])
    assert np.array_equal(n.cpu().numpy(), store["lengths"][idx])
    assert np.array_equal(es.cpu().numpy(), store["es_params"][:, idx])
    binding.esrnn_destroy(h)


def test_two_epochs_over_a_store_follow_the_oracle():
    import torch
    cfg = CONFIGS["tiny_quarterly"].with_(B=16)
    N, epochs = 4 * cfg.B, 2
    store = synth.make_inputs(cfg.with_(B=N), seed=5, ragged=True)
    lrs, clip = [2e-3, 5e-3], 20.0
    opt = binding.AdamConfig(lrs[0], lrs[1], 0.9, 0.999, 1e-8, clip)
    step = binding.TrainingStep(cfg, want_forecasts=False)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    y_s, n_s, es_s, w_d = dev(store["y"]), dev(store["lengths"]), dev(store["es_params"]), dev(store["weights"].copy())
    m_w, v_w = torch.zeros_like(w_d), torch.zeros_like(w_d)
    m_e, v_e = torch.zeros_like(es_s), torch.zeros_like(es_s)
    counts = torch.zeros(N, dtype=torch.int32, device="cuda")
    y = torch.empty((cfg.T, cfg.B), dtype=torch.float32, device="cuda")
    n = torch.empty(cfg.B, dtype=torch.int32, device="cuda")
    es = torch.empty((cfg.K, cfg.B), dtype=torch.float32, device="cuda")
    # oracle state
    o = dict(w=store["weights"].astype(np.float64), m_w=np.zeros(cfg.weight_count), v_w=np.zeros(cfg.weight_count),
             es=store["es_params"].astype(np.float64), m_e=np.zeros((cfg.K, N)), v_e=np.zeros((cfg.K, N)),
             counts=np.zeros(N, dtype=np.int64))
    rng = np.random.default_rng(9)
    t = 0
    for _ in range(epochs):
        perm = rng.permutation(N).astype(np.int32)
        for s in range(0, N, cfg.B):
            idx = perm[s:s + cfg.B]
            t += 1
            before = es_s.clone()
            idx_d = dev(idx)
            binding.esrnn_gather_batch(step.handle, y_s, n_s, es_s, idx_d, y, n, es)
            step.forward(y, n, es, w_d)
            step.backward(y, n, es, w_d)
            binding.esrnn_adam_update_indexed(step.handle, opt, t, w_d, step.grad_weights, m_w, v_w, es_s,
                                              step.grad_es_params, m_e, v_e, counts, idx_d, step.workspace)
            f = oracle.forward(cfg, store["y"][:, idx], store["lengths"][idx], o["es"][:, idx], o["w"], want_forecasts=False)
            g = oracle.backward(cfg, f, want_adjoints=False)
            out = oracle.adam_update_indexed(o["w"], g.grad_weights, o["m_w"], o["v_w"], t, o["es"], g.grad_es_params,
                                             o["m_e"], o["v_e"], o["counts"], idx, [f32(x) for x in lrs], B1, B2, EPS, f32(clip))
            o = dict(zip(("w", "m_w", "v_w", "es", "m_e", "v_e", "counts"), out))
            assert abs(step.loss.item() - f.loss) / abs(f.loss) <= 1e-4, t
            assert rel(w_d.cpu().numpy(), o["w"]) <= 1e-3, t
            assert rel(es_s.cpu().numpy(), o["es"]) <= 1e-3, t
            assert rel(m_e.cpu().numpy(), o["m_e"]) <= 1e-3 and rel(v_e.cpu().numpy(), o["v_e"]) <= 2e-3, t
            assert np.array_equal(counts.cpu().numpy(), o["counts"])
            rest = np.setdiff1d(np.arange(N), idx)
            assert torch.equal(es_s[:, rest], before[:, rest]), "series outside the batch must not change"
    assert counts.min().item() == epochs and counts.max().item() == epochs
    step.close()
