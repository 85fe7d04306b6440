"""GPU parity: the HIP training step against the float64 CPU oracle, tensor by
tensor, through the C ABI.  Sizes span several 16-series tiles with a ragged
last tile; lengths are ragged where stated."""
import numpy as np
import pytest

from paper_1907_03329_amd import synth
from paper_1907_03329_amd.synth import CONFIGS, Config

pytestmark = pytest.mark.gpu

from tests import gpu_common as gc  # noqa: E402


def small(name, **kw):
    base = dict(name=name, B=37, T=40, n_seas=1, m1=4, m2=0, I=4, H=8, hidden=8, blocks=((1, 2), (4, 8)),
                tau=0.48, lambda_lv=50.0)
    base.update(kw)
    return Config(**base)


def report(errs):
    errs = {k: v for k, v in errs.items() if k != "series_at_kink"}
    worst = sorted(errs.items(), key=lambda kv: -kv[1])[:4]
    print("  worst:", ", ".join(f"{k}={v:.2e}" for k, v in worst), flush=True)


@pytest.mark.parametrize("ragged", [False, True])
def test_tiny_quarterly_config(ragged):
    errs = gc.run_and_check(CONFIGS["tiny_quarterly"], seed=0, ragged=ragged)
    report(errs)


@pytest.mark.parametrize("space", [synth.PARAMS_DIRECT, synth.PARAMS_LOGIT])
def test_single_seasonality_small_hidden(space):
    errs = gc.run_and_check(small("single_h8", param_space=space), seed=1, ragged=True)
    report(errs)


def test_level_only():
    cfg = small("none_h8", n_seas=0, m1=0, I=6, H=6, blocks=((1, 2), (2, 6)), step_mu=0.01, step_sd=0.05, noise_sd=0.03)
    report(gc.run_and_check(cfg, seed=2, ragged=True))


@pytest.mark.parametrize("space", [synth.PARAMS_DIRECT, synth.PARAMS_LOGIT])
def test_double_seasonality(space):
    cfg = small("double_h8", T=60, n_seas=2, m1=3, m2=7, seas_sd2=0.1, I=5, H=6, param_space=space,
                blocks=((1, 3), (5,)))
    report(gc.run_and_check(cfg, seed=3, ragged=True))


def test_hidden_30_shape_of_yearly():
    cfg = CONFIGS["yearly"].with_(B=50)
    report(gc.run_and_check(cfg, seed=4, ragged=True))


def test_hidden_40_shape_of_quarterly_several_tiles():
    cfg = CONFIGS["quarterly"].with_(B=70)
    report(gc.run_and_check(cfg, seed=5, ragged=True))


def test_hidden_50_shape_of_monthly():
    cfg = CONFIGS["monthly"].with_(B=21, T=90)
    report(gc.run_and_check(cfg, seed=6, ragged=True))


def test_shape_of_hourly_short():
    cfg = CONFIGS["hourly"].with_(B=19, T=300)
    report(gc.run_and_check(cfg, seed=7, ragged=False))


def test_three_blocks_and_single_layer_blocks():
    cfg = small("three_blocks", blocks=((1,), (2,), (3, 1)), hidden=5, I=3, H=5)
    report(gc.run_and_check(cfg, seed=8, ragged=True))


def test_four_blocks():
    # the last layer of the first block receives gradient from the output stage and from three later blocks
    cfg = small("four_blocks", blocks=((1, 2), (1,), (3,), (2, 4)), hidden=7, I=4, H=3, B=21)
    report(gc.run_and_check(cfg, seed=21, ragged=True))


def test_maximum_sizes():
    # hidden, input window and horizon at the limits of the library (largest kernel shapes; the output
    # stage reads all its weight operands from LDS)
    cfg = small("max_sizes", hidden=64, I=64, H=64, T=140, B=20, blocks=((1, 2), (3,)), m1=12)
    report(gc.run_and_check(cfg, seed=22, ragged=True))


def test_wide_horizon_medium_hidden():
    # hidden 50 with a 40-step horizon: output stage with its transposed operands in LDS
    cfg = small("h50_H40", hidden=50, I=12, H=40, T=100, B=35, blocks=((1, 3), (6,)), m1=12)
    report(gc.run_and_check(cfg, seed=23, ragged=True))


def test_input_window_padded_to_hidden_tiles():
    # I = 13 has no dedicated kernel shape with hidden 30: the input is padded to the hidden tile count
    cfg = small("padded_input", hidden=30, I=13, H=3, T=48)
    report(gc.run_and_check(cfg, seed=9, ragged=True))


def test_no_penalty_and_other_quantile():
    cfg = small("tau_0.3", lambda_lv=0.0, tau=0.3)
    report(gc.run_and_check(cfg, seed=10, ragged=False))


def test_batch_of_one_and_exact_tile():
    report(gc.run_and_check(small("one", B=1), seed=11))
    report(gc.run_and_check(small("sixteen", B=16), seed=12))


def test_minimum_length_series():
    """Series whose length equals I + H have exactly one window."""
    cfg = small("minlen", B=20)

    def mutate(inp):
        inp["lengths"][:] = cfg.I + cfg.H
        inp["lengths"][0] = cfg.T
        inp["y"][np.arange(cfg.T)[:, None] >= inp["lengths"][None, :]] = 1.0

    report(gc.run_and_check(cfg, seed=13, mutate=mutate))


def test_padding_values_are_ignored():
    import torch
    from paper_1907_03329_amd import binding
    cfg = small("pad", B=20)
    inp = synth.make_inputs(cfg, seed=14, ragged=True)
    s1 = gc.run_gpu(cfg, inp)
    inp2 = {k: v.copy() for k, v in inp.items()}
    pad = np.arange(cfg.T)[:, None] >= inp["lengths"][None, :]
    inp2["y"][pad] = -5.0      # would be NaN under a logarithm
    s2 = gc.run_gpu(cfg, inp2)
    assert torch.equal(s1.loss, s2.loss)
    assert torch.equal(s1.forecasts, s2.forecasts)
    assert torch.equal(s1.grad_es_params, s2.grad_es_params)
    assert torch.equal(s1.grad_weights, s2.grad_weights)


def test_results_are_deterministic():
    import torch
    cfg = small("det", B=40)
    inp = synth.make_inputs(cfg, seed=15, ragged=True)
    s1, s2 = gc.run_gpu(cfg, inp), gc.run_gpu(cfg, inp)
    assert torch.equal(s1.loss, s2.loss)
    assert torch.equal(s1.grad_weights, s2.grad_weights)
    assert torch.equal(s1.grad_es_params, s2.grad_es_params)


def test_single_window_position():
    """T = I + H: exactly one window position, every recurrence has one step."""
    cfg = small("one_position", T=12, I=4, H=8, B=18)
    report(gc.run_and_check(cfg, seed=16))


def test_dilation_longer_than_the_window_sequence():
    """Dilations beyond the number of positions: the state never arrives, every chain has one step."""
    cfg = small("long_dilation", T=20, I=4, H=8, blocks=((1, 12), (30,)), B=18)
    report(gc.run_and_check(cfg, seed=17, ragged=True))


def test_period_close_to_series_length():
    """Seasonal period of the order of the shortest series: most initial factors are never updated."""
    cfg = small("long_period", T=40, m1=24, I=4, H=8, B=33)

    def mutate(inp):
        inp["lengths"][1::2] = 14      # shorter than the period (I + H = 12 <= 14 < 24)
        inp["y"][np.arange(cfg.T)[:, None] >= inp["lengths"][None, :]] = 1.0

    report(gc.run_and_check(cfg, seed=18, mutate=mutate))


def test_large_dilations_many_chains():
    """Hourly-like dilations (24, 168) on a short batch: many workgroups per series tile."""
    cfg = small("chains", T=260, n_seas=2, m1=24, m2=168, seas_sd2=0.1, I=24, H=48, hidden=40,
                blocks=((1, 4), (24, 168)), B=20)
    report(gc.run_and_check(cfg, seed=19))


def test_extreme_smoothing_parameters():
    """alpha -> 1 and gamma -> 0 (closed-form cases of the smoothing recursions) on the GPU."""
    cfg = small("extreme", B=20)

    def mutate(inp):
        rows = synth.es_param_rows(cfg)
        inp["es_params"][rows["alpha"], :10] = 1.0
        inp["es_params"][rows["gamma1"], 5:15] = 0.0

    errs = gc.run_and_check(cfg, seed=20, mutate=mutate)
    report(errs)


def test_backward_before_forward_is_refused():
    import torch
    from paper_1907_03329_amd import binding
    cfg = small("order", B=16)
    step = binding.TrainingStep(cfg)
    dev = gc.to_device(synth.make_inputs(cfg, seed=21))
    with pytest.raises(binding.EsrnnError) as ei:
        step.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    assert ei.value.status == 4
    step.forward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    step.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    torch.cuda.synchronize()
    step.close()


def test_forward_only_gives_the_same_loss_and_forecasts_and_refuses_backward():
    import torch
    from paper_1907_03329_amd import binding
    cfg = small("fwd_only", B=40)
    inp = synth.make_inputs(cfg, seed=25, ragged=True)
    dev = gc.to_device(inp)
    ref = gc.run_gpu(cfg, inp, backward=False)
    step = binding.TrainingStep(cfg)
    binding.esrnn_set_forward_only(step.handle, True)
    step.forward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    torch.cuda.synchronize()
    assert torch.equal(step.loss, ref.loss)
    assert torch.equal(step.forecasts, ref.forecasts)
    with pytest.raises(binding.EsrnnError) as ei:
        step.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    assert ei.value.status == 4
    binding.esrnn_set_forward_only(step.handle, False)
    step.forward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    step.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    ref.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    torch.cuda.synchronize()
    assert torch.equal(step.grad_weights, ref.grad_weights)
    step.close(); ref.close()


def test_long_seasonal_periods_use_large_lds():
    """Periods whose rings need more than 64 KB of LDS per 64 series (the attribute that allows it is set
    once per kernel): 200 + 120 periods -> 80 KB."""
    cfg = small("long_rings", T=420, n_seas=2, m1=200, m2=120, seas_sd2=0.1, I=4, H=8, B=20, blocks=((1, 2),))
    report(gc.run_and_check(cfg, seed=26))
    report(gc.run_and_check(cfg, seed=27, ragged=True))


def test_seasonal_periods_at_the_limit():
    """m1 + m2 = 448, the most the library accepts: rings of 112 KB beside the staging buffers of the smoothing
    kernels (128 KB of LDS per workgroup in the forward, 148 KB in the reverse recursion)."""
    cfg = small("ring_limit", T=470, n_seas=2, m1=300, m2=148, seas_sd2=0.1, I=4, H=8, B=70, blocks=((1, 2),))
    report(gc.run_and_check(cfg, seed=28, ragged=True))


def test_forecasts_may_be_omitted_and_stream_is_honoured():
    import torch
    from paper_1907_03329_amd import binding
    cfg = small("nofc", B=24)
    inp = synth.make_inputs(cfg, seed=22)
    dev = gc.to_device(inp)
    ref = gc.run_gpu(cfg, inp)
    step = binding.TrainingStep(cfg, want_forecasts=False)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step.forward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"], stream=side)
        step.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"], stream=side)
    side.synchronize()
    assert torch.equal(step.loss, ref.loss)
    assert torch.equal(step.grad_weights, ref.grad_weights)
    assert torch.equal(step.grad_es_params, ref.grad_es_params)


def test_smoothing_and_window_entry_points_alone():
    """esrnn_es_window_forward / _backward on the workspace prefix: windows against the oracle, and the
    smoothing gradients for window gradients taken from the oracle's reverse sweep."""
    import torch
    from oracle import oracle
    from paper_1907_03329_amd import binding
    cfg = small("es_only", T=60, n_seas=2, m1=3, m2=7, seas_sd2=0.1, I=5, H=6, B=45, blocks=((1, 3), (5,)))
    inp = synth.make_inputs(cfg, seed=23, ragged=True)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], inp["weights"])
    g = oracle.backward(cfg, f)
    dev = gc.to_device(inp)
    h = binding.esrnn_create(cfg)
    nbytes = binding.esrnn_es_window_workspace_bytes(h)
    assert nbytes < binding.esrnn_workspace_bytes(h)
    ws = torch.zeros(nbytes // 4, dtype=torch.float32, device="cuda")
    binding.esrnn_es_window_forward(h, dev["y"], dev["lengths"], dev["es_params"], ws)

    def view(name):
        v = binding.esrnn_workspace_buffer(h, name)
        lead, Bp, R, logical = (int(x) for x in v.dims)
        assert v.offset_bytes + 4 * lead * Bp * max(R, 1) <= nbytes
        return v, ws[v.offset_bytes // 4: v.offset_bytes // 4 + lead * Bp * max(R, 1)]

    def untile(name):
        v, flat = view(name)
        lead, Bp, R, logical = (int(x) for x in v.dims)
        return flat.view(lead, Bp // 16, R, 16).permute(0, 1, 3, 2).reshape(lead, Bp, R)[:, :cfg.B, :logical].cpu().numpy()

    def tile_into(name, arr):   # arr [P, B, rows]
        v, flat = view(name)
        lead, Bp, R, logical = (int(x) for x in v.dims)
        full = np.zeros((lead, Bp, R), dtype=np.float32)
        full[:, :cfg.B, :logical] = arr
        t = torch.from_numpy(full).cuda().view(lead, Bp // 16, 16, R).permute(0, 1, 3, 2).contiguous()
        flat.copy_(t.view(-1))

    wm = gc.valid_window_mask(cfg, inp["lengths"])
    assert gc.rel_err(untile("X"), f.X.transpose(1, 0, 2), wm) <= gc.TOL_FWD
    assert gc.rel_err(untile("Z"), f.Z.transpose(1, 0, 2), wm) <= gc.TOL_FWD
    tile_into("grad_X", g.gX.transpose(1, 0, 2))
    tile_into("grad_O", g.gO.transpose(1, 0, 2))
    ges = torch.empty((cfg.K, cfg.B), dtype=torch.float32, device="cuda")
    binding.esrnn_es_window_backward(h, dev["y"], dev["lengths"], dev["es_params"], ws, ges)
    torch.cuda.synchronize()
    got = ges.cpu().numpy()
    for name, sl in synth.es_param_rows(cfg).items():
        e = gc.rel_err(got[sl], g.grad_es_params[sl])
        assert e <= gc.TOL_GRAD, f"grad_{name}: {e:.3e}"
    binding.esrnn_destroy(h)


def test_large_batch_small_network():
    """65541 series (4097 series tiles, the last one ragged): the launch shapes of the streaming kernels at
    a batch far above the benchmark's; small network, ragged lengths."""
    cfg = small("large_batch", B=65536 + 5, T=26, I=5, H=6, hidden=5, blocks=((1,), (2,)), m1=3)
    errs = gc.run_and_check(cfg, seed=24, ragged=True)
    report(errs)
