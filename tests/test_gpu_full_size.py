"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times: loss, every forecast and every gradient tensor against the float64 CPU
oracle run on the whole batch (the oracle needs 5-20 s per workload on the GPU
box's host cores), plus a gradient invariant that holds at any size."""
import numpy as np
import pytest

from paper_1907_03329_amd import synth
from paper_1907_03329_amd.synth import CONFIGS

pytestmark = pytest.mark.gpu

from tests import gpu_common as gc  # noqa: E402


def gauge_invariant(cfg, inp, step):
    """sum_k s_init[k] * dL/ds_init[k] = 0 for every series and seasonality:
    scaling all initial factors rescales the level and nothing else."""
    rows = synth.es_param_rows(cfg)
    ges = step.grad_es_params.cpu().numpy().astype(np.float64)
    for name in ("s1_init", "s2_init"):
        if name in rows:
            s = inp["es_params"][rows[name]].astype(np.float64)
            terms = s * ges[rows[name]]
            inv = np.abs(terms.sum(axis=0))
            scale = np.abs(terms).sum(axis=0).max()
            assert inv.max() <= 2e-4 * scale, f"{name}: gauge sum {inv.max():.3e} vs scale {scale:.3e}"


@pytest.mark.parametrize("name", ["quarterly", "yearly", "hourly", "monthly"])
def test_full_size_workload(name):
    from oracle import oracle
    cfg = CONFIGS[name]
    inp = synth.make_inputs(cfg, seed=0)
    step = gc.run_gpu(cfg, inp)
    gauge_invariant(cfg, inp, step)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], inp["weights"])
    errs = gc.check_forward(cfg, inp, step, f, stages=False)
    errs.update(gc.check_backward(cfg, inp, step, f, None, stages=False))
    kink = errs.pop("series_at_kink")
    worst = sorted(errs.items(), key=lambda kv: -kv[1])[:4]
    print(f"  {name}: {int(kink)} series with an output at the pinball kink; worst " + ", ".join(f"{k}={v:.2e}" for k, v in worst), flush=True)
    step.close()


def test_quarterly_batch_sweep_ragged():
    """The batch sweep of the quarterly workload (prefixes of the same batch), with ragged lengths."""
    for B in (64, 256, 1024):
        cfg = CONFIGS["quarterly"].with_(B=B)
        errs = gc.run_and_check(cfg, seed=0, ragged=True, stages=False)
        errs.pop("series_at_kink")
        print(f"  B={B}: worst {max(errs.values()):.2e}", flush=True)
