"""GPU parity of the two window-adjoint kernels (the reverse of Eq. (6)'s windows: gradients of the
de-seasonalised log series and of the log level) against the float64 CPU oracle.

The library gathers per (time, series) at small batches and streams tile by tile at large ones; the
choice is made from the number of 16-series tiles when a handle is created (environment variable
ESRNN_WINDOW_STREAM_FROM: 0 = stream always, a large number = never).  Both kernels are forced onto every
shape here, ragged lengths included, and compared on every series and time step (grad_u, grad_v) and in
what follows from them (gradients of the smoothing parameters)."""
import os

import pytest

from paper_1907_03329_amd.synth import CONFIGS, Config

pytestmark = pytest.mark.gpu

from tests import gpu_common as gc  # noqa: E402


class forced:
    def __init__(self, value):
        self.value = str(value)

    def __enter__(self):
        self.old = os.environ.get("ESRNN_WINDOW_STREAM_FROM")
        os.environ["ESRNN_WINDOW_STREAM_FROM"] = self.value

    def __exit__(self, *exc):
        if self.old is None:
            os.environ.pop("ESRNN_WINDOW_STREAM_FROM", None)
        else:
            os.environ["ESRNN_WINDOW_STREAM_FROM"] = self.old


def small(name, **kw):
    base = dict(name=name, B=37, T=40, n_seas=1, m1=4, m2=0, I=4, H=8, hidden=8, blocks=((1, 2), (4,)),
                tau=0.48, lambda_lv=50.0)
    base.update(kw)
    return Config(**base)


SHAPES = {
    "quarterly_70": lambda: CONFIGS["quarterly"].with_(B=70),
    "quarterly_categories_64": lambda: CONFIGS["quarterly"].with_(B=64, n_cat=6),
    "monthly_21": lambda: CONFIGS["monthly"].with_(B=21, T=90),
    "yearly_130": lambda: CONFIGS["yearly"].with_(B=130),
    "hourly_19": lambda: CONFIGS["hourly"].with_(B=19, T=300),
    "widest_windows": lambda: small("widest_windows", hidden=64, I=64, H=64, T=140, B=20, m1=12),
    "one_step_windows": lambda: small("one_step_windows", I=1, H=1, T=9, B=5, m1=2),
    "odd_widths": lambda: small("odd_widths", I=13, H=3, T=48, hidden=12),
    "no_level_penalty": lambda: small("no_level_penalty", lambda_lv=0.0, I=5, H=6),
    "single_series": lambda: small("single_series", B=1, I=3, H=5),
}


@pytest.mark.parametrize("kind", ["gather", "stream"])
@pytest.mark.parametrize("shape", sorted(SHAPES))
def test_each_window_adjoint_kernel_on_every_shape(shape, kind):
    cfg = SHAPES[shape]()
    with forced(0 if kind == "stream" else 1 << 30):
        errs = gc.run_and_check(cfg, seed=90, ragged=True, stages=True)
    print(f"  {shape} {kind}: grad_u {errs['grad_u']:.2e} grad_v {errs['grad_v']:.2e}", flush=True)


def test_default_choice_at_many_tiles_agrees_with_the_gather_kernel():
    """65536 quarterly series (4096 tiles) is where the default turns to the streaming kernel.  The oracle
    cannot run that size in the time of a test; both kernels are compared with it on every shape above,
    and here with each other on the full-size batch: the same sums in a different order."""
    import numpy as np
    import torch
    from paper_1907_03329_amd import synth
    cfg = CONFIGS["quarterly"].with_(B=65536)
    inp = synth.make_inputs(cfg, seed=91, ragged=True)
    got = {}
    for kind, value in (("default", None), ("gather", 1 << 30)):
        if value is None:
            assert "ESRNN_WINDOW_STREAM_FROM" not in os.environ
            step = gc.run_gpu(cfg, inp)
        else:
            with forced(value):
                step = gc.run_gpu(cfg, inp)
        got[kind] = {k: step.buffer(k).clone() for k in ("grad_u", "grad_v")}
        got[kind]["grad_es"] = step.grad_es_params.clone()
        step.close()
        torch.cuda.synchronize()
    live = torch.from_numpy(np.arange(cfg.T)[:, None] < inp["lengths"][None, :]).cuda()
    for k in ("grad_u", "grad_v"):
        a, b = got["default"][k], got["gather"][k]
        scale = b[live].abs().max().item()
        err = ((a - b).abs() * live).max().item() / scale
        print(f"  {k}: {err:.2e}", flush=True)
        assert err <= 2e-6, (k, err)
    a, b = got["default"]["grad_es"], got["gather"]["grad_es"]
    err = ((a - b).abs().amax(dim=1) / b.abs().amax(dim=1).clamp_min(1e-30)).max().item()
    print(f"  grad_es rows: {err:.2e}", flush=True)
    assert err <= 1e-5, err
