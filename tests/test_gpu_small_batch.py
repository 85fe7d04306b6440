"""GPU parity of the two kinds of LSTM layer kernels against the float64 CPU oracle.

Layers with few workgroups run on the 4-series kernels, the others on the 16-series kernels; the library
chooses per layer from the batch size and the dilation.  These tests cover the choice itself at batch
sizes 1 .. 512 with dilations 1 and 4, and force each kind of kernel onto shapes that the default would
give to the other (environment variable ESRNN_NARROW_BELOW, read when a handle is created: 0 = 16-series
kernels everywhere, a large number = 4-series kernels everywhere), so that both are checked on every
hidden size, input width, residual wiring and penalty."""
import os

import pytest

from paper_1907_03329_amd.synth import CONFIGS, Config

pytestmark = pytest.mark.gpu

from tests import gpu_common as gc  # noqa: E402


class forced:
    """Context manager: create handles with the given threshold."""

    def __init__(self, value):
        self.value = value

    def __enter__(self):
        self.old = os.environ.get("ESRNN_NARROW_BELOW")
        if self.value is None:
            os.environ.pop("ESRNN_NARROW_BELOW", None)
        else:
            os.environ["ESRNN_NARROW_BELOW"] = str(self.value)

    def __exit__(self, *exc):
        if self.old is None:
            os.environ.pop("ESRNN_NARROW_BELOW", None)
        else:
            os.environ["ESRNN_NARROW_BELOW"] = self.old


def small(name, **kw):
    base = dict(name=name, B=37, T=40, n_seas=1, m1=4, m2=0, I=4, H=8, hidden=8, blocks=((1, 2), (4, 8)),
                tau=0.48, lambda_lv=50.0)
    base.update(kw)
    return Config(**base)


@pytest.mark.parametrize("B", [1, 16, 48, 512])
def test_default_choice_dilations_1_and_4(B):
    cfg = CONFIGS["quarterly"].with_(B=B, blocks=((1, 4), (1, 4)))
    errs = gc.run_and_check(cfg, seed=70 + B % 7, ragged=True, stages=B <= 48)
    print(f"  B={B}: worst {max(v for k, v in errs.items() if k != 'series_at_kink'):.2e}", flush=True)


SHAPES = {
    "quarterly_70": lambda: CONFIGS["quarterly"].with_(B=70),
    "monthly_21": lambda: CONFIGS["monthly"].with_(B=21, T=90),
    "yearly_50": lambda: CONFIGS["yearly"].with_(B=50),
    "hourly_19": lambda: CONFIGS["hourly"].with_(B=19, T=300),
    "max_sizes": lambda: small("max_sizes", hidden=64, I=64, H=64, T=140, B=20, blocks=((1, 2), (3,)), m1=12),
    "four_blocks": lambda: small("four_blocks", blocks=((1, 2), (1,), (3,), (2, 4)), hidden=7, I=4, H=3, B=21),
    "padded_input": lambda: small("padded_input", hidden=30, I=13, H=3, T=48),
    "hidden_5": lambda: small("hidden_5", hidden=5, I=3, H=5, blocks=((1,), (2,), (3, 1))),
    "long_dilation": lambda: small("long_dilation", T=20, I=4, H=8, blocks=((1, 12), (30,)), B=18),
    "penalty_categories": lambda: small("penalty_categories", hidden=40, I=4, H=8, B=23, n_cat=6, lambda_c=0.3,
                                        blocks=((1, 2), (4,), (3,))),
}


@pytest.mark.parametrize("kind", ["wide", "narrow"])
@pytest.mark.parametrize("shape", sorted(SHAPES))
def test_each_kernel_kind_on_every_shape(shape, kind):
    cfg = SHAPES[shape]()
    with forced(0 if kind == "wide" else 1 << 30):
        errs = gc.run_and_check(cfg, seed=80, ragged=True)
    print(f"  {shape} {kind}: worst {max(v for k, v in errs.items() if k != 'series_at_kink'):.2e}", flush=True)


def test_mid_size_batch_on_the_four_series_kernels():
    """512 series of the quarterly shape, every layer forced onto the 4-series kernels (several chains per
    workgroup, 128 series tiles of four)."""
    cfg = CONFIGS["quarterly"].with_(B=512)
    with forced(1 << 30):
        errs = gc.run_and_check(cfg, seed=81, ragged=True, stages=False)
    print(f"  worst {max(v for k, v in errs.items() if k != 'series_at_kink'):.2e}", flush=True)
