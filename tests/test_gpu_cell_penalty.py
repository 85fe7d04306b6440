"""Cell-state penalty (Section 8.4) in the HIP library against the float64 oracle."""
import numpy as np
import pytest

from paper_1907_03329_amd.synth import CONFIGS
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["tiny_quarterly", "yearly", "monthly"])
def test_training_step_with_cell_state_penalty(name):
    cfg = CONFIGS[name]
    cfg = cfg.with_(B=min(cfg.B, 37), T=min(cfg.T, 120), lambda_c=3.0)
    errs = gc.run_and_check(cfg, seed=61, ragged=True)
    print(name, {k: f"{v:.1e}" for k, v in errs.items() if v > 1e-6})


def test_penalty_with_three_blocks_categories_and_many_chains():
    cfg = CONFIGS["tiny_quarterly"].with_(B=70, T=90, blocks=((1, 7), (12,), (3, 5)), hidden=30, lambda_c=10.0, n_cat=6)
    gc.run_and_check(cfg, seed=62, ragged=True)


def test_penalty_changes_the_gradient_and_the_loss():
    import torch
    from paper_1907_03329_amd import synth
    cfg = CONFIGS["tiny_quarterly"].with_(B=20)
    inp = synth.make_inputs(cfg, seed=63)
    a = gc.run_gpu(cfg, inp)
    b = gc.run_gpu(cfg.with_(lambda_c=2.0), inp)
    assert b.loss.item() > a.loss.item()
    assert not torch.equal(a.grad_weights, b.grad_weights)
    assert torch.equal(a.forecasts, b.forecasts)
    a.close(); b.close()
