"""Shared helpers of the GPU parity tests: run the HIP library and the float64
CPU oracle on the same seeded inputs and compare tensor by tensor.

Tolerance convention (per tensor): max |gpu - oracle| / max |oracle|.
Forecasts and loss must be within 1e-4, every gradient tensor within 1e-3; the
intermediates are held to the same bounds so that a failure names its stage.
"""
from __future__ import annotations

import numpy as np

from oracle import oracle
from paper_1907_03329_amd import binding, synth

TOL_FWD = 1e-4
TOL_GRAD = 1e-3


def rel_err(got, want, mask=None):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if mask is not None:
        got, want = got[mask], want[mask]
    if want.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values from the GPU"
    scale = np.abs(want).max()
    return float(np.abs(got - want).max() / (scale if scale > 0 else 1.0))


def to_device(inp):
    import torch
    return {k: torch.from_numpy(v).cuda() for k, v in inp.items()}


def run_gpu(cfg, inp, backward=True):
    import torch
    step = binding.TrainingStep(cfg)
    dev = to_device(inp)
    if "categories" in dev:
        step.set_categories(dev["categories"])
    step.forward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    if backward:
        step.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    torch.cuda.synchronize()
    return step


def valid_window_mask(cfg, lengths):
    """[P, B] True where the window fits into the series."""
    P = cfg.T - cfg.I - cfg.H + 1
    Pb = lengths.astype(np.int64) - cfg.I - cfg.H + 1
    return np.arange(P)[:, None] < Pb[None, :]


def check_forward(cfg, inp, step, f, stages=True):
    """Compare the GPU forward state in `step` with the oracle result `f`.
    Returns {name: error}; raises on the first tensor out of tolerance."""
    errs = {}
    T, B = cfg.T, cfg.B
    lengths = inp["lengths"]
    live = (np.arange(T)[:, None] < lengths[None, :])          # [T, B]
    wm = valid_window_mask(cfg, lengths)                        # [P, B]

    def chk(name, got, want, mask, tol):
        e = rel_err(got, want, mask)
        errs[name] = e
        assert e <= tol, f"{name}: relative error {e:.3e} > {tol:g} ({cfg.name})"

    if stages:
        chk("level", step.buffer("level").cpu().numpy(), f.l.T, live, TOL_FWD)
        chk("u", step.buffer("u").cpu().numpy(), f.u.T, live, TOL_FWD)
        chk("v", step.buffer("v").cpu().numpy(), f.v.T, live, TOL_FWD)
        if cfg.n_seas >= 1:
            chk("S1", step.buffer("S1").cpu().numpy(), f.S1.T, live, TOL_FWD)
        if cfg.n_seas >= 2:
            chk("S2", step.buffer("S2").cpu().numpy(), f.S2.T, live, TOL_FWD)
        chk("X", step.buffer("X").cpu().numpy(), f.X.transpose(1, 0, 2), wm, TOL_FWD)
        chk("Z", step.buffer("Z").cpu().numpy(), f.Z.transpose(1, 0, 2), wm, TOL_FWD)
        for l in range(f.n_layers):
            g = step.buffer("gates", l).cpu().numpy()           # [P, B, h, 4]
            chk(f"gates{l}", g, f.gates[l].transpose(1, 0, 3, 2), wm, TOL_FWD)
            chk(f"c{l}", step.buffer("c", l).cpu().numpy(), f.c[l].transpose(1, 0, 2), wm, TOL_FWD)
            chk(f"h{l}", step.buffer("hid", l).cpu().numpy(), f.h[l].transpose(1, 0, 2), wm, TOL_FWD)
        for k in range(len(cfg.blocks)):
            chk(f"block{k}", step.buffer("block_out", k).cpu().numpy(), f.blk[k].transpose(1, 0, 2), wm, TOL_FWD)
        chk("O", step.buffer("O").cpu().numpy(), f.o.transpose(1, 0, 2), wm, TOL_FWD)
    chk("loss", step.loss.cpu().numpy(), np.array([f.loss]), None, TOL_FWD)
    fc = step.forecasts.cpu().numpy()
    chk("forecasts", fc, f.forecasts, None, TOL_FWD)
    assert np.all(fc[~wm] == 0.0), "forecasts of masked windows must be zero"
    return errs


def check_backward(cfg, inp, step, f, g, stages=True):
    errs = {}
    T = cfg.T
    lengths = inp["lengths"]
    live = (np.arange(T)[:, None] < lengths[None, :])
    wm = valid_window_mask(cfg, lengths)

    def chk(name, got, want, mask, tol):
        e = rel_err(got, want, mask)
        errs[name] = e
        assert e <= tol, f"{name}: relative error {e:.3e} > {tol:g} ({cfg.name})"

    # At the kink of the pinball loss (target == output up to float32 rounding) either one-sided
    # derivative is a valid result, and the choice changes that series' gradients by a visible amount.
    # One such element moves the pinball part of its series' gradients by about 2 / (valid outputs of the
    # series).  Series where that could exceed a fifth of the gradient tolerance are compared through the
    # shared-weight gradients only (where one element weighs 1 / n_pin); everything per series is
    # compared on the other series.
    near = np.abs(f.Z - f.o) <= 2e-6 * np.maximum(1.0, np.abs(f.Z))            # [B, P, H]
    near &= wm.T[:, :, None]
    n_out = np.maximum(wm.sum(axis=0) * cfg.H, 1)                                # [B]
    clean = 2.0 * near.sum(axis=(1, 2)) / n_out <= 0.2 * TOL_GRAD               # [B]
    errs["series_at_kink"] = float((~clean).sum())
    assert (~clean).sum() <= max(3, 0.05 * cfg.B), "implausibly many outputs at the kink of the pinball loss"
    if stages:
        chk("grad_O", step.buffer("grad_O").cpu().numpy(), g.gO.transpose(1, 0, 2),
            np.broadcast_to(clean[None, :, None], (wm.shape[0], cfg.B, cfg.H)), TOL_GRAD)
        chk("grad_top", step.buffer("grad_top").cpu().numpy(), g.gR.transpose(1, 0, 2), wm & clean[None, :], TOL_GRAD)
        chk("grad_X", step.buffer("grad_X").cpu().numpy(), g.gX.transpose(1, 0, 2), wm & clean[None, :], TOL_GRAD)
        chk("grad_u", step.buffer("grad_u").cpu().numpy(), g.gu.T, live & clean[None, :], TOL_GRAD)
        chk("grad_v", step.buffer("grad_v").cpu().numpy(), g.gv.T, live & clean[None, :], TOL_GRAD)
    ges = step.grad_es_params.cpu().numpy()
    for name, sl in synth.es_param_rows(cfg).items():
        chk(f"grad_{name}", ges[sl][:, clean], g.grad_es_params[sl][:, clean], None, TOL_GRAD)
    gw = step.grad_weights.cpu().numpy()
    for name, off, shape in synth.weight_layout(cfg):
        n = int(np.prod(shape))
        chk(f"grad_{name}", gw[off:off + n], g.grad_weights[off:off + n], None, TOL_GRAD)
    return errs


def run_and_check(cfg, seed=0, ragged=False, stages=True, mutate=None):
    inp = synth.make_inputs(cfg, seed=seed, ragged=ragged)
    if mutate is not None:
        mutate(inp)
    f = oracle.forward(cfg, inp["y"], inp["lengths"], inp["es_params"], inp["weights"],
                       categories=inp.get("categories"))
    g = oracle.backward(cfg, f)
    step = run_gpu(cfg, inp)
    errs = check_forward(cfg, inp, step, f, stages)
    errs.update(check_backward(cfg, inp, step, f, g, stages))
    step.close()
    return errs
