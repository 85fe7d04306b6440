"""Seeded synthetic inputs for the ES-RNN training step.

This module only draws random numbers and lays them out in the argument
formats of the C-ABI (time-major series, per-series ES parameter rows, one flat
weight vector).  It holds none of the method's arithmetic and imports neither
the HIP binding nor the CPU oracle; the tests and the benchmark hand the same
arrays to both.

The series stand in for the M4 data the paper trains on (Section 4, Tables 2
and 3), which is not available here: positive series with a slowly drifting
level, fixed multiplicative seasonal profiles and multiplicative noise, at the
lengths the paper equalises to (Section 5.2) and the network shapes of Table 1.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

import numpy as np

PARAMS_DIRECT = 0
PARAMS_LOGIT = 1


@dataclass(frozen=True)
class Config:
    """Shape of one training step (mirrors the fields of ``esrnn_config``)."""

    name: str
    B: int
    T: int
    n_seas: int
    m1: int
    m2: int
    I: int
    H: int
    hidden: int
    blocks: Tuple[Tuple[int, ...], ...]
    tau: float = 0.48
    lambda_lv: float = 50.0
    param_space: int = PARAMS_DIRECT
    lambda_c: float = 0.0   # weight of the cell-state penalty (Section 8.4); 0: none
    n_cat: int = 0     # series categories fed to the network as a one-hot block after the input window (Section 5.3); 0: none
    # generator knobs (standard deviations; see make_inputs)
    step_mu: float = 0.0
    step_sd: float = 0.02
    seas_sd1: float = 0.1
    seas_sd2: float = 0.0
    noise_sd: float = 0.05

    @property
    def P(self) -> int:
        return self.T - self.I - self.H + 1

    @property
    def K(self) -> int:
        return 1 + self.n_seas + (self.m1 if self.n_seas >= 1 else 0) + (self.m2 if self.n_seas >= 2 else 0)

    @property
    def dilations(self) -> List[int]:
        return [d for blk in self.blocks for d in blk]

    @property
    def n_layers(self) -> int:
        return len(self.dilations)

    @property
    def weight_count(self) -> int:
        h, n = self.hidden, 0
        for layer in range(self.n_layers):
            k = (self.I + self.n_cat if layer == 0 else h) + h
            n += 4 * h * k + 4 * h
        return n + h * h + h + self.H * h + self.H

    def with_(self, **kw) -> "Config":
        return replace(self, **kw)


# The five workloads: network shapes from Table 1 of the paper (quarterly,
# monthly, yearly); window sizes, the hourly shape and the generator recipe are
# the benchmark's own.
CONFIGS: Dict[str, Config] = {
    "tiny_quarterly": Config("tiny_quarterly", B=16, T=72, n_seas=1, m1=4, m2=0, I=4, H=8, hidden=40,
                             blocks=((1, 2), (4, 8)), step_sd=0.02, seas_sd1=0.1, noise_sd=0.05),
    "quarterly": Config("quarterly", B=4096, T=72, n_seas=1, m1=4, m2=0, I=4, H=8, hidden=40,
                        blocks=((1, 2), (4, 8)), step_sd=0.02, seas_sd1=0.1, noise_sd=0.05),
    "monthly": Config("monthly", B=4096, T=240, n_seas=1, m1=12, m2=0, I=12, H=18, hidden=50,
                      blocks=((1, 3), (6, 12)), step_mu=0.002, step_sd=0.01, seas_sd1=0.15, noise_sd=0.05),
    "yearly": Config("yearly", B=8192, T=40, n_seas=0, m1=0, m2=0, I=6, H=6, hidden=30,
                     blocks=((1, 2), (2, 6)), step_mu=0.01, step_sd=0.05, seas_sd1=0.0, noise_sd=0.03),
    "hourly": Config("hourly", B=512, T=720, n_seas=2, m1=24, m2=168, I=24, H=48, hidden=40,
                     blocks=((1, 4), (24, 168)), step_sd=0.02, seas_sd1=0.2, seas_sd2=0.2, noise_sd=0.05),
}
CONFIG_ORDER = ["tiny_quarterly", "quarterly", "monthly", "yearly", "hourly"]


def weight_layout(cfg: Config) -> List[Tuple[str, int, Tuple[int, ...]]]:
    """(name, offset, shape) of every block of the flat weight vector.

    Per LSTM layer: ``W`` of shape [4h, in+h] row-major, gate rows in the order
    input, forget, cell candidate, output, columns first the layer input (for
    the first layer: the window, then the one-hot category block) then the
    recurrent state; then the bias [4h].  After the layers: adapter
    ``Wa`` [h, h], ``ba`` [h], head ``Wo`` [H, h], ``bo`` [H].
    """
    h, out, off = cfg.hidden, [], 0
    for layer in range(cfg.n_layers):
        k = (cfg.I + cfg.n_cat if layer == 0 else h) + h      # first layer: window, then the category one-hot
        out.append((f"W{layer}", off, (4 * h, k)))
        off += 4 * h * k
        out.append((f"b{layer}", off, (4 * h,)))
        off += 4 * h
    for name, shape in (("Wa", (h, h)), ("ba", (h,)), ("Wo", (cfg.H, h)), ("bo", (cfg.H,))):
        out.append((name, off, shape))
        off += int(np.prod(shape))
    assert off == cfg.weight_count
    return out


def es_param_rows(cfg: Config) -> Dict[str, slice]:
    """Row ranges of the [K, B] per-series ES parameter matrix."""
    rows, r = {"alpha": slice(0, 1)}, 1
    if cfg.n_seas >= 1:
        rows["gamma1"] = slice(r, r + 1)
        r += 1
    if cfg.n_seas >= 2:
        rows["gamma2"] = slice(r, r + 1)
        r += 1
    if cfg.n_seas >= 1:
        rows["s1_init"] = slice(r, r + cfg.m1)
        r += cfg.m1
    if cfg.n_seas >= 2:
        rows["s2_init"] = slice(r, r + cfg.m2)
        r += cfg.m2
    assert r == cfg.K
    return rows


def make_inputs(cfg: Config, seed: int = 0, ragged: bool = False) -> Dict[str, np.ndarray]:
    """Draw one batch.  Fixed draw order, float64 draws cast to float32 once.

    Returns ``y`` [T, B] float32 (time-major, pad value 1 past each length),
    ``lengths`` [B] int32, ``es_params`` [K, B] float32 (in ``cfg.param_space``),
    ``weights`` [weight_count] float32 and, if ``cfg.n_cat > 0``, ``categories``
    [B] int32 in [0, n_cat).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    B, T, h = cfg.B, cfg.T, cfg.hidden
    # (1) start level, (2) log-level random walk
    u0 = rng.normal(np.log(1000.0), 0.5, size=B)
    steps = rng.normal(cfg.step_mu, cfg.step_sd, size=(T - 1, B))
    log_level = np.concatenate([u0[None, :], u0[None, :] + np.cumsum(steps, axis=0)], axis=0)
    # (3) seasonal profiles, arithmetic mean one per series
    f1 = f2 = None
    if cfg.n_seas >= 1:
        f1 = rng.lognormal(0.0, cfg.seas_sd1, size=(cfg.m1, B))
        f1 /= f1.mean(axis=0, keepdims=True)
    if cfg.n_seas >= 2:
        f2 = rng.lognormal(0.0, cfg.seas_sd2, size=(cfg.m2, B))
        f2 /= f2.mean(axis=0, keepdims=True)
    # (4) multiplicative noise
    noise = rng.lognormal(0.0, cfg.noise_sd, size=(T, B))
    y = np.exp(log_level) * noise
    t = np.arange(T)
    if f1 is not None:
        y *= f1[t % cfg.m1, :]
    if f2 is not None:
        y *= f2[t % cfg.m2, :]
    # (5) per-series ES parameters
    rows = es_param_rows(cfg)
    es = np.empty((cfg.K, B))
    es[rows["alpha"]] = rng.uniform(0.2, 0.8, size=(1, B))
    if cfg.n_seas >= 1:
        es[rows["gamma1"]] = rng.uniform(0.05, 0.5, size=(1, B))
    if cfg.n_seas >= 2:
        es[rows["gamma2"]] = rng.uniform(0.05, 0.5, size=(1, B))
    if cfg.n_seas >= 1:
        es[rows["s1_init"]] = f1 * rng.lognormal(0.0, 0.05, size=(cfg.m1, B))
    if cfg.n_seas >= 2:
        es[rows["s2_init"]] = f2 * rng.lognormal(0.0, 0.05, size=(cfg.m2, B))
    if cfg.param_space == PARAMS_LOGIT:
        n_smooth = 1 + cfg.n_seas
        es[:n_smooth] = np.log(es[:n_smooth]) - np.log1p(-es[:n_smooth])
        es[n_smooth:] = np.log(es[n_smooth:])
    # (6) shared weights
    bound = 1.0 / np.sqrt(h)
    w = rng.uniform(-bound, bound, size=cfg.weight_count)
    for name, off, shape in weight_layout(cfg):
        if name.startswith("b") and name[1:].isdigit():
            w[off + h: off + 2 * h] += 1.0  # forget-gate bias
    # lengths last so that the draws above do not depend on `ragged`
    lengths = np.full(B, T, dtype=np.int32)
    if ragged:
        lo = min(T, cfg.I + cfg.H + max(cfg.m1, cfg.m2, 2))
        lengths = rng.integers(lo, T + 1, size=B).astype(np.int32)
        lengths[0] = T
        if B > 1:
            lengths[-1] = lo
        y[t[:, None] >= lengths[None, :]] = 1.0
    out = {
        "y": np.ascontiguousarray(y, dtype=np.float32),
        "lengths": lengths,
        "es_params": np.ascontiguousarray(es, dtype=np.float32),
        "weights": np.ascontiguousarray(w, dtype=np.float32),
    }
    # categories after everything else, and only when asked for: batches without them stay as they were
    if cfg.n_cat > 0:
        out["categories"] = rng.integers(0, cfg.n_cat, size=B).astype(np.int32)
    return out


def take_series(inputs: Dict[str, np.ndarray], idx) -> Dict[str, np.ndarray]:
    """Restrict a batch to the series in ``idx`` (weights are shared)."""
    idx = np.asarray(idx)
    out = {
        "y": np.ascontiguousarray(inputs["y"][:, idx]),
        "lengths": np.ascontiguousarray(inputs["lengths"][idx]),
        "es_params": np.ascontiguousarray(inputs["es_params"][:, idx]),
        "weights": inputs["weights"],
    }
    if "categories" in inputs:
        out["categories"] = np.ascontiguousarray(inputs["categories"][idx])
    return out
