"""Seeded random shapes against the oracle: hidden sizes, input windows, horizons, block structures, dilations,
window counts, seasonalities, batch sizes, ragged lengths and both kinds of LSTM kernel are drawn together, so
that combinations no hand-written case names are reached too (every draw is a valid configuration).  Batches
start at 16 series: the per-row bounds of the common checks take their scale from the largest gradient in the
batch, which a batch of one or two series whose seasonal gradients cancel does not provide (single-series batches
have a test of their own in test_gpu_parity.py)."""
import os
import random

import pytest

from paper_1907_03329_amd.synth import Config
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu

# hidden size -> input windows whose (hidden tiles, input tiles) pair has a kernel of its own
SHAPES = [(5, [4, 8]), (8, [4, 8]), (30, [6, 8, 12, 30]), (40, [4, 10, 12, 24, 30, 40]), (50, [10, 12, 18, 20, 50]),
          (64, [64])]


def draw(rng, it, batches, positions):
    hidden, windows = rng.choice(SHAPES)
    I = rng.choice(windows)
    H = rng.choice([1, 3, 6, 8, 13, 18])
    blocks = tuple(tuple(rng.choice([1, 2, 3, 4, 6, 8]) for _ in range(rng.choice([1, 2])))
                   for _ in range(rng.choice([1, 2, 3])))
    T = I + H + rng.choice(positions) - 1
    ns = rng.choice([0, 1, 1, 2])
    m1 = rng.choice([m for m in (2, 3, 4, 7) if m <= T]) if ns >= 1 else 0
    m2 = rng.choice([m for m in (5, 9, 11) if m <= T]) if ns >= 2 else 0
    kw = dict(name=f"random{it}", B=rng.choice(batches), T=T, n_seas=ns, m1=m1, m2=m2, I=I, H=H, hidden=hidden,
              blocks=blocks, tau=rng.choice([0.48, 0.5, 0.3]), lambda_lv=rng.choice([0.0, 50.0]))
    if ns == 2:
        kw["seas_sd2"] = 0.1
    return Config(**kw), rng.choice([0, 160, 100000]), rng.random() < 0.6


@pytest.mark.parametrize("seed,count,batches,positions", [
    (11, 120, [16, 17, 45, 64, 100, 170, 260], [1, 2, 5, 9, 17, 30]),
    (12, 16, [260, 700, 1500, 2600], [17, 30, 61]),
])
def test_random_shapes(seed, count, batches, positions):
    rng = random.Random(seed)
    before = os.environ.get("ESRNN_NARROW_BELOW")
    try:
        for it in range(count):
            cfg, narrow_below, ragged = draw(rng, it, batches, positions)
            os.environ["ESRNN_NARROW_BELOW"] = str(narrow_below)     # read when the handle is created
            print(f"  [{it}] hidden={cfg.hidden} I={cfg.I} H={cfg.H} blocks={cfg.blocks} T={cfg.T} seasons={cfg.n_seas} "
                  f"m=({cfg.m1},{cfg.m2}) B={cfg.B} narrow_below={narrow_below} ragged={ragged}", flush=True)
            gc.run_and_check(cfg, seed=1000 * seed + it, ragged=ragged)
    finally:
        if before is None:
            os.environ.pop("ESRNN_NARROW_BELOW", None)
        else:
            os.environ["ESRNN_NARROW_BELOW"] = before
