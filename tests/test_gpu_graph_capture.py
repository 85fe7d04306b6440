"""The training step recorded into a HIP graph (through torch's capture) and replayed: callers that
capture launch-bound loops must get, on every replay, exactly what the eager calls give."""
import numpy as np
import pytest

from paper_1907_03329_amd import binding, synth
from paper_1907_03329_amd.synth import CONFIGS
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu


def test_captured_step_replays_like_eager():
    import torch
    cfg = CONFIGS["tiny_quarterly"].with_(B=40)
    inp = synth.make_inputs(cfg, seed=51, ragged=True)
    dev = gc.to_device(inp)
    step = binding.TrainingStep(cfg)

    def eager():
        step.forward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
        step.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
        torch.cuda.synchronize()
        return (step.loss.clone(), step.forecasts.clone(), step.grad_es_params.clone(), step.grad_weights.clone())

    ref = eager()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step.forward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
        step.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
    for replay in range(3):
        # eager work and a change of inputs between the replays: the graph reads the buffers, not a snapshot
        scale = 1.0 + 0.01 * replay
        dev["weights"].mul_(scale)
        want = eager()
        for t in (step.loss, step.forecasts, step.grad_es_params, step.grad_weights):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (step.loss, step.forecasts, step.grad_es_params, step.grad_weights)
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {replay} differs from the eager result"
        dev["weights"].div_(scale)
    assert not torch.equal(ref[3], want[3])    # the inputs did change between replays
    step.close()
