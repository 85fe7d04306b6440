"""Host-side checks of the HIP library that need no GPU: it loads, exports every
symbol the public header declares, validates configurations, and reports the
sizes the input generator and the oracle agree on."""
import ctypes as C
import os
import re

import pytest

from oracle import oracle
from paper_1907_03329_amd import binding, synth
from paper_1907_03329_amd.synth import CONFIGS, Config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_1907_03329_amd import build
        build.build()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "esrnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(esrnn_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"esrnn_create", "esrnn_destroy", "esrnn_forward", "esrnn_backward", "esrnn_workspace_bytes",
            "esrnn_es_param_rows", "esrnn_weight_count", "esrnn_status_string",
            "esrnn_workspace_buffer"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in esrnn.h but not exported"


def test_config_struct_matches_header_size(lib):
    # 9 int32 + 4 + 16 int32 + 2 float + 1 int32
    assert C.sizeof(binding.EsrnnConfig) == 4 * (9 + 4 + 16 + 2 + 1 + 1 + 1)


@pytest.mark.parametrize("name", synth.CONFIG_ORDER)
def test_sizes_agree_with_generator_and_oracle(lib, name):
    cfg = CONFIGS[name]
    h = binding.esrnn_create(cfg)
    try:
        assert binding.esrnn_es_param_rows(h) == cfg.K
        assert binding.esrnn_weight_count(h) == cfg.weight_count
        cc = oracle._c_config(cfg)
        assert oracle.lib().eso_es_param_rows(C.byref(cc)) == cfg.K
        assert oracle.lib().eso_weight_count(C.byref(cc)) == cfg.weight_count
        nbytes = binding.esrnn_workspace_bytes(h)
        # at least the activation stash: 6 floats per hidden unit, layer, window position and series
        P = cfg.T - cfg.I - cfg.H + 1
        assert nbytes >= 4 * 6 * cfg.hidden * cfg.n_layers * P * cfg.B
        assert nbytes % 256 == 0
        v = binding.esrnn_workspace_buffer(h, "gates", cfg.n_layers - 1)
        assert v.layout == binding.LAYOUT_GATE_TILE and v.dims[0] == P and v.dims[3] == cfg.hidden
        assert v.offset_bytes % 256 == 0 and v.offset_bytes < nbytes
        with pytest.raises(binding.EsrnnError):
            binding.esrnn_workspace_buffer(h, "gates", cfg.n_layers)
    finally:
        binding.esrnn_destroy(h)


def bad(**kw):
    base = dict(name="bad", B=4, T=30, n_seas=1, m1=4, m2=0, I=3, H=5, hidden=8, blocks=((1, 2),))
    base.update(kw)
    return Config(**base)


@pytest.mark.parametrize("cfg", [
    bad(I=20, H=11),                 # I + H > T
    bad(m1=31),                      # period longer than the series
    bad(n_seas=3),
    bad(hidden=65),
    bad(hidden=0),
    bad(B=0),
    bad(blocks=((1, 0),)),           # dilation < 1
    bad(blocks=()),
    bad(tau=1.0),
    bad(tau=0.0),
    bad(lambda_lv=-1.0),
    bad(param_space=2),
    bad(I=65, T=200),
    bad(H=65, T=200),
    bad(hidden=8, I=40, T=100),      # input window wider than the padded hidden size and no dedicated shape
    bad(n_seas=2, m1=400, m2=300, T=800),   # seasonal rings of 64 series beyond the LDS of a compute unit
])
def test_invalid_configurations_are_rejected(lib, cfg):
    with pytest.raises(binding.EsrnnError) as ei:
        binding.esrnn_create(cfg)
    assert ei.value.status == 2


def test_null_and_order_errors_need_no_device(lib):
    assert lib.esrnn_create(None, None) == 1
    cfg = bad()
    h = binding.esrnn_create(cfg)
    n = C.c_size_t()
    assert lib.esrnn_workspace_bytes(h, None) == 1
    assert lib.esrnn_workspace_bytes(None, C.byref(n)) == 1
    # size and alignment of a workspace, checked on the host (the pointer is never dereferenced)
    assert lib.esrnn_workspace_bytes(h, C.byref(n)) == 0
    full = n.value
    assert lib.esrnn_es_window_workspace_bytes(h, C.byref(n)) == 0
    prefix = n.value
    assert 0 < prefix < full
    assert lib.esrnn_check_workspace(h, C.c_void_p(4096), full, 0) == 0
    assert lib.esrnn_check_workspace(h, C.c_void_p(4096), full - 1, 0) == 3
    assert lib.esrnn_check_workspace(h, C.c_void_p(4096 + 64), full, 0) == 3
    assert lib.esrnn_check_workspace(h, C.c_void_p(4096), prefix, 1) == 0
    assert lib.esrnn_check_workspace(h, C.c_void_p(4096), prefix, 0) == 3
    assert lib.esrnn_check_workspace(h, None, full, 0) == 1
    assert lib.esrnn_check_workspace(None, C.c_void_p(4096), full, 0) == 1
    # the diagnostic probe checks its arguments before it launches
    assert lib.esrnn_probe_issue_overlap(0, 10, 1, None, None) == 1
    for mode, iters, per_cu in ((4, 10, 1), (-1, 10, 1), (0, 0, 1), (0, 10, 3), (3, 10, 1), (0, (1 << 20) + 1, 1)):
        assert lib.esrnn_probe_issue_overlap(mode, iters, per_cu, C.c_void_p(4096), None) == 2
    # null array arguments are refused before anything is launched
    assert lib.esrnn_forward(h, None, None, None, None, None, None, None, None) == 1
    assert lib.esrnn_backward(h, None, None, None, None, None, None, None, None) == 1
    # misaligned workspace, and backward before forward (pointers are never dereferenced on these paths)
    fake = C.c_void_p(4096)
    assert lib.esrnn_forward(h, fake, fake, fake, fake, C.c_void_p(4097), fake, None, None) == 3
    assert lib.esrnn_backward(h, fake, fake, fake, fake, fake, fake, fake, None) == 4
    assert binding.status_string(4).startswith("backward")
    # forward-only handles refuse esrnn_backward; null handle
    assert lib.esrnn_set_forward_only(None, 1) == 1
    assert lib.esrnn_set_forward_only(h, 1) == 0
    assert lib.esrnn_backward(h, fake, fake, fake, fake, fake, fake, fake, None) == 4
    # periods up to 448 in total are accepted
    binding.esrnn_destroy(binding.esrnn_create(bad(n_seas=2, m1=400, m2=48, T=800)))
    binding.esrnn_destroy(h)


def test_binding_refuses_host_tensors(lib):
    import torch
    cfg = bad()
    h = binding.esrnn_create(cfg)
    t = torch.zeros(4)
    with pytest.raises(ValueError):
        binding.esrnn_forward(h, t, t, t, t, t, t)
    binding.esrnn_destroy(h)
