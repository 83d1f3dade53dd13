"""The C-ABI library loads, exports every function include/edgepipe.h declares,
and rejects bad arguments without touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2110_14895_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "edgepipe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ep_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary_calls():
    names = declared_functions()
    for n in ("ep_stage_create", "ep_stage_forward", "ep_stage_profile", "ep_stage_destroy",
              "ep_partition", "ep_status_string", "ep_last_error"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in edgepipe.h but not exported"


def test_status_strings():
    assert binding.status_string(binding.EP_OK) == "EP_OK"
    assert binding.status_string(binding.EP_ERR_INFEASIBLE) == "EP_ERR_INFEASIBLE"
    assert binding.status_string(99) == "EP_ERR_UNKNOWN"


def _cfg(**kw):
    base = dict(n_layers=2, d_model=128, n_heads=2, d_mlp=256, n_tokens=65)
    base.update(kw)
    return binding.VitConfig(**base)


def _null_layers(n):
    return (binding.ep_layer_weights * n)()


@pytest.mark.parametrize("cfg,begin,end,status", [
    (_cfg(), 0, 0, binding.EP_ERR_INVALID_ARG),                  # empty range
    (_cfg(), 1, 3, binding.EP_ERR_INVALID_ARG),                  # beyond n_layers
    (_cfg(d_model=130), 0, 1, binding.EP_ERR_UNSUPPORTED),       # bf16 path needs D % 64 == 0
    (_cfg(n_heads=3), 0, 1, binding.EP_ERR_INVALID_ARG),         # D % H != 0
    (_cfg(n_heads=4), 0, 1, binding.EP_ERR_UNSUPPORTED),         # d_head = 32
    (_cfg(n_tokens=5000), 0, 1, binding.EP_ERR_UNSUPPORTED),     # too many tokens for the bf16 kernel
    (_cfg(param_dtype=binding.EP_F32), 0, 1, binding.EP_ERR_UNSUPPORTED),   # fp32 params, bf16 input
    (_cfg(param_dtype=7), 0, 1, binding.EP_ERR_INVALID_ARG),
])
def test_stage_create_rejects_bad_arguments_before_any_gpu_call(cfg, begin, end, status):
    lib = binding.lib()
    h = C.c_void_p()
    c = cfg.c_struct()
    rc = lib.ep_stage_create(C.byref(c), begin, end, _null_layers(2), 4, C.byref(h))
    assert rc == status, binding.last_error()
    assert not h.value
    assert binding.last_error() != ""


def test_stage_create_rejects_null_parameter_pointers_and_bad_batch():
    lib = binding.lib()
    h = C.c_void_p()
    c = _cfg().c_struct()
    assert lib.ep_stage_create(C.byref(c), 0, 1, _null_layers(1), 4, C.byref(h)) == binding.EP_ERR_INVALID_ARG
    assert "null parameter" in binding.last_error()
    assert lib.ep_stage_create(C.byref(c), 0, 1, _null_layers(1), 0, C.byref(h)) == binding.EP_ERR_INVALID_ARG
    assert lib.ep_stage_create(None, 0, 1, _null_layers(1), 1, C.byref(h)) == binding.EP_ERR_INVALID_ARG


def test_stage_create_rejects_a_batch_the_dense_layers_cannot_index():
    # 2000 images x 257 tokens x 5120 hidden columns is past the 32-bit element index of the dense
    # layers: refused when the stage is built, not in the middle of a forward
    lib = binding.lib()
    h = C.c_void_p()
    c = _cfg(n_layers=1, d_model=1280, n_heads=16, d_mlp=5120, n_tokens=257).c_struct()
    assert lib.ep_stage_create(C.byref(c), 0, 1, _null_layers(1), 2000, C.byref(h)) == binding.EP_ERR_UNSUPPORTED
    assert "rows" in binding.last_error() and not h.value
    # the same width at a batch that fits gets as far as the parameter check
    assert lib.ep_stage_create(C.byref(c), 0, 1, _null_layers(1), 256, C.byref(h)) == binding.EP_ERR_INVALID_ARG


def test_forward_and_profile_reject_null_handle():
    lib = binding.lib()
    assert lib.ep_stage_forward(None, None, 1, None, None) == binding.EP_ERR_INVALID_ARG
    out = (C.c_double * 1)()
    assert lib.ep_stage_profile(None, 1, 1, None, out) == binding.EP_ERR_INVALID_ARG
    lib.ep_stage_destroy(None)      # allowed


def test_binding_checks_parameter_dtype():
    p = {n: np.zeros(4, dtype=np.float32) for n in binding.PARAM_NAMES}
    with pytest.raises(TypeError):
        binding.Stage(_cfg(), 0, 1, [p], 1)
