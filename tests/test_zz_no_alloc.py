"""ep_stage_forward_static (the entry point that allocates nothing: its intermediates live in a
workspace that is part of the library's code object) against ep_stage_forward on the same inputs,
through the C ABI: two calls in a row, the second on a smaller micro-batch, results bit for bit
those of the allocating path and within the bf16 / fp32 tolerance of the CPU checker."""
import numpy as np
import pytest

import oracle
from paper_2110_14895_amd import binding, synth
from tests import harness as H

pytestmark = pytest.mark.gpu


def _run(call, cfg, x):
    import torch
    xin = H.to_device(x, cfg.in_dtype == binding.EP_BF16)
    out = torch.full(x.shape, float("nan"), dtype=torch.float32, device="cuda")
    call(xin, x.shape[0], out, torch.cuda.current_stream())
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("bf16", [True, False])
def test_static_workspace_forward_matches_allocating_forward_twice(bf16):
    sh = synth.custom_shape("noalloc", 2, 320, 4, 640, 257) if bf16 else synth.SHAPES["tiny"]
    layers = [synth.layer_params(sh, l, bf16=bf16, randomize_affine=True, w_std=0.05) for l in range(2)]
    tol = H.TOL_BF16 if bf16 else H.TOL_F32
    own = H.make_stage(sh, layers, 0, 2, 5, bf16=bf16)          # reference: the stage's own workspace
    lean = H.make_stage(sh, layers, 0, 2, 1, bf16=bf16)         # max_batch 1: B is limited by the static workspace
    for B, tag in ((5, "first"), (2, "second")):                # the second call is smaller and finds the first one's leftovers
        x = synth.activations(sh, B, bf16=bf16, tag=tag)
        want = _run(own.forward, own.cfg, x)
        got = _run(lean.forward_static, lean.cfg, x)
        np.testing.assert_array_equal(got, want)
        ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
        assert H.rel_err(got, ref) <= tol
    own.destroy()
    lean.destroy()


def test_static_workspace_limit_is_enforced_at_the_real_width():
    import torch
    sh = synth.SHAPES["vit_huge"]
    layers = [synth.layer_params(sh, 0, bf16=True)]
    own = H.make_stage(sh, layers, 0, 1, 14, bf16=True)
    lean = H.make_stage(sh, layers, 0, 1, 1, bf16=True)
    x = synth.activations(sh, 14, bf16=True)                    # 14 * 257 rows: the largest micro-batch that fits 64 MiB
    want = _run(own.forward, own.cfg, x)
    got = _run(lean.forward_static, lean.cfg, x)
    np.testing.assert_array_equal(got, want)
    for i in (0, 13):
        assert H.rel_err(got[i], oracle.stage_forward(H.oracle_cfg(sh), layers, x[i:i + 1])[0]) <= H.TOL_BF16
    # a smaller call after it, then one past the limit: refused, nothing launched, output untouched
    # (compared at its own size: a micro-batch of 3 takes the second MLP layer through another schedule than one of 14)
    np.testing.assert_array_equal(_run(lean.forward_static, lean.cfg, x[:3]), _run(own.forward, own.cfg, x[:3]))
    big = torch.zeros((15,) + x.shape[1:], dtype=torch.int16, device="cuda")
    out = torch.full((15,) + x.shape[1:], 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.EdgePipeError) as ei:
        lean.forward_static(big, 15, out, torch.cuda.current_stream())
    assert ei.value.status == binding.EP_ERR_UNSUPPORTED and "workspace" in str(ei.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    with pytest.raises(binding.EdgePipeError):
        lean.forward_static(big, 0, out, torch.cuda.current_stream())
    own.destroy()
    lean.destroy()
