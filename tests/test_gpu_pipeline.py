"""Pipeline of stages on one GPU (section 3.1: micro-batches flow through parts of
consecutive layers): results must be those of the whole model on every micro-batch,
for any cut and any number of micro-batches, and the schedule must keep working
when the caller's stream has work before and after it."""
import numpy as np
import pytest

from tests import harness as H
import oracle
from paper_2110_14895_amd import binding, synth

pytestmark = pytest.mark.gpu


def layers_of(sh, n, bf16):
    return [synth.layer_params(sh, l, bf16=bf16, randomize_affine=True) for l in range(n)]


def build(sh, layers, cuts, mb, *, bf16, boundary_bf16=False):
    """Stages for the layer ranges [cuts[k], cuts[k+1]); the first takes the model's input dtype,
    boundaries are fp32 (or bf16), the last returns fp32."""
    stages = []
    for k in range(len(cuts) - 1):
        first, last = k == 0, k == len(cuts) - 2
        stages.append(H.make_stage(sh, layers[cuts[k]:cuts[k + 1]], cuts[k], cuts[k + 1], mb, bf16=bf16,
                                   in_bf16=(bf16 if first else boundary_bf16),
                                   out_bf16=(False if last else boundary_bf16)))
    return stages


@pytest.mark.parametrize("cuts,n_micro", [((0, 2, 3, 6), 5), ((0, 1, 6), 1), ((0, 6), 3), ((0, 1, 2, 3, 4, 5, 6), 4)])
def test_pipeline_equals_whole_model_bf16(cuts, n_micro):
    import torch
    sh = synth.custom_shape("pipe", 6, 256, 4, 512, 197)
    mb = 4
    layers = layers_of(sh, 6, True)
    whole = H.make_stage(sh, layers, 0, 6, mb, bf16=True)
    stages = build(sh, layers, cuts, mb, bf16=True)
    pipe = binding.Pipeline(stages, mb)
    x = synth.activations(sh, mb * n_micro, bf16=True)
    xin = H.to_device(x, True)
    out = torch.full(x.shape, float("nan"), dtype=torch.float32, device="cuda")
    pipe.run(xin, n_micro, out, torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for m in range(n_micro):
        ref = H.run_stage(whole, x[m * mb:(m + 1) * mb])
        np.testing.assert_array_equal(got[m * mb:(m + 1) * mb], ref)     # fp32 boundaries: same arithmetic
    # and the whole thing against the checker on one image of the last micro-batch
    i = mb * n_micro - 1
    r = oracle.stage_forward(H.oracle_cfg(sh), layers, x[i:i + 1])[0]
    assert H.rel_err(got[i], r) <= H.TOL_BF16
    pipe.destroy()


def test_pipeline_fp32_path_and_repeated_runs_on_a_side_stream():
    import torch
    sh = synth.SHAPES["tiny"]
    mb, n_micro = 3, 4
    layers = layers_of(sh, 2, False)
    stages = build(sh, layers, (0, 1, 2), mb, bf16=False)
    pipe = binding.Pipeline(stages, mb)
    x = synth.activations(sh, mb * n_micro, bf16=False)
    ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
    side = torch.cuda.Stream()
    xin = torch.empty(x.shape, dtype=torch.float32, device="cuda")
    out = torch.empty(x.shape, dtype=torch.float32, device="cuda")
    host = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    for rep in range(3):
        with torch.cuda.stream(side):
            xin.copy_(host.cuda(non_blocking=False) * (rep + 1) / (rep + 1))   # work before the run ...
            pipe.run(xin, n_micro, out, side)
            res = out * 1.0                                                     # ... and after it, same stream
        side.synchronize()
        assert H.rel_err(res.cpu().numpy(), ref) <= H.TOL_F32
    pipe.destroy()


def test_pipeline_bf16_boundaries_stay_within_tolerance():
    import torch
    sh = synth.custom_shape("pipe_b", 4, 256, 4, 512, 65)
    mb, n_micro = 8, 3
    layers = layers_of(sh, 4, True)
    stages = build(sh, layers, (0, 2, 4), mb, bf16=True, boundary_bf16=True)
    pipe = binding.Pipeline(stages, mb)
    x = synth.activations(sh, mb * n_micro, bf16=True)
    out = torch.empty(x.shape, dtype=torch.float32, device="cuda")
    pipe.run(H.to_device(x, True), n_micro, out, torch.cuda.current_stream())
    torch.cuda.synchronize()
    ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
    assert H.rel_err(out.cpu().numpy(), ref) <= H.TOL_BF16
    pipe.destroy()


def test_pipeline_rejects_bad_chains():
    sh = synth.custom_shape("pipe_e", 4, 128, 2, 256, 33)
    layers = layers_of(sh, 4, True)
    a = H.make_stage(sh, layers[0:2], 0, 2, 4, bf16=True)
    b = H.make_stage(sh, layers[2:4], 2, 4, 4, bf16=True, in_bf16=False)
    gap = H.make_stage(sh, layers[3:4], 3, 4, 4, bf16=True, in_bf16=False)
    small = H.make_stage(sh, layers[2:4], 2, 4, 2, bf16=True, in_bf16=False)
    wrong_dtype = H.make_stage(sh, layers[2:4], 2, 4, 4, bf16=True, in_bf16=True)
    binding.Pipeline([a, b], 4).destroy()
    for bad, mb in (([a, gap], 4), ([a, small], 4), ([a, wrong_dtype], 4), ([b, a], 4), ([a, b], 0)):
        with pytest.raises(binding.EdgePipeError) as ei:
            binding.Pipeline(bad, mb)
        assert ei.value.status == binding.EP_ERR_INVALID_ARG
    p = binding.Pipeline([a, b], 4)
    with pytest.raises(binding.EdgePipeError):
        p.run(None, 1, None)
    p.destroy()
