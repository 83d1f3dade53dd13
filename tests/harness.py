"""Shared plumbing of the GPU parity tests: build a stage from seeded host
parameters, run it through the C ABI on torch-owned device memory, run the CPU
checker on the same host buffers, and measure the error the way the tolerance
is stated (max |gpu - ref| over the RMS of ref)."""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np

import oracle
from paper_2110_14895_amd import binding, synth

TOL_F32 = 1e-4    # fp32 path: max-abs error / output RMS
TOL_BF16 = 2e-2   # bf16 path, against the un-rounded float64 result


def oracle_cfg(sh: synth.VitShape, **kw) -> oracle.OracleConfig:
    return oracle.OracleConfig(sh.d_model, sh.n_heads, sh.d_mlp, sh.n_tokens, sh.ln_eps, **kw)


def vit_config(sh: synth.VitShape, *, bf16: bool, in_bf16: Optional[bool] = None,
               out_bf16: bool = False) -> binding.VitConfig:
    if in_bf16 is None:
        in_bf16 = bf16
    return binding.VitConfig(sh.n_layers, sh.d_model, sh.n_heads, sh.d_mlp, sh.n_tokens, sh.ln_eps,
                             binding.EP_BF16 if bf16 else binding.EP_F32,
                             binding.EP_BF16 if in_bf16 else binding.EP_F32,
                             binding.EP_BF16 if out_bf16 else binding.EP_F32)


def make_stage(sh, layers: Sequence[Dict[str, np.ndarray]], begin: int, end: int, max_batch: int, *,
               bf16: bool, in_bf16: Optional[bool] = None, out_bf16: bool = False) -> binding.Stage:
    cfg = vit_config(sh, bf16=bf16, in_bf16=in_bf16, out_bf16=out_bf16)
    dev_layers = [synth.as_param_dtype(p, bf16) for p in layers]
    return binding.Stage(cfg, begin, end, dev_layers, max_batch)


def to_device(x: np.ndarray, as_bf16: bool):
    import torch
    if as_bf16:
        bits = synth.f32_to_bf16_bits(x).reshape(x.shape)
        return torch.from_numpy(bits.view(np.int16)).cuda()
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def run_stage(stage: binding.Stage, x: np.ndarray, *, stream=None, keep_device: bool = False):
    """x float32 host [B, T, D] (bf16-representable if the stage takes bf16) -> float32 host output."""
    import torch
    cfg = stage.cfg
    B = x.shape[0]
    xin = to_device(x, cfg.in_dtype == binding.EP_BF16)
    if cfg.out_dtype == binding.EP_BF16:
        out = torch.empty(x.shape, dtype=torch.int16, device="cuda")
    else:
        out = torch.empty(x.shape, dtype=torch.float32, device="cuda")
    s = stream if stream is not None else torch.cuda.current_stream()
    stage.forward(xin, B, out, s)
    torch.cuda.synchronize()
    if keep_device:
        return out
    if cfg.out_dtype == binding.EP_BF16:
        return synth.bf16_bits_to_f32(out.cpu().numpy().view(np.uint16)).reshape(x.shape)
    return out.cpu().numpy()


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / sqrt(mean ref^2)"""
    ref = np.asarray(ref, dtype=np.float64)
    rms = math.sqrt(float(np.mean(ref * ref)))
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref))) / rms


def err_std(got: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    rms = math.sqrt(float(np.mean(ref * ref)))
    return float(np.std(np.asarray(got, dtype=np.float64) - ref)) / rms
