"""ctypes front end of vit_oracle.c (test infrastructure, not the product).

All activations are float64 numpy arrays; parameters are float32 arrays with
the names q|k|v-fused ViT layers use: ln1_g ln1_b w_qkv b_qkv w_o b_o ln2_g
ln2_b w_fc1 b_fc1 w_fc2 b_fc2, weights stored [out, in].
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import numpy as np

from . import build as _build

_PARAMS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
           "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
_FP = C.POINTER(C.c_float)
_DP = C.POINTER(C.c_double)


class _Cfg(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_mlp", C.c_int32),
                ("n_tokens", C.c_int32), ("ln_eps", C.c_double), ("round_mode", C.c_int32)]


class _Layer(C.Structure):
    _fields_ = [(n, _FP) for n in _PARAMS]


@dataclass
class OracleConfig:
    d_model: int
    n_heads: int
    d_mlp: int
    n_tokens: int
    ln_eps: float = 1e-6
    round_mode: int = 0   # 1 = diagnostic bf16 rounding of GEMM operands

    def _c(self) -> _Cfg:
        return _Cfg(self.d_model, self.n_heads, self.d_mlp, self.n_tokens, self.ln_eps,
                    self.round_mode)


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        L.epo_layernorm.argtypes = [_DP, C.c_int64, C.c_int32, _FP, _FP, C.c_double, _DP]
        L.epo_linear.argtypes = [_DP, C.c_int64, C.c_int32, _FP, _FP, C.c_int32, _DP]
        L.epo_gelu.argtypes = [_DP, C.c_int64, _DP]
        L.epo_attention.argtypes = [_DP, C.c_int32, C.c_int32, C.c_int32, C.c_int, _DP, _DP]
        L.epo_layer_forward.argtypes = [C.POINTER(_Cfg), C.POINTER(_Layer), C.c_int32, _DP]
        L.epo_stage_forward.argtypes = [C.POINTER(_Cfg), C.c_int32, C.POINTER(_Layer), _FP,
                                        C.c_int32, _DP]
        L.epo_round_bf16.argtypes = [C.c_double]
        L.epo_round_bf16.restype = C.c_double
        for f in (L.epo_layer_forward, L.epo_stage_forward, L.epo_num_threads):
            f.restype = C.c_int
        _lib = L
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _fp(a: np.ndarray):
    return a.ctypes.data_as(_FP)


def _dp(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_DP) if a is not None else None


def num_threads() -> int:
    return int(lib().epo_num_threads())


def round_bf16(v: float) -> float:
    """The narrowing the diagnostic mode applies at the five operand points: float64 -> float32 ->
    bf16, both steps round-to-nearest-even; infinities and NaN pass through."""
    return float(lib().epo_round_bf16(float(v)))


def layernorm(x, g, b, eps: float) -> np.ndarray:
    x = _f64(x)
    D = x.shape[-1]
    g, b = _f32(g), _f32(b)
    y = np.empty_like(x)
    lib().epo_layernorm(_dp(x), x.size // D, D, _fp(g), _fp(b), eps, _dp(y))
    return y


def linear(x, w, bias) -> np.ndarray:
    x = _f64(x)
    w, bias = _f32(w), _f32(bias)
    N, K = w.shape
    assert x.shape[-1] == K and bias.shape == (N,)
    y = np.empty(x.shape[:-1] + (N,), dtype=np.float64)
    lib().epo_linear(_dp(x), x.size // K, K, _fp(w), _fp(bias), N, _dp(y))
    return y


def gelu(x) -> np.ndarray:
    x = _f64(x)
    y = np.empty_like(x)
    lib().epo_gelu(_dp(x), x.size, _dp(y))
    return y


def attention(qkv, n_heads: int, round_mode: int = 0, return_probs: bool = False):
    """qkv [T, 3D] of one image -> o [T, D] (and p [H, T, T])."""
    qkv = _f64(qkv)
    T, D3 = qkv.shape
    D = D3 // 3
    o = np.empty((T, D), dtype=np.float64)
    p = np.empty((n_heads, T, T), dtype=np.float64) if return_probs else None
    lib().epo_attention(_dp(qkv), T, D, n_heads, round_mode, _dp(o), _dp(p))
    return (o, p) if return_probs else o


def _layer_struct(params: Dict[str, np.ndarray], keep: list) -> _Layer:
    s = _Layer()
    for n in _PARAMS:
        a = _f32(params[n])
        keep.append(a)
        setattr(s, n, _fp(a))
    return s


def layer_forward(cfg: OracleConfig, params: Dict[str, np.ndarray], x) -> np.ndarray:
    """One encoder layer on x [B, T, D]; returns a new float64 array."""
    x = _f64(x).copy()
    assert x.ndim == 3 and x.shape[1:] == (cfg.n_tokens, cfg.d_model)
    keep: list = []
    s = _layer_struct(params, keep)
    c = cfg._c()
    rc = lib().epo_layer_forward(C.byref(c), C.byref(s), x.shape[0], _dp(x))
    if rc:
        raise RuntimeError(f"epo_layer_forward failed: {rc}")
    return x


def stage_forward(cfg: OracleConfig, layers: Sequence[Dict[str, np.ndarray]], x_in) -> np.ndarray:
    """A stage (consecutive layers, in order) on float32 x_in [B, T, D] -> float64."""
    x_in = _f32(x_in)
    assert x_in.ndim == 3 and x_in.shape[1:] == (cfg.n_tokens, cfg.d_model)
    keep: list = []
    arr = (_Layer * max(1, len(layers)))()
    for i, p in enumerate(layers):
        arr[i] = _layer_struct(p, keep)
    out = np.empty(x_in.shape, dtype=np.float64)
    c = cfg._c()
    rc = lib().epo_stage_forward(C.byref(c), len(layers), arr, _fp(x_in), x_in.shape[0], _dp(out))
    if rc:
        raise RuntimeError(f"epo_stage_forward failed: {rc}")
    return out
