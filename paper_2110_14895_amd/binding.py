"""ctypes binding of libedgepipe.so: same names as include/edgepipe.h, argument
marshalling only.  Every step of a stage's forward pass and of the planner
runs inside the library; nothing here computes, and there is no fallback: if
the library has not been built, loading raises.

Device buffers are passed as integers (addresses) or as any object with a
``data_ptr()`` method (e.g. a torch tensor); streams as integers or objects
with a ``cuda_stream`` attribute (e.g. ``torch.cuda.Stream``).
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

EP_OK, EP_ERR_INVALID_ARG, EP_ERR_UNSUPPORTED, EP_ERR_OOM, EP_ERR_HIP, EP_ERR_INFEASIBLE = range(6)
EP_F32, EP_BF16 = 0, 1

KERNEL_NAMES = ("ln1", "qkv", "attn", "proj", "ln2", "fc1", "fc2")   # ep_kernel_id order
# ids that time the first launch of a dense layer alone (EP_K_*_MAIN)
MAIN_KERNEL_IDS = {"qkv": 7, "proj": 8, "fc1": 9, "fc2": 10}
PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libedgepipe.so")


class EdgePipeError(RuntimeError):
    def __init__(self, status: int, where: str, text: str):
        super().__init__(f"{where}: {text or status_string(status)} [{status_string(status)}]")
        self.status = status


class ep_vit_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_mlp", C.c_int32), ("n_tokens", C.c_int32), ("ln_eps", C.c_float),
                ("param_dtype", C.c_int32), ("in_dtype", C.c_int32), ("out_dtype", C.c_int32)]


class ep_embed_config(C.Structure):
    _fields_ = [("image_size", C.c_int32), ("patch", C.c_int32), ("channels", C.c_int32), ("d_model", C.c_int32),
                ("param_dtype", C.c_int32), ("out_dtype", C.c_int32)]


class ep_head_config(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_tokens", C.c_int32), ("n_classes", C.c_int32), ("ln_eps", C.c_float),
                ("param_dtype", C.c_int32)]


class ep_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PARAM_NAMES]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if libedgepipe.so is missing (build it with
    ``python -m paper_2110_14895_amd.build`` or ``__graft_entry__.build()``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: the HIP library has not been built "
                               "(run `python paper_2110_14895_amd/build.py`); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        dp, ip = C.POINTER(C.c_double), C.POINTER(C.c_int32)
        L.ep_stage_create.argtypes = [C.POINTER(ep_vit_config), C.c_int32, C.c_int32,
                                      C.POINTER(ep_layer_weights), C.c_int32, C.POINTER(C.c_void_p)]
        L.ep_stage_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.ep_stage_forward_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.ep_stage_forward_static.restype = C.c_int
        L.ep_stage_profile.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, dp]
        L.ep_stage_trace_begin.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.ep_stage_trace_end.argtypes = [C.c_void_p, ip, dp]
        L.ep_stage_gemm_main_rows.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int64)]
        L.ep_stage_info.argtypes = [C.c_void_p, C.POINTER(ep_vit_config), ip, ip, ip]
        L.ep_pipeline_create.argtypes = [C.c_int32, C.POINTER(C.c_void_p), C.c_int32, C.POINTER(C.c_void_p)]
        L.ep_pipeline_run.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.ep_pipeline_destroy.argtypes = [C.c_void_p]
        L.ep_pipeline_destroy.restype = None
        vp = C.c_void_p
        L.ep_embed_create.argtypes = [C.POINTER(ep_embed_config), vp, vp, vp, vp, C.c_int32, C.POINTER(vp)]
        L.ep_embed_forward.argtypes = [vp, vp, C.c_int32, vp, vp]
        L.ep_embed_destroy.argtypes = [vp]
        L.ep_embed_destroy.restype = None
        L.ep_head_create.argtypes = [C.POINTER(ep_head_config), vp, vp, vp, vp, C.c_int32, C.POINTER(vp)]
        L.ep_head_forward.argtypes = [vp, vp, C.c_int32, vp, vp]
        L.ep_head_destroy.argtypes = [vp]
        L.ep_head_destroy.restype = None
        L.ep_stage_device_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_uint64)]
        L.ep_stage_destroy.argtypes = [C.c_void_p]
        L.ep_stage_destroy.restype = None
        L.ep_mfma_peak.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, dp, dp]
        L.ep_gemm_clock_sample.argtypes = [dp, dp]
        L.ep_gemm_clock_sample.restype = C.c_int
        L.ep_partition.argtypes = [C.c_int32, C.c_int32, dp, dp, dp, dp, dp, dp, ip, ip, ip, ip]
        L.ep_partition_categories.argtypes = [C.c_int32, C.c_int32, dp, dp, dp, dp, dp, dp, ip, ip, ip, ip, ip]
        L.ep_status_string.argtypes = [C.c_int]
        L.ep_status_string.restype = C.c_char_p
        L.ep_last_error.argtypes = []
        L.ep_last_error.restype = C.c_char_p
        for f in (L.ep_stage_create, L.ep_stage_forward, L.ep_stage_profile, L.ep_stage_trace_begin,
                  L.ep_stage_trace_end, L.ep_stage_gemm_main_rows, L.ep_stage_device_bytes, L.ep_partition,
                  L.ep_partition_categories, L.ep_stage_info, L.ep_pipeline_create, L.ep_pipeline_run,
                  L.ep_embed_create, L.ep_embed_forward, L.ep_head_create, L.ep_head_forward, L.ep_mfma_peak):
            f.restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().ep_status_string(int(status)).decode()


def last_error() -> str:
    return lib().ep_last_error().decode()


def _check(status: int, where: str) -> None:
    if status != EP_OK:
        raise EdgePipeError(status, where, last_error())


def _addr(buf) -> int:
    if buf is None:
        return 0
    if isinstance(buf, int):
        return buf
    return int(buf.data_ptr())


def _stream(stream) -> int:
    if stream is None:
        return 0
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


@dataclass
class VitConfig:
    n_layers: int
    d_model: int
    n_heads: int
    d_mlp: int
    n_tokens: int
    ln_eps: float = 1e-6
    param_dtype: int = EP_BF16
    in_dtype: int = EP_BF16
    out_dtype: int = EP_F32

    def c_struct(self) -> ep_vit_config:
        return ep_vit_config(self.n_layers, self.d_model, self.n_heads, self.d_mlp, self.n_tokens,
                             self.ln_eps, self.param_dtype, self.in_dtype, self.out_dtype)


class Stage:
    """ep_stage_create / ep_stage_forward / ep_stage_profile / ep_stage_destroy."""

    def __init__(self, cfg: VitConfig, layer_begin: int, layer_end: int,
                 layers: Sequence[Dict[str, np.ndarray]], max_batch: int):
        want = np.uint16 if cfg.param_dtype == EP_BF16 else np.float32
        self._keep: List[np.ndarray] = []
        arr = (ep_layer_weights * max(1, len(layers)))()
        for i, p in enumerate(layers):
            for name in PARAM_NAMES:
                a = np.ascontiguousarray(p[name])
                if a.dtype != want:
                    raise TypeError(f"layer {i} {name}: expected {np.dtype(want)} host array, got {a.dtype}")
                self._keep.append(a)
                setattr(arr[i], name, a.ctypes.data)
        self.cfg = cfg
        self.n_layers = layer_end - layer_begin
        self.max_batch = max_batch
        self._h = C.c_void_p()
        c = cfg.c_struct()
        if len(layers) != layer_end - layer_begin:
            raise ValueError("len(layers) must equal layer_end - layer_begin")
        _check(lib().ep_stage_create(C.byref(c), layer_begin, layer_end, arr, max_batch,
                                     C.byref(self._h)), "ep_stage_create")
        self._keep.clear()      # the library copied the parameters

    def forward(self, x_in, batch: int, x_out, stream=None) -> None:
        _check(lib().ep_stage_forward(self._h, _addr(x_in), batch, _addr(x_out), _stream(stream)),
               "ep_stage_forward")

    def forward_static(self, x_in, batch: int, x_out, stream=None) -> None:
        _check(lib().ep_stage_forward_static(self._h, _addr(x_in), int(batch), _addr(x_out), _stream(stream)),
               "ep_stage_forward_static")

    def profile(self, batch: int, iters: int = 5, stream=None) -> np.ndarray:
        out = np.zeros(self.n_layers, dtype=np.float64)
        _check(lib().ep_stage_profile(self._h, batch, iters, _stream(stream),
                                      out.ctypes.data_as(C.POINTER(C.c_double))), "ep_stage_profile")
        return out

    def trace_begin(self, kernel: int, max_launches: int) -> None:
        _check(lib().ep_stage_trace_begin(self._h, kernel, max_launches), "ep_stage_trace_begin")

    def trace_end(self) -> Tuple[int, float]:
        n, sec = C.c_int32(), C.c_double()
        _check(lib().ep_stage_trace_end(self._h, C.byref(n), C.byref(sec)), "ep_stage_trace_end")
        return int(n.value), float(sec.value)

    def gemm_main_rows(self, batch: int, kernel: int) -> int:
        v = C.c_int64()
        _check(lib().ep_stage_gemm_main_rows(self._h, batch, kernel, C.byref(v)), "ep_stage_gemm_main_rows")
        return int(v.value)

    def device_bytes(self) -> int:
        v = C.c_uint64()
        _check(lib().ep_stage_device_bytes(self._h, C.byref(v)), "ep_stage_device_bytes")
        return int(v.value)

    def destroy(self) -> None:
        if self._h:
            lib().ep_stage_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _host(a: np.ndarray, param_dtype: int, name: str) -> np.ndarray:
    want = np.uint16 if param_dtype == EP_BF16 else np.float32
    a = np.ascontiguousarray(a)
    if a.dtype != want:
        raise TypeError(f"{name}: expected {np.dtype(want)} host array, got {a.dtype}")
    return a


class Embed:
    """ep_embed_*: images [B, C, S, S] fp32 -> token sequence [B, T, D].  Host parameters in
    param_dtype storage (uint16 bf16 bit patterns or float32): w_patch [D, C*P*P], b_patch [D],
    cls [D], pos [T, D]."""

    def __init__(self, image_size: int, patch: int, channels: int, d_model: int, param_dtype: int, out_dtype: int,
                 params: Dict[str, np.ndarray], max_batch: int):
        cfg = ep_embed_config(image_size, patch, channels, d_model, param_dtype, out_dtype)
        keep = [_host(params[k], param_dtype, k) for k in ("w_patch", "b_patch", "cls", "pos")]
        self._h = C.c_void_p()
        _check(lib().ep_embed_create(C.byref(cfg), *[a.ctypes.data for a in keep], max_batch, C.byref(self._h)),
               "ep_embed_create")
        self.n_tokens = 1 + (image_size // patch) ** 2

    def forward(self, images, batch: int, x_out, stream=None) -> None:
        _check(lib().ep_embed_forward(self._h, _addr(images), batch, _addr(x_out), _stream(stream)), "ep_embed_forward")

    def destroy(self) -> None:
        if self._h:
            lib().ep_embed_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Head:
    """ep_head_*: x [B, T, D] fp32 -> logits [B, n_classes] fp32.  Host parameters ln_g, ln_b [D],
    w_head [n_classes, D], b_head [n_classes] in param_dtype storage."""

    def __init__(self, d_model: int, n_tokens: int, n_classes: int, ln_eps: float, param_dtype: int,
                 params: Dict[str, np.ndarray], max_batch: int):
        cfg = ep_head_config(d_model, n_tokens, n_classes, ln_eps, param_dtype)
        keep = [_host(params[k], param_dtype, k) for k in ("ln_g", "ln_b", "w_head", "b_head")]
        self._h = C.c_void_p()
        _check(lib().ep_head_create(C.byref(cfg), *[a.ctypes.data for a in keep], max_batch, C.byref(self._h)),
               "ep_head_create")

    def forward(self, x, batch: int, logits, stream=None) -> None:
        _check(lib().ep_head_forward(self._h, _addr(x), batch, _addr(logits), _stream(stream)), "ep_head_forward")

    def destroy(self) -> None:
        if self._h:
            lib().ep_head_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Pipeline:
    """ep_pipeline_*: stages on one device, micro-batches flowing through them on one stream per
    stage.  Borrows the Stage objects (keep them alive; destroy the pipeline first)."""

    def __init__(self, stages, micro_batch: int):
        self._stages = list(stages)
        arr = (C.c_void_p * len(self._stages))(*[st._h for st in self._stages])
        h = C.c_void_p()
        _check(lib().ep_pipeline_create(len(self._stages), arr, micro_batch, C.byref(h)), "ep_pipeline_create")
        self._h = h
        self.micro_batch = micro_batch

    def run(self, x_in, n_micro: int, x_out, stream=None) -> None:
        _check(lib().ep_pipeline_run(self._h, _addr(x_in), n_micro, _addr(x_out), _stream(stream)), "ep_pipeline_run")

    def destroy(self) -> None:
        if self._h:
            lib().ep_pipeline_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def mfma_peak(form: int, random_operands: bool, iters: int, stream=None) -> Tuple[float, float]:
    """(TFLOP/s, shader MHz) of a loop of nothing but bf16 matrix instructions on the current device."""
    tf, mhz = C.c_double(), C.c_double()
    _check(lib().ep_mfma_peak(int(form), int(bool(random_operands)), int(iters), _stream(stream),
                              C.byref(tf), C.byref(mhz)), "ep_mfma_peak")
    return tf.value, mhz.value


def gemm_clock_sample() -> Tuple[float, float]:
    """(shader MHz, seconds) of workgroup 0 of the most recent large dense-layer launch that finished."""
    mhz, sec = C.c_double(), C.c_double()
    _check(lib().ep_gemm_clock_sample(C.byref(mhz), C.byref(sec)), "ep_gemm_clock_sample")
    return mhz.value, sec.value


def partition_categories(t_comp, layer_mem, dev_mem, xfer_bytes, bw):
    """ep_partition_categories.  Returns (T_opt, [(device, first_layer, last_layer), ...], n_categories)."""
    t_comp = np.ascontiguousarray(t_comp, dtype=np.float64)
    if t_comp.ndim != 2:
        raise ValueError("t_comp must be [L, D]")
    L, D = t_comp.shape
    layer_mem = np.ascontiguousarray(layer_mem, dtype=np.float64)
    dev_mem = np.ascontiguousarray(dev_mem, dtype=np.float64)
    xfer_bytes = np.ascontiguousarray(xfer_bytes, dtype=np.float64)
    bw = np.ascontiguousarray(bw, dtype=np.float64)
    if layer_mem.shape != (L,) or xfer_bytes.shape != (L,) or dev_mem.shape != (D,) or bw.shape != (D, D):
        raise ValueError("array shapes do not match t_comp [L, D]")
    dp, ip = C.POINTER(C.c_double), C.POINTER(C.c_int32)
    t_opt, n, ncat = C.c_double(), C.c_int32(), C.c_int32()
    dev = np.zeros(D, dtype=np.int32)
    first = np.zeros(D, dtype=np.int32)
    last = np.zeros(D, dtype=np.int32)
    _check(lib().ep_partition_categories(L, D, t_comp.ctypes.data_as(dp), layer_mem.ctypes.data_as(dp),
                                         dev_mem.ctypes.data_as(dp), xfer_bytes.ctypes.data_as(dp),
                                         bw.ctypes.data_as(dp), C.byref(t_opt), C.byref(n),
                                         dev.ctypes.data_as(ip), first.ctypes.data_as(ip),
                                         last.ctypes.data_as(ip), C.byref(ncat)), "ep_partition_categories")
    return t_opt.value, [(int(dev[s]), int(first[s]), int(last[s])) for s in range(n.value)], int(ncat.value)


def partition(t_comp, layer_mem, dev_mem, xfer_bytes, bw) -> Tuple[float, List[Tuple[int, int, int]]]:
    """ep_partition.  Returns (T_opt, [(device, first_layer, last_layer), ...])."""
    t_comp = np.ascontiguousarray(t_comp, dtype=np.float64)
    if t_comp.ndim != 2:
        raise ValueError("t_comp must be [L, D]")
    L, D = t_comp.shape
    layer_mem = np.ascontiguousarray(layer_mem, dtype=np.float64)
    dev_mem = np.ascontiguousarray(dev_mem, dtype=np.float64)
    xfer_bytes = np.ascontiguousarray(xfer_bytes, dtype=np.float64)
    bw = np.ascontiguousarray(bw, dtype=np.float64)
    if layer_mem.shape != (L,) or xfer_bytes.shape != (L,) or dev_mem.shape != (D,) or bw.shape != (D, D):
        raise ValueError("array shapes do not match t_comp [L, D]")
    dp, ip = C.POINTER(C.c_double), C.POINTER(C.c_int32)
    t_opt, n = C.c_double(), C.c_int32()
    dev = np.zeros(D, dtype=np.int32)
    first = np.zeros(D, dtype=np.int32)
    last = np.zeros(D, dtype=np.int32)
    _check(lib().ep_partition(L, D, t_comp.ctypes.data_as(dp), layer_mem.ctypes.data_as(dp),
                              dev_mem.ctypes.data_as(dp), xfer_bytes.ctypes.data_as(dp),
                              bw.ctypes.data_as(dp), C.byref(t_opt), C.byref(n),
                              dev.ctypes.data_as(ip), first.ctypes.data_as(ip),
                              last.ctypes.data_as(ip)), "ep_partition")
    return t_opt.value, [(int(dev[s]), int(first[s]), int(last[s])) for s in range(n.value)]
