"""Seeded synthetic inputs for ViT encoder stages and for the partition planner.

This module only *draws numbers*: it holds none of the method's arithmetic
(no LayerNorm, attention, GEMM, cost model or partition logic) and is the one
piece of code that both the CPU checker and the GPU library's harness feed
from, so that both see bit-identical host buffers.

Generator.  A counter-based generator written out here so that no library
RNG stream is relied on:

* ``key``   = FNV-1a (64 bit) of a tensor's name string, xor the seed hashed
  through the splitmix64 finaliser;
* word ``c`` of a stream = splitmix64 finaliser of ``key + (c+1)*0x9E3779B97F4A7C15``;
* each 64-bit word gives two uniforms (high and low 32 bits) and one
  Box-Muller pair of standard normals, evaluated in float64.

Workload shapes follow the ViT models the paper evaluates (section 4, "Deep
Learning Models": ViT-Base / Large / Huge at 224x224 input) plus a tiny
configuration for fast checks.  Value distributions: weights N(0, std 0.02),
activations N(0, 1), biases 0 and LayerNorm gain 1 / shift 0 for benchmark
configurations, all randomised for unit tests.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np

_N_WORKERS = max(1, min(16, (os.cpu_count() or 1)))

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = 0x9E3779B97F4A7C15

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


# --------------------------------------------------------------------------
# counter-based generator
# --------------------------------------------------------------------------
def _fmix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wraps modulo 2**64)."""
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= np.uint64(0xBF58476D1CE4E5B9)
    z ^= z >> np.uint64(27)
    z *= np.uint64(0x94D049BB133111EB)
    z ^= z >> np.uint64(31)
    return z


def _fmix_int(z: int) -> int:
    z &= 0xFFFFFFFFFFFFFFFF
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
    z ^= z >> 31
    return z


def stream_key(name: str, seed: int = 0) -> int:
    """64-bit stream key of a tensor name and a seed."""
    h = 0xCBF29CE484222325
    for byte in name.encode("utf-8"):
        h ^= byte
        h = (h * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h ^ _fmix_int(seed + 0x5851F42D4C957F2D)


def _words(key: int, first: int, count: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        ctr = np.arange(first + 1, first + 1 + count, dtype=np.uint64)
        return _fmix(ctr * np.uint64(_GOLDEN) + np.uint64(key))


def uniform(name: str, n: int, seed: int = 0) -> np.ndarray:
    """n float64 uniforms in [0, 1) (32 bits of resolution each)."""
    key = stream_key(name, seed)
    w = _words(key, 0, (n + 1) // 2)
    out = np.empty(2 * w.size, dtype=np.float64)
    out[0::2] = (w >> np.uint64(32)).astype(np.float64) * (1.0 / 4294967296.0)
    out[1::2] = (w & np.uint64(0xFFFFFFFF)).astype(np.float64) * (1.0 / 4294967296.0)
    return out[:n]


def _normal_chunk(key: int, first: int, cnt: int, out: np.ndarray) -> None:
    w = _words(key, first, cnt)
    u1 = ((w >> np.uint64(32)).astype(np.float64) + 1.0) * (1.0 / 4294967296.0)  # (0, 1]
    u2 = (w & np.uint64(0xFFFFFFFF)).astype(np.float64) * (1.0 / 4294967296.0)  # [0, 1)
    r = np.sqrt(-2.0 * np.log(u1))
    ang = (2.0 * np.pi) * u2
    out[2 * first:2 * (first + cnt):2] = r * np.cos(ang)
    out[2 * first + 1:2 * (first + cnt):2] = r * np.sin(ang)


def normal(name: str, n: int, seed: int = 0, chunk: int = 1 << 20) -> np.ndarray:
    """n float64 standard normals: Box-Muller on the stream's 32-bit uniforms.
    Word c of the stream always yields elements 2c and 2c+1, so the result does
    not depend on chunking or on the number of worker threads."""
    key = stream_key(name, seed)
    pairs = (n + 1) // 2
    out = np.empty(2 * pairs, dtype=np.float64)
    starts = list(range(0, pairs, chunk))
    if len(starts) <= 1:
        for first in starts:
            _normal_chunk(key, first, min(chunk, pairs - first), out)
    else:
        with ThreadPoolExecutor(max_workers=min(_N_WORKERS, len(starts))) as pool:
            list(pool.map(lambda f: _normal_chunk(key, f, min(chunk, pairs - f), out), starts))
    return out[:n]


# --------------------------------------------------------------------------
# bf16 storage helpers (round-to-nearest-even narrowing, exact widening)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 array of bf16 bit patterns, round to nearest even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = bits + np.uint32(0x7FFF) + lsb
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bf16-representable float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


# --------------------------------------------------------------------------
# model shapes
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class VitShape:
    """Encoder shape: L layers, width D, H heads, MLP width M, T tokens."""
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    d_mlp: int
    n_tokens: int
    ln_eps: float = 1e-6

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    def flops_per_image_per_layer(self) -> float:
        """2 FLOP per multiply-add over the four dense layers and the two
        attention products; normalisation, softmax, GELU, bias and residual
        are not counted."""
        t, d, m = self.n_tokens, self.d_model, self.d_mlp
        return 2.0 * t * d * (3 * d) + 2.0 * t * d * d + 4.0 * t * d * m + 4.0 * t * t * d

    def param_shapes(self) -> Dict[str, tuple]:
        d, m = self.d_model, self.d_mlp
        return {"ln1_g": (d,), "ln1_b": (d,), "w_qkv": (3 * d, d), "b_qkv": (3 * d,),
                "w_o": (d, d), "b_o": (d,), "ln2_g": (d,), "ln2_b": (d,),
                "w_fc1": (m, d), "b_fc1": (m,), "w_fc2": (d, m), "b_fc2": (d,)}


SHAPES = {
    # 32x32 image, patch 4, plus CLS
    "tiny": VitShape("tiny", 2, 192, 3, 768, 65),
    # 224x224 image, patch 16, plus CLS
    "vit_base": VitShape("vit_base", 12, 768, 12, 3072, 197),
    "vit_large": VitShape("vit_large", 24, 1024, 16, 4096, 197),
    # 224x224 image, patch 14, plus CLS
    "vit_huge": VitShape("vit_huge", 32, 1280, 16, 5120, 257),
    # the smaller encoders of section 5.4 (DeiT-Tiny / -Small / -Base widths), 224x224 image,
    # patch 16, plus CLS; 12 layers each, heads of 64
    "deit_tiny": VitShape("deit_tiny", 12, 192, 3, 768, 197),
    "deit_small": VitShape("deit_small", 12, 384, 6, 1536, 197),
}


def custom_shape(name: str, n_layers: int, d_model: int, n_heads: int, d_mlp: int,
                 n_tokens: int, ln_eps: float = 1e-6) -> VitShape:
    return VitShape(name, n_layers, d_model, n_heads, d_mlp, n_tokens, ln_eps)


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------
def layer_params(shape: VitShape, layer: int, seed: int = 0, *, bf16: bool = False,
                 randomize_affine: bool = False, w_std: float = 0.02) -> Dict[str, np.ndarray]:
    """float32 parameters of one encoder layer (values bf16-representable if bf16).

    Benchmark recipe: weights N(0, w_std), biases 0, gain 1, shift 0.
    With randomize_affine: biases N(0, 0.1), gains 1 + N(0, 0.1), shifts N(0, 0.1).
    """
    out: Dict[str, np.ndarray] = {}
    for pname, shp in shape.param_shapes().items():
        n = int(np.prod(shp))
        tag = f"{shape.name}/L{layer}/{pname}"
        if pname.startswith("w_"):
            a = normal(tag, n, seed) * w_std
        elif randomize_affine:
            a = normal(tag, n, seed) * 0.1
            if pname.endswith("_g"):
                a = a + 1.0
        else:
            a = np.ones(n) if pname.endswith("_g") else np.zeros(n)
        a = a.astype(np.float32).reshape(shp)
        out[pname] = round_to_bf16(a).reshape(shp) if bf16 else a
    return out


def activations(shape: VitShape, batch: int, seed: int = 0, *, bf16: bool = False,
                tag: str = "x", first_image: int = 0) -> np.ndarray:
    """float32 [batch, T, D] N(0,1) input activations.  Image b of the batch is
    its own stream, so a sample of images can be regenerated alone."""
    t, d = shape.n_tokens, shape.d_model
    out = np.empty((batch, t, d), dtype=np.float32)
    for b in range(batch):
        a = normal(f"{shape.name}/{tag}/img{first_image + b}", t * d, seed)
        out[b] = a.astype(np.float32).reshape(t, d)
    return round_to_bf16(out).reshape(out.shape) if bf16 else out


# --------------------------------------------------------------------------
# planner inputs
# --------------------------------------------------------------------------
@dataclass
class PartitionInstance:
    """Plain arrays of a partition problem (section 3.2-3.3 symbols):
    t_comp[L, D] seconds, layer_mem[L] and dev_mem[D] bytes, xfer_bytes[L]
    (P_j), bw[D, D] bytes/s from sender u (row) to receiver v (column)."""
    t_comp: np.ndarray
    layer_mem: np.ndarray
    dev_mem: np.ndarray
    xfer_bytes: np.ndarray
    bw: np.ndarray

    @property
    def n_layers(self) -> int:
        return self.t_comp.shape[0]

    @property
    def n_devices(self) -> int:
        return self.t_comp.shape[1]


def random_partition_instance(n_layers: int, n_devices: int, seed: int, *,
                              mem_tight: float = 0.0, comm_heavy: float = 0.0,
                              quantize: Optional[int] = None) -> PartitionInstance:
    """Small random instance for checking the planner against enumeration.

    mem_tight in [0,1): how binding the memory limits are; comm_heavy scales
    transfer sizes up so that links, not compute, bound the period.  quantize=q
    snaps every quantity to a multiple of 1/q so that ties are common.
    """
    L, D = n_layers, n_devices
    tag = f"part/{L}x{D}"
    base = 0.5 + uniform(tag + "/base", L, seed)
    speed = 1.0 + 7.0 * uniform(tag + "/speed", D, seed)
    jit = 0.9 + 0.2 * uniform(tag + "/jit", L * D, seed).reshape(L, D)
    t_comp = base[:, None] / speed[None, :] * jit
    layer_mem = 1.0 + uniform(tag + "/lmem", L, seed)
    frac = 1.0 - mem_tight * (0.2 + 0.8 * uniform(tag + "/dmem", D, seed))
    dev_mem = layer_mem.sum() * frac
    bw = 0.5 + 9.5 * uniform(tag + "/bw", D * D, seed).reshape(D, D)
    xfer = (0.2 + uniform(tag + "/xfer", L, seed)) * (1.0 + 20.0 * comm_heavy)
    if quantize:
        q = float(quantize)
        t_comp = np.maximum(np.round(t_comp * q), 1.0) / q
        layer_mem = np.maximum(np.round(layer_mem * q), 1.0) / q
        dev_mem = np.round(dev_mem * q) / q
        bw = np.maximum(np.round(bw * q), 1.0) / q
        xfer = np.maximum(np.round(xfer * q), 1.0) / q
    return PartitionInstance(np.ascontiguousarray(t_comp), layer_mem, dev_mem, xfer,
                             np.ascontiguousarray(bw))


def category_partition_instance(n_layers: int, counts, seed: int, *, shuffle: bool = True,
                                **kw) -> PartitionInstance:
    """A cluster of N = len(counts) device types with counts[c] identical devices of type c
    (section 3.3's setting for the category dynamic program): a random instance over the N types
    is drawn with random_partition_instance and expanded per device; two devices of one type
    are linked at that type's own diagonal bandwidth.  shuffle=True scatters the types over the
    device ids (seeded), so that categories are not runs of consecutive ids."""
    counts = [int(c) for c in counts]
    N, D = len(counts), int(sum(counts))
    base = random_partition_instance(n_layers, N, seed, **kw)
    cat = np.repeat(np.arange(N), counts)
    if shuffle:
        order = np.argsort(uniform(f"part/cat{N}x{D}/order", D, seed), kind="stable")
        cat = cat[order]
    t_comp = np.ascontiguousarray(base.t_comp[:, cat])
    dev_mem = base.dev_mem[cat].copy()
    bw = np.ascontiguousarray(base.bw[np.ix_(cat, cat)])
    # the diagonal of the type-level matrix is the link between two devices of one type; make it
    # symmetric by construction (it is a single number per type)
    return PartitionInstance(t_comp, base.layer_mem.copy(), dev_mem, base.xfer_bytes.copy(), bw)


def heterogeneous_cluster(layer_cost_s: np.ndarray, shape: VitShape, batch: int, *,
                          n_devices: int = 16, seed: int = 1, act_bytes: int = 4,
                          param_bytes: int = 2,
                          seconds_per_layer_image: float = 0.37) -> PartitionInstance:
    """Synthetic heterogeneous cluster for the planner.

    Devices: relative compute speed s_u ~ U[1,8] (larger is faster), memory
    m_u ~ U[1,8] GB, egress bandwidth bw_u ~ U[10,1000] Mb/s; the link u->v runs
    at the sender's egress rate.  Per-layer costs are the measured per-layer
    cost vector normalised to mean 1 and scaled so that a speed-1 device takes
    `seconds_per_layer_image` per layer per image (the single-board ViT-Huge
    rate implied by section 5.1: 1.01 images/s on 16 boards at 11.88x).
    Layer memory = parameter bytes of the layer; each device keeps a reserve
    for the activations of one micro-batch.  Transfer size P_j = bytes of the
    [batch, T, D] stage-boundary activation.
    """
    L = int(len(layer_cost_s))
    D = n_devices
    u = uniform(f"cluster/{D}", 3 * D, seed)
    speed = 1.0 + 7.0 * u[0:D]
    mem_gb = 1.0 + 7.0 * u[D:2 * D]
    bw_mbps = 10.0 + 990.0 * u[2 * D:3 * D]
    c = np.asarray(layer_cost_s, dtype=np.float64)
    rel = c / c.mean()
    t_comp = rel[:, None] * (seconds_per_layer_image * batch) / speed[None, :]
    n_par = sum(int(np.prod(s)) for s in shape.param_shapes().values())
    layer_mem = np.full(L, float(n_par * param_bytes))
    act = float(batch * shape.n_tokens * act_bytes)
    reserve = act * (2 * shape.d_model + max(3 * shape.d_model, shape.d_mlp))
    dev_mem = mem_gb * 1e9 - reserve
    xfer = np.full(L, act * shape.d_model)
    bw = np.repeat((bw_mbps * 1e6 / 8.0)[:, None], D, axis=1)
    return PartitionInstance(np.ascontiguousarray(t_comp), layer_mem, dev_mem, xfer,
                             np.ascontiguousarray(bw))


def surround_params(shape: VitShape, patch: int, channels: int, n_classes: int, seed: int = 0, *,
                    bf16: bool = False, w_std: float = 0.02) -> Dict[str, np.ndarray]:
    """float32 parameters of the patch embedding and of the classifier head for `shape`
    (T = 1 + number of patches): w_patch [D, C*P*P], b_patch [D], cls [D], pos [T, D],
    ln_g / ln_b [D] of the final LayerNorm, w_head [n_classes, D], b_head [n_classes].
    Weights N(0, w_std), class token and position embeddings N(0, w_std), biases and LayerNorm
    affine random so that every term shows; values bf16-representable if bf16."""
    D, T = shape.d_model, shape.n_tokens
    K = channels * patch * patch
    tag = f"{shape.name}/surround"
    p = {
        "w_patch": (w_std * normal(tag + "/w_patch", D * K, seed)).reshape(D, K),
        "b_patch": 0.1 * normal(tag + "/b_patch", D, seed),
        "cls": w_std * normal(tag + "/cls", D, seed),
        "pos": (w_std * normal(tag + "/pos", T * D, seed)).reshape(T, D),
        "ln_g": 1.0 + 0.1 * normal(tag + "/ln_g", D, seed),
        "ln_b": 0.1 * normal(tag + "/ln_b", D, seed),
        "w_head": (w_std * normal(tag + "/w_head", n_classes * D, seed)).reshape(n_classes, D),
        "b_head": 0.1 * normal(tag + "/b_head", n_classes, seed),
    }
    out = {}
    for k, v in p.items():
        v = v.astype(np.float32)
        out[k] = round_to_bf16(v) if bf16 else v
    return out


def images(batch: int, channels: int, size: int, seed: int = 0, first_image: int = 0) -> np.ndarray:
    """float32 [batch, channels, size, size] standard-normal pixels (normalised images), one
    stream per image so that image i is the same in any batch."""
    out = np.empty((batch, channels, size, size), dtype=np.float32)
    for i in range(batch):
        out[i] = normal(f"image/{channels}x{size}/{first_image + i}", channels * size * size, seed).reshape(
            channels, size, size).astype(np.float32)
    return out


def as_param_dtype(params: Dict[str, np.ndarray], bf16: bool) -> Dict[str, np.ndarray]:
    """Host arrays in the storage type a stage is created from: bf16 bit
    patterns (uint16; the values must already be bf16-representable) or float32."""
    if not bf16:
        return {k: np.ascontiguousarray(v, dtype=np.float32) for k, v in params.items()}
    out = {}
    for k, v in params.items():
        bits = f32_to_bf16_bits(v)
        if not np.array_equal(bf16_bits_to_f32(bits).reshape(np.shape(v)), np.asarray(v, dtype=np.float32)):
            raise ValueError(f"{k} holds values that are not bf16-representable")
        out[k] = bits.reshape(np.shape(v))
    return out
