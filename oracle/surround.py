"""What stands before the first and after the last encoder layer of a vision
transformer (test infrastructure, not the product): patch embedding with class
token and position embeddings, and final LayerNorm + classifier on the class
token.  The paper places the embedding outside the transformer layers (section
4, "Deep Learning Models": images are brought to a uniform input dimension by
the embedding layer) and takes the model definition from the original ViT; this
file states that definition in float64, with plain loops over patches and
library matmul / the C routines of vit_oracle.c as steps.
"""
from __future__ import annotations

import numpy as np

from . import vit


def patches(images, patch: int) -> np.ndarray:
    """images [B, C, H, W] -> [B, (H/P)*(W/P), C*P*P] float64.  Patches in row-major order
    of the patch grid; inside a patch the order is (channel, row, column), the order in which a
    convolution weight [D, C, P, P] is flattened."""
    x = np.asarray(images, dtype=np.float64)
    B, C, H, W = x.shape
    if H % patch or W % patch:
        raise ValueError("image size must be a multiple of the patch size")
    gh, gw = H // patch, W // patch
    out = np.empty((B, gh * gw, C * patch * patch), dtype=np.float64)
    for py in range(gh):
        for px in range(gw):
            blk = x[:, :, py * patch:(py + 1) * patch, px * patch:(px + 1) * patch]   # [B, C, P, P]
            out[:, py * gw + px, :] = blk.reshape(B, -1)
    return out


def embed_forward(images, w_patch, b_patch, cls, pos, patch: int) -> np.ndarray:
    """Token sequence fed to layer 0: row 0 = class token + pos[0]; row 1+p = linear projection
    of patch p (+ bias) + pos[1+p].  w_patch [D, C*P*P], pos [T, D] with T = 1 + number of patches."""
    pt = patches(images, patch)
    B, NP, K = pt.shape
    w = np.asarray(w_patch, dtype=np.float64)
    D = w.shape[0]
    pos = np.asarray(pos, dtype=np.float64)
    if w.shape != (D, K) or pos.shape != (NP + 1, D):
        raise ValueError("shapes of w_patch / pos do not match the images")
    x = np.empty((B, NP + 1, D), dtype=np.float64)
    x[:, 0, :] = np.asarray(cls, dtype=np.float64)[None, :] + pos[0][None, :]
    proj = vit.linear(pt.reshape(B * NP, K), np.asarray(w_patch, dtype=np.float32), np.asarray(b_patch, dtype=np.float32))
    x[:, 1:, :] = proj.reshape(B, NP, D) + pos[1:][None, :, :]
    return x


def head_forward(x, ln_g, ln_b, eps: float, w_head, b_head) -> np.ndarray:
    """Logits [B, n_classes]: LayerNorm of the class-token row of the last layer's output, then
    the classifier; the other rows do not enter."""
    x = np.asarray(x, dtype=np.float64)
    z = vit.layernorm(np.ascontiguousarray(x[:, 0, :]), np.asarray(ln_g, dtype=np.float32),
                      np.asarray(ln_b, dtype=np.float32), eps)
    return vit.linear(z, np.asarray(w_head, dtype=np.float32), np.asarray(b_head, dtype=np.float32))
