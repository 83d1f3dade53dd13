"""GPU parity of the parts around the encoder (ep_embed_*, ep_head_*) against the float64
checker, and images -> logits through embedding, a whole-model stage and the head."""
import numpy as np
import pytest

import oracle
from paper_2110_14895_amd import binding, synth
from tests import harness as H

pytestmark = pytest.mark.gpu


def make(sh, patch, channels, size, n_classes, mb, bf16, seed=0):
    prm = synth.surround_params(sh, patch, channels, n_classes, seed, bf16=bf16)
    dev = synth.as_param_dtype(prm, bf16)
    dt = binding.EP_BF16 if bf16 else binding.EP_F32
    emb = binding.Embed(size, patch, channels, sh.d_model, dt, dt, dev, mb)
    head = binding.Head(sh.d_model, sh.n_tokens, n_classes, sh.ln_eps, dt, dev, mb)
    return prm, emb, head


def run_embed(emb, img, shape_out, bf16):
    import torch
    B = img.shape[0]
    out = torch.empty(shape_out, dtype=torch.int16 if bf16 else torch.float32, device="cuda")
    emb.forward(torch.from_numpy(img).cuda(), B, out, torch.cuda.current_stream())
    torch.cuda.synchronize()
    if bf16:
        return synth.bf16_bits_to_f32(out.cpu().numpy().view(np.uint16)).reshape(shape_out)
    return out.cpu().numpy()


@pytest.mark.parametrize("size,patch,channels,d,bf16", [
    (32, 4, 3, 192, False),       # the tiny configuration: K = 48 (padded to 64), T = 65
    (32, 4, 3, 192, True),
    (224, 16, 3, 768, True),      # ViT-Base: K = 768, T = 197
    (224, 14, 3, 1280, True),     # ViT-Huge: K = 588 (padded to 640), T = 257
    (24, 8, 1, 64, True),         # one channel, 3 x 3 patches, K = 64
])
def test_embedding_matches_checker(size, patch, channels, d, bf16):
    T = 1 + (size // patch) ** 2
    sh = synth.custom_shape(f"emb{size}_{patch}", 1, d, max(1, d // 64), 4 * d, T)
    B = 5
    prm, emb, head = make(sh, patch, channels, size, 8, B, bf16)
    img = synth.images(B, channels, size, seed=2)
    got = run_embed(emb, img, (B, T, d), bf16)
    ref = oracle.embed_forward(img, prm["w_patch"], prm["b_patch"], prm["cls"], prm["pos"], patch)
    # class-token row: one addition, then (bf16 path) one rounding
    np.testing.assert_allclose(got[:, 0, :], ref[:, 0, :], rtol=2 ** -8 if bf16 else 1e-6, atol=1e-6)
    e = H.rel_err(got, ref)
    print(f"embedding {size}/{patch} D={d} {'bf16' if bf16 else 'fp32'}: err {e:.3e}")
    assert e <= (H.TOL_BF16 if bf16 else H.TOL_F32)
    # a smaller batch through the same handle gives the same images
    got2 = run_embed(emb, img[:2], (2, T, d), bf16)
    np.testing.assert_array_equal(got2, got[:2])
    emb.destroy(); head.destroy()


@pytest.mark.parametrize("d,T,nc,bf16", [(192, 65, 16, False), (192, 65, 16, True), (1280, 257, 1000, True), (768, 197, 1000, True),
                                         (2048, 17, 1000, True)])
def test_head_matches_checker(d, T, nc, bf16):
    import torch
    sh = synth.custom_shape(f"head{d}", 1, d, max(1, d // 64), 4 * d, T)
    B = 7
    prm = synth.surround_params(sh, 2, 1, nc, 5, bf16=bf16)
    dt = binding.EP_BF16 if bf16 else binding.EP_F32
    head = binding.Head(d, T, nc, sh.ln_eps, dt, synth.as_param_dtype(prm, bf16), B)
    x = (2.0 * synth.normal(f"head/x{d}", B * T * d, 1)).reshape(B, T, d).astype(np.float32)
    logits = torch.full((B, nc), float("nan"), dtype=torch.float32, device="cuda")
    head.forward(torch.from_numpy(x).cuda(), B, logits, torch.cuda.current_stream())
    torch.cuda.synchronize()
    ref = oracle.head_forward(x, prm["ln_g"], prm["ln_b"], sh.ln_eps, prm["w_head"], prm["b_head"])
    e = H.rel_err(logits.cpu().numpy(), ref)
    print(f"head D={d} classes={nc} {'bf16' if bf16 else 'fp32'}: err {e:.3e}")
    assert e <= (H.TOL_BF16 if bf16 else H.TOL_F32)
    head.destroy()


@pytest.mark.parametrize("bf16", [False, True])
def test_images_to_logits(bf16):
    import torch
    # 48 x 48 images, patch 8 -> 37 tokens; 3 layers of width 128
    sh = synth.custom_shape("e2e", 3, 128, 2, 256, 37)
    B, nc = 6, 24
    prm, emb, head = make(sh, 8, 3, 48, nc, B, bf16, seed=9)
    layers = [synth.layer_params(sh, l, bf16=bf16, randomize_affine=True, w_std=0.05) for l in range(3)]
    st = H.make_stage(sh, layers, 0, 3, B, bf16=bf16)
    img = synth.images(B, 3, 48, seed=4)
    s = torch.cuda.current_stream()
    x0 = torch.empty((B, 37, 128), dtype=torch.int16 if bf16 else torch.float32, device="cuda")
    x1 = torch.empty((B, 37, 128), dtype=torch.float32, device="cuda")
    logits = torch.empty((B, nc), dtype=torch.float32, device="cuda")
    emb.forward(torch.from_numpy(img).cuda(), B, x0, s)
    st.forward(x0, B, x1, s)
    head.forward(x1, B, logits, s)
    torch.cuda.synchronize()
    r0 = oracle.embed_forward(img, prm["w_patch"], prm["b_patch"], prm["cls"], prm["pos"], 8)
    r1 = oracle.stage_forward(H.oracle_cfg(sh), layers, r0)
    ref = oracle.head_forward(r1, prm["ln_g"], prm["ln_b"], sh.ln_eps, prm["w_head"], prm["b_head"])
    e = H.rel_err(logits.cpu().numpy(), ref)
    print(f"images -> logits {'bf16' if bf16 else 'fp32'}: err {e:.3e}")
    assert e <= (H.TOL_BF16 if bf16 else H.TOL_F32)
    emb.destroy(); head.destroy()


def test_surround_error_paths():
    sh = synth.custom_shape("err", 1, 64, 1, 128, 10)
    prm = synth.as_param_dtype(synth.surround_params(sh, 4, 1, 8, 0, bf16=True), True)
    with pytest.raises(binding.EdgePipeError):
        binding.Embed(13, 4, 1, 64, binding.EP_BF16, binding.EP_BF16, prm, 2)          # 13 % 4 != 0
    with pytest.raises(binding.EdgePipeError):
        binding.Embed(12, 4, 1, 96, binding.EP_BF16, binding.EP_BF16, prm, 2)          # width % 64
    with pytest.raises(binding.EdgePipeError):
        binding.Head(64, 10, 9, 1e-6, binding.EP_BF16, prm, 2)                          # classes % 8
    e = binding.Embed(12, 4, 1, 64, binding.EP_BF16, binding.EP_BF16, prm, 2)
    with pytest.raises(binding.EdgePipeError):
        e.forward(None, 1, None)
    e.destroy()
