"""Pins of the CPU checker's ViT stage forward (oracle/vit_oracle.c) against
closed forms, invariants, hand-expanded attention on 2-4 tokens, and float64
library routines.  Each pin is chosen so that a plausible slip in the checker
(dropped term, wrong scale, swapped q/k/v block, transposed weight, wrong
variance) fails at least one of them.  No GPU, no product code."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2110_14895_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(tag, *shape, seed=0):
    return synth.normal(tag, int(np.prod(shape)), seed).reshape(shape)


def small_shape(T=7, D=24, H=3, M=40, L=3):
    return synth.custom_shape(f"s{T}_{D}_{H}_{M}", L, D, H, M, T)


def cfg_of(sh, **kw):
    return oracle.OracleConfig(sh.d_model, sh.n_heads, sh.d_mlp, sh.n_tokens, sh.ln_eps, **kw)


# ----------------------------------------------------------------- LayerNorm
def test_layernorm_mean_zero_and_closed_form_variance():
    D, eps = 192, 1e-6
    x = rnd("ln/x", 11, D) * 3.0 + 1.5
    y = oracle.layernorm(x, np.ones(D), np.zeros(D), eps)
    assert np.abs(y.mean(axis=1)).max() < 1e-12
    var = x.var(axis=1)                       # biased
    np.testing.assert_allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)


def test_layernorm_large_eps_scales_variance():
    # variance sigma^2/(sigma^2+eps) with a non-negligible eps: catches eps outside the sqrt
    D = 16
    x = rnd("ln/x2", 5, D)
    var = x.var(axis=1)
    y = oracle.layernorm(x, np.ones(D), np.zeros(D), 0.5)
    np.testing.assert_allclose(y.var(axis=1), var / (var + 0.5), rtol=1e-12)


def test_layernorm_shift_invariance_and_affine():
    D = 48
    x = rnd("ln/x3", 4, D)
    g, b = 1.0 + 0.1 * rnd("ln/g", D), 0.1 * rnd("ln/b", D)
    g32, b32 = g.astype(np.float32), b.astype(np.float32)
    y0 = oracle.layernorm(x, g32, b32, 1e-6)
    y1 = oracle.layernorm(x + 7.25, g32, b32, 1e-6)
    np.testing.assert_allclose(y0, y1, atol=1e-12)
    plain = oracle.layernorm(x, np.ones(D), np.zeros(D), 1e-6)
    np.testing.assert_allclose(y0, plain * g32.astype(np.float64) + b32.astype(np.float64),
                               atol=1e-14)


def test_layernorm_matches_torch_float64():
    D = 40
    x = rnd("ln/x4", 9, D)
    g, b = (1 + 0.1 * rnd("ln/g4", D)).astype(np.float32), (0.1 * rnd("ln/b4", D)).astype(np.float32)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (D,), torch.from_numpy(g).double(),
                                         torch.from_numpy(b).double(), eps=1e-6).numpy()
    np.testing.assert_allclose(oracle.layernorm(x, g, b, 1e-6), ref, rtol=1e-12, atol=1e-13)


# -------------------------------------------------------------------- linear
def test_linear_is_x_times_w_transposed_plus_bias():
    x = rnd("lin/x", 5, 12)
    w = rnd("lin/w", 20, 12).astype(np.float32)       # [out, in], non-square
    b = rnd("lin/b", 20).astype(np.float32)
    ref = (torch.from_numpy(x) @ torch.from_numpy(w).double().T + torch.from_numpy(b).double()).numpy()
    np.testing.assert_allclose(oracle.linear(x, w, b), ref, rtol=1e-13, atol=1e-13)
    # one entry by hand
    manual = sum(x[2, k] * float(w[7, k]) for k in range(12)) + float(b[7])
    assert abs(oracle.linear(x, w, b)[2, 7] - manual) < 1e-14


# ---------------------------------------------------------------------- GELU
def test_gelu_tabulated_normal_cdf():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "normal_cdf.txt"))
            if l.strip() and not l.startswith("#")]
    u = np.array([float(r[0]) for r in rows])
    phi = np.array([float(r[1]) for r in rows])
    np.testing.assert_allclose(oracle.gelu(u), u * phi, rtol=0, atol=2e-15)


def test_gelu_identities():
    u = np.linspace(-6, 6, 101)
    g = oracle.gelu(u)
    assert oracle.gelu(np.zeros(1))[0] == 0.0
    np.testing.assert_allclose(g - oracle.gelu(-u), u, atol=1e-14)      # gelu(u) - gelu(-u) = u
    big = np.array([9.0, 12.0, 30.0])
    np.testing.assert_allclose(oracle.gelu(big), big, rtol=1e-15)
    # differs from the tanh approximation (which is not what is computed)
    tanh_form = 0.5 * u * (1 + np.tanh(math.sqrt(2 / math.pi) * (u + 0.044715 * u ** 3)))
    assert np.abs(g - tanh_form).max() > 1e-4
    ref = torch.nn.functional.gelu(torch.from_numpy(u)).numpy()
    np.testing.assert_allclose(g, ref, atol=1e-15)


# ----------------------------------------------------------------- attention
def test_attention_two_tokens_written_out():
    # T=2, one head, dh=2; every entry as an explicit formula
    q0, q1 = (0.3, -1.2), (0.8, 0.5)
    k0, k1 = (1.1, 0.4), (-0.7, 0.9)
    v0, v1 = (2.0, -1.0), (0.5, 3.0)
    qkv = np.array([[*q0, *k0, *v0], [*q1, *k1, *v1]])
    r2 = math.sqrt(2.0)
    s00 = (q0[0] * k0[0] + q0[1] * k0[1]) / r2
    s01 = (q0[0] * k1[0] + q0[1] * k1[1]) / r2
    s10 = (q1[0] * k0[0] + q1[1] * k0[1]) / r2
    s11 = (q1[0] * k1[0] + q1[1] * k1[1]) / r2
    p00 = math.exp(s00) / (math.exp(s00) + math.exp(s01))
    p01 = math.exp(s01) / (math.exp(s00) + math.exp(s01))
    p10 = math.exp(s10) / (math.exp(s10) + math.exp(s11))
    p11 = math.exp(s11) / (math.exp(s10) + math.exp(s11))
    want_o = np.array([[p00 * v0[0] + p01 * v1[0], p00 * v0[1] + p01 * v1[1]],
                       [p10 * v0[0] + p11 * v1[0], p10 * v0[1] + p11 * v1[1]]])
    o, p = oracle.attention(qkv, 1, return_probs=True)
    np.testing.assert_allclose(p[0], [[p00, p01], [p10, p11]], rtol=1e-14)
    np.testing.assert_allclose(o, want_o, rtol=1e-14)


@pytest.mark.parametrize("T,dh", [(3, 2), (4, 3), (4, 1)])
def test_attention_small_hand_expanded(T, dh):
    qkv = rnd(f"att/{T}/{dh}", T, 3 * dh)
    q = [[qkv[t][e] for e in range(dh)] for t in range(T)]
    k = [[qkv[t][dh + e] for e in range(dh)] for t in range(T)]
    v = [[qkv[t][2 * dh + e] for e in range(dh)] for t in range(T)]
    o, p = oracle.attention(qkv, 1, return_probs=True)
    for t in range(T):
        ex = [math.exp(math.fsum(q[t][e] * k[u][e] for e in range(dh)) / math.sqrt(dh))
              for u in range(T)]
        z = math.fsum(ex)
        for u in range(T):
            assert abs(p[0, t, u] - ex[u] / z) < 1e-14
        for e in range(dh):
            want = math.fsum(ex[u] / z * v[u][e] for u in range(T))
            assert abs(o[t, e] - want) < 1e-13


def test_softmax_rows_sum_to_one_and_shift_invariance():
    T, D, H = 65, 48, 3
    qkv = rnd("att/sum", T, 3 * D) * 2.0
    _, p = oracle.attention(qkv, H, return_probs=True)
    assert np.abs(p.sum(axis=-1) - 1.0).max() < 1e-12
    assert (p >= 0).all()
    # adding the same vector to every key shifts each score row by a constant
    shifted = qkv.copy()
    shifted[:, D:2 * D] += rnd("att/shift", 1, D)
    _, p2 = oracle.attention(shifted, H, return_probs=True)
    # rows shift by q.t * c / sqrt(dh), a per-row constant -> same softmax
    np.testing.assert_allclose(p2, p, atol=1e-12)


def test_attention_matches_torch_float64_multihead():
    T, D, H = 13, 40, 5
    dh = D // H
    qkv = rnd("att/torch", T, 3 * D)
    t = torch.from_numpy(qkv)
    q, k, v = (t[:, i * D:(i + 1) * D].reshape(T, H, dh).permute(1, 0, 2) for i in range(3))
    s = q @ k.transpose(1, 2) / math.sqrt(dh)
    ref = (torch.softmax(s, -1) @ v).permute(1, 0, 2).reshape(T, D).numpy()
    np.testing.assert_allclose(oracle.attention(qkv, H), ref, rtol=1e-12, atol=1e-13)


def test_attention_heads_are_column_blocks():
    # H heads == H independent single-head problems on column blocks h*dh..(h+1)*dh
    T, D, H = 6, 12, 3
    dh = D // H
    qkv = rnd("att/heads", T, 3 * D)
    o = oracle.attention(qkv, H)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        one = np.concatenate([qkv[:, 0 * D:1 * D][:, sl], qkv[:, 1 * D:2 * D][:, sl],
                              qkv[:, 2 * D:3 * D][:, sl]], axis=1)
        np.testing.assert_allclose(o[:, sl], oracle.attention(one, 1), atol=1e-14)


def test_attention_uniform_when_queries_are_zero():
    T, D, H = 9, 16, 2
    qkv = rnd("att/uni", T, 3 * D)
    qkv[:, :D] = 0.0
    o, p = oracle.attention(qkv, H, return_probs=True)
    assert np.abs(p - 1.0 / T).max() < 1e-15
    np.testing.assert_allclose(o, np.broadcast_to(qkv[:, 2 * D:].mean(axis=0), (T, D)), atol=1e-14)


def test_attention_single_token_returns_v():
    D = 8
    qkv = rnd("att/one", 1, 3 * D)
    np.testing.assert_array_equal(oracle.attention(qkv, 2), qkv[:, 2 * D:])


# --------------------------------------------------------------- whole layer
def torch_layer(sh, p, x):
    """Independent float64 statement of a pre-LN encoder layer with torch ops."""
    D, H, T = sh.d_model, sh.n_heads, sh.n_tokens
    dh = D // H
    P = {k: torch.from_numpy(np.asarray(v)).double() for k, v in p.items()}
    x = torch.from_numpy(x).double()
    B = x.shape[0]
    F = torch.nn.functional
    y = F.layer_norm(x, (D,), P["ln1_g"], P["ln1_b"], sh.ln_eps)
    qkv = F.linear(y, P["w_qkv"], P["b_qkv"])
    q, k, v = (qkv[..., i * D:(i + 1) * D].reshape(B, T, H, dh).transpose(1, 2) for i in range(3))
    a = torch.softmax(q @ k.transpose(-1, -2) / math.sqrt(dh), -1) @ v
    a = a.transpose(1, 2).reshape(B, T, D)
    x = x + F.linear(a, P["w_o"], P["b_o"])
    z = F.layer_norm(x, (D,), P["ln2_g"], P["ln2_b"], sh.ln_eps)
    h = F.gelu(F.linear(z, P["w_fc1"], P["b_fc1"]))
    return (x + F.linear(h, P["w_fc2"], P["b_fc2"])).numpy()


def test_layer_matches_torch_float64():
    sh = small_shape(T=7, D=24, H=3, M=40)
    p = synth.layer_params(sh, 0, randomize_affine=True, w_std=0.3)
    x = synth.activations(sh, 2).astype(np.float64)
    got = oracle.layer_forward(cfg_of(sh), p, x)
    np.testing.assert_allclose(got, torch_layer(sh, p, x), rtol=1e-11, atol=1e-12)


def test_tiny_config_stage_matches_torch_float64():
    sh = synth.SHAPES["tiny"]
    layers = [synth.layer_params(sh, l) for l in range(2)]
    x = synth.activations(sh, 1)
    got = oracle.stage_forward(cfg_of(sh), layers, x)
    ref = x.astype(np.float64)
    for p in layers:
        ref = torch_layer(sh, p, ref)
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)
    rms = math.sqrt((got ** 2).mean())
    assert 0.9 < rms < 1.3


def test_zero_output_weights_make_layer_identity():
    sh = small_shape()
    p = synth.layer_params(sh, 0, randomize_affine=True)
    for n in ("w_o", "b_o", "w_fc2", "b_fc2"):
        p[n] = np.zeros_like(p[n])
    x = synth.activations(sh, 2)
    out = oracle.stage_forward(cfg_of(sh), [p, p], x)
    np.testing.assert_array_equal(out, x.astype(np.float64))
    allzero = {k: np.zeros_like(v) for k, v in p.items()}
    np.testing.assert_array_equal(oracle.stage_forward(cfg_of(sh), [allzero], x),
                                  x.astype(np.float64))


def test_token_permutation_equivariance():
    sh = small_shape(T=9)
    layers = [synth.layer_params(sh, l, randomize_affine=True, w_std=0.2) for l in range(2)]
    x = synth.activations(sh, 1)
    perm = np.array([3, 0, 8, 5, 1, 7, 2, 6, 4])
    a = oracle.stage_forward(cfg_of(sh), layers, x)
    b = oracle.stage_forward(cfg_of(sh), layers, x[:, perm])
    np.testing.assert_allclose(b, a[:, perm], atol=1e-12)


def test_batch_independence_is_exact():
    sh = small_shape()
    layers = [synth.layer_params(sh, l, randomize_affine=True, w_std=0.2) for l in range(2)]
    x = synth.activations(sh, 4)
    full = oracle.stage_forward(cfg_of(sh), layers, x)
    for b in (0, 3):
        np.testing.assert_array_equal(full[b:b + 1], oracle.stage_forward(cfg_of(sh), layers, x[b:b + 1]))


def test_stage_composition():
    # T_2(T_1(X)) over layer ranges [0,a) and [a,L) equals the whole range (section 3.1)
    sh = small_shape(L=4)
    layers = [synth.layer_params(sh, l, randomize_affine=True, w_std=0.2) for l in range(4)]
    x = synth.activations(sh, 2)
    cfg = cfg_of(sh)
    whole = oracle.stage_forward(cfg, layers, x)
    mid = x.astype(np.float64)
    for p in layers[:1]:
        mid = oracle.layer_forward(cfg, p, mid)
    for p in layers[1:]:
        mid = oracle.layer_forward(cfg, p, mid)
    np.testing.assert_array_equal(mid, whole)


def test_rounding_mode_is_small_perturbation_and_off_by_default():
    sh = small_shape(T=12, D=64, H=2, M=128)
    layers = [synth.layer_params(sh, l, bf16=True) for l in range(2)]
    x = synth.activations(sh, 1, bf16=True)
    exact = oracle.stage_forward(cfg_of(sh), layers, x)
    rounded = oracle.stage_forward(cfg_of(sh, round_mode=1), layers, x)
    rms = math.sqrt((exact ** 2).mean())
    err = np.abs(exact - rounded).max() / rms
    assert 0 < err < 2e-2


# ------------------------------------------- the diagnostic mode's bf16 narrowing
def test_round_bf16_ties_go_to_even_and_signs_mirror():
    # bf16 keeps 8 significant bits: neighbours of 1 are 1 - 2^-8 and 1 + 2^-7
    r = oracle.round_bf16
    assert r(1.0) == 1.0 and r(0.0) == 0.0 and r(-0.0) == 0.0 and math.copysign(1.0, r(-0.0)) == -1.0
    assert r(1 + 2.0 ** -8) == 1.0                        # halfway between 1 (even) and 1 + 2^-7 (odd)
    assert r(1 + 3 * 2.0 ** -8) == 1 + 2.0 ** -6          # halfway between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    assert r(1 + 2.0 ** -8 + 2.0 ** -20) == 1 + 2.0 ** -7   # just above the tie: up
    assert r(1 + 2.0 ** -8 - 2.0 ** -20) == 1.0             # just below: down
    assert r(1 + 5 * 2.0 ** -8) == 1 + 2.0 ** -6          # tie between 1 + 2^-6 (even) and 1 + 3*2^-7 (odd)
    for v in (1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, 3.14159, 1e-3, 2.5e20):
        assert r(-v) == -r(v)
    # truncation would give 1 + 2^-7 here, rounding half up the same, half-to-even too: a plain value
    assert r(1 + 2.0 ** -7 + 2.0 ** -9) == 1 + 2.0 ** -7
    # a carry out of the mantissa moves to the next binade
    assert r(2 - 2.0 ** -9) == 2.0
    assert r(2 - 2.0 ** -8) == 2.0                        # tie: 2 - 2^-7 is odd, 2 is even
    assert r(2 - 3 * 2.0 ** -9) == 2 - 2.0 ** -7


def test_round_bf16_narrows_through_float32_first():
    # 1 + 2^-8 + 2^-30 lies above the tie, but float32 (24 significant bits) cannot hold the 2^-30:
    # the value is narrowed to float32 first, lands exactly on the tie, and goes to the even side.
    # Rounding the float64 value to bf16 in one step would give 1 + 2^-7 instead.
    assert oracle.round_bf16(1 + 2.0 ** -8 + 2.0 ** -30) == 1.0
    assert oracle.round_bf16(1 + 3 * 2.0 ** -8 - 2.0 ** -30) == 1 + 2.0 ** -6


def test_round_bf16_special_values_and_range():
    r = oracle.round_bf16
    assert r(math.inf) == math.inf and r(-math.inf) == -math.inf
    assert math.isnan(r(math.nan))
    big = float(np.finfo(np.float32).max)                 # above the largest bf16, past its tie: infinity
    assert r(big) == math.inf and r(-big) == -math.inf
    largest = (2 - 2.0 ** -7) * 2.0 ** 127                # the largest finite bf16
    assert r(largest) == largest
    tiny = 2.0 ** -133                                    # a bf16 subnormal (multiples of 2^-133)
    assert r(tiny) == tiny and r(1.5 * tiny) == 2 * tiny and r(2.5 * tiny) == 2 * tiny


def test_round_bf16_agrees_with_library_conversion():
    vals = np.concatenate([rnd("rb/a", 4000), rnd("rb/b", 2000) * 1e-4, rnd("rb/c", 2000) * 1e5,
                           # exact ties and their neighbours at many exponents
                           np.array([(1 + (2 * k + 1) * 2.0 ** -8) * 2.0 ** e for k in range(8) for e in (-20, -1, 0, 7)]),
                           ]).astype(np.float32)
    want = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle.round_bf16(float(v)) for v in vals])
    np.testing.assert_array_equal(got, want)


def test_rounding_mode_narrows_exactly_the_five_operand_points():
    # the layer rebuilt from the checker's own steps with the narrowing done by the library's
    # float32 -> bf16 conversion at: both LayerNorm outputs, q|k|v, the attention probabilities
    # (inside the attention step), the attention output and the GELU output
    def nb(a):
        return torch.from_numpy(np.asarray(a, dtype=np.float64)).to(torch.float32).to(torch.bfloat16) \
            .to(torch.float64).numpy()
    sh = small_shape(T=9, D=32, H=2, M=48, L=1)
    p = synth.layer_params(sh, 0, bf16=True, randomize_affine=True, w_std=0.2)
    x = synth.activations(sh, 2, bf16=True).astype(np.float64)
    got = oracle.layer_forward(cfg_of(sh, round_mode=1), p, x)
    out = np.empty_like(x)
    for b in range(x.shape[0]):
        y = nb(oracle.layernorm(x[b], p["ln1_g"], p["ln1_b"], sh.ln_eps))
        qkv = nb(oracle.linear(y, p["w_qkv"], p["b_qkv"]))
        o = nb(oracle.attention(qkv, sh.n_heads, round_mode=1))
        x1 = x[b] + oracle.linear(o, p["w_o"], p["b_o"])
        z = nb(oracle.layernorm(x1, p["ln2_g"], p["ln2_b"], sh.ln_eps))
        h = nb(oracle.gelu(oracle.linear(z, p["w_fc1"], p["b_fc1"])))
        out[b] = x1 + oracle.linear(h, p["w_fc2"], p["b_fc2"])
    np.testing.assert_array_equal(got, out)
    # and the probabilities: rounded after normalisation, before they weigh the values
    qkv = rnd("rm/qkv", 5, 3 * 8)
    o_r = oracle.attention(qkv, 1, round_mode=1)
    _, pr = oracle.attention(qkv, 1, return_probs=True)
    np.testing.assert_allclose(o_r, nb(pr[0]) @ qkv[:, 16:], rtol=1e-13, atol=1e-15)
