"""GPU parity: ep_stage_forward through the C ABI against the float64 CPU
checker on the same seeded host buffers.  Tolerances: max-abs error over the
RMS of the reference <= 1e-4 on the fp32 path and <= 2e-2 on the bf16 path."""
import math

import numpy as np
import pytest

import oracle
from paper_2110_14895_amd import binding, synth
from tests import harness as H

pytestmark = pytest.mark.gpu


def layers_of(sh, n, *, bf16, affine=True, w_std=0.02, first=0):
    return [synth.layer_params(sh, first + l, bf16=bf16, randomize_affine=affine, w_std=w_std)
            for l in range(n)]


# ------------------------------------------------------------------ fp32 path
def test_tiny_fp32_config():
    # D=192, 3 heads of 64, MLP 768, T=65, 2 layers, batch 1, weights N(0, 0.02), biases 0
    sh = synth.SHAPES["tiny"]
    layers = layers_of(sh, 2, bf16=False, affine=False)
    x = synth.activations(sh, 1)
    st = H.make_stage(sh, layers, 0, 2, 1, bf16=False)
    got = H.run_stage(st, x)
    ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
    assert H.rel_err(got, ref) <= H.TOL_F32


@pytest.mark.parametrize("T,D,Hh,M,B", [(7, 24, 3, 40, 3), (65, 192, 3, 768, 2), (130, 72, 2, 100, 1)])
def test_fp32_ragged_shapes_with_affine_and_bias(T, D, Hh, M, B):
    sh = synth.custom_shape(f"f32_{T}_{D}", 2, D, Hh, M, T)
    layers = layers_of(sh, 2, bf16=False, w_std=0.1)
    x = synth.activations(sh, B)
    st = H.make_stage(sh, layers, 0, 2, B + 1, bf16=False)
    got = H.run_stage(st, x)
    ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
    assert H.rel_err(got, ref) <= H.TOL_F32


# ------------------------------------------------------------------ bf16 path
def _zero(layers, names):
    out = []
    for p in layers:
        q = dict(p)
        for n in names:
            q[n] = np.zeros_like(q[n])
        out.append(q)
    return out


SMALL_BF16 = [
    # T, D, H, M, B : d_head 64 / 80, tokens spanning 3 / 7 / 9 key tiles, ragged row counts
    (65, 128, 2, 256, 3),
    (197, 256, 4, 512, 2),
    (257, 320, 4, 640, 2),
    (33, 128, 2, 192, 5),
    (1, 128, 2, 128, 1),
    (288, 128, 2, 256, 1),
    # more tokens than one pass of ten query waves covers (320): the query tiles go in passes, the keys
    # stream through once per pass; 577 = a 384 x 384 image in 16 x 16 patches plus the class token
    (321, 128, 2, 128, 2),
    (577, 320, 4, 192, 2),
    (1000, 128, 2, 128, 1),
]


@pytest.mark.parametrize("T,D,Hh,M,B", SMALL_BF16)
@pytest.mark.parametrize("part", ["mlp_only", "attention_only", "full"])
def test_bf16_small_shapes(T, D, Hh, M, B, part):
    sh = synth.custom_shape(f"bf_{T}_{D}_{Hh}", 2, D, Hh, M, T)
    layers = layers_of(sh, 2, bf16=True, w_std=0.05)
    if part == "mlp_only":
        layers = _zero(layers, ["w_o", "b_o"])
    elif part == "attention_only":
        layers = _zero(layers, ["w_fc2", "b_fc2"])
    x = synth.activations(sh, B, bf16=True)
    st = H.make_stage(sh, layers, 0, 2, B, bf16=True)
    got = H.run_stage(st, x)
    ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
    ref_r = oracle.stage_forward(H.oracle_cfg(sh, round_mode=1), layers, x)
    e, er = H.rel_err(got, ref), H.rel_err(got, ref_r)
    sd, sdr = H.err_std(got, ref), H.err_std(got, ref_r)
    print(f"{part} T={T} D={D}: err {e:.3e} (std {sd:.3e}), vs operand-rounded reference {er:.3e} (std {sdr:.3e})")
    assert e <= H.TOL_BF16
    # Against the operand-rounded reference.  With the attention branch switched off the two share
    # their rounding points, and what is left are operands that land on the other side of a tie
    # (mostly GELU outputs: the device's GELU is accurate to 3.5e-4 relative, a sixth of half a bf16
    # step): a third of the unrounded error's spread or less (observed 0.25 .. 0.33; maximum
    # 5.7e-4 .. 4.9e-3).  The attention kernel narrows the probabilities before it normalises them
    # (the reference after), so with attention on the operand-rounded reference is no closer to the
    # device than the unrounded one and only the graded bound is asserted.
    if part == "mlp_only":
        assert sdr <= 0.5 * sd and er <= 7.5e-3
    else:
        assert er <= H.TOL_BF16


def test_bf16_zero_output_weights_is_exact_identity():
    sh = synth.custom_shape("bf_id", 2, 128, 2, 256, 65)
    layers = _zero(layers_of(sh, 2, bf16=True), ["w_o", "b_o", "w_fc2", "b_fc2"])
    x = synth.activations(sh, 2, bf16=True)
    st = H.make_stage(sh, layers, 0, 2, 2, bf16=True)
    np.testing.assert_array_equal(H.run_stage(st, x), x)


def test_bf16_io_dtypes_and_batch_smaller_than_max():
    sh = synth.custom_shape("bf_io", 1, 128, 2, 256, 65)
    layers = layers_of(sh, 1, bf16=True, w_std=0.05)
    x = synth.activations(sh, 3, bf16=True)
    ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
    base = H.run_stage(H.make_stage(sh, layers, 0, 1, 8, bf16=True), x)
    assert H.rel_err(base, ref) <= H.TOL_BF16
    f32_in = H.run_stage(H.make_stage(sh, layers, 0, 1, 8, bf16=True, in_bf16=False), x)
    np.testing.assert_array_equal(f32_in, base)         # same values in, same kernels
    bf_out = H.run_stage(H.make_stage(sh, layers, 0, 1, 8, bf16=True, out_bf16=True), x)
    np.testing.assert_array_equal(bf_out, synth.round_to_bf16(base).reshape(base.shape))


def test_batch_limits_and_in_place():
    import torch
    sh = synth.custom_shape("bf_lim", 1, 128, 2, 256, 65)
    layers = layers_of(sh, 1, bf16=True)
    st = H.make_stage(sh, layers, 0, 1, 2, bf16=True, in_bf16=False)
    x = synth.activations(sh, 2, bf16=True)
    want = H.run_stage(st, x)
    buf = torch.from_numpy(x).cuda()
    st.forward(buf, 2, buf)                              # x_out aliases x_in
    torch.cuda.synchronize()
    np.testing.assert_array_equal(buf.cpu().numpy(), want)
    with pytest.raises(binding.EdgePipeError) as ei:
        st.forward(buf, 3, buf)
    assert ei.value.status == binding.EP_ERR_INVALID_ARG
    with pytest.raises(binding.EdgePipeError):
        st.forward(buf, 0, buf)


def test_stage_composition_and_caller_stream():
    # T_2(T_1(X)) on two stage handles equals the single stage over both ranges (section 3.1)
    import torch
    sh = synth.custom_shape("bf_comp", 4, 128, 2, 256, 65)
    layers = layers_of(sh, 4, bf16=True, w_std=0.05)
    x = synth.activations(sh, 3, bf16=True)
    whole = H.make_stage(sh, layers, 0, 4, 3, bf16=True)
    s1 = H.make_stage(sh, layers[:1], 0, 1, 3, bf16=True)
    s2 = H.make_stage(sh, layers[1:], 1, 4, 3, bf16=True, in_bf16=False)
    stream = torch.cuda.Stream()
    ref = H.run_stage(whole, x)
    mid = H.run_stage(s1, x, stream=stream, keep_device=True)
    out = torch.empty_like(mid)
    s2.forward(mid, 3, out, stream)
    stream.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), ref)
    assert H.rel_err(ref, oracle.stage_forward(H.oracle_cfg(sh), layers, x)) <= H.TOL_BF16


@pytest.mark.parametrize("T,D,Hh,M,B", [(50, 128, 2, 1024, 1), (197, 256, 4, 2048, 3), (65, 192, 3, 1536, 2)])
def test_second_mlp_layer_cut_into_k_ranges(T, D, Hh, M, B):
    # few output tiles and a long K: the second MLP layer runs as one workgroup per (K range, tile) and the
    # next layer's first LayerNorm (or, after the last layer, a kernel of its own) adds the ranges.  The
    # workspace of such a stage holds the range sums, which is how the test knows the path is taken.
    import torch
    sh = synth.custom_shape("bf_split", 3, D, Hh, M, T)
    layers = layers_of(sh, 3, bf16=True, w_std=0.05)
    x = synth.activations(sh, B, bf16=True)
    whole = H.make_stage(sh, layers, 0, 3, B, bf16=True)
    R = B * T
    lean = R * D * 4 + R * D * 2 + R * max(3 * D, M) * 2               # x | a | big
    params = 3 * (2 * (4 * D * D + 2 * D * M) + 4 * (9 * D + M))
    assert whole.device_bytes() >= params + lean + 2 * R * D * 4, "no room for range sums: the path under test is not taken"
    got = H.run_stage(whole, x)
    ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
    e = H.rel_err(got, ref)
    print(f"K ranges T={T} D={D} M={M} B={B}: err {e:.3e}")
    assert e <= H.TOL_BF16
    np.testing.assert_array_equal(H.run_stage(whole, x), got)             # same sums in the same order every time
    # layer by layer through one-layer stages (each adds its own ranges) = the ranges added by the next LayerNorm
    cur = x
    for l in range(3):
        st = H.make_stage(sh, layers[l:l + 1], l, l + 1, B, bf16=True, in_bf16=(l == 0))
        cur = H.run_stage(st, cur)
    np.testing.assert_array_equal(cur, got)
    # bf16 output of the last layer: the fp32 result, rounded once
    bf = H.run_stage(H.make_stage(sh, layers, 0, 3, B, bf16=True, out_bf16=True), x)
    np.testing.assert_array_equal(bf, synth.round_to_bf16(got).reshape(got.shape))


def test_determinism_and_workspace_poison():
    import torch
    sh = synth.custom_shape("bf_det", 2, 320, 4, 640, 257)
    layers = layers_of(sh, 2, bf16=True, w_std=0.05)
    x = synth.activations(sh, 2, bf16=True)
    st = H.make_stage(sh, layers, 0, 2, 4, bf16=True)
    a = H.run_stage(st, x)
    big = H.run_stage(st, synth.activations(sh, 4, bf16=True, tag="other") * 50.0)   # dirty the workspace
    assert np.isfinite(big).all()
    b = H.run_stage(st, x)
    np.testing.assert_array_equal(a, b)


def test_forward_under_graph_capture_replays_bit_exactly():
    # ep_stage_forward only enqueues kernels on the caller's stream (no allocation, no
    # synchronisation), so a caller may capture it in a graph: every replay, with eager work of
    # the same stage in between, reproduces the eager result bit for bit.  All dense-layer paths:
    # persistent launches with a row remainder (ViT-Huge width, B = 16), the small-tile kernel, and
    # the second MLP layer cut into K ranges with the sums added by the next LayerNorm / the last kernel.
    import torch
    for sh, B in ((synth.custom_shape("bf_graph_small", 2, 320, 4, 640, 65), 3),
                  (synth.custom_shape("bf_graph_ranges", 3, 256, 4, 2048, 197), 2),
                  (synth.custom_shape("bf_graph_wide", 1, 1280, 16, 5120, 257), 16)):
        layers = layers_of(sh, sh.n_layers, bf16=True, w_std=0.05)
        st = H.make_stage(sh, layers, 0, sh.n_layers, B, bf16=True)
        x = synth.activations(sh, B, bf16=True)
        other = synth.activations(sh, B, bf16=True, tag="other")
        ref = H.run_stage(st, x)                                  # eager; also first-call set-up
        xin, oin = H.to_device(x, True), H.to_device(other, True)
        out = torch.empty(x.shape, dtype=torch.float32, device="cuda")
        scratch = torch.empty_like(out)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                st.forward(xin, B, out, side)
        for _ in range(3):
            out.fill_(float("nan"))
            st.forward(oin, B, scratch, torch.cuda.current_stream())   # eager work on the same workspace
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out.cpu().numpy(), ref)
        del graph
        st.destroy()


# ----------------------------------------------------- the named configurations
def test_vit_base_stage_of_three_layers_batch_8():
    sh = synth.SHAPES["vit_base"]
    layers = layers_of(sh, 3, bf16=True, affine=False)
    x = synth.activations(sh, 8, bf16=True)
    st = H.make_stage(sh, layers, 0, 3, 8, bf16=True)
    got = H.run_stage(st, x)
    ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
    e = H.rel_err(got, ref)
    print(f"ViT-Base 3 layers B=8: err {e:.3e}, std {H.err_std(got, ref):.3e}, rms {math.sqrt((ref**2).mean()):.3f}")
    assert e <= H.TOL_BF16


def test_vit_large_stage_of_six_layers_batch_sweep():
    sh = synth.SHAPES["vit_large"]
    layers = layers_of(sh, 6, bf16=True, affine=False)
    st = H.make_stage(sh, layers, 0, 6, 64, bf16=True)
    # images are independent (section 2.1): image i gives the same result in any batch
    ref = {i: oracle.stage_forward(H.oracle_cfg(sh), layers, synth.activations(sh, 1, bf16=True, first_image=i))[0]
           for i in (0, 3, 9, 15, 22, 31, 40, 49, 58, 63)}
    for B in (1, 4, 16, 32, 64):
        x = synth.activations(sh, B, bf16=True)
        got = H.run_stage(st, x)
        assert np.isfinite(got).all()
        for i, r in ref.items():
            if i < B:
                e = H.rel_err(got[i], r)
                print(f"ViT-Large 6 layers B={B} image {i}: err {e:.3e}")
                assert e <= H.TOL_BF16
        if B > 1:   # the rest of the batch: same statistics as the checked images
            rms = np.sqrt((got.astype(np.float64) ** 2).mean(axis=(1, 2)))
            assert np.all(np.abs(rms / rms[0] - 1) < 0.2)


@pytest.mark.parametrize("B", [16, 32, 48])
def test_vit_huge_row_remainder_shapes(B):
    # B * 257 rows = B tiles of 256 rows + B rows: the dense layers that fill the chip take the B
    # remaining rows (they belong to the last image) in the last phase of their launch, as tiles of
    # 64, 32 or 16 rows depending on the layer's width; the narrower layers of the smaller batches
    # run the one-tile-per-workgroup kernel instead
    sh = synth.SHAPES["vit_huge"]
    layers = layers_of(sh, 2, bf16=True, affine=True)
    st = H.make_stage(sh, layers, 0, 2, B, bf16=True)
    x = synth.activations(sh, B, bf16=True)
    got = H.run_stage(st, x)
    assert np.isfinite(got).all()
    for i in (0, B - 1):
        ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x[i:i + 1])[0]
        e = H.rel_err(got[i], ref)
        print(f"ViT-Huge 2 layers B={B} image {i}: err {e:.3e}")
        assert e <= H.TOL_BF16
        # the last rows of the last image are the remainder rows: check them on their own too
        e_tail = H.rel_err(got[i][-B:], ref[-B:])
        assert e_tail <= H.TOL_BF16
    st.destroy()


def test_vit_huge_batch_256_rows_past_the_tile_walk():
    # 256 * 257 rows = 257 tiles of 256 rows: a 257th tile row would cost the layers of width 1280 a fifth
    # round of tiles, so their tile walk stops a tile row early and the last phase of the launch takes
    # the 256 rows left (all of them rows of the last image); the wider layers walk all 257 tile rows
    sh = synth.SHAPES["vit_huge"]
    B = 256
    layers = layers_of(sh, 1, bf16=True, affine=True)
    st = H.make_stage(sh, layers, 0, 1, B, bf16=True)
    x = synth.activations(sh, B, bf16=True)
    got = H.run_stage(st, x)
    assert np.isfinite(got).all()
    for i in (0, 37, 74, 111, 127, 148, 185, 222, B - 1):
        ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x[i:i + 1])[0]
        e = H.rel_err(got[i], ref)
        print(f"ViT-Huge 1 layer B={B} image {i}: err {e:.3e}")
        assert e <= H.TOL_BF16
    rms = np.sqrt((got.astype(np.float64) ** 2).mean(axis=(1, 2)))
    assert np.all(np.abs(rms / rms[0] - 1) < 0.2)
    st.destroy()


def test_vit_huge_all_layers_batch_64_sampled_images():
    # the benchmark configuration: 32 layers, B=64, T=257.  The checker recomputes eight images
    # spread over the batch (one in each eighth: the attention kernel deals images 8k .. 8k+7 to
    # one XCD, the dense layers one tile row per image), each compared element by element.
    sh = synth.SHAPES["vit_huge"]
    layers = layers_of(sh, 32, bf16=True, affine=False)
    st = H.make_stage(sh, layers, 0, 32, 64, bf16=True)
    x = synth.activations(sh, 64, bf16=True)
    got = H.run_stage(st, x)
    assert np.isfinite(got).all()
    worst = 0.0
    refs = {}
    for i in (0, 9, 18, 27, 36, 45, 54, 63):
        ref = refs[i] = oracle.stage_forward(H.oracle_cfg(sh), layers, x[i:i + 1])[0]
        e, s = H.rel_err(got[i], ref), H.err_std(got[i], ref)
        print(f"ViT-Huge 32 layers B=64 image {i}: err {e:.3e}, std {s:.3e}, rms {math.sqrt((ref**2).mean()):.3f}",
              flush=True)
        worst = max(worst, e)
    assert worst <= H.TOL_BF16
    # Every image, every position: the same images dealt to other positions of the batch (rolled by
    # 9: another XCD range, another tile row).  A row of a dense layer, a row of LayerNorm and an
    # (image, head) pair of attention are computed by the same instruction sequence wherever they
    # sit, so the results are bit-identical - except for the image in the last position, whose last
    # 64 rows are the row remainder and take the narrow tiles (another summation order): the two
    # images that meet that position in one of the runs (63, and 54 after the roll) are held against
    # the checker there instead.
    shift = 9
    got_r = H.run_stage(st, np.roll(x, shift, axis=0))
    for i in range(64):
        j = (i + shift) % 64
        if i == 63 or j == 63:
            e = H.rel_err(got_r[j], refs[i])
            print(f"image {i} at position {j}: err {e:.3e}")
            assert e <= H.TOL_BF16, (i, j, e)
        else:
            np.testing.assert_array_equal(got_r[j], got[i], err_msg=f"image {i} at position {j}")
    # 64 * 257 rows = 64 tiles of 256 rows + 64: every dense layer runs as one persistent launch
    # whose last phase takes the 64 remaining rows
    for name, kid in binding.MAIN_KERNEL_IDS.items():
        assert st.gemm_main_rows(64, kid) == 16448
    st.destroy()


@pytest.mark.parametrize("name,batch", [("deit_tiny", 32), ("deit_small", 16), ("deit_small", 256)])
def test_small_encoder_shapes_all_layers(name, batch):
    # the narrow models of section 5.4: D = 192 / 384, 12 layers; small N and K stress the tile
    # selection (N = 192 .. 1536) rather than the matrix pipe
    sh = synth.SHAPES[name]
    layers = layers_of(sh, sh.n_layers, bf16=True, affine=False)
    st = H.make_stage(sh, layers, 0, sh.n_layers, batch, bf16=True)
    x = synth.activations(sh, batch, bf16=True)
    got = H.run_stage(st, x)
    assert np.isfinite(got).all()
    for i in sorted({0, batch - 1}):
        ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x[i:i + 1])[0]
        e = H.rel_err(got[i], ref)
        print(f"{name} {sh.n_layers} layers B={batch} image {i}: err {e:.3e}, std {H.err_std(got[i], ref):.3e}")
        assert e <= H.TOL_BF16


# ------------------------------------------------- profiling, tracing, planning
def test_profile_and_trace_report_positive_times():
    import torch
    sh = synth.custom_shape("bf_prof", 3, 256, 4, 512, 197)
    layers = layers_of(sh, 3, bf16=True)
    st = H.make_stage(sh, layers, 0, 3, 8, bf16=True)
    t = st.profile(8, iters=3)
    assert t.shape == (3,) and np.all(t > 0) and np.all(t < 1.0)
    x = synth.activations(sh, 8, bf16=True)
    ref = H.run_stage(st, x)
    total = 0.0
    for kid in range(len(binding.KERNEL_NAMES)):
        st.trace_begin(kid, 3)
        got = H.run_stage(st, x)
        n, sec = st.trace_end()
        assert n == 3 and sec > 0
        np.testing.assert_array_equal(got, ref)      # tracing does not change results
        total += sec
    assert total < 1.0
    with pytest.raises(binding.EdgePipeError):
        st.trace_end()                                # no active trace
    # the ids that time the launch of a dense layer alone: never longer than the bracket around the
    # whole layer, and the rows it covers are all rows (a dense layer is one launch)
    for name, kid in binding.MAIN_KERNEL_IDS.items():
        st.trace_begin(binding.KERNEL_NAMES.index(name), 3)
        H.run_stage(st, x)
        _, whole = st.trace_end()
        st.trace_begin(kid, 3)
        got = H.run_stage(st, x)
        n, sec = st.trace_end()
        assert n == 3 and 0 < sec <= whole * 1.5 + 1e-4
        np.testing.assert_array_equal(got, ref)
        rows = st.gemm_main_rows(8, kid)
        assert rows == 8 * sh.n_tokens
    with pytest.raises(binding.EdgePipeError):
        st.gemm_main_rows(8, 0)                       # LayerNorm is not a dense layer


def test_heterogeneous_partition_stages_match_checker():
    """Per-layer costs profiled on this GPU feed ep_partition for 16 synthetic devices
    (seed 1); every resulting uneven stage is run at micro-batches 1, 2, 4, ..., 256 and
    compared with the checker on image 0 (images are independent, so one reference per
    stage serves every batch size) and on the last image of every batch; then the stages
    are chained and compared with the checker's result over all 32 layers."""
    from oracle import partition as P
    sh = synth.SHAPES["vit_huge"]
    B_plan = 8
    layers = layers_of(sh, 32, bf16=True, affine=False)
    whole = H.make_stage(sh, layers, 0, 32, B_plan, bf16=True)
    cost = whole.profile(B_plan, iters=2)
    whole.destroy()
    assert cost.shape == (32,) and np.all(cost > 0)
    inst = synth.heterogeneous_cluster(cost, sh, batch=B_plan, n_devices=16, seed=1)
    t_opt, plan = binding.partition(inst.t_comp, inst.layer_mem, inst.dev_mem, inst.xfer_bytes, inst.bw)
    t_ref, _ = P.paper_dp(inst.t_comp, inst.layer_mem, inst.dev_mem, inst.xfer_bytes, inst.bw)
    assert t_opt == t_ref                                   # bit-exact optimum
    assert P.evaluate(plan, inst.t_comp, inst.layer_mem, inst.dev_mem, inst.xfer_bytes, inst.bw) == t_opt
    sizes = [l - f + 1 for _, f, l in plan]
    print(f"plan: T_opt={t_opt:.4f}s, stages (device, first, last): {plan}")
    assert sum(sizes) == 32 and len(set(sizes)) > 1         # uneven stages
    batches = (1, 2, 4, 8, 16, 32, 64, 128, 256)
    for s_idx, (_dev, first, last) in enumerate(plan):
        stage_layers = layers[first:last + 1]
        st = H.make_stage(sh, stage_layers, first, last + 1, max(batches), bf16=True)
        tag = f"stage{s_idx}"                              # independent N(0,1) input per stage
        x_all = synth.activations(sh, max(batches), bf16=True, tag=tag)   # image i is the same in every batch
        ref0 = oracle.stage_forward(H.oracle_cfg(sh), stage_layers, x_all[:1])[0]
        for B in batches:
            got = H.run_stage(st, x_all[:B])
            assert np.isfinite(got).all()
            e = H.rel_err(got[0], ref0)
            assert e <= H.TOL_BF16, (s_idx, B, e)
            if B > 1:
                # the last image of the batch: at B = 256 its rows are the ones past the tile walk
                ref_last = oracle.stage_forward(H.oracle_cfg(sh), stage_layers, x_all[B - 1:B])[0]
                e2 = H.rel_err(got[B - 1], ref_last)
                print(f"stage {s_idx} layers {first}-{last}: B={B} image 0 err {e:.2e}, image {B-1} err {e2:.2e}",
                      flush=True)
                assert e2 <= H.TOL_BF16, (s_idx, B, e2)
        st.destroy()

    # The plan's stages chained (fp32 boundaries, micro-batch 2): stage k's output is stage k+1's
    # input, the last output is compared with the checker's result over all 32 layers.
    import torch
    B = 2
    x = synth.activations(sh, B, bf16=True)
    cur = H.to_device(x, True)
    for s_idx, (_dev, first, last) in enumerate(plan):
        st = H.make_stage(sh, layers[first:last + 1], first, last + 1, B, bf16=True, in_bf16=(s_idx == 0))
        nxt = torch.empty(x.shape, dtype=torch.float32, device="cuda")
        st.forward(cur, B, nxt, torch.cuda.current_stream())
        torch.cuda.synchronize()
        st.destroy()
        cur = nxt
    got = cur.cpu().numpy()
    ref = oracle.stage_forward(H.oracle_cfg(sh), layers, x)
    for i in range(B):
        e = H.rel_err(got[i], ref[i])
        print(f"chained plan, {len(plan)} stages, B={B}, image {i}: err {e:.3e}, std {H.err_std(got[i], ref[i]):.3e}")
        assert e <= H.TOL_BF16
