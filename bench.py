"""Throughput of the ViT-Huge 32-layer encoder forward (one pipeline stage that
holds the whole model) at micro-batch 64 on one MI355X.

A step is one ep_stage_forward over one synthetic micro-batch already resident
in HBM.  Prints ONE JSON line: images/s, the roofline of the dominant kernel
(the first MLP GEMM, timed with HIP events inside the library on the stream it
runs on), the per-kernel time split of a layer, and the CPU checker timed on
the host cores on a bounded sample (three images through all 32 layers).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16
# HBM bytes per launch of the dominant kernel at the headline workload, from two rocprofv3 --pmc
# runs of this script (FETCH_SIZE, WRITE_SIZE), each scaled by what the same counter reads for the
# input conversion kernel, whose traffic is known: 308.2 MB fetched + 179.9 MB written
# (profiles/vit_huge_b64_fc1_hbm_traffic.md).  Valid for the kernel as profiled; set to None when
# the kernel changes until the counters are taken again.
FC1_MAIN_TRAFFIC_BYTES = 308.2e6 + 179.9e6


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--model", default="vit_huge",
                    help="vit_huge (headline) | vit_large | vit_base | deit_small | deit_tiny")
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--layers", type=int, default=0, help="0 = all layers of the model")
    ap.add_argument("--stages", type=int, default=1,
                    help="cut the layers evenly into this many pipeline stages (ep_pipeline_run) ...")
    ap.add_argument("--micro-batch", type=int, default=0,
                    help="... fed with micro-batches of this size (must divide --batch; default: the batch)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays (pays off where the launches of a step, "
                         "not its kernels, set the pace: narrow models, small batches)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-split", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU only (a pipeline stage is one device's work); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2110_14895_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    binding.lib()          # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)

    sh = synth.SHAPES[args.model]
    n_layers = args.layers or sh.n_layers
    B = args.batch
    layers = [synth.layer_params(sh, l, bf16=True) for l in range(n_layers)]
    x = synth.activations(sh, B, bf16=True)
    cfg = binding.VitConfig(sh.n_layers, sh.d_model, sh.n_heads, sh.d_mlp, sh.n_tokens, sh.ln_eps,
                            binding.EP_BF16, binding.EP_BF16, binding.EP_F32)
    xin = torch.from_numpy(synth.f32_to_bf16_bits(x).reshape(x.shape).view(np.int16)).cuda()
    out = torch.empty(x.shape, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    mb = args.micro_batch or B
    pipelined = args.stages > 1 or mb != B
    if pipelined and args.graph:
        print("bench.py: --graph times the single-stage forward; drop --stages / --micro-batch", file=sys.stderr)
        return 2
    if pipelined:
        # the same work through the pipeline runtime: even cut into --stages stages, fp32 boundaries
        if B % mb or args.stages > n_layers:
            print("bench.py: --micro-batch must divide --batch and --stages must not exceed the layers", file=sys.stderr)
            return 2
        cuts = [round(k * n_layers / args.stages) for k in range(args.stages + 1)]
        stages = []
        for k in range(args.stages):
            c = binding.VitConfig(sh.n_layers, sh.d_model, sh.n_heads, sh.d_mlp, sh.n_tokens, sh.ln_eps,
                                  binding.EP_BF16, binding.EP_BF16 if k == 0 else binding.EP_F32, binding.EP_F32)
            stages.append(binding.Stage(c, cuts[k], cuts[k + 1],
                                        [synth.as_param_dtype(p, True) for p in layers[cuts[k]:cuts[k + 1]]], mb))
        pipe = binding.Pipeline(stages, mb)
        stage = None

        def step():
            pipe.run(xin, B // mb, out, stream)
    else:
        stage = binding.Stage(cfg, 0, n_layers, [synth.as_param_dtype(p, True) for p in layers], B)

        def step():
            stage.forward(xin, B, out, stream)

    for _ in range(max(args.warmup, 1) if args.graph else args.warmup):
        step()                                   # also the first-call set-up, which a capture must not see
    torch.cuda.synchronize()
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        eager_stream, stream = stream, side
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        stream = eager_stream
        step = graph.replay
        step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3
    images_per_s = B * args.steps / dt
    flops_per_step = B * n_layers * sh.flops_per_image_per_layer()
    tflops = flops_per_step / (dt / args.steps) / 1e12

    # ---- dominant kernel: the persistent GEMM launch of FC1 (+GELU), HIP events around each of
    # its launches (recorded inside the library on the stream it launches on) in a second pass
    # over the same steps; the other kernels of the layer are timed the same way for the split.
    R = B * sh.n_tokens
    roofline = None
    kernels = {}
    fc1_main = binding.MAIN_KERNEL_IDS["fc1"]
    ids = list(range(len(binding.KERNEL_NAMES))) + [fc1_main] if not args.no_kernel_split else [fc1_main]
    if pipelined or args.graph:
        ids = []           # the per-kernel split belongs to the eager single-stage run
    for kid in ids:
        steps = args.steps if kid == fc1_main else min(args.steps, 3)
        stage.trace_begin(kid, n_layers * steps)
        for _ in range(steps):
            stage.forward(xin, B, out, stream)
        torch.cuda.synchronize()
        n, sec = stage.trace_end()
        if kid < len(binding.KERNEL_NAMES):
            kernels[binding.KERNEL_NAMES[kid]] = sec / n * 1e6 if n else None
        elif n:
            rows = stage.gemm_main_rows(B, kid)          # rows this launch covers
            fl = 2.0 * rows * sh.d_model * sh.d_mlp
            achieved = fl / (sec / n) / 1e12
            roofline = {"kernel": "fc1_gelu_gemm_main_launch", "bound": "mfma", "achieved": round(achieved, 2),
                        "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(achieved / PEAK_BF16_MFMA_TFLOPS, 4),
                        "traffic": FC1_MAIN_TRAFFIC_BYTES if (B, sh.name, n_layers) == (64, "vit_huge", 32) else None,
                        "avg_us": round(sec / n * 1e6, 2), "launches": n, "rows": rows,
                        "flop_per_launch": fl}

    result = {
        "metric": ("images/sec + % bf16 MFMA peak, ViT-Huge 32-layer encoder fwd, 1 MI355X"
                   if (sh.name, n_layers) == ("vit_huge", 32) else
                   f"images/sec + % bf16 MFMA peak, {sh.name} {n_layers}-layer encoder fwd, 1 MI355X"),
        "value": round(images_per_s, 2), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{sh.name} {n_layers}-layer stage, micro-batch {B}, T={sh.n_tokens}, "
                               f"D={sh.d_model}, H={sh.n_heads}, M={sh.d_mlp}; bf16 in, fp32 residual and output",
                   "micro_batch": mb, "layers": n_layers, "stages": args.stages, "batch": B,
                   "launch": "graph replay" if args.graph else "eager"},
        "tflops": round(tflops, 2), "frac_bf16_mfma_peak": round(tflops / PEAK_BF16_MFMA_TFLOPS, 4),
        "roofline": roofline,
        "kernel_us_per_launch": {k: (round(v, 2) if v else None) for k, v in kernels.items()},
    }

    if not args.no_cpu_baseline:
        import oracle
        ocfg = oracle.OracleConfig(sh.d_model, sh.n_heads, sh.d_mlp, sh.n_tokens, sh.ln_eps)
        n_cpu = min(3, B)                        # a bounded sample: about 15 s at the headline shape
        t0 = time.perf_counter()
        ref = oracle.stage_forward(ocfg, layers, x[:n_cpu])
        cdt = time.perf_counter() - t0
        got = out[:n_cpu].cpu().numpy().astype(np.float64)
        err = float(np.abs(got - ref).max() / np.sqrt((ref * ref).mean()))
        result["cpu_baseline"] = {"value": round(n_cpu / cdt, 4), "unit": "images/s",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "sample": f"{n_cpu} images of the same micro-batch through all {n_layers} layers "
                                            f"({cdt:.1f} s of float64 CPU work)"}
        result["parity_sample_max_abs_over_rms"] = round(err, 5)

    print(json.dumps(result))
    if pipelined:
        pipe.destroy()
        for st in stages:
            st.destroy()
    else:
        stage.destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())
