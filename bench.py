"""Throughput of the ViT-Huge 32-layer encoder forward (one pipeline stage that
holds the whole model) at micro-batch 64 on one MI355X.

A step is one ep_stage_forward over one synthetic micro-batch already resident
in HBM.  Prints ONE JSON line: images/s (wall clock around the timed steps),
the median and minimum step time from HIP events around every step, the
roofline of the dominant kernel (the first MLP GEMM, timed with HIP events
inside the library on the stream it runs on) against the published bf16 peak
and against what a loop of nothing but matrix instructions sustains on this
box, the per-kernel time split of a layer, the shader clock the dense layers
ran at, and the CPU checker timed on the host cores on a bounded sample.

Other workloads: --model / --layers / --batch (e.g. the ViT-Base 3-layer stage
at micro-batch 8, the ViT-Large 6-layer stage at micro-batches 1 .. 64);
--mfma-peak prints the matrix-core probe alone.
"""
import argparse
import hashlib
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16, published
PEAK_HBM_GBPS = 8000.0             # MI355X HBM3E, published
PROBE_ITERS = 100000               # matrix instructions x 16 per wave of the probe: about 20 ms

# Sources that define the dense-layer kernel whose HBM traffic profiles/ records; the recorded
# figure is reported only while their hash matches the one stored next to it.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "vit_huge_b64_fc1_hbm_traffic.md")
KERNEL_SOURCES = ("ep_gemm_bf16_persist.hip", "ep_gemm_bf16_skinny_tile.h", "ep_gemm_bf16.hip", "ep_device.h")


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2110_14895_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def recorded_traffic():
    """HBM bytes per FC1 launch at the headline workload from the rocprofv3 counter summary, or None
    when the kernel sources have changed since the counters were taken."""
    try:
        text = open(TRAFFIC_FILE).read()
        sha = re.search(r"kernel_source_sha256_16:\s*([0-9a-f]{16})", text).group(1)
        val = float(re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text).group(1))
    except (OSError, AttributeError, ValueError):
        return None
    return val if sha == kernel_source_hash() else None


def algorithmic_bytes_per_layer(sh, rows: int) -> float:
    """HBM bytes one layer has to move with every intermediate written once and read once (fp32 residual
    stream, bf16 operands): LN1 read 4RD, q|k|v written and read 6RD + 6RD, attention output 2RD + 2RD,
    residual read and written by the two residual layers 4 x 4RD, LN2 read 4RD, hidden activations
    2RM + 2RM, and the layer's parameters."""
    d, m = sh.d_model, sh.d_mlp
    weights = 2.0 * (3 * d * d + d * d + 2 * d * m) + 4.0 * (9 * d + m)
    return rows * d * 40.0 + rows * m * 4.0 + weights


def mfma_peak_report(binding, stream):
    out = {}
    for form, name in ((0, "16x16x32"), (1, "32x32x16")):
        for rnd, dname in ((0, "constant"), (1, "random")):
            tf, mhz = binding.mfma_peak(form, rnd, PROBE_ITERS, stream)
            out[f"{name}_{dname}"] = {"tflops": round(tf, 1), "shader_mhz": round(mhz)}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
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
    ap.add_argument("--mfma-peak", action="store_true",
                    help="print what a loop of nothing but bf16 matrix instructions sustains (both instruction "
                         "forms, constant and random operands) and exit")
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
    stream = torch.cuda.current_stream()

    if args.mfma_peak:
        print(json.dumps({"metric": "bf16 matrix-instruction loop, TFLOP/s", "published_peak": PEAK_BF16_MFMA_TFLOPS,
                          "iters": PROBE_ITERS, "probe": mfma_peak_report(binding, stream)}))
        return 0

    sh = synth.SHAPES[args.model]
    n_layers = args.layers or sh.n_layers
    B = args.batch
    layers = [synth.layer_params(sh, l, bf16=True) for l in range(n_layers)]
    x = synth.activations(sh, B, bf16=True)
    cfg = binding.VitConfig(sh.n_layers, sh.d_model, sh.n_heads, sh.d_mlp, sh.n_tokens, sh.ln_eps,
                            binding.EP_BF16, binding.EP_BF16, binding.EP_F32)
    xin = torch.from_numpy(synth.f32_to_bf16_bits(x).reshape(x.shape).view(np.int16)).cuda()
    out = torch.empty(x.shape, dtype=torch.float32, device="cuda")
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
    # ---- the timed region: exactly --steps steps between two synchronisations; an event on the
    # steps' stream before each step and after the last gives every step's own duration
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record(stream)
        step()
    marks[args.steps].record(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]

    ms_per_step = dt / args.steps * 1e3
    images_per_s = B * args.steps / dt
    flops_per_step = B * n_layers * sh.flops_per_image_per_layer()
    tflops = flops_per_step / (dt / args.steps) / 1e12
    R = B * sh.n_tokens
    bytes_per_step = n_layers * algorithmic_bytes_per_layer(sh, R)

    # ---- what the matrix cores of this machine sustain on a loop of nothing but the dense layers' matrix
    # instruction, on random operands (the chip lowers its clock under real data)
    peak_measured, probe_mhz = binding.mfma_peak(0, True, PROBE_ITERS, stream)

    # ---- dominant kernel: the launch of FC1 (+GELU), HIP events around each of its launches
    # (recorded inside the library on the stream it launches on) in a second pass over the same
    # steps; the other kernels of the layer are timed the same way for the split.
    roofline = None
    kernels = {}
    gemm_mhz = None
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
            by = 2.0 * rows * sh.d_model + 2.0 * sh.d_mlp * sh.d_model + 4.0 * sh.d_mlp + 2.0 * rows * sh.d_mlp
            t = sec / n
            tf, gb = fl / t / 1e12, by / t / 1e9
            mfma_bound = tf / PEAK_BF16_MFMA_TFLOPS >= gb / PEAK_HBM_GBPS    # the roof the launch is nearer to
            headline = (B, sh.name, n_layers) == (64, "vit_huge", 32)
            roofline = {"kernel": "fc1_gelu_gemm_launch", "bound": "mfma" if mfma_bound else "hbm",
                        "achieved": round(tf if mfma_bound else gb, 2),
                        "peak": PEAK_BF16_MFMA_TFLOPS if mfma_bound else PEAK_HBM_GBPS,
                        "unit": "TFLOP/s" if mfma_bound else "GB/s",
                        "frac": round(tf / PEAK_BF16_MFMA_TFLOPS if mfma_bound else gb / PEAK_HBM_GBPS, 4),
                        "traffic": recorded_traffic() if headline else None,
                        "peak_measured": round(peak_measured, 1) if mfma_bound else None,
                        "frac_measured": round(tf / peak_measured, 4) if mfma_bound else None,
                        "tflops": round(tf, 2), "algorithmic_gbps": round(gb, 1),
                        "avg_us": round(t * 1e6, 2), "launches": n, "rows": rows,
                        "flop_per_launch": fl, "algorithmic_bytes_per_launch": by}
            try:
                gemm_mhz = round(binding.gemm_clock_sample()[0])     # the last large dense-layer launch of the pass
            except binding.EdgePipeError:
                gemm_mhz = None                                      # micro-batch too small for such launches

    headline = (sh.name, n_layers) == ("vit_huge", 32)
    result = {
        "metric": ("images/sec + % bf16 MFMA peak, ViT-Huge 32-layer encoder fwd, 1 MI355X" if headline else
                   f"images/sec + % bf16 MFMA peak, {sh.name} {n_layers}-layer encoder fwd, 1 MI355X"),
        "value": round(images_per_s, 2), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{sh.name} {n_layers}-layer stage, micro-batch {B}, T={sh.n_tokens}, "
                               f"D={sh.d_model}, H={sh.n_heads}, M={sh.d_mlp}; bf16 in, fp32 residual and output",
                   "micro_batch": mb, "layers": n_layers, "stages": args.stages, "batch": B,
                   "launch": "graph replay" if args.graph else "eager"},
        "ms_per_step_median": round(statistics.median(step_ms), 3), "ms_per_step_min": round(min(step_ms), 3),
        "tflops": round(tflops, 2), "frac_bf16_mfma_peak": round(tflops / PEAK_BF16_MFMA_TFLOPS, 4),
        "mfma_peak_measured_tflops": round(peak_measured, 1),
        "frac_mfma_peak_measured": round(tflops / peak_measured, 4),
        "algorithmic_gbps": round(bytes_per_step / (dt / args.steps) / 1e9, 1),
        "frac_hbm_peak": round(bytes_per_step / (dt / args.steps) / 1e9 / PEAK_HBM_GBPS, 4),
        "clocks": {"mfma_probe_shader_mhz": round(probe_mhz), "dense_layer_shader_mhz": gemm_mhz},
        "roofline": roofline,
        "kernel_us_per_launch": {k: (round(v, 2) if v else None) for k, v in kernels.items()},
    }

    if not args.no_cpu_baseline:
        import oracle
        ocfg = oracle.OracleConfig(sh.d_model, sh.n_heads, sh.d_mlp, sh.n_tokens, sh.ln_eps)
        # parity sample: up to eight images spread evenly over the micro-batch, each compared element by
        # element; the checker is timed on the first half of them (a bounded sample: about 20 s at the
        # headline shape on 16 cores)
        n_par = min(8, B)
        sample = sorted({round(k * (B - 1) / max(n_par - 1, 1)) for k in range(n_par)})
        n_cpu = max(1, len(sample) // 2)
        got_all = out.cpu().numpy()
        t0 = time.perf_counter()
        refs = oracle.stage_forward(ocfg, layers, x[sample[:n_cpu]])
        cdt = time.perf_counter() - t0
        if len(sample) > n_cpu:
            refs = np.concatenate([refs, oracle.stage_forward(ocfg, layers, x[sample[n_cpu:]])])
        errs, stds = {}, {}
        for k, i in enumerate(sample):
            ref = refs[k]
            rms = float(np.sqrt((ref * ref).mean()))
            d = got_all[i].astype(np.float64) - ref
            errs[str(i)] = round(float(np.abs(d).max()) / rms, 5)
            stds[str(i)] = round(float(d.std()) / rms, 5)
        result["cpu_baseline"] = {"value": round(n_cpu / cdt, 4), "unit": "images/s",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "sample": f"images {sample[:n_cpu]} of the same micro-batch through all {n_layers} "
                                            f"layers ({cdt:.1f} s of float64 CPU work)"}
        result["parity_max_abs_over_rms"] = errs
        result["parity_err_std_over_rms"] = stds
        result["parity_worst"] = max(errs.values())

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
