#!/usr/bin/env python3
"""Benchmark of one GPU's share of the synchronous data-parallel ResNet-50 SGD iteration.

One "step" = rn50_step: forward + backward over a local mini-batch of 32 synthetic 224x224
images (ResNet-50 v1.5, FP16 storage, FP32 accumulation / BN statistics / optimizer),
label-smoothed softmax cross-entropy (eps 0.1) and the momentum-SGD update of the flat
25,557,032-parameter buffer.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: images/s, the roofline figures of the kernel that takes the largest share
of the step (HIP-event timing of every launch, collected in a second pass of the same K steps so
that the events do not perturb the throughput figure), the per-kernel breakdown, and the CPU
oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0     # MI355X dense FP16 MFMA peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E peak


def cpu_baseline(sample_batch):
    """The CPU oracle as it stands (FP32 instantiation, storage rounding on), one full ResNet-50
    training step at a small batch; images/s = batch / seconds."""
    import numpy as np
    import oracle as O
    from oracle import resnet50 as R
    from paper_1811_05233_amd import synth
    net = R.Net(sample_batch, (224, 224))
    lay = [(s.kind, s.offset, s.count, s.fan_in) for s in net.segments]
    w = synth.flat_params(200, lay)
    x = synth.normal_f16(201, (sample_batch, 224, 224, 3))
    lab = synth.labels(202, sample_batch)
    t0 = time.perf_counter()
    R.step_ref(net, x, lab, w, np.zeros_like(w), 0.1, 0.9, 1e-4, loss_scale=1024.0, lowp=True, dtype=np.float32)
    dt = time.perf_counter() - t0
    return {"value": sample_batch / dt, "unit": "images/s", "cores": O.max_threads(), "kind": "oracle",
            "sample": "one full ResNet-50 fwd+bwd+SGD step at batch %d, 224x224, FP32 oracle with binary16 "
                      "storage rounding, %.1f s" % (sample_batch, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--cpu-sample-batch", type=int, default=4, help="0 disables the cpu_baseline leg")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event pass")
    ap.add_argument("--no-autotune", action="store_true", help="use the built-in tile heuristics")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three plain 256 MiB device copies (a kernel of known traffic, to calibrate "
                         "hardware byte counters against)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the gradient all-reduce is out of scope); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_1811_05233_amd as P
    from paper_1811_05233_amd import synth

    dev = "cuda:0"
    B = args.batch
    loss_scale = 1024.0
    cfg = P.make_config(B, loss_scale=loss_scale)
    lay = P.rn50_param_layout(cfg)
    n = P.rn50_param_count(cfg)
    w = torch.from_numpy(synth.flat_params(200, lay)).to(dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    w16 = torch.empty(n, dtype=torch.float16, device=dev)
    g16 = torch.empty(n, dtype=torch.float16, device=dev)
    x = torch.from_numpy(synth.normal_f16(201, (B, 224, 224, 3))).to(torch.float16).to(dev)
    lab = torch.from_numpy(synth.labels(202, B)).to(dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    ctx = P.Rn50Context(cfg, dev)
    P.rn50_cast_params(n, w, w16)
    hp = P.rn50_hparams(0.1, 0.9, 1e-4, 1.0 / loss_scale)

    def step():
        ctx.step(x, lab, w, v, w16, g16, hp, loss)

    if not args.no_autotune:
        ctx.autotune(x, lab, w, w16, g16, loss)      # one-off kernel-variant selection, outside the timed region

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt * 1e3 / args.steps
    loss_val = float(loss.item())
    if not np.isfinite(loss_val):
        raise RuntimeError("loss is not finite after the timed steps")

    if args.copy_probe:
        src = torch.zeros(128 << 20, dtype=torch.float16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    kernels, roof = [], None
    if not args.no_profile:
        P.rn50_profile_begin()
        for _ in range(args.steps):
            step()
        prof = P.rn50_profile_end()
        for e in prof:
            per_step_ms = e["total_ms"] / args.steps
            kernels.append({"kernel": e["name"], "launches_per_step": e["launches"] / args.steps,
                            "ms_per_step": round(per_step_ms, 4),
                            "avg_us": round(1e3 * e["total_ms"] / e["launches"], 2),
                            "tflops": round(e["flops"] / (e["total_ms"] * 1e-3) / 1e12, 1) if e["flops"] else None,
                            "gbs": round(e["bytes"] / (e["total_ms"] * 1e-3) / 1e9, 1)})
        kernels.sort(key=lambda k: -k["ms_per_step"])
        dom = max(prof, key=lambda e: e["total_ms"])
        if dom["flops"] > 0:
            ach = dom["flops"] / (dom["total_ms"] * 1e-3) / 1e12
            roof = {"kernel": dom["name"], "bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_FP16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(ach / PEAK_FP16_TFLOPS, 4), "traffic": None,
                    "avg_launch_us": round(1e3 * dom["total_ms"] / dom["launches"], 2),
                    "launches_per_step": dom["launches"] / args.steps}
        else:
            ach = dom["bytes"] / (dom["total_ms"] * 1e-3) / 1e9
            roof = {"kernel": dom["name"], "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None,
                    "avg_launch_us": round(1e3 * dom["total_ms"] / dom["launches"], 2),
                    "launches_per_step": dom["launches"] / args.steps}
        # all convolution kernels together: MFMA rate while they run, and over the whole step
        conv = [e for e in prof if e["flops"] > 0 and ("gather" in e["name"] or "wgrad_kernel" in e["name"])]
        conv_fl = sum(e["flops"] for e in conv)
        conv_ms = sum(e["total_ms"] for e in conv)
        roof["conv_mfma_util_pct"] = round(100.0 * conv_fl / (conv_ms * 1e-3) / 1e12 / PEAK_FP16_TFLOPS, 2)
        roof["conv_tflops_whole_step"] = round(conv_fl / args.steps / (ms * 1e-3) / 1e12, 1)
        sgd = [e for e in prof if e["name"].startswith("sgd")]
        if sgd:
            roof["sgd_hbm_frac"] = round(sgd[0]["bytes"] / (sgd[0]["total_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)

    out = {
        "metric": "images/sec per MI355X, ResNet-50 fwd+bwd+SGD @ batch 32",
        "value": round(B * args.steps / dt, 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
        "config": {"workload": "full ResNet-50 v1.5 training step (fwd+bwd+label-smoothed loss+momentum SGD), "
                               "batch %d, 224x224x3 fp16 N(0,1) images, 1000 classes" % B,
                   "global_batch": B, "loss_scale": loss_scale},
        "loss": round(loss_val, 5),
        "paper_context": "Table 6: 2565 images/s on 4 V100 (641 per GPU, incl. all-reduce and input pipeline)",
        "roofline": roof, "kernels": kernels,
    }
    if args.cpu_sample_batch > 0:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample_batch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
