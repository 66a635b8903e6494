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

Other workloads (each prints one JSON line of its own; the default is the full step):
  --mode conv-sweep   the 23 distinct ResNet-50 convolution shapes at batch 32 through conv_fwd /
                      conv_dgrad / conv_wgrad, per shape: microseconds, TFLOP/s, fraction of its own
                      roofline min(MFMA peak, arithmetic intensity x HBM peak)
  --mode batch-sweep  the full step at 16, 32, 64 and 128 images per GPU
  --mode tail         the update alone on the flat 25,557,032-element buffer, 100 steps
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PACKAGED_TUNING = os.path.join("paper_1811_05233_amd", "tuning_resnet50_b32.json")
PEAK_FP16_TFLOPS = 2500.0     # MI355X dense FP16 MFMA peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E peak


def kernel_family(name):
    """Kernel template of a profile entry: the name up to its template arguments or remark."""
    return name.split("<")[0].split(" (")[0].strip()


def measured_traffic(family):
    """HBM-side bytes per launch of a kernel template (all its instantiations, weighted by their launches) from the
    committed rocprofv3 counter summary (FETCH_SIZE and WRITE_SIZE, calibrated against a plain copy), or None if the
    summary does not list it."""
    path = os.path.join(ROOT, "profiles", "rn50_step_batch32_hbm_traffic.txt")
    launches = kib = 0.0
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) < 4:
                continue
            try:
                n, rd, wr = float(parts[-3]), float(parts[-2]), float(parts[-1])
            except ValueError:
                continue
            if kernel_family("".join(parts[:-3])) == family:
                launches += n
                kib += n * (rd + wr)
    except OSError:
        pass
    return int(kib / launches * 1024) if launches else None


def trace_average_us(family):
    """Average duration of a kernel template on the caller's stream in the committed rocprofv3 kernel trace summary
    (begin/end timestamps, i.e. without the dispatch latency that an event pair includes), or None."""
    path = os.path.join(ROOT, "profiles", "rn50_step_batch32_kernel_stats.txt")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) >= 8 and parts[0] == family and parts[2] == "launches" and parts[-1] == "average":
                return float(parts[-3])
    except (OSError, ValueError):
        pass
    return None


def _cpu_step_seconds(batch):
    import numpy as np
    from oracle import resnet50 as R
    from paper_1811_05233_amd import synth
    net = R.Net(batch, (224, 224))
    lay = [(s.kind, s.offset, s.count, s.fan_in) for s in net.segments]
    w = synth.flat_params(200, lay)
    x = synth.normal_f16(201, (batch, 224, 224, 3))
    lab = synth.labels(202, batch)
    t0 = time.perf_counter()
    R.step_ref(net, x, lab, w, np.zeros_like(w), 0.1, 0.9, 1e-4, loss_scale=1024.0, lowp=True, dtype=np.float32)
    return time.perf_counter() - t0


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(sample_batch):
    """The CPU oracle as it stands (FP32 instantiation, storage rounding on), one full ResNet-50 training step;
    images/s = batch / seconds.  sample_batch < 0: a batch-4 step first, then the largest batch of 8, 16, 32 (the
    benchmarked workload) that the batch-4 time predicts to finish within 25 s; its figure is the one reported.
    A single-threaded batch-1 step is timed as well."""
    import oracle as O
    threads = O.max_threads()
    if sample_batch < 0:
        sample_batch, dt = 4, _cpu_step_seconds(4)
        bigger = [b for b in (32, 16, 8) if dt * b / 4 <= 25.0]
        if bigger:
            sample_batch = bigger[0]
            dt = _cpu_step_seconds(sample_batch)
    else:
        dt = _cpu_step_seconds(sample_batch)
    O.set_threads(1)
    dt1 = _cpu_step_seconds(1)
    O.set_threads(threads)
    return {"value": sample_batch / dt, "unit": "images/s", "cores": threads, "kind": "oracle",
            "sample": "one full ResNet-50 fwd+bwd+SGD step at batch %d, 224x224, FP32 oracle with binary16 "
                      "storage rounding, %.1f s" % (sample_batch, dt),
            "cpu_model": _cpu_model(),
            "single_thread": {"value": 1.0 / dt1, "unit": "images/s", "cores": 1,
                              "sample": "the same step at batch 1 on one thread, %.1f s" % dt1}}


# (cin, cout, r, stride, pad, hin, layers with this shape): the 23 distinct convolution shapes of ResNet-50 v1.5
CONV_SHAPES = [
    (3, 64, 7, 2, 3, 224, 1), (64, 64, 1, 1, 0, 56, 1), (64, 64, 3, 1, 1, 56, 3), (64, 256, 1, 1, 0, 56, 4),
    (256, 64, 1, 1, 0, 56, 2), (256, 128, 1, 1, 0, 56, 1), (128, 128, 3, 2, 1, 56, 1), (128, 512, 1, 1, 0, 28, 4),
    (256, 512, 1, 2, 0, 56, 1), (512, 128, 1, 1, 0, 28, 3), (128, 128, 3, 1, 1, 28, 3), (512, 256, 1, 1, 0, 28, 1),
    (256, 256, 3, 2, 1, 28, 1), (256, 1024, 1, 1, 0, 14, 6), (512, 1024, 1, 2, 0, 28, 1), (1024, 256, 1, 1, 0, 14, 5),
    (256, 256, 3, 1, 1, 14, 5), (1024, 512, 1, 1, 0, 14, 1), (512, 512, 3, 2, 1, 14, 1), (512, 2048, 1, 1, 0, 7, 3),
    (1024, 2048, 1, 2, 0, 14, 1), (2048, 512, 1, 1, 0, 7, 2), (512, 512, 3, 1, 1, 7, 2)]


def conv_sweep(args):
    """Every convolution shape on its own through the C ABI (built-in tile heuristics), each launch timed by
    the library's HIP-event pairs on the launch stream; operands are re-used between launches (warm) or, with
    --cold, rotated among enough distinct sets to exceed the Infinity Cache."""
    import torch
    import paper_1811_05233_amd as P
    from paper_1811_05233_amd import synth
    dev, B, reps = "cuda:0", args.batch, max(args.steps, 5)
    rows, tot = [], {"fwd": [0.0, 0.0], "dgrad": [0.0, 0.0], "wgrad": [0.0, 0.0]}
    for i, (cin, cout, r, stride, pad, hin, cnt) in enumerate(CONV_SHAPES):
        d = P.make_conv_desc(B, hin, hin, cin, cout, r, r, stride, pad)
        p = (hin + 2 * pad - r) // stride + 1
        x0 = torch.from_numpy(synth.normal_f16(100 + i, (B, hin, hin, cin))).to(dev)
        w0 = torch.from_numpy(synth.he_normal_f16(130 + i, (cout, r, r, cin), cin * r * r)).to(dev)
        dy0 = torch.from_numpy(synth.normal_f16(160 + i, (B, p, p, cout))).to(dev)
        set_bytes = 2 * (x0.numel() + w0.numel() + dy0.numel())
        nset = max(2, -(-(300 << 20) // set_bytes)) if args.cold else 1          # > 256 MB of distinct operands
        xs, wts, dys = [x0] + [x0.clone() for _ in range(nset - 1)], [w0] + [w0.clone() for _ in range(nset - 1)], \
            [dy0] + [dy0.clone() for _ in range(nset - 1)]
        ys, dxs, dws = [torch.empty_like(t) for t in dys], [torch.empty_like(t) for t in xs], [torch.empty_like(t) for t in wts]
        ws = [torch.empty(max(P.conv_workspace_bytes(d, k), 16), dtype=torch.uint8, device=dev) for k in range(3)]
        turn = [0]

        def nxt():
            turn[0] = (turn[0] + 1) % nset
            return turn[0]

        flops = 2.0 * B * p * p * cout * r * r * cin
        inp = B * p * p * cin if (r == 1 and stride > 1) else B * hin * hin * cin
        nbytes = 2.0 * (inp + cout * r * r * cin + B * p * p * cout)
        floor_us = max(flops / (PEAK_FP16_TFLOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)) * 1e6
        row = {"shape": "%d>%d %dx%d/%d @%d" % (cin, cout, r, r, stride, hin), "layers": cnt,
               "gflop": round(flops / 1e9, 3), "mbytes": round(nbytes / 1e6, 1), "roofline_us": round(floor_us, 2)}

        def f_fwd():
            j = nxt()
            P.conv_fwd(d, xs[j], wts[j], ys[j], ws[0])

        def f_dgrad():
            j = nxt()
            P.conv_dgrad(d, dys[j], wts[j], dxs[j], ws[1])

        def f_wgrad():
            j = nxt()
            P.conv_wgrad(d, xs[j], dys[j], dws[j], ws[2])

        for kind, fn in (("fwd", f_fwd), ("dgrad", f_dgrad), ("wgrad", f_wgrad)):
            if kind == "dgrad" and cin == 3:
                continue
            for _ in range(3):
                fn()
            P.rn50_profile_begin()
            for _ in range(reps):
                fn()
            prof = P.rn50_profile_end()       # everything the entry point launches (filter transpose, partial-tile sum, ...)
            us = 1e3 * sum(e["total_ms"] for e in prof) / reps
            row[kind] = {"us": round(us, 1), "tflops": round(flops / us / 1e6, 1), "roofline_frac": round(floor_us / us, 3)}
            tot[kind][0] += us * cnt
            tot[kind][1] += flops * cnt
        rows.append(row)
    summary = {k: {"us_all_layers": round(v[0], 1), "tflops": round(v[1] / v[0] / 1e6, 1),
                   "mfma_util_pct": round(100.0 * v[1] / v[0] / 1e6 / PEAK_FP16_TFLOPS, 2)} for k, v in tot.items()}
    return {"metric": "conv kernel sweep, ResNet-50 v1.5 shapes @ batch %d" % B, "unit": "TFLOP/s",
            "value": summary["fwd"]["tflops"], "n_gpus": 1, "dtype": "f16 storage, f32 accumulate",
            "data": "synthetic", "config": {"workload": "23 distinct conv shapes (53 layers), fwd / dgrad / wgrad "
            "timed separately, %s operands, built-in tile heuristics" % ("cold (rotating sets > 256 MB)" if args.cold else "warm")},
            "summary": summary, "shapes": rows}


def batch_sweep(args, batches=(16, 32, 64, 128)):
    import torch
    import paper_1811_05233_amd as P
    from paper_1811_05233_amd import synth
    dev, loss_scale, res = "cuda:0", 1024.0, []
    for B in batches:
        cfg = P.make_config(B, loss_scale=loss_scale)
        lay, n = P.rn50_param_layout(cfg), P.rn50_param_count(cfg)
        w = torch.from_numpy(synth.flat_params(300 + B, lay)).to(dev)
        v = torch.zeros(n, dtype=torch.float32, device=dev)
        w16 = torch.empty(n, dtype=torch.float16, device=dev)
        g16 = torch.empty(n, dtype=torch.float16, device=dev)
        x = torch.from_numpy(synth.normal_f16(301 + B, (B, 224, 224, 3))).to(torch.float16).to(dev)
        lab = torch.from_numpy(synth.labels(302 + B, B)).to(dev)
        loss = torch.zeros(1, dtype=torch.float32, device=dev)
        ctx = P.Rn50Context(cfg, dev)
        P.rn50_cast_params(n, w, w16)
        hp = P.rn50_hparams(0.1, 0.9, 1e-4, 1.0 / loss_scale)
        if not args.no_autotune:
            ctx.autotune(x, lab, w, w16, g16, loss)
        for _ in range(args.warmup):
            ctx.step(x, lab, w, v, w16, g16, hp, loss)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ctx.step(x, lab, w, v, w16, g16, hp, loss)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        res.append({"batch": B, "images_per_s": round(B * args.steps / dt, 1), "ms_per_step": round(dt * 1e3 / args.steps, 4),
                    "loss": round(float(loss.item()), 5)})
        ctx.close()
        del ctx, w, v, w16, g16, x
    return {"metric": "images/sec per MI355X, ResNet-50 fwd+bwd+SGD, per-GPU batch %s" % "/".join(str(b) for b in batches),
            "unit": "images/s", "value": [r["images_per_s"] for r in res], "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
            "config": {"workload": "full ResNet-50 v1.5 training step at the batch-size-control sizes"}, "batches": res}


def tail(args):
    import torch
    import paper_1811_05233_amd as P
    from paper_1811_05233_amd import synth
    dev, n, steps = "cuda:0", 25557032, 100
    g = torch.from_numpy((synth.normal_f32(400, (n,)) * 1e-3).astype("float16")).to(dev)
    w = torch.from_numpy(synth.normal_f32(401, (n,)) * 0.05).to(dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    w16 = torch.empty(n, dtype=torch.float16, device=dev)
    for _ in range(3):
        P.sgd_momentum_flat(n, g, 1.0 / 54000.0, w, v, w16, 0.1, 0.9, 1e-4)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        P.sgd_momentum_flat(n, g, 1.0 / 54000.0, w, v, w16, 0.1, 0.9, 1e-4)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / steps
    gbs = 20.0 * n / us / 1e3
    # the same buffer under LARS with the ResNet-50 segment table (norm pass 6 B + update 20 B per parameter)
    cfg = P.make_config(32)
    segments = [(off, cnt, kind in (P.RN50_KIND_CONV, P.RN50_KIND_FCW)) for (kind, off, cnt, fan) in P.rn50_param_layout(cfg)]
    plan = P.LarsPlan(segments, dev)
    for _ in range(3):
        plan.step(g, 1.0 / 54000.0, w, v, w16, 0.1, 0.9, 1e-4, 0.01, 1e-6)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        plan.step(g, 1.0 / 54000.0, w, v, w16, 0.1, 0.9, 1e-4, 0.01, 1e-6)
    e1.record()
    torch.cuda.synchronize()
    us_l = e0.elapsed_time(e1) * 1e3 / steps
    gbs_l = 26.0 * n / us_l / 1e3
    return {"metric": "momentum-SGD update of the flat 25,557,032-parameter buffer", "unit": "GB/s", "value": round(gbs, 1),
            "n_gpus": 1, "steps": steps, "us_per_step": round(us, 2), "dtype": "f32 (f16 gradient in, f16 weight copy out)",
            "data": "synthetic", "config": {"workload": "g ~ N(0,1e-3^2) f16, w ~ N(0,0.05^2), v=0, grad_scale 1/54000, "
            "lr 0.1, momentum 0.9, wd 1e-4, 100 steps on the same gradient"},
            "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None, "bytes_per_parameter": 20},
            "lars": {"us_per_step": round(us_l, 2), "achieved": round(gbs_l, 1), "unit": "GB/s",
                     "frac": round(gbs_l / PEAK_HBM_GBS, 4), "bytes_per_parameter": 26, "segments": len(segments),
                     "eta": 0.01, "eps": 1e-6}}


def probes(args):
    """Machine figures that the kernel design is argued from, measured with the library's probe kernels and torch events:
    register-only MFMA rate, tile loads out of L2 / the Infinity Cache / HBM (LDS-DMA and vector loads), a streaming
    copy, the cost of a dependent empty kernel, and one large plain GEMM through the convolution kernels."""
    import torch
    import paper_1811_05233_amd as P
    dev = "cuda:0"
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps          # seconds per call

    out = torch.zeros(4096 * 256, dtype=torch.float32, device=dev)
    res = {"mfma_register_only_tflops": {}, "tile_load_tbs": {}}
    for blocks in (256, 1024, 2048):
        iters = 20000
        t = timed(lambda: P.probe_mfma(blocks, iters, out), 3)
        res["mfma_register_only_tflops"]["%d workgroups" % blocks] = round(blocks * 4 * iters * 4 * 32768.0 / t / 1e12, 1)
    src = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
    # (name, working set, workgroups, tiles per workgroup, start stride in tiles): a 2 MiB set stays in every XCD's
    # 4 MB L2 (starts spread so that workgroups sharing a compute unit are not on the same tile); 64 MiB exceeds the
    # L2s and stays in the 256 MB Infinity Cache; the last case reads each tile of 1 GiB exactly once.
    cases = (("2 MiB working set (L2)", 2 << 20, 2048, 512, 37), ("64 MiB working set (Infinity Cache)", 64 << 20, 2048, 512, 1031),
             ("1 GiB read once (HBM)", 1 << 30, 2048, 32, 32))
    for name, nbytes, blocks, iters, stride in cases:
        for lds in (1, 0):
            t = timed(lambda: P.probe_tile_load(src, nbytes, blocks, iters, stride, lds, out), 3)
            res["tile_load_tbs"][name + (", global->LDS" if lds else ", vector loads")] = round(blocks * iters * 16384.0 / t / 1e12, 2)
    t = timed(lambda: P.probe_tile_load(src, 2 << 20, 1, 4096, 0, 1, out), 3)
    res["tile_load_one_workgroup_gbs"] = round(4096 * 16384.0 / t / 1e9, 1)
    t = timed(lambda: P.probe_tile_load(src, 2 << 20, 256, 2048, 37, 1, out), 3)
    res["tile_load_one_workgroup_per_cu_tbs"] = round(256 * 2048 * 16384.0 / t / 1e12, 2)
    dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    t = timed(lambda: P.probe_copy(src, dst, 1 << 30), 5)
    res["stream_copy_tbs_read_plus_write"] = round(2.0 * (1 << 30) / t / 1e12, 2)
    del dst
    res["dependent_empty_kernel_us"] = round(timed(lambda: P.probe_empty(2000), 3) / 2000 * 1e6, 2)
    del src
    # one large plain GEMM (1x1 convolution, 100352 x 1024 x 1024) through every forward variant that applies
    d = P.make_conv_desc(32, 56, 56, 1024, 1024, 1, 1, 1, 0)
    x = torch.randn(32 * 56 * 56 * 1024, device=dev).to(torch.float16)
    w = (torch.randn(1024 * 1024, device=dev) * 0.03).to(torch.float16)
    y = torch.empty(32 * 56 * 56 * 1024, dtype=torch.float16, device=dev)
    gemm = {}
    for v in range(P.conv_variant_count(P.CONV_FWD)):
        if not P.conv_variant_applies(d, P.CONV_FWD, v):
            continue
        t = timed(lambda: P.conv_fwd(d, x, w, y, variant=v), 5)
        gemm["variant %d" % v] = round(2.0 * 100352 * 1024 * 1024 / t / 1e12, 1)
    best = max(gemm, key=gemm.get)
    res["gemm_100352x1024x1024_tflops"] = {"best": gemm[best], "best_variant": best, "frac_of_peak": round(gemm[best] / PEAK_FP16_TFLOPS, 3),
                                           "all": gemm}
    return {"metric": "hardware probes (MI355X)", "data": "synthetic", "n_gpus": 1, "probes": res}


def extras(args):
    """The other workloads of the configuration list in short form, outside the timed region of the step: the
    update tail (100 steps), the convolution sweep (warm and cold operands: totals and the three shapes furthest
    from their own roofline), the step at the other batch-size-control sizes (few steps each) and the hardware probes."""
    import copy
    out = {}
    t = tail(args)
    out["tail"] = {"sgd_gbs": t["value"], "sgd_hbm_frac": t["roofline"]["frac"], "sgd_us_per_step": t["us_per_step"],
                   "lars_gbs": t["lars"]["achieved"], "lars_hbm_frac": t["lars"]["frac"], "steps": t["steps"]}
    sweep = {}
    for cold in (False, True):
        a = copy.copy(args)
        a.cold, a.steps, a.batch = cold, 5, 32
        r = conv_sweep(a)
        worst = sorted(((row[k]["roofline_frac"], row["shape"], k, row[k]["us"]) for row in r["shapes"]
                        for k in ("fwd", "dgrad", "wgrad") if k in row))[:3]
        sweep["cold" if cold else "warm"] = {"summary": r["summary"],
                                             "worst": [{"shape": w[1], "kind": w[2], "us": w[3], "roofline_frac": w[0]} for w in worst]}
    out["conv_sweep"] = sweep
    a = copy.copy(args)
    a.steps, a.warmup, a.no_autotune = 8, 2, False
    out["batch_sweep"] = batch_sweep(a, (16, 64, 128))["batches"]
    pr = probes(args)["probes"]
    g = pr.pop("gemm_100352x1024x1024_tflops")
    pr["gemm_100352x1024x1024_tflops"] = {k: g[k] for k in ("best", "best_variant", "frac_of_peak")}
    out["hardware_probes"] = pr
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mode", choices=["step", "conv-sweep", "batch-sweep", "tail", "probes"], default="step")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--cpu-sample-batch", type=int, default=-1,
                    help="batch of the cpu_baseline leg; 0 disables it, negative picks up to 32 within about 25 s")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event pass")
    ap.add_argument("--no-extras", action="store_true",
                    help="step mode: skip the short runs of the other workloads (update tail, conv sweep, other batch sizes)")
    ap.add_argument("--no-autotune", action="store_true", help="use the built-in tile heuristics")
    ap.add_argument("--tuning-file", default="",
                    help="step mode: JSON file with the kernel-variant table; read if it exists (instead of autotuning), "
                         "written after autotuning otherwise.  Default at batch 32: the table shipped with the package "
                         "(%s), so that the benchmark and the committed profiles run the same kernels" % PACKAGED_TUNING)
    ap.add_argument("--autotune", action="store_true", help="step mode: time the kernel variants now instead of using the shipped table")
    ap.add_argument("--tune-report", default="", help="step mode: write what the autotune pass measured to this text file")
    ap.add_argument("--lars", action="store_true",
                    help="step mode: update with LARS (eta 0.01, eps 1e-6, the paper's optimizer) instead of momentum SGD")
    ap.add_argument("--cold", action="store_true",
                    help="conv-sweep: rotate every launch among enough operand sets to exceed the 256 MB Infinity Cache")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three plain 256 MiB device copies (a kernel of known traffic, to calibrate "
                         "hardware byte counters against)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the gradient all-reduce is out of scope); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.mode != "step":
        print(json.dumps({"conv-sweep": conv_sweep, "batch-sweep": batch_sweep, "tail": tail, "probes": probes}[args.mode](args)))
        return

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
    hp = P.rn50_hparams(0.1, 0.9, 1e-4, 1.0 / loss_scale, 0.01 if args.lars else 0.0, 1e-6 if args.lars else 0.0)

    def step():
        ctx.step(x, lab, w, v, w16, g16, hp, loss)

    if not args.tuning_file and not args.autotune and not args.no_autotune and P.shipped_tuning_path(B):
        args.tuning_file = P.shipped_tuning_path(B)
    shipped = os.path.abspath(args.tuning_file) == P.shipped_tuning_path(B) if args.tuning_file else False
    if args.tuning_file and os.path.exists(args.tuning_file) and not args.autotune:
        ctx.set_tuning(json.load(open(args.tuning_file))["table"])
    elif not args.no_autotune:
        ctx.autotune(x, lab, w, w16, g16, loss)      # one-off kernel-variant selection, outside the timed region
        if args.tuning_file:
            json.dump({"batch": B, "table": ctx.get_tuning()}, open(args.tuning_file, "w"))
        if args.tune_report:
            open(args.tune_report, "w").write(ctx.tuning_report())

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
    # the same K steps once more, each bracketed by its own pair of events on the launch stream: the median step time
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    median_ms = per_step[len(per_step) // 2]

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
        # the dominant kernel is looked for on the caller's stream, the dependent chain that sets the step time (an
        # event pair of a side-stream launch also contains its wait for compute units); the side stream's largest
        # kernel is reported next to it
        def by_family(entries):
            fam = {}
            for e in entries:
                f = fam.setdefault(kernel_family(e["name"]), {"name": kernel_family(e["name"]), "total_ms": 0.0, "launches": 0,
                                                              "flops": 0.0, "bytes": 0.0, "instantiations": 0})
                for k in ("total_ms", "launches", "flops", "bytes"):
                    f[k] += e[k]
                f["instantiations"] += 1
            return list(fam.values())

        def roof_of(d):
            if d["flops"] > 0:
                a = d["flops"] / (d["total_ms"] * 1e-3) / 1e12
                r = {"kernel": d["name"], "bound": "mfma", "achieved": round(a, 2), "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(a / PEAK_FP16_TFLOPS, 4)}
            else:
                a = d["bytes"] / (d["total_ms"] * 1e-3) / 1e9
                r = {"kernel": d["name"], "bound": "hbm", "achieved": round(a, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(a / PEAK_HBM_GBS, 4)}
            r["traffic"] = measured_traffic(d["name"]) if shipped else None     # the committed counters describe the shipped table
            r["avg_launch_us"] = round(1e3 * d["total_ms"] / d["launches"], 2)
            r["launches_per_step"] = d["launches"] / args.steps
            r["instantiations"] = d["instantiations"]
            r["algorithmic_bytes_per_launch"] = int(d["bytes"] / d["launches"])
            return r, a

        # A kernel is its template: the tile variants of one kernel (chosen per layer by the tuning table) count
        # together.  The dominant kernel is looked for on the caller's stream, the dependent chain that sets the step
        # time (an event pair of a side-stream launch also contains its wait for compute units); the side stream's
        # largest kernel is reported next to it.
        chain = by_family([e for e in prof if 2 * e["side_launches"] < e["launches"]])
        side = by_family([e for e in prof if 2 * e["side_launches"] >= e["launches"] and e["flops"] > 0])
        dom = max(chain, key=lambda e: e["total_ms"])
        roof, ach = roof_of(dom)
        roof["stream"] = "caller's stream (dependent chain)"
        tr = trace_average_us(dom["name"]) if shipped else None
        if tr:
            # the same kernel by the committed rocprofv3 trace: an event pair adds the dispatch latency of the launch
            roof["trace_avg_us"] = tr
            roof["frac_by_trace_duration"] = round(roof["frac"] * roof["avg_launch_us"] / tr, 4)
        if side:
            roof["side_stream_largest"] = roof_of(max(side, key=lambda e: e["total_ms"]))[0]
        if dom["flops"] > 0 and dom["bytes"] > 0:
            # where this kernel's launches sit on the roofline: their aggregate arithmetic intensity caps them at
            # intensity x HBM peak if that is below the MFMA peak
            inten = dom["flops"] / dom["bytes"]
            own = min(PEAK_FP16_TFLOPS, inten * PEAK_HBM_GBS / 1e3)
            roof["intensity_flops_per_byte"] = round(inten, 1)
            roof["own_roof_tflops"] = round(own, 1)
            roof["frac_of_own_roof"] = round(ach / own, 4)
            roof["hbm_gbs_algorithmic"] = round(dom["bytes"] / (dom["total_ms"] * 1e-3) / 1e9, 1)
        # what an event pair reads around an (almost) empty launch: the dispatch latency that avg_launch_us includes
        # and that a profiler's begin/end timestamps of the kernel do not
        tiny = torch.empty(8, dtype=torch.float16, device=dev)
        P.rn50_profile_begin()
        for _ in range(50):
            P.rn50_cast_params(8, w, tiny)
        floor = P.rn50_profile_end()
        roof["event_floor_us"] = round(1e3 * floor[0]["total_ms"] / floor[0]["launches"], 2)
        # all convolution kernels together: MFMA rate while they run, and over the whole step
        conv = [e for e in prof if e["flops"] > 0 and any(t in e["name"] for t in ("gather", "strip_gemm", "wgrad_kernel", "wgrad_strip"))]
        conv_fl = sum(e["flops"] for e in conv)
        conv_ms = sum(e["total_ms"] for e in conv)
        roof["conv_mfma_util_pct"] = round(100.0 * conv_fl / (conv_ms * 1e-3) / 1e12 / PEAK_FP16_TFLOPS, 2)
        roof["conv_tflops_whole_step"] = round(conv_fl / args.steps / (ms * 1e-3) / 1e12, 1)
        sgd = [e for e in prof if e["name"].startswith(("sgd", "lars"))]
        if sgd:
            roof["sgd_hbm_frac"] = round(sum(e["bytes"] for e in sgd) / (sum(e["total_ms"] for e in sgd) * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)

    out = {
        "metric": "images/sec per MI355X, ResNet-50 fwd+bwd+%s @ batch %d" % ("LARS" if args.lars else "SGD", B),
        "value": round(B * args.steps / dt, 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "median_ms_per_step": round(median_ms, 4),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 storage, f32 accumulate", "data": "synthetic",
        "config": {"workload": "full ResNet-50 v1.5 training step (fwd+bwd+label-smoothed loss+momentum SGD), "
                               "batch %d, 224x224x3 fp16 N(0,1) images, 1000 classes" % B,
                   "global_batch": B, "loss_scale": loss_scale},
        "loss": round(loss_val, 5),
        "paper_context": "other hardware, context only: Table 6: 2565 images/s on 4 V100 (641 per GPU, incl. all-reduce and "
                         "input pipeline); Table 5: 90 epochs in 122 s on 3456 V100; Table 2: 84.75 % scaling efficiency on 1024 V100",
        "roofline": roof, "kernels": kernels,
    }
    ctx.close()
    del ctx
    if not args.no_extras:
        out["extras"] = extras(args)
    if args.cpu_sample_batch != 0:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample_batch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
