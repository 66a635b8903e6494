"""Kernel-variant selection by the time of the whole training step.

rn50_autotune times every convolution's variants one launch site at a time, in isolation.  Inside the step the
kernels of the two streams share the compute units and the L2, and the variant that wins alone is not always the
one that gives the shortest step.  This tool searches the variant table (three entries per convolution: forward,
data gradient, filter gradient) by coordinate descent on the measured step time itself: for one entry after the
other it tries every variant id that is a kernel of its own for the shape (rn50_conv_variant_applies), and keeps
a change only if a second, longer measurement confirms the gain.

    python -m paper_1811_05233_amd.tune_in_situ --out paper_1811_05233_amd/tuning_resnet50_b32.json

writes the table that bench.py loads by default at batch 32.  Only C-ABI calls are used (rn50_set_tuning,
rn50_step); inputs are the benchmark's synthetic tensors.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--out", required=True)
    ap.add_argument("--start", default="", help="JSON table to start from (default: shape heuristics everywhere)")
    ap.add_argument("--steps", type=int, default=16, help="timed steps per trial")
    ap.add_argument("--confirm-steps", type=int, default=48)
    ap.add_argument("--min-gain-us", type=float, default=2.5, help="a trial must beat the incumbent by this much to be re-measured")
    ap.add_argument("--passes", type=int, default=1)
    ap.add_argument("--roles", default="0,1,2", help="which entries to search: 0 forward, 1 data gradient, 2 filter gradient")
    ap.add_argument("--candidates", default="", help="comma-separated variant ids to try instead of all of them "
                                                     "(a quick pass after adding a variant)")
    args = ap.parse_args()

    import torch
    import paper_1811_05233_amd as P
    from paper_1811_05233_amd import synth

    dev, B, ls = "cuda:0", args.batch, 1024.0
    cfg = P.make_config(B, loss_scale=ls)
    lay, n = P.rn50_param_layout(cfg), P.rn50_param_count(cfg)
    w = torch.from_numpy(synth.flat_params(200, lay)).to(dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    w16 = torch.empty(n, dtype=torch.float16, device=dev)
    g16 = torch.empty(n, dtype=torch.float16, device=dev)
    x = torch.from_numpy(synth.normal_f16(201, (B, 224, 224, 3))).to(torch.float16).to(dev)
    lab = torch.from_numpy(synth.labels(202, B)).to(dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    ctx = P.Rn50Context(cfg, dev)
    P.rn50_cast_params(n, w, w16)
    hp = P.rn50_hparams(0.1, 0.9, 1e-4, 1.0 / ls, 0.0, 0.0)

    table = ctx.get_tuning()
    if args.start:
        table = json.load(open(args.start))["table"]
    else:
        table = [-1] * len(table)
    counts = [P.conv_variant_count(P.CONV_FWD), P.conv_variant_count(P.CONV_DGRAD), P.conv_variant_count(P.CONV_WGRAD)]

    def measure(t, steps):
        ctx.set_tuning(t)
        for _ in range(3):
            ctx.step(x, lab, w, v, w16, g16, hp, loss)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            ctx.step(x, lab, w, v, w16, g16, hp, loss)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / steps      # microseconds per step

    # the convolutions in network order (stem; per block conv1, conv2, conv3 and, in a stage's first block, the
    # projection), to ask the library which variant ids are kernels of their own for each shape
    descs = [P.make_conv_desc(B, 224, 224, 3, 64, 7, 7, 2, 3)]
    hw, cin = 56, 64
    for stage, nblocks in enumerate((3, 4, 6, 3)):
        width = 64 << stage
        for b in range(nblocks):
            stride = 2 if (b == 0 and stage > 0) else 1
            descs.append(P.make_conv_desc(B, hw, hw, cin, width, 1, 1, 1, 0))
            descs.append(P.make_conv_desc(B, hw, hw, width, width, 3, 3, stride, 1))
            descs.append(P.make_conv_desc(B, hw // stride, hw // stride, width, 4 * width, 1, 1, 1, 0))
            if b == 0:
                descs.append(P.make_conv_desc(B, hw, hw, cin, 4 * width, 1, 1, stride, 0))
            hw //= stride
            cin = 4 * width
    assert 3 * len(descs) == len(table)
    roles = [int(r) for r in args.roles.split(",")]
    best = measure(table, args.confirm_steps)
    print("start: %.1f us per step" % best, flush=True)
    nsites = len(table) // 3
    for ps in range(args.passes):
        changed = 0
        for site in range(nsites):
            for role in roles:
                if site == 0 and role == 1:
                    continue                                  # the stem has no data gradient
                idx = 3 * site + role
                incumbent = table[idx]
                cur = measure(table, args.steps)              # re-measured per entry: the clock drifts a little
                tried = []
                cands = [int(v) for v in args.candidates.split(",")] if args.candidates else [-1] + list(range(counts[role]))
                for cand in cands:
                    if cand == incumbent or cand >= counts[role] or (cand >= 0 and not P.conv_variant_applies(descs[site], role, cand)):
                        continue
                    trial = list(table)
                    trial[idx] = cand
                    tried.append((measure(trial, args.steps), cand))
                tried.sort()
                for tm, cand in tried[:2]:
                    if tm > cur - args.min_gain_us:
                        break
                    trial = list(table)
                    trial[idx] = cand
                    a = measure(trial, args.confirm_steps)
                    b = measure(table, args.confirm_steps)
                    if a < b - 0.6 * args.min_gain_us:
                        table, best, changed = trial, a, changed + 1
                        print("  site %d role %d: %d -> %d  (%.1f -> %.1f us)" % (site, role, incumbent, cand, b, a), flush=True)
                        break
            print("pass %d site %d/%d done, step %.1f us" % (ps, site + 1, nsites, best), flush=True)
            json.dump({"batch": B, "table": table}, open(args.out, "w"))
        if not changed:
            break
    final = measure(table, 4 * args.confirm_steps)
    table = ctx.get_tuning()        # as the library runs it: ids that do not apply to a shape read -1 / the fallback's id
    print("final: %.1f us per step" % final, flush=True)
    json.dump({"batch": B, "table": table, "us_per_step_when_tuned": round(final, 1)}, open(args.out, "w"))
    ctx.close()


if __name__ == "__main__":
    main()
