#!/usr/bin/env python3
"""Benchmark of the PCONV hot path on one MI355X.

One "step" = one pass of the VGG-16 3x3 convolution stack (13 pattern+connectivity-sparse conv
layers with fused bias+ReLU, 2x2 max-pools between blocks) at batch 32, fp32, chained on the
device with all inputs resident in HBM.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_VEC_TFLOPS = 157.3      # MI355X fp32 vector peak (256 CU x 2.4 GHz x 256 flop/clk/CU)
PEAK_HBM_GBS = 8000.0
# HBM bytes of the 13 conv launches of one step, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled
# by a 256 MiB device copy (x2.000 / x1.000); see profiles/pconv_conv2d_vgg16_stack_n32_fp32.md.
# Valid for the default workload (batch 32) only.
MEASURED_TRAFFIC_BYTES_BATCH32 = 3.346e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--policy", type=int, default=0, help="kernel policy (0 auto, 1 generic, 2 tiled)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--num-patterns", type=int, default=0, choices=[0, 4, 8, 12],
                    help="size of the pattern table of the sparse layers (0 = the workload's own, 8): the "
                         "paper's pattern-count experiment on the same shapes")
    ap.add_argument("--no-fuse-pool", action="store_true",
                    help="run every max-pool as a kernel of its own instead of in the epilogue of the convolution")
    ap.add_argument("--profile-copy-mb", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (calibrates rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters against a kernel of known traffic)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the batch would shard across GPUs with no "
              "exchange step); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1909_05073_amd as P
    from pconv_inputs import base_seed, config_layers, make_layer, nnz_of_layer

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    P.pconv_set_kernel_policy(args.policy)
    dev = torch.device("cuda:0")
    specs = config_layers(3, batch=args.batch)
    if args.num_patterns:
        import dataclasses
        specs = [s if s.pattern_dist == "dense" else dataclasses.replace(s, num_patterns=args.num_patterns) for s in specs]
    n = args.batch

    layers = []
    for i, spec in enumerate(specs):
        L = make_layer(spec, base_seed(3) + 100 * i)
        h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
        nnz = nnz_of_layer(L)
        flop = 2.0 * nnz * n * spec.h_out * spec.w_out
        # The max-pool after a layer goes into the convolution's epilogue, except where the layer has so
        # few tiles that the library shares them between workgroups through the full-size output
        # (conv13 at batch 32), which a fused pool would rule out.
        units = -(-(n * -(-spec.h // 4) * -(-spec.w // 4)) // 64) * -(-spec.c_out // 64)
        fuse = bool(spec.pool_after) and not args.no_fuse_pool and args.policy != 1 and units > 128
        out_elems = n * spec.c_out * ((spec.h_out // 2) * (spec.w_out // 2) if fuse else spec.h_out * spec.w_out)
        byts = 4.0 * (n * spec.c_in * spec.h * spec.w + out_elems) + 4.0 * nnz + 2.0 * int(L["conn"].sum())
        layers.append(dict(spec=spec, L=L, h=h, bias=torch.from_numpy(L["bias"]).to(dev), nnz=nnz,
                           flop=flop, bytes=byts, fuse=fuse,
                           y=(None if fuse else torch.empty((n, spec.c_out, spec.h_out, spec.w_out), device=dev)),
                           p=(torch.empty((n, spec.c_out, spec.h_out // 2, spec.w_out // 2), device=dev)
                              if spec.pool_after else None)))
    g = torch.Generator(device=dev); g.manual_seed(base_seed(3))
    x0 = torch.randn((n, 3, 224, 224), device=dev, generator=g).clamp_(min=0)
    stream = torch.cuda.current_stream().cuda_stream

    def step(events=None):
        cur = x0
        for i, ly in enumerate(layers):
            s = ly["spec"]
            if events is not None:
                events[i][0].record()
            if ly["fuse"]:
                P.pconv_conv2d_pool2x2(ly["h"], cur.data_ptr(), ly["p"].data_ptr(), ly["bias"].data_ptr(), n, s.h, s.w,
                                       P.NCHW, P.F32, True, stream)
                if events is not None:
                    events[i][1].record()
                cur = ly["p"]
                continue
            P.pconv_conv2d(ly["h"], cur.data_ptr(), ly["y"].data_ptr(), ly["bias"].data_ptr(), n, s.h, s.w,
                           1, 1, P.NCHW, P.F32, True, stream)
            if events is not None:
                events[i][1].record()
            cur = ly["y"]
            if ly["p"] is not None:
                P.pconv_maxpool2x2(cur.data_ptr(), ly["p"].data_ptr(), n, s.c_out, s.h_out, s.w_out,
                                   P.NCHW, P.F32, stream)
                cur = ly["p"]

    if args.profile_copy_mb:
        src = torch.empty(args.profile_copy_mb * 2**20 // 4, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in layers] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(ev[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    total_flop = sum(ly["flop"] for ly in layers)
    per_layer = []
    conv_ms_total = 0.0
    for i, ly in enumerate(layers):
        ms = float(np.mean([ev[k][i][0].elapsed_time(ev[k][i][1]) for k in range(args.steps)]))
        conv_ms_total += ms
        t_roof_ms = max(ly["flop"] / (PEAK_VEC_TFLOPS * 1e12), ly["bytes"] / (PEAK_HBM_GBS * 1e9)) * 1e3
        per_layer.append(dict(layer=ly["spec"].name + ("+pool" if ly["fuse"] else ""), ms=round(ms, 4),
                              eff_tflops=round(ly["flop"] / ms / 1e9, 2),
                              alg_gbs=round(ly["bytes"] / ms / 1e6, 1),
                              binds="hbm" if ly["bytes"] / (PEAK_HBM_GBS * 1e9) > ly["flop"] / (PEAK_VEC_TFLOPS * 1e12) else "alu",
                              roof_frac=round(t_roof_ms / ms, 4)))
    achieved = total_flop / (conv_ms_total * 1e-3) / 1e12
    out = {
        "metric": "effective GFLOP/s (nonzero MACs), VGG-16 3x3 stack",
        "value": round(total_flop / (ms_per_step * 1e-3) / 1e9, 1),
        "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"vgg16_3x3_stack_13conv_batch{n}_fp32_{args.num_patterns or 8}pattern_conn3.6x",
                   "global_batch": n, "layout": "nchw", "kernel_policy": args.policy,
                   "fused_maxpools": sum(1 for ly in layers if ly["fuse"])},
        "roofline": {"bound": "alu", "achieved": round(achieved, 3), "peak": PEAK_VEC_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_VEC_TFLOPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES_BATCH32 if (n == 32 and args.policy == 0 and not args.no_fuse_pool
                                                                   and args.num_patterns in (0, 8)) else None,
                     "algorithmic_flop": total_flop, "algorithmic_bytes": sum(ly["bytes"] for ly in layers),
                     "kernel": "pconv_conv2d / pconv_conv2d_pool2x2 (13 launches per step, summed)",
                     "conv_ms_per_step": round(conv_ms_total, 4),
                     "stack_roof_frac": round(sum(max(ly["flop"] / (PEAK_VEC_TFLOPS * 1e12),
                                                      ly["bytes"] / (PEAK_HBM_GBS * 1e9)) for ly in layers)
                                              * 1e3 / conv_ms_total, 4)},
        "layers": per_layer,
    }

    if not args.no_cpu_baseline:
        # the oracle as it stands, on the host cores, on a bounded sample of the step: the 13 layers at
        # a smaller batch (the work per image is the same for every image)
        import oracle
        from pconv_inputs import make_input
        cpu_batch = min(n, 16)
        cpu_s = 0.0
        cpu_flop = 0.0
        for i, spec_c in enumerate(config_layers(3, batch=cpu_batch)):
            L = layers[i]["L"]
            x = make_input(spec_c, base_seed(3) + 100 * i)
            wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
            t = time.perf_counter()
            oracle.conv2d(x, wt, L["bias"], relu=True)
            cpu_s += time.perf_counter() - t
            cpu_flop += 2.0 * layers[i]["nnz"] * cpu_batch * spec_c.h_out * spec_c.w_out
            del x
        out["cpu_baseline"] = {"value": round(cpu_flop / cpu_s / 1e9, 3), "unit": "GFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "the 13 conv layers at batch %d (%d/%d of one step), %.1f s"
                                         % (cpu_batch, cpu_batch, n, cpu_s)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
