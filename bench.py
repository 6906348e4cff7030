#!/usr/bin/env python3
"""Benchmark of the PCONV hot path on one MI355X.

One "step" = one pass of the VGG-16 3x3 convolution stack (13 pattern+connectivity-sparse conv
layers with fused bias+ReLU, 2x2 max-pools between blocks) at batch 32, fp32, chained on the
device with all inputs resident in HBM.  Prints ONE JSON line: the headline metric with its
roofline and CPU-baseline objects, and, timed after the headline loop, the other benchmark
configurations (one 256->256 layer at batch 1, the ResNet-50 3x3 layers in bf16, the imbalanced
stress layer), the pattern-count sweep of the paper's Tables 1-2 and cold-cache times of the two
HBM-bound layers.
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_VEC_TFLOPS = 157.3      # MI355X fp32 vector peak (256 CU x 2.4 GHz x 256 flop/clk/CU)
PEAK_MFMA_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
# HBM bytes of the 13 conv launches of one step, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled
# by a 256 MiB device copy (x2.000 / x1.000); see profiles/pconv_conv2d_vgg16_stack_n32_fp32.md.
# Valid for the default workload (batch 32) only.
MEASURED_TRAFFIC_BYTES_BATCH32 = 2.914e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--policy", type=int, default=0, help="kernel policy (0 auto, 1 generic, 2 tiled)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="headline loop only: no other configurations, sweep or cold-cache times")
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
    from pconv_inputs import LayerSpec, base_seed, config_layers, make_layer, nnz_of_layer

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    P.pconv_set_kernel_policy(args.policy)
    dev = torch.device("cuda:0")
    n = args.batch
    stream = torch.cuda.current_stream().cuda_stream

    def t_roof_s(flop, byts):
        return max(flop / (PEAK_VEC_TFLOPS * 1e12), byts / (PEAK_HBM_GBS * 1e9))

    # ---- the VGG-16 stack ------------------------------------------------------------------
    def build_stack(num_patterns=0, table=None):
        """Packs the 13 layers.  table: replaces the pattern table of the sparse layers (same ids)."""
        specs = config_layers(3, batch=n)
        if num_patterns:
            specs = [s if s.pattern_dist == "dense" else dataclasses.replace(s, num_patterns=num_patterns) for s in specs]
        layers = []
        for i, spec in enumerate(specs):
            L = make_layer(spec, base_seed(3) + 100 * i)
            if table is not None and spec.pattern_dist != "dense":
                L = dict(L, table=np.asarray(table, np.uint16))
            h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
            nnz = nnz_of_layer(L)
            flop = 2.0 * nnz * n * spec.h_out * spec.w_out
            # the max-pool after a layer goes into the convolution's epilogue where the library recommends it
            fuse = (bool(spec.pool_after) and not args.no_fuse_pool and
                    P.pconv_pool2x2_fusion(h, n, spec.h, spec.w, P.NCHW, P.F32) == 2)
            out_elems = n * spec.c_out * ((spec.h_out // 2) * (spec.w_out // 2) if fuse else spec.h_out * spec.w_out)
            byts = 4.0 * (n * spec.c_in * spec.h * spec.w + out_elems) + 4.0 * nnz + 2.0 * int(L["conn"].sum())
            layers.append(dict(spec=spec, L=L, h=h, bias=torch.from_numpy(L["bias"]).to(dev), nnz=nnz,
                               flop=flop, bytes=byts, fuse=fuse))
        return layers

    # activations of the stack: one set of buffers, shared by every table variant
    shapes = config_layers(3, batch=n)
    ybuf = [torch.empty((n, s.c_out, s.h_out, s.w_out), device=dev) for s in shapes]
    pbuf = [torch.empty((n, s.c_out, s.h_out // 2, s.w_out // 2), device=dev) if s.pool_after else None for s in shapes]
    g = torch.Generator(device=dev); g.manual_seed(base_seed(3))
    x0 = torch.randn((n, 3, 224, 224), device=dev, generator=g).clamp_(min=0)

    def step(layers, events=None):
        cur = x0
        for i, ly in enumerate(layers):
            s = ly["spec"]
            if events is not None:
                events[i][0].record()
            if ly["fuse"]:
                P.pconv_conv2d_pool2x2(ly["h"], cur.data_ptr(), pbuf[i].data_ptr(), ly["bias"].data_ptr(), n, s.h, s.w,
                                       P.NCHW, P.F32, True, stream)
                if events is not None:
                    events[i][1].record()
                cur = pbuf[i]
                continue
            P.pconv_conv2d(ly["h"], cur.data_ptr(), ybuf[i].data_ptr(), ly["bias"].data_ptr(), n, s.h, s.w,
                           1, 1, P.NCHW, P.F32, True, stream)
            if events is not None:
                events[i][1].record()
            cur = ybuf[i]
            if pbuf[i] is not None:
                P.pconv_maxpool2x2(cur.data_ptr(), pbuf[i].data_ptr(), n, s.c_out, s.h_out, s.w_out,
                                   P.NCHW, P.F32, stream)
                cur = pbuf[i]

    def time_stack(layers, steps, warmup, per_layer=False):
        for _ in range(warmup):
            step(layers)
        torch.cuda.synchronize()
        ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in layers] for _ in range(steps)] if per_layer else None
        t0 = time.perf_counter()
        for k in range(steps):
            step(layers, ev[k] if per_layer else None)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms = (t1 - t0) * 1e3 / steps
        if not per_layer:
            return ms, None
        return ms, [float(np.mean([ev[k][i][0].elapsed_time(ev[k][i][1]) for k in range(steps)])) for i in range(len(layers))]

    layers = build_stack(args.num_patterns)
    if args.profile_copy_mb:
        src = torch.empty(args.profile_copy_mb * 2**20 // 4, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ms_per_step, layer_ms = time_stack(layers, args.steps, args.warmup, per_layer=True)

    total_flop = sum(ly["flop"] for ly in layers)
    per_layer = []
    for ly, ms in zip(layers, layer_ms):
        s = ly["spec"]
        units = -(-(n * -(-s.h // 4) * -(-s.w // 4)) // 64) * -(-s.c_out // 64)   # (tile of 64 patches, 64 filters) pairs
        per_layer.append(dict(layer=s.name + ("+pool" if ly["fuse"] else ""), ms=round(ms, 4),
                              eff_tflops=round(ly["flop"] / ms / 1e9, 2),
                              alg_gbs=round(ly["bytes"] / ms / 1e6, 1),
                              binds="hbm" if ly["bytes"] / (PEAK_HBM_GBS * 1e9) > ly["flop"] / (PEAK_VEC_TFLOPS * 1e12) else "alu",
                              roof_frac=round(t_roof_s(ly["flop"], ly["bytes"]) * 1e3 / ms, 4),
                              units=units))
    conv_ms_total = sum(layer_ms)
    achieved = total_flop / (conv_ms_total * 1e-3) / 1e12
    default_workload = n == 32 and args.policy == 0 and not args.no_fuse_pool and args.num_patterns in (0, 8)
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
                     "traffic": MEASURED_TRAFFIC_BYTES_BATCH32 if default_workload else None,
                     "algorithmic_flop": total_flop, "algorithmic_bytes": sum(ly["bytes"] for ly in layers),
                     "kernel": "pconv_conv2d / pconv_conv2d_pool2x2 (13 launches per step, summed)",
                     "conv_ms_per_step": round(conv_ms_total, 4),
                     "stack_roof_frac": round(sum(t_roof_s(ly["flop"], ly["bytes"]) for ly in layers)
                                              * 1e3 / conv_ms_total, 4)},
        "layers": per_layer,
    }

    if not args.no_extras:
        # the plain v_fmac rate of this device, next to the datasheet peak
        pm = P.pconv_debug_measure_fma_peak()
        out["roofline"]["peak_measured"] = round(pm, 1)
        out["roofline"]["frac_of_peak_measured"] = round(achieved / pm, 4)

        def time_call(fn, iters=20, warm=3, flush=None):
            for _ in range(warm):
                fn()
            torch.cuda.synchronize()
            tot = 0.0
            e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
            if flush is None:
                e0.record()
                for _ in range(iters):
                    fn()
                e1.record(); torch.cuda.synchronize()
                return e0.elapsed_time(e1) / iters
            for _ in range(iters):
                flush()
                e0.record(); fn(); e1.record(); torch.cuda.synchronize()
                tot += e0.elapsed_time(e1)
            return tot / iters

        def layer_case(spec, seed, dtype):
            """Packs one layer, returns (ms, eff flop, alg bytes, dense flop) of pconv_conv2d on fresh inputs."""
            L = make_layer(spec, seed)
            h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], dtype)
            tdt = torch.float32 if dtype == "f32" else torch.bfloat16
            x = torch.randn((spec.n, spec.c_in, spec.h, spec.w), device=dev).clamp_(min=0).to(tdt)
            b = torch.from_numpy(L["bias"]).to(dev)
            y = torch.empty((spec.n, spec.c_out, spec.h_out, spec.w_out), device=dev, dtype=tdt)
            code = P.F32 if dtype == "f32" else P.BF16
            ms = time_call(lambda: P.pconv_conv2d(h, x.data_ptr(), y.data_ptr(), b.data_ptr(), spec.n, spec.h, spec.w,
                                                  spec.stride, 1, P.NCHW, code, True, stream))
            nnz = nnz_of_layer(L)
            el = 4 if dtype == "f32" else 2
            flop = 2.0 * nnz * spec.n * spec.h_out * spec.w_out
            byts = el * (x.numel() + y.numel()) + el * nnz + 2.0 * int(L["conn"].sum())
            dense = 2.0 * 9 * spec.c_in * spec.c_out * spec.n * spec.h_out * spec.w_out
            h.free()
            return ms, flop, byts, dense

        other = {}
        spec2 = config_layers(2)[0]
        ms, flop, byts, _ = layer_case(spec2, base_seed(2), "f32")
        other["c2_256x256_56x56_batch1_fp32"] = dict(ms=round(ms, 4), eff_tflops=round(flop / ms / 1e9, 2),
                                                     bytes=byts, roof_frac=round(t_roof_s(flop, byts) * 1e3 / ms, 4))
        spec5 = config_layers(5)[0]
        ms, flop, byts, _ = layer_case(spec5, base_seed(5), "f32")
        other["c5_512x512_28x28_batch64_fp32_12pattern_geometric"] = dict(
            ms=round(ms, 4), eff_tflops=round(flop / ms / 1e9, 2), bytes=byts, roof_frac=round(t_roof_s(flop, byts) * 1e3 / ms, 4))
        c4_ms = c4_flop = c4_bytes = c4_dense = c4_roof = 0.0
        c4_layers = []
        for i, spec in enumerate(config_layers(4, batch=32)):
            ms, flop, byts, dense = layer_case(spec, base_seed(4) + i, "bf16")
            c4_ms += ms; c4_flop += flop; c4_bytes += byts; c4_dense += dense; c4_roof += t_roof_s(flop, byts) * 1e3
            c4_layers.append(round(ms, 4))
        other["c4_resnet50_3x3_16layers_batch32_bf16"] = dict(
            ms=round(c4_ms, 4), eff_tflops=round(c4_flop / c4_ms / 1e9, 2), bytes=c4_bytes,
            roof_frac=round(c4_roof / c4_ms, 4),            # against the fp32 vector / HBM roof, effective FLOPs
            kernel="conv_mfma_kernel (bf16 matrix cores, dense over masked weights)",
            mfma_frac_effective=round(c4_flop / c4_ms / 1e9 / PEAK_MFMA_BF16_TFLOPS, 4),
            mfma_frac_dense_equivalent=round(c4_dense / c4_ms / 1e9 / PEAK_MFMA_BF16_TFLOPS, 4),
            layer_ms=c4_layers)
        out["other_configs"] = other

        # the paper's pattern-count experiment (Tables 1-2) on the same stack: 4, 8 and 12 patterns from the
        # benchmark table, and a table of 8 masks drawn from the 56 four-tap masks that contain the centre
        if default_workload:
            sweep = {"8": round(ms_per_step, 4)}
            rng = np.random.default_rng(base_seed(3))
            cands = [m for m in range(512) if bin(m).count("1") == 4 and (m >> 4) & 1]
            rand8 = sorted(int(v) for v in rng.choice(cands, 8, replace=False))
            for key, kw in (("4", dict(num_patterns=4)), ("12", dict(num_patterns=12)), ("8_random_masks", dict(table=rand8))):
                ls = build_stack(**kw)
                sweep[key] = round(time_stack(ls, 5, 2)[0], 4)
                for ly in ls:
                    ly["h"].free()
            out["pattern_count_sweep_ms_per_step"] = sweep
            out["pattern_count_sweep_random_masks"] = ["0x%03x" % m for m in rand8]

            # cold-cache times of the two HBM-bound layers: a 512 MiB fill between launches evicts L2 and MALL
            junk = torch.empty(512 * 2**20 // 4, device=dev)
            cold = {}
            for i in (0, 1):
                ly, s = layers[i], layers[i]["spec"]
                cur = x0 if i == 0 else ybuf[0]
                if ly["fuse"]:
                    fn = lambda ly=ly, s=s, cur=cur, i=i: P.pconv_conv2d_pool2x2(
                        ly["h"], cur.data_ptr(), pbuf[i].data_ptr(), ly["bias"].data_ptr(), n, s.h, s.w, P.NCHW, P.F32, True, stream)
                else:
                    fn = lambda ly=ly, s=s, cur=cur, i=i: P.pconv_conv2d(
                        ly["h"], cur.data_ptr(), ybuf[i].data_ptr(), ly["bias"].data_ptr(), n, s.h, s.w, 1, 1, P.NCHW, P.F32, True, stream)
                cold[per_layer[i]["layer"]] = dict(warm_ms=per_layer[i]["ms"],
                                                   cold_ms=round(time_call(fn, iters=5, warm=1, flush=lambda: junk.fill_(1.0)), 4))
            del junk
            out["cold_cache_ms"] = cold

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
