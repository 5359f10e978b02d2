#!/usr/bin/env python3
"""Benchmark of the mixed-tenant multi-LoRA linear layer on one MI355X.

A "step" is one pass of the layer over one synthetic batch: forward for the
decode and prefill configurations, forward + backward for the training and
mixed configurations.  The headline line is the decode configuration
(256 tokens, 4096x4096, 32 adapters of rank 16, Zipf segment sizes); the other
bf16 configurations are reported in the same JSON line under "others".

Inputs are seeded synthetic tensors already resident in HBM before the timed
region.  The token->adapter map is built once, outside the timed region (a
serving engine builds it once per batch and reuses it for every layer).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--configs 1,2,3,4]
                  [--layout torch|math] [--launch graph|eager] [--no-cpu-baseline] [--no-multi-projection]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2516.6   # 256 CUs x 4096 flop/clk x 2.4 GHz, dense bf16


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--configs", default="1,2,3,4")
    ap.add_argument("--layout", default="torch", choices=["torch", "math"])
    ap.add_argument("--launch", default=None, choices=["graph", "eager"])
    ap.add_argument("--no-vendor-reference", action="store_true",
                    help="skip timing torch.mm (the vendor GEMM library) on the base product x W of each workload")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device copies: a kernel of known HBM traffic for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    ap.add_argument("--rotate", type=int, default=20, help="distinct weight sets cycled in the decode config")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--multi-projection-only", action="store_true",
                    help="time only the q/k/v multi-projection decode workload and print its line (for profiles)")
    ap.add_argument("--no-multi-projection", action="store_true",
                    help="skip the q/k/v multi-projection measurement of the decode configuration")
    ap.add_argument("--seed", type=int, default=0)
    return ap.parse_args()


def algorithmic_work(T, K, N, ranks, counts, bwd, out_bytes=2):
    """Algorithmic flops and minimum bytes of one step (padding, the two-term
    split of u and masked rows are not counted)."""
    ranks = np.asarray(ranks, dtype=np.float64)
    counts = np.asarray(counts, dtype=np.float64)
    tr = float(np.sum(ranks * counts))                 # sum_t T_t r_t
    present = counts > 0
    lora_w = float(np.sum(ranks[present])) * (K + N)   # elements of the adapters that are used
    fwd_flops = 2.0 * T * K * N + 2.0 * tr * (K + N)
    fwd_bytes = 2.0 * (K * N + T * K) + out_bytes * T * N + 2.0 * lora_w
    gemm_fwd = dict(flops=2.0 * T * K * N + 2.0 * tr * N,
                    bytes=2.0 * (K * N + T * K) + out_bytes * T * N + 2.0 * float(np.sum(ranks[present])) * N + 4.0 * tr)
    if not bwd:
        return dict(flops=fwd_flops, bytes=fwd_bytes, gemm=gemm_fwd, gemm_launches=1)
    bwd_flops = 2.0 * T * K * N + 4.0 * tr * (K + N)
    bwd_bytes = 2.0 * (K * N + T * N + T * K) + out_bytes * T * K + 2.0 * lora_w + 4.0 * lora_w
    gemm_bwd_flops = 2.0 * T * K * N + 2.0 * tr * K
    return dict(flops=fwd_flops + bwd_flops, bytes=fwd_bytes + bwd_bytes,
                gemm=dict(flops=(gemm_fwd["flops"] + gemm_bwd_flops) / 2.0, bytes=None), gemm_launches=2)


def measured_traffic(cfg, kernel_names):
    """HBM bytes per launch (fetch + write) of the named kernels, from the committed summary of the
    rocprofv3 --pmc runs (profiles/hbm_traffic.md); None when the summary has no such row.  Kernels
    that run once each per launch of the timed span (GEMM + finish) add up; variants of one kernel
    (forward / backward instantiations) are averaged over their launches."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.md")
    if not os.path.exists(path):
        return None
    total, found = 0.0, False
    for name in kernel_names:
        num = den = 0.0
        for line in open(path):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) >= 8 and cells[1] == str(cfg) and name in cells[2]:
                launches = float(cells[3])
                num += launches * (float(cells[5]) + float(cells[6]))
                den += launches
        if den:
            total += num / den
            found = True
    return total if found else None


def device_normal(shape, std, gen, torch):
    t = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    t.normal_(0.0, std, generator=gen)
    return t


def build_case(cfg, args, torch, api, wl):
    """Device tensors, descriptors and buffers of one configuration."""
    layout = api.MARLAAS_LAYOUT_TORCH if args.layout == "torch" else api.MARLAAS_LAYOUT_MATH
    sh, ranks, scales, ids = wl.config_ids(cfg, args.seed)
    T, K, N, n = sh["T"], sh["d_in"], sh["d_out"], sh["n"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1000 * args.seed + cfg)
    ctx = api.marlaas_create(0)
    ids_dev = torch.from_numpy(ids).cuda()
    segmap = api.marlaas_segmap_build(ctx, ids_dev, n)
    n_sets = args.rotate if cfg == 1 else 1
    sets = []
    for _ in range(n_sets):
        x = device_normal((T, K), 1.0, gen, torch)
        W = device_normal((N, K) if layout else (K, N), K ** -0.5, gen, torch)
        A = [device_normal((int(r), K) if layout else (K, int(r)), K ** -0.5, gen, torch) for r in ranks]
        B = [device_normal((N, int(r)) if layout else (int(r), N), float(r) ** -0.5, gen, torch) for r in ranks]
        desc = api.LoraDesc(x, W, A, B, ranks, scales, segmap, layout=layout, out_dtype=torch.bfloat16)
        sets.append(dict(x=x, W=W, A=A, B=B, desc=desc))
    case = dict(cfg=cfg, ctx=ctx, segmap=segmap, sets=sets, T=T, K=K, N=N, n=n, ranks=ranks, ids=ids,
                bwd=sh["bwd"], layout=layout, counts=np.bincount(ids, minlength=n))
    case["y"] = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    ws_bytes = api.marlaas_workspace_bytes(sets[0]["desc"], sh["bwd"])
    case["ws"] = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    api.marlaas_set_workspace(ctx, case["ws"])
    if sh["bwd"]:
        case["dY"] = device_normal((T, N), 1.0, gen, torch)
        case["dX"] = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
        case["u"] = torch.empty((T, api.marlaas_u_stride(sets[0]["desc"])), dtype=torch.float32, device="cuda")
        case["dA"] = [torch.empty(tuple(a.shape), dtype=torch.float32, device="cuda") for a in sets[0]["A"]]
        case["dB"] = [torch.empty(tuple(b.shape), dtype=torch.float32, device="cuda") for b in sets[0]["B"]]
    return case


def one_step(case, i, api):
    s = case["sets"][i % len(case["sets"])]
    if case["bwd"]:
        api.marlaas_lora_fwd(case["ctx"], s["desc"], case["y"], u_save=case["u"])
        api.marlaas_lora_bwd(case["ctx"], s["desc"], case["dY"], dX=case["dX"], dA=case["dA"], dB=case["dB"],
                             u_saved=case["u"])
    else:
        api.marlaas_lora_fwd(case["ctx"], s["desc"], case["y"])


def time_case(case, steps, warmup, launch, torch, api, profile=True):
    for i in range(warmup):
        one_step(case, i, api)
    torch.cuda.synchronize()
    graph = None
    if launch == "graph":
        # one HIP graph holding `steps` consecutive steps (each on its own weight set)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(steps):
                one_step(case, i, api)
        graph.replay()          # untimed replay: uploads the graph
        torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        graph.replay()
    else:
        for i in range(steps):
            one_step(case, i, api)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    if not profile:
        return wall_ms / steps, None
    # per-kernel durations: a second pass of the same steps with every launch bracketed by events
    api.marlaas_profile_enable(case["ctx"], True)
    for i in range(steps):
        one_step(case, i, api)
    torch.cuda.synchronize()
    kern = {}
    for name, kid in (("shrink", api.MARLAAS_KERNEL_SHRINK), ("gemm", api.MARLAAS_KERNEL_GEMM),
                      ("reduce", api.MARLAAS_KERNEL_REDUCE)):
        ms, cnt = api.marlaas_profile_read(case["ctx"], kid)
        kern[name] = dict(total_ms=ms, launches=cnt, avg_ms=(ms / cnt if cnt else None))
    api.marlaas_profile_enable(case["ctx"], False)
    return wall_ms / steps, kern


def vendor_reference(case, steps, warmup, launch, torch):
    """Context, not part of the product path: the base product alone (no adapters) through torch.mm,
    i.e. the vendor GEMM library, on the same operands and with the same launch mode.  For
    forward + backward workloads: x W and dY W^T."""
    sets = case["sets"]
    y = case["y"]
    tl = case["layout"] == 1           # torch layout: W[d_out, d_in]

    def step(i):
        s = sets[i % len(sets)]
        torch.mm(s["x"], s["W"].t() if tl else s["W"], out=y)
        if case["bwd"]:
            torch.mm(case["dY"], s["W"] if tl else s["W"].t(), out=case["dX"])
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    graph = None
    if launch == "graph":
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(steps):
                step(i)
        graph.replay()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        graph.replay()
    else:
        for i in range(steps):
            step(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def multi_projection_decode(case, args, steps, warmup, torch, api):
    """The decode batch against a block's q / k / v projections (d_out 4096, 1024, 1024: grouped-query
    attention of an 8B-class model), each with its own adapters of rank 16: one
    marlaas_lora_fwd_multi call per step against three marlaas_lora_fwd calls, HIP-graph replay over
    rotating weight sets like the headline.  Roofline as for the headline: algorithmic bytes of the
    step over the duration of the one GEMM + finish span."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77 + args.seed)
    T, K, n, ranks, layout = case["T"], case["K"], case["n"], case["ranks"], case["layout"]
    Ns = (4096, 1024, 1024)
    ctx, segmap = case["ctx"], case["segmap"]
    scales = [2.0] * n
    sets = []
    for s in case["sets"][:max(2, len(case["sets"]) // 2)]:
        projs = []
        for N in Ns:
            W = device_normal((N, K) if layout else (K, N), K ** -0.5, gen, torch)
            A = [device_normal((int(r), K) if layout else (K, int(r)), K ** -0.5, gen, torch) for r in ranks]
            B = [device_normal((N, int(r)) if layout else (int(r), N), float(r) ** -0.5, gen, torch) for r in ranks]
            projs.append(dict(W=W, A=A, B=B, desc=api.LoraDesc(s["x"], W, A, B, ranks, scales, segmap, layout=layout,
                                                              out_dtype=torch.bfloat16)))
        sets.append(projs)
    ys = [torch.empty((T, N), dtype=torch.bfloat16, device="cuda") for N in Ns]
    descs0 = [pr["desc"] for pr in sets[0]]
    ws = torch.empty(max(api.marlaas_workspace_bytes_multi(descs0), 256), dtype=torch.uint8, device="cuda")
    old_ws = case["ws"]
    api.marlaas_set_workspace(ctx, ws)

    def fused_step(i):
        api.marlaas_lora_fwd_multi(ctx, [pr["desc"] for pr in sets[i % len(sets)]], ys)

    def separate_step(i):
        for pr, y in zip(sets[i % len(sets)], ys):
            api.marlaas_lora_fwd(ctx, pr["desc"], y)

    out = {}
    for name, step in (("fused", fused_step), ("separate", separate_step)):
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(steps):
                step(i)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        out[name + "_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / steps
        del graph
    api.marlaas_profile_enable(ctx, True)
    for i in range(steps):
        fused_step(i)
    torch.cuda.synchronize()
    ms, cnt = api.marlaas_profile_read(ctx, api.MARLAAS_KERNEL_GEMM)
    api.marlaas_profile_enable(ctx, False)
    api.marlaas_set_workspace(ctx, old_ws)
    present = case["counts"] > 0
    nbytes = sum(2.0 * (K * N + 0.0) + 2.0 * T * N + 2.0 * float(np.sum(ranks[present])) * (K + N) for N in Ns) + 2.0 * T * K
    span_ms = ms / cnt if cnt else None
    out.update(workload="decode q/k/v: T=%d, %d -> %s, %d adapters r=16 per projection" % (T, K, list(Ns), n),
               gemm_launches_per_step=cnt / steps, tokens_per_s=T / (out["fused_ms_per_step"] * 1e-3),
               roofline=dict(bound="hbm", achieved=nbytes / (span_ms * 1e-3) / 1e9 if span_ms else None, peak=HBM_PEAK_GBS,
                             unit="GB/s", frac=nbytes / (span_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if span_ms else None,
                             traffic=None, kernel="gemm_skinny_kernel + splitk_finish_kernel (three projections, shrink fused)",
                             avg_kernel_ms=span_ms))
    return out


def cpu_baseline_decode(args, wl):
    """The fp64 oracle, as it stands, on the full decode configuration."""
    from oracle import lora_oracle
    w = wl.make_config(1, seed=args.seed, layout=wl.TORCH if args.layout == "torch" else wl.MATH)
    reps, t0 = 0, time.perf_counter()
    while True:
        lora_oracle.fwd(w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"], layout=w["layout"])
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or reps >= 200:
            break
    return dict(value=reps * w["T"] / dt, unit="tokens/s", cores=lora_oracle.num_threads(), kind="oracle",
                sample="all 256 tokens of the decode configuration, %d forward passes in %.1f s" % (reps, dt))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the layer is data parallel over tokens; "
              "no collective is part of it). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_08527_amd import api
    from paper_2605_08527_amd import workloads as wl
    api.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    cfgs = [int(c) for c in args.configs.split(",") if c]
    if args.multi_projection_only:
        steps = args.steps if args.steps is not None else 200
        warmup = args.warmup if args.warmup is not None else 40
        case = build_case(1, args, torch, api, wl)
        m = multi_projection_decode(case, args, steps, warmup, torch, api)
        print(json.dumps({
            "metric": "mixed-LoRA layer tokens/s at 32 adapters (with TFLOP/s and % of MFMA / HBM peak)",
            "value": m["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": m["fused_ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": m["workload"], "layout": args.layout, "launch": "graph", "out_dtype": "bf16",
                       "weight_sets_rotated": max(2, args.rotate // 2), "segmap": "prebuilt, outside the timed region"},
            "roofline": m["roofline"], "separate_calls_ms_per_step": m["separate_ms_per_step"]}))
        return
    results = {}
    for cfg in cfgs:
        if cfg not in (1, 2, 3, 4):
            raise SystemExit("--configs takes 1..4 (config 0 is a parity-only case)")
        steps = args.steps if args.steps is not None else {1: 200, 2: 20, 3: 5, 4: 30}[cfg]
        warmup = args.warmup if args.warmup is not None else {1: 40, 2: 5, 3: 2, 4: 5}[cfg]
        launch = args.launch or ("graph" if cfg == 1 else "eager")
        case = build_case(cfg, args, torch, api, wl)
        ms, kern = time_case(case, steps, warmup, launch, torch, api)
        extra = {}
        if not args.no_vendor_reference:
            extra["vendor_base_gemm_only_ms_per_step"] = vendor_reference(case, steps, warmup, launch, torch)
        if cfg == 1 and len(case["sets"]) > 1:
            # the same steps on one weight set only: everything stays in the memory-side cache
            hot = dict(case, sets=case["sets"][:1])
            extra["hot_cache_ms_per_step"] = time_case(hot, steps, warmup, launch, torch, api, profile=False)[0]
        if cfg == 1 and not args.no_multi_projection:
            extra["multi_projection"] = multi_projection_decode(case, args, steps, warmup, torch, api)
        if cfg == 4:
            # the timed steps reuse a prebuilt segment map; building it (three small kernels and a
            # read-back of the offsets) costs this much per batch
            ids_dev = torch.from_numpy(case["ids"]).cuda()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(10):
                m = api.marlaas_segmap_build(case["ctx"], ids_dev, case["n"])
                del m
            torch.cuda.synchronize()
            extra["segmap_build_ms"] = (time.perf_counter() - t0) * 1e3 / 10
            extra["ms_per_step_with_segmap_build"] = ms + extra["segmap_build_ms"]
        work = algorithmic_work(case["T"], case["K"], case["N"], case["ranks"], case["counts"], case["bwd"])
        g = kern["gemm"]
        if cfg == 1:
            # small batches: the split-K GEMM (which also computes the shrink) and its finish kernel are
            # timed as one span; without a separate shrink launch that span is the whole step
            fused = kern["shrink"]["launches"] == 0
            ach = (work["bytes"] if fused else work["gemm"]["bytes"]) / (g["avg_ms"] * 1e-3) / 1e9
            roof = dict(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                        traffic=measured_traffic(1, ["gemm_skinny_kernel", "splitk_finish_kernel"]),
                        kernel="gemm_skinny_kernel + splitk_finish_kernel" + (" (shrink fused)" if fused else ""),
                        avg_kernel_ms=g["avg_ms"])
        else:
            ach = work["gemm"]["flops"] / (g["avg_ms"] * 1e-3) / 1e12
            roof = dict(bound="mfma", achieved=ach, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=ach / MFMA_BF16_PEAK_TFLOPS, traffic=measured_traffic(cfg, ["gemm_bf16_kernel"]),
                        kernel="gemm_bf16_kernel",
                        avg_kernel_ms=g["avg_ms"])
        results[cfg] = dict(
            workload="config %d" % cfg, steps=steps, warmup=warmup, launch=launch, ms_per_step=ms,
            tokens_per_s=case["T"] / (ms * 1e-3), tflops=work["flops"] / (ms * 1e-3) / 1e12,
            step_gbs=work["bytes"] / (ms * 1e-3) / 1e9,
            frac_mfma_peak=work["flops"] / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            frac_hbm_peak=work["bytes"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            T=case["T"], d_in=case["K"], d_out=case["N"], n_adapters=case["n"],
            kernels={k: v for k, v in kern.items() if v["launches"]}, roofline=roof, **extra)
        del case
        torch.cuda.empty_cache()
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    head_cfg = 1 if 1 in results else cfgs[0]
    h = results[head_cfg]
    names = {1: "decode fwd: T=256, 4096x4096, 32 adapters r=16, Zipf(1.2) segments",
             2: "prefill fwd: T=40960, 4096->14336, 32 adapters r=16, ragged contiguous segments",
             3: "train fwd+bwd: T=262144, 14336->4096, 16 adapters r=32",
             4: "mixed fwd+bwd: T=16896 interleaved, 5120x5120, 64 adapters r in {8,16,32,64}"}
    line = {
        "metric": "mixed-LoRA layer tokens/s at 32 adapters (with TFLOP/s and % of MFMA / HBM peak)",
        "value": h["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": h["steps"], "warmup": h["warmup"],
        "ms_per_step": h["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": names[head_cfg], "layout": args.layout, "launch": h["launch"],
                   "out_dtype": "bf16", "weight_sets_rotated": args.rotate if head_cfg == 1 else 1,
                   "segmap": "prebuilt, outside the timed region"},
        "tflops": h["tflops"], "roofline": h["roofline"],
    }
    if not args.no_cpu_baseline and head_cfg == 1:
        line["cpu_baseline"] = cpu_baseline_decode(args, wl)
    for k in ("vendor_base_gemm_only_ms_per_step", "hot_cache_ms_per_step", "multi_projection"):
        if k in h:
            line[k] = h[k]
    line["others"] = [dict(results[c], workload=names[c]) for c in cfgs if c != head_cfg]
    line["kernels"] = h["kernels"]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
