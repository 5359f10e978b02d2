#!/usr/bin/env python3
"""Benchmark of the mixed-tenant multi-LoRA linear layer on one MI355X.

A "step" is one pass of the layer over one synthetic batch: forward for the
decode and prefill configurations, forward + backward for the training and
mixed configurations.  The headline line is the decode configuration
(256 tokens, 4096x4096, 32 adapters of rank 16, Zipf segment sizes); the other
bf16 configurations are reported in the same JSON line under "others".

Inputs are seeded synthetic tensors already resident in HBM before the timed
region; adapters are registered in an adapter table and the token->adapter map
is built once, both outside the timed region (a serving engine does both once
per batch / per adapter version and reuses them for every layer).  Every weight
set the timed steps rotate over is prepared before anything is captured or timed.

Timing: W untimed warm-up steps, then exactly K steps between two
synchronisations (ms_per_step, value); after that at least 50 further
iterations, each bracketed by a pair of HIP events on the launch stream, give
the median and the minimum.  The decode configuration runs as one HIP graph of K
steps (one replay = K steps over rotating weight sets, so that every step streams
its weight from HBM); the large configurations launch eagerly.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--configs 1,2,3,4]
                  [--layout torch|math] [--launch graph|eager] [--no-cpu-baseline] [--no-multi-projection]
"""
import argparse
import json
import os
import select
import statistics
import subprocess
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2516.6   # 256 CUs x 4096 flop/clk x 2.4 GHz, dense bf16
# Second denominator for the matrix-core bound: what a loop of nothing but bf16 MFMAs (the GEMM's
# own instruction shape, 256 workgroups, N(0,1) operands) sustained on this machine under its power
# limit; the all-zero-operand figure is 2460.
MFMA_MEASURED_CEILING_TFLOPS = 1750.0
METRIC = "mixed-LoRA layer TFLOP/s + tokens/s at 32 adapters; % of MFMA / HBM peak"
MIN_EVENT_ITERS = 50


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
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
    ap.add_argument("--no-clocks", action="store_true", help="do not sample rocm-smi while the headline runs")
    ap.add_argument("--multi-projection-only", action="store_true",
                    help="time only the q/k/v multi-projection decode workload and print its line (for profiles)")
    ap.add_argument("--no-multi-projection", action="store_true",
                    help="skip the q/k/v multi-projection measurement of the decode configuration")
    ap.add_argument("--no-event-stats", action="store_true", help="skip the extra event-timed iterations (for profiles)")
    ap.add_argument("--no-packed-weight", action="store_true",
                    help="decode configuration without the packed copy of the weight (the kernels then stage W through LDS)")
    ap.add_argument("--stack-layers", type=int, default=8,
                    help="layers of the decode layer-stack measurement of the decode configuration (0: skip)")
    ap.add_argument("--no-single-task", action="store_true",
                    help="skip the single-task update measurement of the training configuration")
    ap.add_argument("--layer-stack-only", action="store_true",
                    help="time only the decode layer stack and print its line (for profiles)")
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
    rocprofv3 --pmc runs (profiles/hbm_traffic.md); None when the summary has no such row.  Not
    measured by this run.  Kernels that run once each per launch of the timed span add up; variants
    of one kernel (forward / backward instantiations) are averaged over their launches."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.md")
    if not os.path.exists(path):
        return None
    total, found = 0.0, False
    for name in kernel_names:
        num = den = 0.0
        for line in open(path):
            cells = [c.strip() for c in line.split("|")]
            try:
                if len(cells) >= 8 and cells[1] == str(cfg) and name in cells[2]:
                    launches = float(cells[3])
                    num += launches * (float(cells[5]) + float(cells[6]))
                    den += launches
            except ValueError:
                continue
        if den:
            total += num / den
            found = True
    return total if found else None


def device_normal(shape, std, gen, torch):
    t = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    t.normal_(0.0, std, generator=gen)
    return t


def build_case(cfg, args, torch, api, wl):
    """Device tensors, adapter tables, descriptors and buffers of one configuration: everything a
    timed step touches exists before the first step."""
    layout = api.MARLAAS_LAYOUT_TORCH if args.layout == "torch" else api.MARLAAS_LAYOUT_MATH
    sh, ranks, scales, ids = wl.config_ids(cfg, args.seed)
    T, K, N, n = sh["T"], sh["d_in"], sh["d_out"], sh["n"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1000 * args.seed + cfg)
    ctx = api.marlaas_create(0)
    ids_dev = torch.from_numpy(ids).cuda()
    segmap = api.marlaas_segmap_build(ctx, ids_dev, n)
    n_sets = args.rotate if cfg == 1 else 1
    case = dict(cfg=cfg, ctx=ctx, segmap=segmap, T=T, K=K, N=N, n=n, ranks=ranks, ids=ids,
                bwd=sh["bwd"], layout=layout, counts=np.bincount(ids, minlength=n))
    if sh["bwd"]:
        shapeA = [((int(r), K) if layout else (K, int(r))) for r in ranks]
        shapeB = [((N, int(r)) if layout else (int(r), N)) for r in ranks]
        case["dA"] = [torch.empty(s, dtype=torch.float32, device="cuda") for s in shapeA]
        case["dB"] = [torch.empty(s, dtype=torch.float32, device="cuda") for s in shapeB]
    sets = []
    for _ in range(n_sets):
        x = device_normal((T, K), 1.0, gen, torch)
        W = device_normal((N, K) if layout else (K, N), K ** -0.5, gen, torch)
        A = [device_normal((int(r), K) if layout else (K, int(r)), K ** -0.5, gen, torch) for r in ranks]
        B = [device_normal((N, int(r)) if layout else (int(r), N), float(r) ** -0.5, gen, torch) for r in ranks]
        table = api.marlaas_adapter_table_create(ctx, n, 1, int(max(ranks)))
        for t in range(n):
            api.marlaas_adapter_table_update(ctx, table, 0, t, A[t], B[t], int(ranks[t]), float(scales[t]),
                                             case["dA"][t] if sh["bwd"] else None, case["dB"][t] if sh["bwd"] else None)
        # small batches read a packed copy of the frozen weight, written once per weight (outside the timed region)
        Wp = api.marlaas_pack_weight(ctx, W, layout, 0) if (cfg == 1 and not args.no_packed_weight) else None
        # large batches whose contraction runs along W's strided dimension read a transposed copy kept with
        # the frozen weight (written once, outside the timed region)
        Wt = api.marlaas_transpose_weight(ctx, W, layout) if (cfg != 1 and (sh["bwd"] if layout else True)) else None
        desc = api.LoraDesc(x, W, None, None, None, None, segmap, layout=layout, out_dtype=torch.bfloat16, table=table,
                            W_packed_fwd=Wp, W_t=Wt)
        sets.append(dict(x=x, W=W, A=A, B=B, table=table, desc=desc, Wp=Wp, Wt=Wt))
    case["sets"] = sets
    case["y"] = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    ws_bytes = api.marlaas_workspace_bytes(sets[0]["desc"], sh["bwd"])
    case["ws"] = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
    api.marlaas_set_workspace(ctx, case["ws"])
    if sh["bwd"]:
        case["dY"] = device_normal((T, N), 1.0, gen, torch)
        case["dX"] = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
        case["u"] = torch.empty((T, api.marlaas_u_stride(sets[0]["desc"])), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    return case


def one_step(case, i, api):
    s = case["sets"][i % len(case["sets"])]
    if case["bwd"]:
        api.marlaas_lora_fwd(case["ctx"], s["desc"], case["y"], u_save=case["u"])
        api.marlaas_lora_bwd(case["ctx"], s["desc"], case["dY"], dX=case["dX"], dA=api.MARLAAS_GRADS_IN_TABLE,
                             dB=api.MARLAAS_GRADS_IN_TABLE, u_saved=case["u"])
    else:
        api.marlaas_lora_fwd(case["ctx"], s["desc"], case["y"])


def time_steps(step, steps, warmup, launch, torch, event_stats=True, during=None):
    """The timing protocol: `warmup` untimed steps, exactly `steps` steps between two
    synchronisations, then >= 50 further event-timed iterations (graph: one iteration = one replay
    of the `steps` captured steps; eager: one step).  Returns a dict in ms per step."""
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    graph = None
    if launch == "graph":
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(steps):
                step(i)
        graph.replay()          # untimed replay: uploads the graph
        torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        graph.replay()
    else:
        for i in range(steps):
            step(i)
    torch.cuda.synchronize()
    out = dict(ms_per_step=(time.perf_counter() - t0) * 1e3 / steps)
    if not event_stats:
        return out
    iters = MIN_EVENT_ITERS if graph is not None else max(MIN_EVENT_ITERS, steps)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    side = during() if during is not None else None      # e.g. a clock sampler running beside the loop
    for it, (b, e) in enumerate(pairs):
        b.record()
        if graph is not None:
            graph.replay()
        else:
            step(it)
        e.record()
    torch.cuda.synchronize()
    per = [b.elapsed_time(e) / (steps if graph is not None else 1) for b, e in pairs]
    out.update(event_iterations=iters, event_median_ms=statistics.median(per), event_min_ms=min(per),
               event_unit="one replay of the captured steps / steps" if graph is not None else "one step")
    if side is not None:
        # keep the same work running until the sampler has returned, then collect what it saw
        t_end = time.perf_counter() + 20.0
        while side.poll() is None and time.perf_counter() < t_end:
            if graph is not None:
                graph.replay()
            else:
                step(0)
            torch.cuda.synchronize()
        out["clocks"] = side.result()
    return out


# The clock sampler is a helper process started BEFORE this process touches the GPU (a process that
# has initialised the GPU must not exec another program on these machines); it runs rocm-smi each
# time it is sent a line and answers with one line of JSON.
_SAMPLER_CODE = r"""
import json, subprocess, sys
for _ in sys.stdin:
    keep = {}
    try:
        out = subprocess.run(["rocm-smi", "--showclocks", "--json"], stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, timeout=30).stdout
        card = next(iter(json.loads(out.decode()).values()))
        for k, v in card.items():
            kl = k.lower()
            if "sclk" in kl or "mclk" in kl or "fclk" in kl:
                keep[k] = v
    except Exception:
        pass
    sys.stdout.write(json.dumps(keep) + "\n")
    sys.stdout.flush()
"""
_sampler_proc = None


def start_clock_helper():
    global _sampler_proc
    try:
        _sampler_proc = subprocess.Popen([sys.executable, "-c", _SAMPLER_CODE], stdin=subprocess.PIPE, stdout=subprocess.PIPE,
                                         stderr=subprocess.DEVNULL)
    except OSError:
        _sampler_proc = None


class ClockSampler:
    """rocm-smi (through the helper process) while the timed loop runs: the engine and memory clocks under this load."""

    def __init__(self):
        self.asked = False
        try:
            if _sampler_proc is not None and _sampler_proc.poll() is None:
                _sampler_proc.stdin.write(b"go\n")
                _sampler_proc.stdin.flush()
                self.asked = True
        except OSError:
            pass

    def poll(self):
        """None while the helper has not answered yet (the caller keeps the load running meanwhile)."""
        if not self.asked:
            return 0
        try:
            ready, _, _ = select.select([_sampler_proc.stdout], [], [], 0)
            return 0 if ready or _sampler_proc.poll() is not None else None
        except (OSError, ValueError):
            return 0

    def result(self):
        if not self.asked:
            return None
        try:
            return json.loads(_sampler_proc.stdout.readline().decode()) or None
        except Exception:
            return None


def kernel_spans(case, steps, torch, api):
    """Per-kernel durations: a pass of the same steps, eager, with every launch of the library
    bracketed by HIP events on the launch stream."""
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
    return kern


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
    # (the vendor library may set itself up on the first call of a shape: at least one eager call before a capture)
    return time_steps(step, steps, max(warmup, 1), launch, torch, event_stats=False)["ms_per_step"]


def multi_projection_decode(case, args, steps, warmup, torch, api):
    """The decode batch against a block's q / k / v projections (d_out 4096, 1024, 1024: grouped-query
    attention of an 8B-class model), each with its own adapters of rank 16 registered in one table of
    three projections: one marlaas_lora_fwd_multi call per step against three marlaas_lora_fwd calls,
    HIP-graph replay over rotating weight sets like the headline.  Roofline as for the headline:
    algorithmic bytes of the step over the event-timed duration of a step of the replayed graph."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77 + args.seed)
    T, K, n, ranks, layout = case["T"], case["K"], case["n"], case["ranks"], case["layout"]
    Ns = (4096, 1024, 1024)
    ctx, segmap = case["ctx"], case["segmap"]
    sets = []
    for s in case["sets"][:max(2, len(case["sets"]) // 2)]:
        table = api.marlaas_adapter_table_create(ctx, n, len(Ns), int(max(ranks)))
        projs = []
        for p, N in enumerate(Ns):
            W = device_normal((N, K) if layout else (K, N), K ** -0.5, gen, torch)
            A = [device_normal((int(r), K) if layout else (K, int(r)), K ** -0.5, gen, torch) for r in ranks]
            B = [device_normal((N, int(r)) if layout else (int(r), N), float(r) ** -0.5, gen, torch) for r in ranks]
            for t in range(n):
                api.marlaas_adapter_table_update(ctx, table, p, t, A[t], B[t], int(ranks[t]), 2.0)
            Wp = api.marlaas_pack_weight(ctx, W, layout, 0) if not args.no_packed_weight else None
            projs.append(dict(W=W, A=A, B=B, Wp=Wp,
                              desc=api.LoraDesc(s["x"], W, None, None, None, None, segmap, layout=layout,
                                                out_dtype=torch.bfloat16, table=table, proj=p, W_packed_fwd=Wp)))
        sets.append(projs)
    ys = [torch.empty((T, N), dtype=torch.bfloat16, device="cuda") for N in Ns]
    descs0 = [pr["desc"] for pr in sets[0]]
    ws = torch.empty(max(api.marlaas_workspace_bytes_multi(descs0), 256), dtype=torch.uint8, device="cuda")
    old_ws = case["ws"]
    api.marlaas_set_workspace(ctx, ws)
    torch.cuda.synchronize()

    def fused_step(i):
        api.marlaas_lora_fwd_multi(ctx, [pr["desc"] for pr in sets[i % len(sets)]], ys)

    def separate_step(i):
        for pr, y in zip(sets[i % len(sets)], ys):
            api.marlaas_lora_fwd(ctx, pr["desc"], y)

    out = {}
    fused = time_steps(fused_step, steps, warmup, "graph", torch, event_stats=not args.no_event_stats)
    out["fused_ms_per_step"] = fused["ms_per_step"]
    out["fused_event_median_ms"] = fused.get("event_median_ms")
    out["separate_ms_per_step"] = time_steps(separate_step, steps, warmup, "graph", torch, event_stats=False)["ms_per_step"]
    api.marlaas_profile_enable(ctx, True)
    for i in range(steps):
        fused_step(i)
    torch.cuda.synchronize()
    ms, cnt = api.marlaas_profile_read(ctx, api.MARLAAS_KERNEL_GEMM)
    api.marlaas_profile_enable(ctx, False)
    api.marlaas_set_workspace(ctx, old_ws)
    present = case["counts"] > 0
    nbytes = sum(2.0 * (K * N + 0.0) + 2.0 * T * N + 2.0 * float(np.sum(ranks[present])) * (K + N) for N in Ns) + 2.0 * T * K
    span_ms = fused.get("event_median_ms") or fused["ms_per_step"]
    out.update(workload="decode q/k/v: T=%d, %d -> %s, %d adapters r=16 per projection" % (T, K, list(Ns), n),
               gemm_launches_per_step=cnt / steps, tokens_per_s=T / (out["fused_ms_per_step"] * 1e-3),
               roofline=dict(bound="hbm", achieved=nbytes / (span_ms * 1e-3) / 1e9, peak=HBM_PEAK_GBS,
                             unit="GB/s", frac=nbytes / (span_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             traffic=None, kernel="small-batch GEMM kernels of one fused three-projection call",
                             avg_kernel_ms=span_ms, eager_event_span_ms=(ms / cnt if cnt else None)))
    return out


def single_task_update(args, steps, warmup, torch, api):
    """The training engine's step for one task (the paper trains one task per update): forward,
    then the backward with the AdamW update of the task's adapter attached (marlaas_lora_bwd_adamw),
    on one adapter's share of the training configuration (16 384 tokens, 14336 -> 4096, rank 32),
    against forward + plain backward (gradients written to fp32 buffers, no optimizer)."""
    T, K, N, r = 16384, 14336, 4096, 32
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4242 + args.seed)
    ctx = api.marlaas_create(0)
    ids = torch.zeros(T, dtype=torch.int32, device="cuda")
    segmap = api.marlaas_segmap_build(ctx, ids, 1)
    x = device_normal((T, K), 1.0, gen, torch)
    W = device_normal((N, K), K ** -0.5, gen, torch)
    A = device_normal((r, K), K ** -0.5, gen, torch)
    B = device_normal((N, r), r ** -0.5, gen, torch)
    dY = device_normal((T, N), 1.0, gen, torch)
    gA, gB = torch.empty((r, K), dtype=torch.float32, device="cuda"), torch.empty((N, r), dtype=torch.float32, device="cuda")
    table = api.marlaas_adapter_table_create(ctx, 1, 1, r)
    api.marlaas_adapter_table_update(ctx, table, 0, 0, A, B, r, 2.0, gA, gB)
    Wt = api.marlaas_transpose_weight(ctx, W, 1)
    desc = api.LoraDesc(x, W, None, None, None, None, segmap, layout=1, out_dtype=torch.bfloat16, table=table, W_t=Wt)
    ws = torch.empty(max(api.marlaas_workspace_bytes(desc, True), 256), dtype=torch.uint8, device="cuda")
    api.marlaas_set_workspace(ctx, ws)
    y = torch.empty((T, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
    u = torch.empty((T, api.marlaas_u_stride(desc)), dtype=torch.float32, device="cuda")
    f32 = lambda t: t.float().clone()
    state = [dict(master_A=f32(A), master_B=f32(B), m_A=torch.zeros_like(gA), v_A=torch.zeros_like(gA),
                  m_B=torch.zeros_like(gB), v_B=torch.zeros_like(gB), A_next=torch.empty_like(A), B_next=torch.empty_like(B))]
    hp = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=1)
    torch.cuda.synchronize()

    def fused(i):
        api.marlaas_lora_fwd(ctx, desc, y, u_save=u)
        api.marlaas_lora_bwd_adamw(ctx, desc, dY, state, dict(hp, step=i + 1), dX=dX, u_saved=u)

    def plain(i):
        api.marlaas_lora_fwd(ctx, desc, y, u_save=u)
        api.marlaas_lora_bwd(ctx, desc, dY, dX=dX, dA=api.MARLAAS_GRADS_IN_TABLE, dB=api.MARLAAS_GRADS_IN_TABLE, u_saved=u)

    n = max(3, min(steps, 10))
    # alternated, best of two each: the engine clock drifts by a few per cent over a run
    t_plain = t_fused = float("inf")
    for _ in range(2):
        t_plain = min(t_plain, time_steps(plain, n, max(1, min(warmup, 2)), "eager", torch, event_stats=False)["ms_per_step"])
        t_fused = min(t_fused, time_steps(fused, n, max(1, min(warmup, 2)), "eager", torch, event_stats=False)["ms_per_step"])
    flops = 2 * (2.0 * T * K * N) + 2.0 * T * r * (K + N) * 3
    return dict(workload="single-task update: T=%d, %d -> %d, 1 adapter r=%d, forward + backward with AdamW attached" % (T, K, N, r),
                ms_per_update=t_fused, ms_forward_backward_without_optimizer=t_plain,
                tokens_per_s=T / (t_fused * 1e-3), tflops=flops / (t_fused * 1e-3) / 1e12,
                params_finite=bool(torch.isfinite(state[0]["master_A"]).all().item() and torch.isfinite(state[0]["master_B"]).all().item()))


def layer_stack_decode(args, torch, api, wl):
    """One decode token step through a stack of layers under one HIP graph (harness/layer_stack.py):
    per layer q/k/v in one call, o, gate/up in one call, down; 8B-class shapes (4096, kv 1024, ffn
    14336), the decode configuration's batch and token -> adapter map, every projection with its own
    packed weight and rank-16 adapters.  The layers' weights (3.5 GB at 8 layers) exceed every cache,
    so each replay streams them from HBM.  Reported: event-timed replays (median, min), the step's
    algorithmic bytes over the median against the HBM peak."""
    from harness.layer_stack import DecodeStack
    sh, ranks, scales, ids = wl.config_ids(1, args.seed)
    T, d, n = sh["T"], sh["d_in"], sh["n"]
    d_kv, d_ff, L = 1024, 14336, args.stack_layers
    ctx = api.marlaas_create(0)
    stack = DecodeStack(api, torch, ctx, torch.from_numpy(ids).cuda(), T, d, d_kv, d_ff, L, ranks, scales,
                        seed=args.seed, packed=not args.no_packed_weight)
    graph = stack.capture()
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    reps = 30
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    t0 = time.perf_counter()
    for b, e in ev:
        b.record()
        graph.replay()
        e.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / reps
    times = sorted(b.elapsed_time(e) for b, e in ev)
    med, mn = times[len(times) // 2], times[0]
    finite = bool(torch.isfinite(stack.out.float()).all().item())
    nbytes = stack.algorithmic_bytes(np.bincount(ids[ids >= 0], minlength=n) > 0)
    return dict(workload="decode step through %d layers (q/k/v, o, gate/up, down; d=%d, kv=%d, ffn=%d), T=%d, "
                         "%d adapters r=16 per projection, one HIP graph" % (L, d, d_kv, d_ff, T, n),
                layers=L, library_calls_per_step=4 * L, glue_kernels_per_step=4 * L,
                ms_per_step_median=med, ms_per_step_min=mn, ms_per_step_wall=wall_ms, ms_per_layer=med / L,
                tokens_per_s=T / (med * 1e-3), replays_timed=reps, outputs_finite=finite,
                weight_bytes=stack.weight_bytes(),
                roofline=dict(bound="hbm", achieved=nbytes / (med * 1e-3) / 1e9, peak=HBM_PEAK_GBS, unit="GB/s",
                              frac=nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, traffic=None,
                              algorithmic_bytes=nbytes, span="event-timed median of one replay of the captured step"))


def cpu_info():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return None


def cpu_baseline(cfg, args, wl):
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample of configuration
    `cfg`: the whole decode batch for configuration 1; for the large ones a seeded subset of token
    rows against the full-size weights and adapters (rows are independent, so tokens/s carries over;
    each call also widens W to fp64 once, which is counted)."""
    from oracle import lora_oracle
    layout = wl.TORCH if args.layout == "torch" else wl.MATH
    if cfg == 1:
        w = wl.make_config(1, seed=args.seed, layout=layout)
        reps, t0 = 0, time.perf_counter()
        while True:
            lora_oracle.fwd(w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"], layout=w["layout"])
            reps += 1
            dt = time.perf_counter() - t0
            if dt >= 10.0 or reps >= 200:
                break
        return dict(value=reps * w["T"] / dt, unit="tokens/s", cores=lora_oracle.num_threads(), kind="oracle", cpu=cpu_info(),
                    sample="all 256 tokens of the decode configuration, %d forward passes in %.1f s" % (reps, dt))
    sh, ranks, scales, ids = wl.config_ids(cfg, args.seed)
    rows = {2: 2048, 3: 1024, 4: 2048}[cfg]
    rng = np.random.default_rng(args.seed + 10 * cfg)
    sub = ids[np.sort(rng.choice(sh["T"], size=rows, replace=False))]
    w = wl.make_layer(args.seed, rows, sh["d_in"], sh["d_out"], ranks, scales, sub, dtype="bf16", layout=layout,
                      want_dY=sh["bwd"])
    a = (w["x"], w["W"], w["A"], w["B"], w["ranks"], w["scales"], w["ids"])
    t0 = time.perf_counter()
    lora_oracle.fwd(*a, layout=layout)
    if sh["bwd"]:
        lora_oracle.bwd(*a, w["dY"], layout=layout)
    dt = time.perf_counter() - t0
    return dict(value=rows / dt, unit="tokens/s", cores=lora_oracle.num_threads(), kind="oracle", cpu=cpu_info(),
                sample="%d token rows with the adapter labels of a seeded subset of the batch, full-size weights: "
                       "forward%s in %.1f s" % (rows, " + backward (dX, dA, dB)" if sh["bwd"] else "", dt))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the layer is data parallel over tokens; "
              "no collective is part of it). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if not args.no_clocks:
        start_clock_helper()       # before anything here touches the GPU
    import torch
    from paper_2605_08527_amd import api
    from harness import workloads as wl
    api.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    cfgs = [int(c) for c in args.configs.split(",") if c]
    steps, warmup = max(1, args.steps), max(0, args.warmup)
    if args.multi_projection_only:
        case = build_case(1, args, torch, api, wl)
        m = multi_projection_decode(case, args, steps, warmup, torch, api)
        print(json.dumps({
            "metric": METRIC,
            "value": m["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": m["fused_ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": m["workload"], "layout": args.layout, "launch": "graph", "out_dtype": "bf16",
                       "weight_sets_rotated": max(2, args.rotate // 2), "segmap": "prebuilt, outside the timed region"},
            "roofline": m["roofline"], "separate_calls_ms_per_step": m["separate_ms_per_step"]}))
        return
    if args.layer_stack_only:
        m = layer_stack_decode(args, torch, api, wl)
        print(json.dumps({
            "metric": METRIC, "value": m["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": m["replays_timed"],
            "warmup": 3, "ms_per_step": m["ms_per_step_median"], "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": m["workload"], "layout": "torch", "launch": "graph", "out_dtype": "bf16"},
            "roofline": m["roofline"], "layer_stack": m}))
        return
    results = {}
    for cfg in cfgs:
        if cfg not in (1, 2, 3, 4):
            raise SystemExit("--configs takes 1..4 (config 0 is a parity-only case)")
        launch = args.launch or ("graph" if cfg == 1 else "eager")
        case = build_case(cfg, args, torch, api, wl)
        sampler = (lambda: ClockSampler()) if (cfg == cfgs[0] and not args.no_clocks) else None
        tm = time_steps(lambda i: one_step(case, i, api), steps, warmup, launch, torch,
                        event_stats=not args.no_event_stats, during=sampler)
        ms = tm["ms_per_step"]
        kern = kernel_spans(case, steps, torch, api)
        extra = {k: v for k, v in tm.items() if k != "ms_per_step"}
        try:
            if not args.no_vendor_reference:
                extra["vendor_base_gemm_only_ms_per_step"] = vendor_reference(case, steps, warmup, launch, torch)
            if cfg == 1 and len(case["sets"]) > 1:
                # the same steps on one weight set only: everything stays in the memory-side cache
                hot = dict(case, sets=case["sets"][:1])
                extra["hot_cache_ms_per_step"] = time_steps(lambda i: one_step(hot, i, api), steps, warmup, launch, torch,
                                                            event_stats=False)["ms_per_step"]
            if cfg == 1 and not args.no_multi_projection:
                extra["multi_projection"] = multi_projection_decode(case, args, steps, warmup, torch, api)
            if cfg == 1 and args.stack_layers > 0:
                extra["layer_stack"] = layer_stack_decode(args, torch, api, wl)
            if cfg == 3 and not args.no_single_task:
                extra["single_task_update"] = single_task_update(args, steps, warmup, torch, api)
            if cfg == 4:
                # the timed steps reuse a prebuilt segment map; regrouping a batch into an existing map
                # object (five small kernels, a read-back of the offsets and one wait) costs this much
                ids_dev = torch.from_numpy(case["ids"]).cuda()
                m = api.marlaas_segmap_create(case["ctx"], case["T"], case["n"])
                api.marlaas_segmap_update(case["ctx"], m, ids_dev, case["n"])
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(10):
                    api.marlaas_segmap_update(case["ctx"], m, ids_dev, case["n"])
                torch.cuda.synchronize()
                extra["segmap_update_ms"] = (time.perf_counter() - t0) * 1e3 / 10
                extra["ms_per_step_with_segmap_update"] = ms + extra["segmap_update_ms"]
            if not args.no_cpu_baseline:
                extra["cpu_baseline"] = cpu_baseline(cfg, args, wl)
        except Exception as e:       # an extra must never cost the line its timed numbers
            extra["extras_error"] = "%s: %s" % (type(e).__name__, e)
        work = algorithmic_work(case["T"], case["K"], case["N"], case["ranks"], case["counts"], case["bwd"])
        g = kern["gemm"]
        src = "profiles/hbm_traffic.md (rocprofv3 --pmc runs of this command; not measured by this run)"
        if cfg == 1:
            # small batches: the step is the small-batch GEMM launches (which also compute the shrink) and
            # nothing else, so the kernel span of a step is the step itself, in the mode it is timed in:
            # the event-bracketed replay of the captured steps
            fused = kern["shrink"]["launches"] == 0
            span_ms = tm.get("event_median_ms", ms) if fused else g["avg_ms"]
            ach = (work["bytes"] if fused else work["gemm"]["bytes"]) / (span_ms * 1e-3) / 1e9
            roof = dict(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                        traffic=measured_traffic(1, ["gemm_skinny_kernel", "splitk_finish_kernel", "gemm_decode_kernel<true, 0>",
                                                         "gemm_decode_kernel<true, 1>"]),
                        traffic_source=src,
                        kernel="small-batch GEMM launches of the step" + (" (shrink fused)" if fused else ""),
                        avg_kernel_ms=span_ms,
                        span=("event-timed median of one step inside the replayed graph" if "event_median_ms" in tm and launch == "graph"
                              else "event-timed per step"),
                        eager_event_span_ms=g["avg_ms"])
        else:
            ach = work["gemm"]["flops"] / (g["avg_ms"] * 1e-3) / 1e12
            roof = dict(bound="mfma", achieved=ach, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=ach / MFMA_BF16_PEAK_TFLOPS, traffic=measured_traffic(cfg, ["gemm_bf16_kernel"]),
                        traffic_source=src, kernel="gemm_bf16_kernel", avg_kernel_ms=g["avg_ms"],
                        measured_mfma_ceiling=MFMA_MEASURED_CEILING_TFLOPS,
                        frac_of_measured_ceiling=ach / MFMA_MEASURED_CEILING_TFLOPS)
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
        "metric": METRIC,
        "value": h["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": h["steps"], "warmup": h["warmup"],
        "ms_per_step": h["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": names[head_cfg], "layout": args.layout, "launch": h["launch"],
                   "out_dtype": "bf16", "weight_sets_rotated": args.rotate if head_cfg == 1 else 1,
                   "adapters": "registered in an adapter table, outside the timed region",
                   "weight": ("row-major" if (args.no_packed_weight or head_cfg != 1) else
                              "frozen W also held as a packed copy (marlaas_pack_weight, once, outside the timed region)"),
                   "segmap": "prebuilt, outside the timed region"},
        "tflops": h["tflops"], "roofline": h["roofline"],
    }
    for k in ("cpu_baseline", "event_iterations", "event_median_ms", "event_min_ms", "event_unit", "clocks",
              "vendor_base_gemm_only_ms_per_step", "hot_cache_ms_per_step", "multi_projection", "layer_stack", "single_task_update",
              "segmap_update_ms", "ms_per_step_with_segmap_update", "extras_error"):
        if k in h:
            line[k] = h[k]
    line["others"] = [dict(results[c], workload=names[c]) for c in cfgs if c != head_cfg]
    line["kernels"] = h["kernels"]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
