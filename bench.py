#!/usr/bin/env python3
"""Benchmark of the VCAS sampled linear-layer backward on one MI355X.

One "step" is one pass of the whole hot path (row norms -> keep probabilities
-> Philox masks -> compaction -> sampled dX and dW) over every linear layer of
the BERT-large-shaped stack (144 layers, B=32, L=512, bf16: the largest of the
configurations by kept work), each layer with its own synthetic G, X, W
resident in HBM.  The data halves run in the order a backward pass imposes:
down, up, out-projection one behind the other, then V, K and Q, whose upstream
gradients do not depend on each other, together.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload bert_large]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "sampled linear-BP ms & effective TFLOP/s vs dense BP (bf16), % of roofline"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3


class Layer:
    """Device-resident tensors and scratch of one linear layer."""

    def __init__(self, spec, vb, to_device, make_layer, cache=None, arrays=None):
        import torch
        key = (spec.N, spec.T, spec.K_in, spec.K_out, spec.dtype)
        if arrays is not None:
            G, X, W = arrays
        elif cache is not None and key in cache:
            G, X, W = cache[key]
        else:
            G, X, W = make_layer(spec)
            if cache is not None:
                cache[key] = (G, X, W)
        self.spec = spec
        self.shape = vb.shape_of(spec.N, spec.T, spec.K_in, spec.K_out, spec.dtype)
        self.G, self.X, self.W = (to_device(a, spec.dtype) for a in (G, X, W))
        self.plan = vb.Plan.allocate(spec.N, spec.T)
        self.ws = vb.make_workspace(self.shape)
        self.dX = torch.empty((spec.R, spec.K_in), dtype=self.G.dtype, device="cuda")
        self.dW = torch.empty((spec.K_out, spec.K_in), dtype=torch.float32, device="cuda")
        self.dense_flops = 4.0 * spec.R * spec.K_in * spec.K_out


def cpu_baseline(specs, make_layer):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import oracle
    picked = [s for s in specs if any(f".b{b}." in s.name for b in _sample_blocks(specs))] or specs[:1]
    flops = 0.0
    secs = 0.0
    for s in picked:
        G, X, W = make_layer(s)
        t0 = time.perf_counter()
        oracle.linear_backward(G, X, W, s.dtype, s.N, s.T, s.rho, s.nu, s.seed, s.layer, 0)
        secs += time.perf_counter() - t0
        flops += 4.0 * s.R * s.K_in * s.K_out
    whole = len(picked) == len(specs)
    return {"value": flops / secs / 1e12, "unit": "TFLOP/s (effective, dense-equivalent)",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{len(picked)} of {len(specs)} layers (blocks {sorted(_sample_blocks(specs))}), "
                      f"{secs:.1f} s of oracle time"
                      + ("" if whole else f"; rate over the sample only, a whole step extrapolated by dense-equivalent "
                                          f"flops would take {sum(4.0 * s.R * s.K_in * s.K_out for s in specs) / (flops / secs):.0f} s")}


def _sample_blocks(specs):
    """Blocks whose layers the oracle is timed on: all of them while that stays near ten seconds of
    CPU work (the oracle does about 0.15 dense-equivalent TFLOP/s on 16 cores), else first, middle
    and last."""
    blocks = sorted({int(s.name.split(".b")[1].split(".")[0]) for s in specs if ".b" in s.name})
    if not blocks:
        return set()
    dense_tflop = sum(4.0 * s.R * s.K_in * s.K_out for s in specs) / 1e12
    if dense_tflop <= 2.0:
        return set(blocks)
    return {blocks[0], blocks[len(blocks) // 2], blocks[-1]}


def _is_sibling(name):
    """In backward order a block's layers come as down, up, o, v, k, q.  The gradients of the Q, K and V
    projections' outputs all come out of the attention backward at once: k and q do not wait for the dX of
    the entry before them, which is what vcas_layer_args.sibling states."""
    return name.endswith((".k", ".q"))


def _chainable(specs):
    """Can the layers feed each other in this order?  A layer's dX [R, K_in] must be the G [R, K_out] of the
    next one; a sibling takes what its elder sibling took."""
    prev = None
    for sp in specs:
        if prev is not None:
            if _is_sibling(sp.name):
                if (sp.K_in, sp.K_out) != (prev.K_in, prev.K_out):
                    return False
            elif sp.K_out != prev.K_in or (sp.N, sp.T, sp.dtype) != (prev.N, prev.T, prev.dtype):
                return False
        prev = sp
    return True


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed counter summary of this workload
    (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, each scaled by a plain copy of known size); None
    if no summary covers it.  The counters cannot be read from inside this process."""
    rel = os.path.join("profiles", f"bench_{workload}_hbm_traffic.md")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        parts = [p.strip() for p in line.strip().strip("|").split("|")]
        if len(parts) >= 2 and parts[0] == f"traffic_bytes_per_launch {kernel}":
            try:
                return float(parts[1]), rel
            except ValueError:
                return None, None
    return None, None


def per_shape_report(args, specs, vb, to_device, workloads):
    """One layer per distinct linear shape of the workload, at its largest and its smallest data
    keep ratio: time of the whole sampled path for that layer, of the dense yardsticks, of the two
    GEMM kernels (the library's kernel timer) and of the row-norm kernel over G.  Every figure is
    the median of 50 event-bracketed replays (after 10 warm-ups) of a HIP graph that runs the
    measured call once per copy of the layer, divided by the copies; 'cold' = the copies together
    exceed the 256 MB last-level cache, 'warm' = the same copy every time."""
    import torch
    bf16 = specs[0].dtype == workloads.BF16
    e = 2 if bf16 else 4
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_TFLOPS
    picked = {}
    for sp in specs:
        key = (sp.K_in, sp.K_out)
        lo, hi = picked.get(key, (sp, sp))
        picked[key] = (sp if sp.rho < lo.rho else lo, sp if sp.rho > hi.rho else hi)
    rows = []
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()

    def median_us(body, batch, reps=50, warm=10):
        """Median time per unit of `body` (which enqueues `batch` units), replayed from a HIP graph so
        that the host's launch cost stays out of it."""
        body()                                   # eager once: one-time kernel attribute set-up
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            body()
        for _ in range(warm):
            graph.replay()
        torch.cuda.synchronize()
        out = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            graph.replay()
            e1.record()
            e1.synchronize()
            out.append(e0.elapsed_time(e1) * 1e3 / batch)
        return sorted(out)[len(out) // 2]

    for key, pair in picked.items():
        for sp in dict.fromkeys(pair):           # one row if the workload has a single keep ratio
            nbytes = (sp.R * (sp.K_in + sp.K_out) + sp.K_in * sp.K_out) * e
            copies = max(2, min(16, -(-(640 << 20) // nbytes)))
            first = Layer(sp, vb, to_device, workloads.make_layer)
            ring = [first]
            for _ in range(copies - 1):
                c = Layer.__new__(Layer)
                c.__dict__.update(first.__dict__)
                c.G, c.X, c.W = first.G.clone(), first.X.clone(), first.W.clone()
                c.dX, c.dW = torch.empty_like(first.dX), torch.empty_like(first.dW)
                c.plan, c.ws = vb.Plan.allocate(sp.N, sp.T), vb.make_workspace(first.shape)
                ring.append(c)
            for l in ring:
                l.ones_p = torch.ones(sp.N, device="cuda")
                l.iota_N = torch.arange(sp.N, dtype=torch.int32, device="cuda")
                l.full_N = torch.full((1,), sp.N, dtype=torch.int32, device="cuda")
                l.ones_R = torch.ones(sp.R, device="cuda")
                l.iota_R = torch.arange(sp.R, dtype=torch.int32, device="cuda")
                l.full_R = torch.full((1,), sp.R, dtype=torch.int32, device="cuda")
                l.gsq = torch.empty(sp.R, device="cuda")
                l.gnorm = torch.empty(sp.N, device="cuda")
                l.dW_t = torch.empty((sp.K_out, sp.K_in), dtype=first.G.dtype, device="cuda")
            def sampled(l):
                cur = torch.cuda.current_stream()
                side.wait_stream(cur)
                vb.vcas_linear_backward(l.shape, l.G, l.X, l.W, sp.rho, sp.nu, vb.Rng(sp.seed, sp.layer, 0), True,
                                        l.plan, l.dX, l.dW, l.ws, side)
                cur.wait_stream(side)

            def dense_own(l):
                vb.vcas_sampled_dgrad(l.shape, l.G, l.W, l.ones_p, l.iota_N, l.full_N, l.dX)
                vb.vcas_sampled_wgrad(l.shape, l.G, l.X, l.ones_R, l.iota_R, l.full_R, l.dW, l.ws)

            def dense_torch(l):
                torch.matmul(l.G, l.W, out=l.dX)
                torch.matmul(l.G.t(), l.X, out=l.dW_t)

            def norms(l):
                vb.vcas_row_norms(l.shape, l.G, None, None, l.gsq, None, l.gnorm)

            def over(fn, layers_):
                return lambda: [fn(l) for l in layers_]

            n = len(ring)
            t_cold = median_us(over(sampled, ring), n)
            t_warm = median_us(over(sampled, [ring[0]] * n), n)
            vb.vcas_profile_begin()
            for _ in range(5):
                over(sampled, ring)()
            (dg_ms, dg_n), (wg_ms, wg_n) = vb.vcas_profile_end()
            t_own = median_us(over(dense_own, ring), n)
            t_torch = median_us(over(dense_torch, ring), n)
            t_k1 = median_us(over(norms, ring), n)
            cntA, cntW = int(ring[0].plan.cntA.item()), int(ring[0].plan.cntW.item())
            dense = 4.0 * sp.R * sp.K_in * sp.K_out
            dg_us, wg_us = dg_ms * 1e3 / max(dg_n, 1), wg_ms * 1e3 / max(wg_n, 1)
            dg_tf = 2.0 * cntA * sp.T * sp.K_in * sp.K_out / dg_us / 1e6
            wg_tf = 2.0 * cntW * sp.K_in * sp.K_out / wg_us / 1e6
            k1_gbs = sp.R * sp.K_out * e / t_k1 / 1e3
            rows.append(f"| {sp.K_in}→{sp.K_out} | {sp.rho:.2f} / {sp.nu:.2f} | {cntA}/{sp.N}, {cntW}/{sp.R} | "
                        f"{(cntA * sp.T + cntW) / (2.0 * sp.R):.3f} | {t_cold:.0f} / {t_warm:.0f} | {t_own:.0f} | {t_torch:.0f} | "
                        f"{t_torch / t_cold:.2f} | {dense / t_cold / 1e6:.0f} | {dg_us:.0f} µs, {dg_tf:.0f} ({100 * dg_tf / peak:.0f} %) | "
                        f"{wg_us:.0f} µs, {wg_tf:.0f} ({100 * wg_tf / peak:.0f} %) | {t_k1:.1f} µs, {k1_gbs:.0f} ({100 * k1_gbs / 8000:.0f} %) |")
            print(f"bench.py: {sp.name} done", file=sys.stderr, flush=True)
            del ring, first
            torch.cuda.empty_cache()
    head = [f"# Per-shape timings: workload {args.workload} ({'bf16' if bf16 else 'f32'}, N={specs[0].N}, T={specs[0].T})", "",
            f"Command: `python3 bench.py --workload {args.workload} --per-shape FILE`", "",
            "One layer per distinct linear shape, at the workload's smallest and largest data keep ratio. "
            "Each figure: median of 50 event-bracketed replays (after 10 warm-ups) of a HIP graph that holds the measured "
            "call once per copy of the layer (2 to 16 copies, together above 640 MB, so no copy is still in a cache when its "
            "turn comes: cold), divided by the number of copies; launch gaps between the calls are included, host time is not. "
            "sampled = vcas_linear_backward (norms, both samplers, dX, dW; weight half on a side stream, joined after "
            "every layer), warm = the same graph over one copy; dense = dX and dW at keep "
            "ratio one without the sampling passes (this library, torch.matmul), cold; effective TFLOP/s = 4·R·K_in·K_out / "
            "cold sampled time; GEMM columns = kernel-timer average per launch inside eagerly launched cold sampled calls, "
            "algorithmic flops 2·cntA·T·K_in·K_out resp. 2·cntW·K_in·K_out, percentage of the 2.5 PFLOP/s bf16 "
            "(157.3 TFLOP/s fp32) datasheet peak; G norms = vcas_row_norms over G only, R·K_out·e bytes, percentage of 8 TB/s.", "",
            "| shape | ρ / ν | kept samples, tokens | kept flop fraction | sampled µs cold / warm | dense own µs | dense torch µs | "
            "speedup vs torch | effective TFLOP/s | dgrad | wgrad | G norms GB/s |",
            "|---|---|---|---|---|---|---|---|---|---|---|---|"]
    with open(args.per_shape, "w") as f:
        f.write("\n".join(head + rows) + "\n")
    print("\n".join(rows), file=sys.stderr)


def adaptation_leg(args, layers, vb, torch):
    """What one update of the adaptive keep ratios costs on this stack (Sec. 5, Alg. 1; App. D): for each of
    M = 2 batches an exact backward pass (dX and dW at keep ratio one) whose dW feeds the running mean and
    mean of squares on every 100th parameter, then the variance probe with M mask draws (SampleA-only dW
    against the exact one, Eq. 3 under each draw's data mask) and Eq. 4's sparsity at s - alpha and
    s + alpha.  The probe forms its own exact dW and also the Monte-Carlo term with both samplers, which
    Alg. 1 does not need, so the figure is an upper bound.  The resident inputs stand in for both batches."""
    import time
    M, stride = 2, 100
    side = []
    for l in layers:
        m = (l.spec.K_out * l.spec.K_in + stride - 1) // stride
        side.append((torch.zeros(m, device="cuda"), torch.zeros(m, device="cuda"),
                     torch.empty(4, dtype=torch.float64, device="cuda"), torch.empty(2, device="cuda"), m))

    def update():
        for i in range(M):
            for l, (mean, sq, out4, pr, m) in zip(layers, side):
                s = l.spec
                vb.vcas_linear_backward(l.shape, l.G, l.X, l.W, 1.0, 1.0, vb.Rng(s.seed, s.layer, 0), True, l.plan,
                                        l.dX, l.dW, l.ws)
                vb.vcas_grad_stats_update(l.dW, m, stride, i + 1, mean, sq)
                vb.vcas_variance_probe(l.shape, l.G, l.X, s.rho, s.nu, vb.Rng(s.seed, s.layer, 10 * i), M, l.plan,
                                       out4, l.ws)
                vb.vcas_sparsity_ratio(l.plan.gnorm, [0.98, 1.0], pr)

    update()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    update()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3
    return {"ms_per_update": ms, "M": M, "kept_parameter_stride": stride,
            "what": "2 batches x (exact dX+dW, running statistics, probe with 2 draws, Eq. 4 at two levels) over "
                    "every layer, one stream; an upper bound (the probe repeats the exact dW and adds a SampleA+SampleW term)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="bert_large")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--one-stream", action="store_true", help="keep the weight-gradient half on the main stream")
    ap.add_argument("--side-streams", type=int, default=1, help="streams the weight-gradient halves rotate over")
    ap.add_argument("--eager", action="store_true", help="launch every kernel from the host instead of replaying a HIP graph")
    ap.add_argument("--stack", type=int, default=None, metavar="GROUP",
                    help="the default launch: one vcas_backward_stack call per step (from the host, no graph), "
                         "cross-stream dependencies once per GROUP layers (default: 3 for R <= 4096, else 6), SampleW and dW on two side streams; "
                         "0 = per-layer calls (see --graph-free options below)")
    ap.add_argument("--rho", type=float, default=None, help="override every layer's data keep ratio (sweeps)")
    ap.add_argument("--nu", type=float, default=None, help="override every layer's token keep ratio (sweeps)")
    ap.add_argument("--graph", action="store_true",
                    help="per-layer vcas_linear_backward calls captured in one HIP graph per step instead")
    ap.add_argument("--no-siblings", action="store_true",
                    help="stack launch: do not mark the K and Q projections as siblings of V (every data half then "
                         "waits for the one before it)")
    ap.add_argument("--wgrad-fill", type=int, default=64, metavar="WORKGROUPS",
                    help="stack launch: workgroups a weight-gradient launch should have before it stops cutting the "
                         "contraction into split-K slices (vcas_layer_args.wgrad_fill; 0 or 384 = what a stand-alone call uses)")
    ap.add_argument("--independent", action="store_true",
                    help="stack launch: every layer keeps the upstream gradient it was generated with, as if other kernels "
                         "had produced it.  The default is the chain of a backward pass (Sec. 4: SampleA sits between the "
                         "layers, the gradient grows sparser on its way down): down's dX buffer is up's G, up's is o's, o's "
                         "is the G of V, K and Q, Q's is the next block's down's; every layer is told which samples the one "
                         "above kept, sweeps the rows of its G that exist for their norms and leaves the rows of dropped "
                         "samples unwritten; only the top layer's G is an input")
    ap.add_argument("--chained", action="store_true", help="the default since the chain became the timed form; accepted and ignored")
    ap.add_argument("--fused-norms", action="store_true",
                    help="chained stack: every dgrad also leaves the sums of squares of its dX by blocks of 64 columns; the "
                         "entry below adds them to row sums and sample norms in one launch and its dgrad decides SampleA "
                         "itself, instead of sweeping G and launching SampleA (the same bits; bf16 only)")
    ap.add_argument("--sweep-norms", action="store_true", help="the default; accepted and ignored")
    ap.add_argument("--xsq-cached", action="store_true",
                    help="stack launch only: the squared row norms of X are taken before the timed region (as a forward "
                         "pass would, vcas_row_norms over every row) and handed to the weight halves; not the default, "
                         "which sweeps X inside the step")
    ap.add_argument("--share-inputs", action="store_true",
                    help="layers of equal shape get copies of the same generated values (each layer still owns its "
                         "tensors in HBM); saves minutes of host-side generation on the 144-layer workloads")
    ap.add_argument("--per-shape", metavar="FILE", default=None,
                    help="instead of the stack step: one layer per distinct linear shape (at the workload's largest and "
                         "smallest data keep ratio), median of 50 event-timed calls after 10 warm-ups, inputs rotated "
                         "over enough copies to defeat the caches; writes a markdown table to FILE and prints no result line")
    ap.add_argument("--adaptation", action="store_true",
                    help="also time one update of the adaptive keep ratios (Alg. 1 with M = 2) on the same stack and "
                         "print it beside ms_per_step")
    ap.add_argument("--counters-pass", action="store_true",
                    help="for a rocprofv3 --pmc run: the sampled steps only, launched eagerly, then one plain 256 MiB "
                         "device copy whose known size calibrates FETCH_SIZE / WRITE_SIZE; prints no result line")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    import workloads
    from paper_2402_17227_amd import binding as vb
    to_device = vb.to_device

    vb.lib()                                    # fails loudly if libvcas.so was not built
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    specs = workloads.config(args.workload)
    if args.rho is not None or args.nu is not None:
        import dataclasses
        specs = [dataclasses.replace(sp, rho=args.rho if args.rho is not None else sp.rho,
                                     nu=args.nu if args.nu is not None else sp.nu) for sp in specs]
    if args.per_shape:
        per_shape_report(args, specs, vb, to_device, workloads)
        return
    cache = {} if args.share_inputs else None
    layers = []
    if args.share_inputs:
        for k, s in enumerate(specs):
            layers.append(Layer(s, vb, to_device, workloads.make_layer, cache))
    else:
        # every layer gets values of its own; the host-side generators run a few layers ahead of the
        # uploads on a handful of threads (numpy releases the interpreter lock while it draws)
        from concurrent.futures import ThreadPoolExecutor
        workers = max(1, min(8, (os.cpu_count() or 2) - 1))
        with ThreadPoolExecutor(workers) as pool:
            ahead = []
            nxt = 0
            for k, s in enumerate(specs):
                while nxt < len(specs) and len(ahead) < 2 * workers:
                    ahead.append(pool.submit(workloads.make_layer, specs[nxt]))
                    nxt += 1
                layers.append(Layer(s, vb, to_device, workloads.make_layer, arrays=ahead.pop(0).result()))
                if k % 24 == 23:
                    print(f"bench.py: {k + 1} of {len(specs)} layers resident", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    dense_flops = sum(l.dense_flops for l in layers)

    # The draw index lives in device memory so that one captured graph gives fresh masks on
    # every replay: each step first bumps the counter, every layer adds it to its draw.
    draw_counter = torch.zeros(1, dtype=torch.int32, device="cuda")

    # Norms of G, SampleA and dX of every layer run in order on the main stream (the order a real
    # backward pass imposes); each layer's weight-gradient half (norms of X, SampleW, dW) depends on
    # its SampleA only and runs beside that.  Default launch: vcas_backward_stack, which puts SampleW
    # and dW on two side streams and pays the cross-stream waits once per group of layers.
    # --graph: per-layer vcas_linear_backward calls, weight halves on side stream(s), one HIP
    # graph per step.  The step ends when every stream has drained.
    sides = [] if args.one_stream else [torch.cuda.Stream() for _ in range(args.side_streams)]

    stack = None
    fused_norms = False
    if args.stack is None:
        # a group of layers = the stretch between two cross-stream waits: half a block ([down, up, o], [V, K, Q]) where
        # a layer is a few microseconds of work and the side streams must not fall behind, a whole block where
        # layers are long enough to hide that (bert_base 2.29 vs 2.32 ms, bert_large 15.2 vs 14.7 ms)
        args.stack = 3 if specs[0].R <= 4096 else 6
    args.chained = not args.independent and _chainable(specs)   # a fused Q/K/V layer breaks the chain of shapes
    if args.graph or args.eager or args.one_stream:
        args.stack = 0
        args.chained = False                      # per-layer calls: independent layers
        if args.xsq_cached:
            sys.exit("bench.py: --xsq-cached goes with the stack launch only")
    if args.stack > 0:
        for l in layers:
            l.xsq_forward = None
            if args.xsq_cached:
                l.xsq_forward = torch.empty(l.spec.R, dtype=torch.float32, device="cuda")
                vb.vcas_row_norms(l.shape, None, l.X, None, None, l.xsq_forward, None)
        entries, prev = [], None
        fused_norms = args.chained and args.fused_norms and specs[0].dtype == workloads.BF16
        for l in layers:
            sib = not args.no_siblings and _is_sibling(l.spec.name)
            G, above, g_blocks = l.G, None, None
            # chained: every dgrad also leaves the sums of squares of its dX by blocks of 64 columns, from
            # which the entry below takes the norms of its G instead of sweeping it
            l.sq_blocks = vb.make_sq_blocks(l.spec.R, l.spec.K_in) if fused_norms else None
            if args.chained and prev is not None:
                # a sibling takes what its elder sibling took; everybody else the dX of the entry before
                G, above, g_blocks = ((prev_G, prev_above, prev_blocks) if _is_sibling(l.spec.name)
                                      else (prev.dX, prev.plan.maskA, prev.sq_blocks))
                assert G.shape == l.G.shape, (l.spec.name, G.shape, l.G.shape)
                l.G = G
            entries.append(vb.layer_args(l.shape, G, l.X, l.W, l.spec.rho, l.spec.nu,
                                         vb.Rng(l.spec.seed, l.spec.layer, 0, draw_counter.data_ptr()), True,
                                         l.plan, l.dX, l.dW, l.ws, l.xsq_forward, sibling=sib,
                                         kept_above=above, leave_dropped_rows=args.chained,
                                         wgrad_fill=args.wgrad_fill, dx_sq_blocks=l.sq_blocks, g_sq_blocks=g_blocks))
            prev, prev_G, prev_above, prev_blocks = l, G, above, g_blocks
        stack = vb.make_stack(entries)
        s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()

    def step():
        main = torch.cuda.current_stream()
        draw_counter.add_(1)
        if stack is not None:
            vb.vcas_backward_stack(stack, args.stack, s2, s3)
            main.wait_stream(s2)
            main.wait_stream(s3)
            return
        for sd in sides:
            sd.wait_stream(main)
        for k, l in enumerate(layers):
            s = l.spec
            vb.vcas_linear_backward(l.shape, l.G, l.X, l.W, s.rho, s.nu,
                                    vb.Rng(s.seed, s.layer, 0, draw_counter.data_ptr()), True, l.plan,
                                    l.dX, l.dW, l.ws, sides[k % len(sides)] if sides else None)
        for sd in sides:
            main.wait_stream(sd)

    # ---- timed region: K steps of the whole path --------------------------------
    step()                                       # eager once: one-time kernel attribute set-up
    torch.cuda.synchronize()
    if args.counters_pass:
        for i in range(args.steps):
            step()
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        return
    if args.eager or stack is not None:
        run_step = step
    else:                                        # the ~500 launches of a step as one HIP graph
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step = graph.replay
    for i in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    kept_rows = sum(int(l.plan.cntA.item()) * l.spec.T * 2.0 * l.spec.K_in * l.spec.K_out for l in layers)
    kept_toks = sum(int(l.plan.cntW.item()) * 2.0 * l.spec.K_in * l.spec.K_out for l in layers)
    kept_fraction = (kept_rows + kept_toks) / dense_flops

    # ---- per-kernel durations of the two GEMMs, HIP events on the launch stream ----
    # The same steps once more, launched eagerly with the library's kernel timer on: every GEMM
    # launch is bracketed by HIP events stamped by its own dispatch (an event pair recorded from
    # the host around a launch would also count the gap until the host submits the kernel).
    reps = max(3, min(args.steps, 10))
    vb.vcas_profile_begin()
    for _ in range(reps):
        step()
    (dg_ms, dg_n), (wg_ms, wg_n) = vb.vcas_profile_end()
    dg_avg, dg_total = dg_ms / max(dg_n, 1), dg_ms / reps
    wg_avg, wg_total = wg_ms / max(wg_n, 1), wg_ms / reps
    bf16 = specs[0].dtype == workloads.BF16
    e = 2 if bf16 else 4
    sfx = "bf16" if bf16 else "f32"
    # algorithmic HBM bytes per launch: kept operand rows once, W resp. dW once, and dX: all of it (zeros
    # included) for independent layers, the kept rows and their block sums of squares in the chain
    def dx_bytes(l):
        if not args.chained:
            return l.spec.R * l.spec.K_in * e
        kept = int(l.plan.cntA.item()) * l.spec.T
        return kept * l.spec.K_in * e + (kept * ((l.spec.K_in + 63) // 64) * 4 if l.sq_blocks is not None else 0)
    dg_bytes = sum(int(l.plan.cntA.item()) * l.spec.T * l.spec.K_out * e + l.spec.K_in * l.spec.K_out * e
                   + dx_bytes(l) for l in layers) / len(layers)
    wg_bytes = sum(int(l.plan.cntW.item()) * (l.spec.K_out + l.spec.K_in) * e + 4 * l.spec.K_in * l.spec.K_out
                   for l in layers) / len(layers)
    # a launch may cover several layers (siblings): flops and bytes per launch follow the launch count
    dg_per_step, wg_per_step = max(dg_n, 1) / reps, max(wg_n, 1) / reps
    dg_bytes *= len(layers) / dg_per_step
    wg_bytes *= len(layers) / wg_per_step
    if dg_total >= wg_total:
        name, avg_ms, flops, alg_bytes = f"dgrad_{sfx}_kernel", dg_avg, kept_rows / dg_per_step, dg_bytes
    else:
        name, avg_ms, flops, alg_bytes = f"wgrad_{sfx}_kernel", wg_avg, kept_toks / wg_per_step, wg_bytes
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_TFLOPS
    achieved = flops / (avg_ms * 1e-3) / 1e12
    traffic, traffic_src = measured_traffic(args.workload.split(":")[0], name)
    roofline = {"bound": "mfma", "kernel": name, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                "frac": achieved / peak, "traffic": traffic,
                "traffic_source": (f"{traffic_src}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of `bench.py --counters-pass`, "
                                   "taken with the build of the commit that last changed that file, not measured in this run") if traffic_src else None,
                "algorithmic_bytes": alg_bytes, "avg_launch_us": avg_ms * 1e3,
                "launches_per_step": dg_per_step if name.startswith("dgrad") else wg_per_step,
                "dgrad_ms_per_step": dg_total, "wgrad_ms_per_step": wg_total}

    # ---- dense yardsticks at the same shapes -------------------------------------
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / reps

    # Two launch forms each: everything on one stream, and the form the sampled step itself has (the
    # chain of dX on the main stream, every dW on a side stream, joined at the end), so that the
    # sampled step is compared with a dense step that overlaps its two halves the same way.
    dense_side = torch.cuda.Stream()

    def two_streams(dx_half, dw_half):
        def run():
            main = torch.cuda.current_stream()
            dense_side.wait_stream(main)
            for l in layers:
                dx_half(l)
            with torch.cuda.stream(dense_side):
                for l in layers:
                    dw_half(l)
            main.wait_stream(dense_side)
        return run

    def own_dx(l):          # this library's two GEMMs at keep ratio one, sampling passes skipped
        vb.vcas_sampled_dgrad(l.shape, l.G, l.W, l.ones_p, l.iota_N, l.full_N, l.dX)

    def own_dw(l):
        vb.vcas_sampled_wgrad(l.shape, l.G, l.X, l.ones_R, l.iota_R, l.full_R, l.dW, l.ws)

    def torch_dx(l):
        torch.matmul(l.G, l.W, out=l.dX)

    def torch_dw(l):        # dW in the layer dtype here (the library writes fp32), into a buffer that exists
        torch.matmul(l.G.t(), l.X, out=l.dW_t)

    def one_stream(dx_half, dw_half):
        def run():
            for l in layers:
                dx_half(l)
                dw_half(l)
        return run

    for l in layers:
        s = l.spec
        l.ones_p = torch.ones(s.N, device="cuda")
        l.iota_N = torch.arange(s.N, dtype=torch.int32, device="cuda")
        l.full_N = torch.full((1,), s.N, dtype=torch.int32, device="cuda")
        l.ones_R = torch.ones(s.R, device="cuda")
        l.iota_R = torch.arange(s.R, dtype=torch.int32, device="cuda")
        l.full_R = torch.full((1,), s.R, dtype=torch.int32, device="cuda")
        l.dW_t = torch.empty((s.K_out, s.K_in), dtype=l.G.dtype, device="cuda")
    reps = max(3, min(args.steps, 10))
    dense_ms = {
        "this_library_keep_ratio_1_gemms_only": timed(one_stream(own_dx, own_dw), reps),
        "this_library_keep_ratio_1_gemms_only_two_streams": timed(two_streams(own_dx, own_dw), reps),
        "torch_matmul": timed(one_stream(torch_dx, torch_dw), reps),
        "torch_matmul_two_streams": timed(two_streams(torch_dx, torch_dw), reps),
    }
    dense_note = ("dX and dW of every layer at keep ratio one, no sampling passes; two_streams = the sampled step's own "
                  "launch form (dX chain on the main stream, dW on a side stream); torch.matmul writes dW in bf16, "
                  "the library in fp32")

    adaptation = adaptation_leg(args, layers, vb, torch) if args.adaptation else None

    out = {
        "metric": METRIC,
        "value": dense_flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s (effective: dense-equivalent 4*R*K_in*K_out per layer / sampled-path time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "launch": (f"vcas_backward_stack from the host, groups of {args.stack} layers, SampleW and dW on two side streams"
                   + ("" if args.no_siblings else ", data halves of V, K, Q of a block in shared launches")
                   + f", weight gradients sliced for {args.wgrad_fill or 384} workgroups"
                   + (", layers chained (each dX buffer is the next G, dropped samples stay dropped and unwritten"
                      + (", row norms of G from the dgrad above" if fused_norms else ", row norms of G swept")
                      + ")" if args.chained else ", independent layers (every G an input, swept for its row norms)")
                   + (", row norms of X cached before the timed region" if args.xsq_cached else "")
                   if stack is not None else
                   ("eager" if args.eager else "hip_graph") +
                   (", one stream" if args.one_stream else f", dW halves on {args.side_streams} side streams")),
        "config": {"workload": args.workload, "layers": len(layers), "chained": bool(args.chained), "N": specs[0].N, "T": specs[0].T,
                   "rho": [min(s.rho for s in specs), max(s.rho for s in specs)], "nu": specs[0].nu},
        "kept_flop_fraction": kept_fraction,
        "dense_ms_per_step": dict(dense_ms, note=dense_note),
        "speedup_vs_dense": {k: v / ms_per_step for k, v in dense_ms.items()},
        "roofline": roofline,
    }
    if adaptation is not None:
        out["adaptation"] = adaptation
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(specs, workloads.make_layer)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
