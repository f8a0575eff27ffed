"""Parity at the full sizes of the benchmark configurations, launched the way bench.py launches:
vcas_backward_stack from the host, SampleW and dW on two side streams, weight gradients sliced for 64
workgroups, draw index read from device
memory (and, for one layer of each model, the graph-replay launch bench.py offers as --graph).
The sampling plan is compared bit for bit with the oracle's; dX and dW are compared on entries
drawn at random (the oracle computes them one by one), and on properties that hold everywhere
(rows of dropped samples are zero, nothing is left unwritten)."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import workloads
from workloads import BF16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vb():
    from paper_2402_17227_amd import binding
    binding.lib()
    return binding


def _cases():
    specs = workloads.config("bert_base")
    by_shape = {}
    for s in specs:
        by_shape.setdefault((s.K_in, s.K_out), []).append(s)
    out = []
    # BERT-base: one layer of each shape from the top (rho near 1), the middle and the bottom (rho 0.3)
    for shape, ls in sorted(by_shape.items()):
        out += [ls[0], ls[len(ls) // 2], ls[-1]]
    for cfg in ("bert_large", "vit_b16", "gpt2_medium"):
        by_shape = {}
        for s in workloads.config(cfg):
            by_shape.setdefault((s.K_in, s.K_out), []).append(s)
        for shape, ls in sorted(by_shape.items()):
            out.append(ls[len(ls) // 2])
    out += [s for s in workloads.config("bert_base_fused_qkv") if s.name.endswith(".b5.qkv")]   # 768 -> 2304
    # the other eight points of the GPT-2-medium sweep (data keep ratio x token keep ratio over {1, .5, .25}),
    # one layer per distinct shape each: keep ratio one at R = 16384 (every row kept, every split-K slice
    # active, no zero-fill duty) down to the corners where few rows survive and the small tiles take over
    for rho in (1.0, 0.5, 0.25):
        for nu in (1.0, 0.5, 0.25):
            if (rho, nu) == (0.5, 0.5):
                continue                         # the workload's default point, covered above
            by_shape = {}
            for s in workloads.config(f"gpt2_medium:{rho}:{nu}"):
                by_shape.setdefault((s.K_in, s.K_out), []).append(s)
            for shape, ls in sorted(by_shape.items()):
                out.append(ls[(len(ls) // 2 + int(4 * rho + 8 * nu)) % len(ls)])   # another block per point
    return out


def _case_id(s):
    return f"{s.name}-rho{s.rho:g}-nu{s.nu:g}" if s.name.startswith("gpt2_medium") else s.name


@pytest.mark.parametrize("spec", _cases(), ids=_case_id)
def test_full_size_layer_in_the_bench_launch_configuration(vb, spec):
    from tests.gpu_util import to_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    G, X, W = workloads.make_layer(spec)
    shape = vb.shape_of(spec.N, spec.T, spec.K_in, spec.K_out, spec.dtype)
    g, x, w = (to_device(a, spec.dtype) for a in (G, X, W))
    plan = vb.Plan.allocate(spec.N, spec.T)
    ws = vb.make_workspace(shape)
    dX = torch.full((spec.R, spec.K_in), float("nan"), dtype=g.dtype, device="cuda")
    dW = torch.full((spec.K_out, spec.K_in), float("nan"), dtype=torch.float32, device="cuda")
    counter = torch.zeros(1, dtype=torch.int32, device="cuda")
    rng = vb.Rng(spec.seed, spec.layer, 0, counter.data_ptr())
    if spec.name.endswith(".b5.o") or spec.name.endswith(".b11.o"):
        # the graph launch: one side stream, the step captured once and replayed
        side = torch.cuda.Stream()

        def step():
            main = torch.cuda.current_stream()
            counter.add_(1)
            side.wait_stream(main)
            vb.vcas_linear_backward(shape, g, x, w, spec.rho, spec.nu, rng, True, plan, dX, dW, ws, side)
            main.wait_stream(side)

        step()                                   # draw 1, eager
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        dX.fill_(float("nan"))
        dW.fill_(float("nan"))
        graph.replay()                           # draw 2
        graph.replay()                           # draw 3
    else:
        stack = vb.make_stack([vb.layer_args(shape, g, x, w, spec.rho, spec.nu, rng, True, plan, dX, dW, ws,
                                             wgrad_fill=64)])
        s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
        for draw in (1, 2, 3):
            main = torch.cuda.current_stream()
            counter.add_(1)
            if draw == 2:
                dX.fill_(float("nan"))
                dW.fill_(float("nan"))
            vb.vcas_backward_stack(stack, 4, s2, s3)
            main.wait_stream(s2)
            main.wait_stream(s3)
    torch.cuda.synchronize()
    draw = int(counter.item())
    assert draw == 3
    _check_against_oracle(spec, G, X, W, plan, dX, dW, draw)


def _check_against_oracle(spec, G, X, W, plan, dX, dW, draw):
    from tests.gpu_util import plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    want = oracle.sampling_plan(G, X, spec.dtype, spec.N, spec.T, spec.rho, spec.nu, spec.seed, spec.layer, draw)
    got = plan_to_numpy(plan)
    compare_plan(got, want)

    # properties that hold everywhere
    assert bool(torch.isfinite(dX).all()) and bool(torch.isfinite(dW).all())
    dropped_rows = torch.from_numpy(np.repeat(want.maskA == 0, spec.T)).cuda()
    assert bool((dX[dropped_rows] == 0).all())

    # entries drawn at random, computed one by one by the oracle (Eq. 2 upper line; Sec. 4.2)
    rs = np.random.default_rng(spec.layer + 17)
    n = 4096
    kept_rows = np.nonzero(np.repeat(want.maskA == 1, spec.T))[0]
    if kept_rows.size:
        rows = rs.choice(kept_rows, n)
        cols = rs.integers(0, spec.K_in, n)
        ref = oracle.dgrad_at(G, W, spec.dtype, spec.T, want.p, want.maskA, rows, cols)
        val = dX[torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()].float().cpu().numpy()
        assert rel_l2(val, ref) <= 1e-2
        # no single entry off by more than bf16 rounding plus accumulation noise at the row's scale
        scale = np.sqrt(np.mean(ref ** 2))
        assert np.max(np.abs(val - ref) / (np.abs(ref) + scale)) <= 2e-2
    orow = rs.integers(0, spec.K_out, n)
    kcol = rs.integers(0, spec.K_in, n)
    ref = oracle.wgrad_at(G, X, spec.dtype, want.scaleW, orow, kcol)
    val = dW[torch.from_numpy(orow).cuda(), torch.from_numpy(kcol).cuda()].cpu().numpy()
    assert rel_l2(val, ref) <= 1e-2
    scale = np.sqrt(np.mean(ref ** 2))
    assert np.max(np.abs(val - ref) / (np.abs(ref) + scale)) <= 2e-2


@pytest.mark.parametrize("workload", ["bert_base", "bert_large"])
def test_full_size_sibling_layers_in_shared_launches(vb, workload):
    """The V, K and Q projections of one block at full size, launched as bench.py launches them: one
    vcas_backward_stack call, groups of three, K and Q marked as siblings of V, so that the three share their
    row-norm, SampleA, dgrad, X-sweep, SampleW, wgrad and reduction launches.  bert_base: SampleA inside the
    dgrad workgroups; bert_large: a SampleA launch with a workgroup per layer."""
    from tests.gpu_util import to_device
    block = "b5" if workload == "bert_base" else "b11"
    specs = [s for s in workloads.config(workload) if s.name.split(".")[1] == block and s.name.split(".")[2] in "vkq"]
    assert [s.name.split(".")[2] for s in specs] == ["v", "k", "q"]
    counter = torch.zeros(1, dtype=torch.int32, device="cuda")
    host, entries, outs, keep = [], [], [], []
    for k, spec in enumerate(specs):
        G, X, W = workloads.make_layer(spec)
        shape = vb.shape_of(spec.N, spec.T, spec.K_in, spec.K_out, spec.dtype)
        g, x, w = (to_device(a, spec.dtype) for a in (G, X, W))
        plan = vb.Plan.allocate(spec.N, spec.T)
        ws = vb.make_workspace(shape)
        dX = torch.full((spec.R, spec.K_in), float("nan"), dtype=g.dtype, device="cuda")
        dW = torch.full((spec.K_out, spec.K_in), float("nan"), dtype=torch.float32, device="cuda")
        entries.append(vb.layer_args(shape, g, x, w, spec.rho, spec.nu,
                                     vb.Rng(spec.seed, spec.layer, 0, counter.data_ptr()), True, plan, dX, dW, ws,
                                     sibling=k > 0, wgrad_fill=64))
        host.append((G, X, W))
        outs.append((plan, dX, dW))
        keep.append((g, x, w, ws))
    stack = vb.make_stack(entries)
    s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
    for draw in (1, 2):
        main = torch.cuda.current_stream()
        counter.add_(1)
        vb.vcas_backward_stack(stack, 3, s2, s3)
        main.wait_stream(s2)
        main.wait_stream(s3)
    torch.cuda.synchronize()
    for spec, (G, X, W), (plan, dX, dW) in zip(specs, host, outs):
        _check_against_oracle(spec, G, X, W, plan, dX, dW, 2)


@pytest.mark.parametrize("workload,block,fused", [("bert_base", "b5", False), ("bert_large", "b11", True)])
def test_full_size_block_in_the_chained_launch(vb, workload, block, fused):
    """The chained launch of bench.py at full size, one attention block: the out-projection, then V, K, Q as
    siblings that take its dX as their G, know which samples it kept (kept_above) and leave the rows of the
    samples they drop unwritten.  The oracle computes the out-projection on its own and hands its dX (bf16) to
    V, K, Q; the GPU gets the same tensor with NaN in the rows of dropped samples, in one stack call.
    fused (bench.py --fused-norms): the out-projection's dgrad also leaves the block sums of squares of
    its dX, and V, K, Q take the row norms of their G from block sums instead of sweeping it.  Data flows from
    the oracle to the GPU only: the block sums handed to V, K, Q are the oracle's, of the oracle's dX; what the
    GPU's dgrad emitted is checked against those within the tolerance of dX, and bit for bit against a sweep of
    the dX it wrote."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    specs = {s.name.split(".")[2]: s for s in workloads.config(workload) if s.name.split(".")[1] == block}
    o = specs["o"]
    G, X, W = workloads.make_layer(o)
    want_o, dX_o, _ = oracle.linear_backward(G, X, W, o.dtype, o.N, o.T, o.rho, o.nu, o.seed, o.layer, 1)
    G2 = workloads.f32_to_bf16_bits(dX_o.astype(np.float32))
    kept = want_o.maskA.astype(bool)
    assert 0 < kept.sum() < o.N
    g2 = to_device(G2, BF16)
    g2.view(o.N, o.T, -1)[torch.from_numpy(~kept).cuda()] = float("nan")
    above = torch.from_numpy(want_o.maskA.astype(np.uint8)).cuda()
    from tests.gpu_util import blocks_to_device_layout, blocks_from_device_layout
    nb = (o.K_in + 63) // 64
    blocks_o = vb.make_sq_blocks(o.R, o.K_in, float("nan")) if fused else None
    want_blocks = g2_blocks = None
    if fused:
        want_blocks = oracle.block_sumsq(G2, BF16)                       # [R, nb]
        poisoned = want_blocks.copy()
        poisoned[np.repeat(~kept, o.T)] = np.nan                         # rows of dropped samples are never read
        g2_blocks = torch.from_numpy(blocks_to_device_layout(poisoned)).cuda()
    entries, outs, keep, host = [], [], [], []
    for k, name in enumerate(["o", "v", "k", "q"]):
        sp = specs[name]
        Gs, Xs, Ws = (G, X, W) if name == "o" else workloads.make_layer(sp)
        shape = vb.shape_of(sp.N, sp.T, sp.K_in, sp.K_out, sp.dtype)
        x, w = to_device(Xs, BF16), to_device(Ws, BF16)
        g = to_device(G, BF16) if name == "o" else g2
        plan = vb.Plan.allocate(sp.N, sp.T)
        ws = vb.make_workspace(shape)
        dX = torch.full((sp.R, sp.K_in), float("nan"), dtype=torch.bfloat16, device="cuda")
        dW = torch.full((sp.K_out, sp.K_in), float("nan"), dtype=torch.float32, device="cuda")
        entries.append(vb.layer_args(shape, g, x, w, sp.rho, sp.nu, vb.Rng(sp.seed, sp.layer, 1), True, plan, dX, dW, ws,
                                     sibling=name in "kq", kept_above=None if name == "o" else above,
                                     leave_dropped_rows=True, wgrad_fill=64,
                                     dx_sq_blocks=blocks_o if name == "o" else None,
                                     g_sq_blocks=None if name == "o" else g2_blocks))
        outs.append((sp, plan, dX, dW))
        keep.append((g, x, w, ws))
        host.append((G if name == "o" else G2, Xs, Ws))
    s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
    vb.vcas_backward_stack(vb.make_stack(entries), 3, s2, s3)
    torch.cuda.synchronize()
    for (sp, plan, dX, dW), (Gs, Xs, Ws) in zip(outs, host):
        want, want_dX, want_dW = oracle.linear_backward(Gs, Xs, Ws, sp.dtype, sp.N, sp.T, sp.rho, sp.nu, sp.seed,
                                                        sp.layer, 1)
        got = plan_to_numpy(plan)
        compare_plan(got, want)
        m = got["maskA"].astype(bool)
        if sp.name.endswith(".o"):
            assert np.array_equal(m, kept)
        else:
            assert not np.any(m & ~kept)
        rows = np.repeat(m, sp.T)
        got_dX = from_device(dX)
        assert np.isnan(got_dX[~rows]).all() and np.isfinite(got_dX[rows]).all()
        assert rel_l2_rows(got_dX[rows], want_dX[rows]) <= 1e-2
        assert rel_l2_tiles(from_device(dW), want_dW) <= 1e-2
    if fused:
        rows = np.repeat(kept, o.T)
        got_blocks = blocks_from_device_layout(blocks_o, nb)
        assert np.isnan(got_blocks[~rows]).all() and np.isfinite(got_blocks[rows]).all()
        num = np.abs(got_blocks[rows].astype(np.float64) - want_blocks[rows]).sum(axis=1)
        den = want_blocks[rows].astype(np.float64).sum(axis=1)
        assert (num[den > 0] / den[den > 0]).max() <= 4e-2               # squares: twice the tolerance of dX
        # the same tree as a sweep over the dX this launch wrote (dropped rows zeroed for the sweep, which reads them)
        dX_o = outs[0][2].clone()
        dX_o.view(o.N, o.T, -1)[torch.from_numpy(~kept).cuda()] = 0.0
        sq_blocks = torch.full((o.R,), float("nan"), device="cuda")
        sq_sweep = torch.full((o.R,), float("nan"), device="cuda")
        vb.vcas_row_norms_from_blocks(o.N, o.T, o.K_in, blocks_o, above, sq_blocks, None)
        vb.vcas_row_norms(vb.shape_of(o.N, o.T, 8, o.K_in, BF16), dX_o, None, None, sq_sweep, None, None)
        torch.cuda.synchronize()
        assert torch.equal(sq_blocks.view(torch.int32), sq_sweep.view(torch.int32))


def test_variance_probe_at_vit_size_with_eight_draws(vb):
    """Config 4's probe: N=64, T=197, M=8 draws (Alg. 1's Monte-Carlo lines, Eq. 3)."""
    from tests.gpu_util import to_device
    base = workloads.config("vit_b16")[0]
    spec = workloads.LayerSpec("vit_probe", BF16, base.N, base.T, 768, 768, base.rho, base.nu, layer=7, seed=11,
                               gen_seed=5, sample_sigma=base.sample_sigma, token_sigma=base.token_sigma)
    G, X, W = workloads.make_layer(spec)
    M = 8
    shape = vb.shape_of(spec.N, spec.T, spec.K_in, spec.K_out, spec.dtype)
    plan = vb.Plan.allocate(spec.N, spec.T)
    ws = vb.make_workspace(shape)
    out = torch.full((4,), float("nan"), dtype=torch.float64, device="cuda")
    vb.vcas_variance_probe(shape, to_device(G, BF16), to_device(X, BF16), spec.rho, spec.nu,
                           vb.Rng(spec.seed, spec.layer, 100), M, plan, out, ws)
    torch.cuda.synchronize()
    want = oracle.variance_probe(G, X, BF16, spec.N, spec.T, spec.rho, spec.nu, spec.seed, spec.layer, 100, M)
    got = out.cpu().numpy()
    np.testing.assert_allclose(got[:2], want[:2], rtol=1e-9)
    np.testing.assert_allclose(got[2:], want[2:], rtol=3e-2)
