"""The benchmark replays a captured HIP graph of the whole path; replays must
give the same bits as eager launches, on every replay, with eager work and
synchronisation in between, and the device-side draw offset must select the
same masks as the host-side draw."""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager_launches():
    from paper_2402_17227_amd import binding as vb
    from tests.gpu_util import to_device, plan_to_numpy
    spec = workloads.LayerSpec("graph", workloads.BF16, 12, 70, 264, 200, 0.5, 0.5, layer=5, seed=31, gen_seed=7,
                               token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    shape = vb.shape_of(spec.N, spec.T, spec.K_in, spec.K_out, spec.dtype)
    g, x, w = (to_device(a, spec.dtype) for a in (G, X, W))

    def buffers():
        return (vb.Plan.allocate(spec.N, spec.T), vb.make_workspace(shape),
                torch.empty((spec.R, spec.K_in), dtype=torch.bfloat16, device="cuda"),
                torch.empty((spec.K_out, spec.K_in), device="cuda"))

    # eager reference for draws 1..4 (host-side draw)
    want = []
    plan, ws, dX, dW = buffers()
    for d in range(1, 5):
        vb.vcas_linear_backward(shape, g, x, w, spec.rho, spec.nu, vb.Rng(spec.seed, spec.layer, d), True, plan, dX,
                                dW, ws)
        torch.cuda.synchronize()
        want.append((plan_to_numpy(plan), dX.float().cpu().numpy(), dW.cpu().numpy()))
    assert len({tuple(p["idxW"][:50]) for p, _, _ in want}) > 1          # the draws do differ

    plan, ws, dX, dW = buffers()
    counter = torch.zeros(1, dtype=torch.int32, device="cuda")
    rng = vb.Rng(spec.seed, spec.layer, 0, counter.data_ptr())
    counter.add_(1)
    vb.vcas_linear_backward(shape, g, x, w, spec.rho, spec.nu, rng, True, plan, dX, dW, ws)   # eager, offset 1
    torch.cuda.synchronize()
    assert np.array_equal(dW.cpu().numpy(), want[0][2])
    counter.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        counter.add_(1)
        vb.vcas_linear_backward(shape, g, x, w, spec.rho, spec.nu, rng, True, plan, dX, dW, ws)
    counter.zero_()
    for d in range(4):
        graph.replay()
        torch.cuda.synchronize()
        got = plan_to_numpy(plan)
        ref_plan, ref_dX, ref_dW = want[d]
        for k in ("gsq", "p", "q", "maskA", "maskW", "idxA", "idxW", "scaleW"):
            assert np.array_equal(got[k], ref_plan[k]), (d, k)
        assert got["cntA"] == ref_plan["cntA"] and got["cntW"] == ref_plan["cntW"]
        assert np.array_equal(dX.float().cpu().numpy(), ref_dX), d
        assert np.array_equal(dW.cpu().numpy(), ref_dW), d
        # eager work between replays
        _ = (torch.randn(256, 256, device="cuda") @ torch.randn(256, 256, device="cuda")).sum().item()


def test_side_stream_gives_the_same_bits_eager_and_captured():
    from paper_2402_17227_amd import binding as vb
    from tests.gpu_util import to_device, plan_to_numpy
    specs = [workloads.LayerSpec(f"side{k}", workloads.BF16, 10, 60, kin, kout, 0.6, 0.5, layer=k, seed=3, gen_seed=21,
                                 token_sigma=0.5) for k, (kin, kout) in enumerate([(264, 200), (128, 256), (200, 136)])]
    layers = []
    for spec in specs:
        G, X, W = workloads.make_layer(spec)
        shape = vb.shape_of(spec.N, spec.T, spec.K_in, spec.K_out, spec.dtype)
        layers.append(dict(spec=spec, shape=shape, g=to_device(G, spec.dtype), x=to_device(X, spec.dtype),
                           w=to_device(W, spec.dtype), plan=vb.Plan.allocate(spec.N, spec.T),
                           ws=vb.make_workspace(shape),
                           dX=torch.empty((spec.R, spec.K_in), dtype=torch.bfloat16, device="cuda"),
                           dW=torch.empty((spec.K_out, spec.K_in), device="cuda")))
    side = torch.cuda.Stream()

    def run(use_side):
        main = torch.cuda.current_stream()
        if use_side:
            side.wait_stream(main)
        for l in layers:
            s = l["spec"]
            vb.vcas_linear_backward(l["shape"], l["g"], l["x"], l["w"], s.rho, s.nu, vb.Rng(s.seed, s.layer, 4), True,
                                    l["plan"], l["dX"], l["dW"], l["ws"], side if use_side else None)
        if use_side:
            main.wait_stream(side)

    def snapshot():
        torch.cuda.synchronize()
        return [(plan_to_numpy(l["plan"]), l["dX"].float().cpu().numpy().copy(), l["dW"].cpu().numpy().copy())
                for l in layers]

    def clear():
        for l in layers:
            l["dX"].fill_(float("nan"))
            l["dW"].fill_(float("nan"))
            l["plan"].cntW.fill_(-1)

    run(False)
    want = snapshot()

    def check(got):
        for (gp, gx, gw), (wp, wx, ww) in zip(got, want):
            for k in ("gsq", "xsq", "p", "q", "maskA", "maskW", "idxA", "idxW", "scaleW", "score"):
                assert np.array_equal(gp[k], wp[k]), k
            assert gp["cntA"] == wp["cntA"] and gp["cntW"] == wp["cntW"]
            assert np.array_equal(gx, wx) and np.array_equal(gw, ww)

    clear()
    run(True)
    check(snapshot())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(True)
    for _ in range(3):
        clear()
        torch.cuda.synchronize()
        graph.replay()
        check(snapshot())


def test_stack_launch_captured_in_a_graph_matches_eager():
    """vcas_backward_stack is meant for eager launching, but a caller may still capture it: its events then
    become edges of the graph and the side streams join the capture.  Every replay must give the bits of the
    eager call with the same draw, sibling launches included."""
    from paper_2402_17227_amd import binding as vb
    from tests.gpu_util import to_device, plan_to_numpy
    mk = workloads.LayerSpec
    specs = [mk("cap0", workloads.BF16, 10, 60, 264, 200, 0.6, 0.5, layer=0, seed=5, gen_seed=31, token_sigma=0.5),
             mk("cap1", workloads.BF16, 10, 60, 136, 136, 0.5, 0.5, layer=1, seed=5, gen_seed=32, token_sigma=0.5),
             mk("cap2", workloads.BF16, 10, 60, 136, 136, 0.7, 0.5, layer=2, seed=5, gen_seed=33, token_sigma=0.5),
             mk("cap3", workloads.BF16, 10, 60, 136, 136, 0.4, 0.5, layer=3, seed=5, gen_seed=34, token_sigma=0.5),
             mk("cap4", workloads.F32, 6, 50, 72, 136, 0.6, 0.4, layer=4, seed=5, gen_seed=35, token_sigma=0.5)]
    flags = [False, False, True, True, False]
    counter = torch.zeros(1, dtype=torch.int32, device="cuda")
    layers, entries = [], []
    for spec, flag in zip(specs, flags):
        G, X, W = workloads.make_layer(spec)
        shape = vb.shape_of(spec.N, spec.T, spec.K_in, spec.K_out, spec.dtype)
        g, x, w = (to_device(a, spec.dtype) for a in (G, X, W))
        plan, ws = vb.Plan.allocate(spec.N, spec.T), vb.make_workspace(shape)
        dX = torch.empty((spec.R, spec.K_in), dtype=g.dtype, device="cuda")
        dW = torch.empty((spec.K_out, spec.K_in), device="cuda")
        layers.append((plan, dX, dW, g, x, w, ws))
        entries.append(vb.layer_args(shape, g, x, w, spec.rho, spec.nu,
                                     vb.Rng(spec.seed, spec.layer, 0, counter.data_ptr()), True, plan, dX, dW, ws,
                                     sibling=flag))
    stack = vb.make_stack(entries)
    s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()

    def step():
        main = torch.cuda.current_stream()
        counter.add_(1)
        vb.vcas_backward_stack(stack, 3, s2, s3)
        main.wait_stream(s2)
        main.wait_stream(s3)

    def snapshot():
        torch.cuda.synchronize()
        return [(plan_to_numpy(plan), dX.float().cpu().numpy().copy(), dW.cpu().numpy().copy())
                for plan, dX, dW, *_ in layers]

    def clear():
        for plan, dX, dW, *_ in layers:
            dX.fill_(float("nan"))
            dW.fill_(float("nan"))
            plan.cntW.fill_(-1)

    want = []
    for _ in range(3):                       # eager: draws 1, 2, 3
        clear()
        step()
        want.append(snapshot())
    assert any(not np.array_equal(a[0]["maskW"], b[0]["maskW"]) for a, b in zip(want[0], want[1]))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    counter.zero_()
    for d in range(3):
        clear()
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for (gp, gx, gw), (wp, wx, ww) in zip(got, want[d]):
            for k in ("gsq", "xsq", "p", "q", "maskA", "maskW", "idxA", "idxW", "scaleW", "score"):
                assert np.array_equal(gp[k], wp[k]), (d, k)
            assert gp["cntA"] == wp["cntA"] and gp["cntW"] == wp["cntW"]
            assert np.array_equal(gx, wx) and np.array_equal(gw, ww), d
        _ = (torch.randn(256, 256, device="cuda") @ torch.randn(256, 256, device="cuda")).sum().item()
