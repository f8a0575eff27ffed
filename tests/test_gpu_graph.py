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
