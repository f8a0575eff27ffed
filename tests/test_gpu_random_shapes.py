"""Seeded sweep over valid layer shapes: whatever N, T, K_in, K_out (multiples of 8) and keep ratios,
the three launch forms of the whole path must reproduce the oracle's sampling plan bit for bit and its
gradients within tolerance.  Shapes are drawn around the kernels' tile edges and limits (a single row, a
single 16-byte group per row, more samples than a wavefront, keep ratios that keep almost nothing)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from workloads import BF16, F32

pytestmark = pytest.mark.gpu
TOL = {F32: 1e-5, BF16: 1e-2}


@pytest.fixture(scope="module")
def vb():
    from paper_2402_17227_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def _cases(seed, count):
    rs = np.random.RandomState(seed)
    edges = [1, 2, 3, 7, 8, 9, 16, 17, 33, 40, 64, 96, 130]
    out = []
    for c in range(count):
        dtype = int(rs.randint(2))
        mode = rs.randint(4)
        if mode == 0:
            N, T = int(rs.randint(1, 5)), int(rs.randint(1, 9))
        elif mode == 1:
            N, T = int(rs.randint(1, 65)), int(rs.randint(1, 64))
        elif mode == 2:
            N, T = int(rs.randint(1, 20)), int(rs.randint(60, 400))
        else:
            N, T = int(rs.randint(60, 130)), int(rs.randint(1, 40))
        out.append(workloads.LayerSpec(
            f"rnd{seed}_{c}", dtype, N, T, 8 * int(rs.choice(edges)), 8 * int(rs.choice(edges)),
            float(rs.choice([1.0, 0.9, 0.5, 0.3, 0.1, 0.02])), float(rs.choice([1.0, 0.7, 0.5, 0.2, 0.05])),
            layer=c, seed=77 + c, gen_seed=1000 * seed + c, sample_sigma=float(rs.choice([0.0, 1.0, 2.0])),
            token_sigma=float(rs.choice([0.0, 0.5]))))
    return out


@pytest.mark.parametrize("seed", [3, 4])
def test_random_shapes_all_launch_forms(vb, seed):
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
    for sp in _cases(seed, 24):
        G, X, W = workloads.make_layer(sp)
        want, want_dX, want_dW = oracle.linear_backward(G, X, W, sp.dtype, sp.N, sp.T, sp.rho, sp.nu, sp.seed,
                                                        sp.layer, 5)
        shape = vb.shape_of(sp.N, sp.T, sp.K_in, sp.K_out, sp.dtype)
        g, x, w = (to_device(a, sp.dtype) for a in (G, X, W))
        for how in ("one stream", "side stream", "stack"):
            what = f"{sp.name} dtype={sp.dtype} N={sp.N} T={sp.T} {sp.K_in}->{sp.K_out} rho={sp.rho} nu={sp.nu}, {how}"
            plan = vb.Plan.allocate(sp.N, sp.T)
            ws = vb.make_workspace(shape)
            dX = torch.full((sp.R, sp.K_in), float("nan"), dtype=g.dtype, device="cuda")
            dW = torch.full((sp.K_out, sp.K_in), float("nan"), dtype=torch.float32, device="cuda")
            rng = vb.Rng(sp.seed, sp.layer, 5)
            if how == "one stream":
                vb.vcas_linear_backward(shape, g, x, w, sp.rho, sp.nu, rng, True, plan, dX, dW, ws)
            elif how == "side stream":
                s2.wait_stream(torch.cuda.current_stream())
                vb.vcas_linear_backward(shape, g, x, w, sp.rho, sp.nu, rng, True, plan, dX, dW, ws, s2)
            else:
                stack = vb.make_stack([vb.layer_args(shape, g, x, w, sp.rho, sp.nu, rng, True, plan, dX, dW, ws)])
                vb.vcas_backward_stack(stack, 4, s2, s3)
            torch.cuda.synchronize()
            compare_plan(plan_to_numpy(plan), want)
            dXh, dWh = from_device(dX), from_device(dW)
            assert np.isfinite(dXh).all() and np.isfinite(dWh).all(), what
            assert np.all(dXh[np.repeat(want.maskA == 0, sp.T)] == 0), what
            if want.idxA.size:
                assert rel_l2_rows(dXh, want_dX) <= TOL[sp.dtype], what
            if want.idxW.size:
                assert rel_l2_tiles(dWh, want_dW) <= TOL[sp.dtype], what
            else:
                assert np.all(dWh == 0), what


@pytest.mark.parametrize("seed", [7, 8])
def test_random_stacks_with_every_optional_field(vb, seed):
    """Seeded random stacks: 2 to 7 layers, runs of one shape with sibling flags (and a few flags on layers of
    another shape), random group size and stream count, split-K fill, cached row norms of X, SampleA-only
    layers.  Every layer must reproduce the oracle's plan bit for bit and its gradients within tolerance."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    rs = np.random.RandomState(seed)
    edges = [1, 2, 3, 8, 9, 17, 33, 40, 96]
    for c in range(8):
        L = int(rs.randint(2, 8))
        layers, shape0 = [], None
        for l in range(L):
            if shape0 is None or rs.rand() < 0.35:
                N, T = [(int(rs.randint(1, 65)), int(rs.randint(1, 64))), (int(rs.randint(1, 20)), int(rs.randint(60, 400))),
                        (int(rs.randint(60, 130)), int(rs.randint(1, 40)))][rs.randint(3)]
                shape0 = (int(rs.randint(2)), N, T, 8 * int(rs.choice(edges)), 8 * int(rs.choice(edges)))
                sibling = False
            else:
                sibling = bool(rs.rand() < 0.8)
            dtype, N, T, kin, kout = shape0
            sp = workloads.LayerSpec(f"rs{seed}_{c}_{l}", dtype, N, T, kin, kout, float(rs.choice([1.0, 0.7, 0.4, 0.1])),
                                     float(rs.choice([1.0, 0.6, 0.3])), layer=l, seed=300 + c, gen_seed=7000 + 100 * seed + 10 * c + l,
                                     sample_sigma=float(rs.choice([0.0, 1.0])), token_sigma=0.5)
            layers.append((sp, sibling, int(rs.choice([0, 1, 64, 128, 384])), bool(rs.rand() < 0.25), bool(rs.rand() < 0.85)))
        group, streams = int(rs.randint(1, 7)), int(rs.choice([1, 2, 3]))
        entries, outs, keep = [], [], []
        for sp, sibling, fill, cache_x, token_sampling in layers:
            G, X, W = workloads.make_layer(sp)
            shape = vb.shape_of(sp.N, sp.T, sp.K_in, sp.K_out, sp.dtype)
            g, x, w = (to_device(a, sp.dtype) for a in (G, X, W))
            plan, ws = vb.Plan.allocate(sp.N, sp.T), vb.make_workspace(shape)
            dX = torch.full((sp.R, sp.K_in), float("nan"), dtype=g.dtype, device="cuda")
            dW = torch.full((sp.K_out, sp.K_in), float("nan"), dtype=torch.float32, device="cuda")
            xsq_forward = None
            if cache_x:
                xsq_forward = torch.empty(sp.R, device="cuda")
                vb.vcas_row_norms(shape, None, x, None, None, xsq_forward, None)
            entries.append(vb.layer_args(shape, g, x, w, sp.rho, sp.nu, vb.Rng(sp.seed, sp.layer, 2), token_sampling, plan,
                                         dX, dW, ws, xsq_forward=xsq_forward, sibling=sibling, wgrad_fill=fill))
            outs.append((plan, dX, dW, G, X, W))
            keep.append((g, x, w, ws, xsq_forward))
        s2 = torch.cuda.Stream() if streams >= 2 else None
        s3 = torch.cuda.Stream() if streams >= 3 else None
        vb.vcas_backward_stack(vb.make_stack(entries), group, s2, s3)
        torch.cuda.synchronize()
        for (sp, sibling, fill, cache_x, token_sampling), (plan, dX, dW, G, X, W) in zip(layers, outs):
            what = (f"stack {c} group={group} streams={streams} {sp.name} dtype={sp.dtype} N={sp.N} T={sp.T} "
                    f"{sp.K_in}->{sp.K_out} rho={sp.rho} nu={sp.nu} sibling={sibling} fill={fill} cached={cache_x} "
                    f"token_sampling={token_sampling}")
            want, want_dX, want_dW = oracle.linear_backward(G, X, W, sp.dtype, sp.N, sp.T, sp.rho, sp.nu, sp.seed,
                                                            sp.layer, 2, token_sampling=token_sampling)
            compare_plan(plan_to_numpy(plan), want)
            dXh, dWh = from_device(dX), from_device(dW)
            assert np.isfinite(dXh).all() and np.isfinite(dWh).all(), what
            assert np.all(dXh[np.repeat(want.maskA == 0, sp.T)] == 0), what
            if want.idxA.size:
                assert rel_l2_rows(dXh, want_dX) <= TOL[sp.dtype], what
            if want.idxW.size:
                assert rel_l2_tiles(dWh, want_dW) <= TOL[sp.dtype], what
            else:
                assert np.all(dWh == 0), what
