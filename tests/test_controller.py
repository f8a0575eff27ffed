"""Adaptive keep ratios (Sec. 5): the library against the oracle.  The update rules are host
arithmetic and are checked without a GPU; the device pieces carry the gpu marker."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
import workloads
from workloads import BF16


@pytest.fixture(scope="module")
def vb():
    from paper_2402_17227_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("seed", range(8))
def test_update_rules_match_the_oracle_on_the_host(vb, seed):
    """Eq. 5, Eq. 4's running maximum and Eq. 7 through the C ABI (no launch) against oracle.controller_update."""
    rng = np.random.default_rng(seed)
    L = int(rng.integers(1, 40))
    prm = oracle.ControllerParams(alpha=float(rng.choice([0.01, 0.05])), beta=float(rng.choice([0.95, 0.5])),
                                  tau_act=0.025, tau_w=float(rng.choice([0.025, 0.5])), nu_min=1 / 64)
    cprm = vb.ControllerParams(prm.alpha, prm.beta, prm.tau_act, prm.tau_w, prm.nu_min)
    s = float(rng.choice([0.0, 0.005, 0.5, 0.995, 1.0]))
    nu = rng.choice([1 / 64, 0.02, 0.3, 0.97, 1.0], L)
    V_s = float(rng.uniform(1, 100))
    V_act = float(rng.choice([0.0, 0.02, 0.025, 0.03])) * V_s
    V_s_l = rng.uniform(1, 10, L)
    V_w = rng.choice([0.0, 0.01, prm.tau_w, 1.0], L) * V_s_l
    pm, pp = rng.uniform(0, 1, L), rng.uniform(0, 1, L)
    want = oracle.controller_update(prm, s, nu, V_s, V_act, V_w, V_s_l, pm, pp)
    got = vb.vcas_controller_update(cprm, s, nu, V_s, V_act, V_w, V_s_l, pm, pp)
    assert got[0] == want[0]
    assert np.array_equal(np.array(got[1]), want[1]) and np.array_equal(np.array(got[2]), want[2])


def test_update_rules_reject_bad_parameters(vb):
    bad = vb.ControllerParams(0.01, 1.5, 0.025, 0.025, 0.01)       # beta must lie in (0, 1)
    with pytest.raises(vb.VcasError):
        vb.vcas_controller_update(bad, 0.5, [0.5], 1.0, 1.0, [1.0], [1.0], [0.5], [0.5])


# ---- device pieces --------------------------------------------------------------------------------

@pytest.mark.gpu
@pytest.mark.parametrize("N,sigma,zero_frac", [(1, 1.0, 0.0), (8, 0.0, 0.0), (32, 1.0, 0.0), (64, 1.5, 0.3),
                                               (197, 1.0, 0.1), (1000, 2.0, 0.5), (1024, 1.0, 0.0)])
def test_sparsity_ratio_bit_exact(vb, N, sigma, zero_frac):
    import torch
    rng = np.random.default_rng(N)
    a = np.exp(sigma * rng.standard_normal(N)).astype(np.float32)
    a[rng.uniform(size=N) < zero_frac] = 0
    if N == 8:
        a[:] = 2.5                                                   # all equal: ties everywhere
    levels = [0.0, 0.1, 0.5, 0.79, 0.8, 0.81, 0.999, 1.0]
    out = torch.full((len(levels),), float("nan"), device="cuda")
    vb.vcas_sparsity_ratio(torch.from_numpy(a).cuda(), levels, out)
    torch.cuda.synchronize()
    want = np.array([oracle.sparsity_ratio(a, s) for s in levels], np.float32)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32))


@pytest.mark.gpu
def test_sparsity_ratio_of_a_real_plan(vb):
    """Eq. 4 on the norms the sampled backward itself produced (BERT-base layer, N = 32)."""
    import torch
    from tests.gpu_util import run_layer_gpu
    spec = workloads.LayerSpec("ctl", BF16, 32, 128, 768, 768, 0.5, 0.5, layer=3, seed=1, gen_seed=2, token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    plan, _, _ = run_layer_gpu(spec, G, X, W, want_dX=False, want_dW=False)
    gn = oracle.sample_norms(oracle.row_sumsq(G, BF16), spec.N, spec.T)      # the oracle's own norms ...
    assert np.array_equal(plan["gnorm"].view(np.uint32), gn.view(np.uint32))  # ... which are the library's, bit for bit
    out = torch.empty(2, device="cuda")
    vb.vcas_sparsity_ratio(torch.from_numpy(plan["gnorm"]).cuda(), [0.79, 0.81], out)
    torch.cuda.synchronize()
    want = [oracle.sparsity_ratio(gn, s) for s in (0.79, 0.81)]
    assert out.cpu().tolist() == want and want[0] <= want[1]


@pytest.mark.gpu
@pytest.mark.parametrize("n,stride", [(1000, 1), (768 * 768, 100), (5, 7), (123457, 101)])
def test_gradient_statistics_match_the_oracle(vb, n, stride):
    import torch
    rng = np.random.default_rng(n)
    M = 5
    m = (n + stride - 1) // stride
    mean_o, sq_o = np.zeros(m, np.float32), np.zeros(m, np.float32)
    mean_g, sq_g = torch.zeros(m, device="cuda"), torch.zeros(m, device="cuda")
    first = None
    acc = torch.zeros(1, dtype=torch.float64, device="cuda")
    want_acc = 0.0
    for i in range(1, M + 1):
        g = (rng.standard_normal(n) * (0.5 + i)).astype(np.float32)
        gd = torch.from_numpy(g).cuda()
        oracle.grad_stats_update(g, stride, i, mean_o, sq_o)
        vb.vcas_grad_stats_update(gd, m, stride, i, mean_g, sq_g)
        if first is None:
            first, first_d = g, gd
        else:                                                        # V_act-style accumulation against the first one
            vb.vcas_sq_diff_strided(gd, first_d, m, stride, 1.0 / (M - 1), i > 2, acc)
            want_acc += oracle.sq_diff_strided(g, first, m, stride) / (M - 1)
    out = torch.empty(1, dtype=torch.float64, device="cuda")
    vb.vcas_grad_stats_variance(mean_g, sq_g, M, out)
    torch.cuda.synchronize()
    # elementwise updates are the same fp32 operations: bit for bit; the fp64 sums differ in order only
    assert np.array_equal(mean_g.cpu().numpy().view(np.uint32), mean_o.view(np.uint32))
    assert np.array_equal(sq_g.cpu().numpy().view(np.uint32), sq_o.view(np.uint32))
    assert float(out.item()) == pytest.approx(oracle.grad_stats_variance(mean_o, sq_o, M), rel=1e-9)
    assert float(acc.item()) == pytest.approx(want_acc, rel=1e-9)


@pytest.mark.gpu
def test_controller_trajectory_on_a_stream_of_batches(vb):
    """Alg. 1 end to end on a three-layer stack and a synthetic stream of batches: every F-th
    iteration the probe quantities are measured with the library (M batches, M mask draws each,
    1/8 of the parameters kept for the statistics) and with the oracle, and both feed their own
    controller.  The two trajectories of s, rho_l and nu_l must coincide."""
    import torch
    from tests.gpu_util import to_device
    L, M, stride, updates = 3, 2, 8, 3
    N, T, K = 16, 32, 64
    prm = oracle.ControllerParams(alpha=0.05, beta=0.8, tau_act=0.05, tau_w=0.05, nu_min=1 / 16)
    cprm = vb.ControllerParams(prm.alpha, prm.beta, prm.tau_act, prm.tau_w, prm.nu_min)
    state_o = dict(s=1.0, rho=np.ones(L), nu=np.ones(L))
    state_g = dict(s=1.0, rho=[1.0] * L, nu=[1.0] * L)
    shape = vb.shape_of(N, T, K, K, BF16)
    m = (K * K + stride - 1) // stride
    margins = []
    for upd in range(updates):
        # ---- oracle side and GPU side measure the same quantities on the same batches --------
        Vs_l_o, Vs_l_g = np.zeros(L), np.zeros(L)
        Vact_o = Vact_g = 0.0
        Vw_o, Vw_g = np.zeros(L), np.zeros(L)
        pm_o, pp_o, pm_g, pp_g = np.zeros(L), np.zeros(L), np.zeros(L), np.zeros(L)
        lo, hi = max(0.0, state_o["s"] - prm.alpha), min(1.0, state_o["s"] + prm.alpha)
        for l in range(L):
            mean_o, sq_o = np.zeros(m, np.float32), np.zeros(m, np.float32)
            mean_g, sq_g = torch.zeros(m, device="cuda"), torch.zeros(m, device="cuda")
            for i in range(M):                                        # M batches
                spec = workloads.LayerSpec(f"ctl{l}", BF16, N, T, K, K, float(state_o["rho"][l]),
                                           float(state_o["nu"][l]), layer=l, seed=5,
                                           gen_seed=1000 * upd + 10 * i + l, sample_sigma=1.0 + 0.5 * l,
                                           token_sigma=0.5)
                G, X, W = workloads.make_layer(spec)
                g, x = to_device(G, BF16), to_device(X, BF16)
                # oracle
                exact = oracle.exact_wgrad(G, X, BF16).astype(np.float32)
                oracle.grad_stats_update(exact, stride, i + 1, mean_o, sq_o)
                probe_o = oracle.variance_probe(G, X, BF16, N, T, spec.rho, spec.nu, spec.seed, l, 10 * upd, M)
                gn = oracle.sample_norms(oracle.row_sumsq(G, BF16), N, T)
                pm_o[l] += oracle.sparsity_ratio(gn, lo) / M
                pp_o[l] += oracle.sparsity_ratio(gn, hi) / M
                Vact_o += probe_o[2] / M
                Vw_o[l] += probe_o[1] / M
                # library
                plan = vb.Plan.allocate(N, T)
                ws = vb.make_workspace(shape)
                dW = torch.empty((K, K), device="cuda")
                vb.vcas_linear_backward(shape, g, x, None, 1.0, 1.0, vb.Rng(spec.seed, l, 0), True, plan, None, dW, ws)
                vb.vcas_grad_stats_update(dW, m, stride, i + 1, mean_g, sq_g)
                out = torch.empty(4, dtype=torch.float64, device="cuda")
                vb.vcas_variance_probe(shape, g, x, spec.rho, spec.nu, vb.Rng(spec.seed, l, 10 * upd), M, plan, out, ws)
                pr = torch.empty(2, device="cuda")
                vb.vcas_sparsity_ratio(plan.gnorm, [lo, hi], pr)
                torch.cuda.synchronize()
                assert np.array_equal(plan.gnorm.cpu().numpy(), gn)
                pm_g[l] += float(pr[0]) / M
                pp_g[l] += float(pr[1]) / M
                Vact_g += float(out[2]) / M
                Vw_g[l] += float(out[1]) / M
            Vs_l_o[l] = oracle.grad_stats_variance(mean_o, sq_o, M)
            v = torch.empty(1, dtype=torch.float64, device="cuda")
            vb.vcas_grad_stats_variance(mean_g, sq_g, M, v)
            Vs_l_g[l] = float(v.item())
        np.testing.assert_allclose(Vs_l_g, Vs_l_o, rtol=2e-2)          # dW in bf16 on the GPU, fp64 in the oracle
        assert np.array_equal(pm_g, pm_o) and np.array_equal(pp_g, pp_o)
        # the decisions are signs: record how far from zero they are, the test is only meaningful
        # (and only stable) when the margins dwarf the tolerance of the measured variances
        margins.append(abs(Vact_o - prm.tau_act * Vs_l_o.sum()) / (prm.tau_act * Vs_l_o.sum()))
        margins += list(np.abs(Vw_o - prm.tau_w * Vs_l_o) / (prm.tau_w * Vs_l_o))
        so, ro, no = oracle.controller_update(prm, state_o["s"], state_o["nu"], Vs_l_o.sum(), Vact_o, Vw_o, Vs_l_o,
                                              pm_o, pp_o)
        sg, rg, ng = vb.vcas_controller_update(cprm, state_g["s"], state_g["nu"], float(Vs_l_g.sum()), Vact_g, Vw_g,
                                               Vs_l_g, pm_g, pp_g)
        state_o = dict(s=so, rho=np.maximum(ro, 1.0 / N), nu=no)
        state_g = dict(s=sg, rho=[max(r, 1.0 / N) for r in rg], nu=ng)
        assert state_g["s"] == state_o["s"]
        assert np.array_equal(np.array(state_g["rho"]), state_o["rho"])
        assert np.array_equal(np.array(state_g["nu"]), state_o["nu"])
    assert min(margins) > 0.1, margins
