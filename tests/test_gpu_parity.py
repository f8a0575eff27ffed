"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Bit-exact for norms, probabilities, masks, index
lists and scales; rel-L2 <= 1e-5 (fp32) / 1e-2 (bf16 in, fp32 accumulate) for
dX and dW."""
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
    return binding


def _bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def _dev(a, dtype=None):
    from tests.gpu_util import to_device
    if dtype is None:
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return to_device(a, dtype)


# ------------------------------------------------------------ single calls

@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("N,T,K", [(3, 7, 8), (4, 33, 136), (8, 128, 768), (2, 197, 1024), (3, 50, 3072),
                                   (2, 64, 4096), (1, 70, 8200)])
def test_row_norms_bit_exact(vb, dtype, N, T, K):
    rng = np.random.default_rng(N * 1000 + K)
    R = N * T
    a = (rng.standard_normal((R, K)) * np.exp(rng.standard_normal((R, 1)))).astype(np.float32)
    A = workloads.f32_to_bf16_bits(a) if dtype == BF16 else a
    keep = (rng.random(N) < 0.6).astype(np.uint8)
    shape = vb.shape_of(N, T, K, K, dtype)
    gsq = torch.empty(R, device="cuda")
    xsq = torch.empty(R, device="cuda")
    gnorm = torch.empty(N, device="cuda")
    d = _dev(A, dtype)
    vb.vcas_row_norms(shape, d, d, _dev(keep), gsq, xsq, gnorm)
    torch.cuda.synchronize()
    want_g = oracle.row_sumsq(A, dtype)
    assert np.array_equal(_bits(gsq.cpu().numpy()), _bits(want_g))
    assert np.array_equal(_bits(xsq.cpu().numpy()), _bits(oracle.row_sumsq(A, dtype, T, keep)))
    assert np.array_equal(_bits(gnorm.cpu().numpy()), _bits(oracle.sample_norms(want_g, N, T)))


@pytest.mark.parametrize("n,rho,sigma,zero_frac", [(1, 0.5, 1.0, 0.0), (8, 0.5, 1.0, 0.0), (64, 0.3, 1.5, 0.1),
                                                   (1000, 0.9, 2.0, 0.0), (4096, 0.25, 1.0, 0.05),
                                                   (16384, 0.2, 1.2, 0.3), (12608, 0.15, 0.7, 0.7),
                                                   (70000, 0.05, 1.0, 0.0), (50, 1.0, 1.0, 0.2)])
def test_keep_probs_bit_exact(vb, n, rho, sigma, zero_frac):
    rng = np.random.default_rng(n)
    a = np.exp(sigma * rng.standard_normal(n)).astype(np.float32)
    a[rng.random(n) < zero_frac] = 0.0
    prob = torch.full((n,), -1.0, device="cuda")
    vb.vcas_keep_probs(_dev(a), n, n * rho, prob)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(prob.cpu().numpy()), _bits(oracle.keep_probs(a, n * rho)))


def test_keep_probs_degenerate_inputs(vb):
    for a, budget in [(np.zeros(100, np.float32), 10.0), (np.full(77, 2.5, np.float32), 77 * 0.35),
                      (np.array([1e6, 1, 2, 3, 4], np.float32), 2.0), (np.array([10, 6, 1, 1, 1, 1], np.float32), 3.0),
                      (np.array([3.0], np.float32), 0.0)]:
        prob = torch.full((a.size,), -1.0, device="cuda")
        vb.vcas_keep_probs(_dev(a), a.size, budget, prob)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(prob.cpu().numpy()), _bits(oracle.keep_probs(a, budget)))


@pytest.mark.parametrize("n", [1, 63, 64, 1000, 4096, 16384, 100003])
@pytest.mark.parametrize("stream_id", [0, 1])
def test_sample_compact_bit_exact(vb, n, stream_id):
    rng = np.random.default_rng(n + stream_id)
    prob = rng.random(n).astype(np.float32)
    prob[rng.random(n) < 0.1] = 1.0
    prob[rng.random(n) < 0.1] = 0.0
    seed, layer, draw = 0x0123456789ABCDEF + n, 41, 7
    mask = torch.full((n,), 9, dtype=torch.uint8, device="cuda")
    idx = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    vb.vcas_sample_compact(_dev(prob), n, vb.Rng(seed, layer, draw), stream_id, mask, idx, cnt)
    torch.cuda.synchronize()
    want_mask, want_idx = oracle.sample_mask(prob, seed, layer, stream_id, draw)
    assert np.array_equal(mask.cpu().numpy(), want_mask)
    assert int(cnt.item()) == want_idx.size
    got_idx = idx.cpu().numpy()
    assert np.array_equal(got_idx[:want_idx.size], want_idx)
    assert np.all(got_idx[want_idx.size:] == -7)          # entries past the count are left alone


def test_philox_known_answer_on_device(vb):
    # Row 5 of (layer 3, stream 1, draw 0, seed 0) is the fourth published-format known answer:
    # word 0 = dd3c661d, so u = 0xdd3c66 / 2^24.  Thresholds one ulp apart on either side pin it.
    u = np.float32(0xDD3C66 / 2.0**24)
    for thr, want in [(np.nextafter(u, np.float32(1)), 1), (u, 0)]:
        prob = np.zeros(8, np.float32)
        prob[5] = thr
        mask = torch.empty(8, dtype=torch.uint8, device="cuda")
        idx = torch.empty(8, dtype=torch.int32, device="cuda")
        cnt = torch.empty(1, dtype=torch.int32, device="cuda")
        vb.vcas_sample_compact(_dev(prob), 8, vb.Rng(0, 3, 0), 1, mask, idx, cnt)
        torch.cuda.synchronize()
        assert int(mask[5].item()) == want and int(cnt.item()) == want


def test_leverage_scores_and_row_scale_bit_exact(vb):
    # wide dynamic range: exercises the correctly rounded sqrt and divide
    rng = np.random.default_rng(17)
    N, T = 37, 113
    R = N * T
    gsq = np.exp(8 * rng.standard_normal(R)).astype(np.float32)
    xsq = np.exp(8 * rng.standard_normal(R)).astype(np.float32)
    gsq[:50] = 0
    p = rng.uniform(1e-4, 1, N).astype(np.float32)
    p[:5] = 1.0
    maskA = (rng.random(N) < 0.7).astype(np.uint8)
    shape = vb.shape_of(N, T, 8, 8, F32)
    score = torch.empty(R, device="cuda")
    vb.vcas_leverage_scores(shape, _dev(gsq), _dev(xsq), _dev(p), _dev(maskA), score)
    q = rng.uniform(1e-5, 1, R).astype(np.float32)
    maskW = (rng.random(R) < 0.5).astype(np.uint8)
    scale = torch.empty(R, device="cuda")
    vb.vcas_row_scale(shape, _dev(p), _dev(q), _dev(maskW), scale)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(score.cpu().numpy()), _bits(oracle.leverage_scores(gsq, xsq, p, maskA, N, T)))
    assert np.array_equal(_bits(scale.cpu().numpy()), _bits(oracle.row_scale(p, q, maskW, N, T)))


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("N,T,kin,kout,keep", [(4, 40, 136, 264, [1, 0, 1, 1]), (3, 197, 320, 200, [0, 1, 0]),
                                               (6, 64, 128, 128, [1, 1, 1, 1, 1, 1]), (5, 30, 64, 72, [0, 0, 0, 0, 0]),
                                               (9, 130, 768, 256, [0, 1, 1, 0, 0, 0, 1, 0, 1])])
def test_dgrad_with_given_mask(vb, dtype, N, T, kin, kout, keep):
    rng = np.random.default_rng(kin + kout)
    R = N * T
    g = rng.standard_normal((R, kout)).astype(np.float32)
    w = (rng.standard_normal((kout, kin)) * 0.05).astype(np.float32)
    G, W = (workloads.f32_to_bf16_bits(a) if dtype == BF16 else a for a in (g, w))
    p = rng.uniform(0.2, 1, N).astype(np.float32)
    maskA = np.array(keep, np.uint8)
    idxA = np.nonzero(maskA)[0].astype(np.int32)
    idx_buf = np.full(N, -1, np.int32)
    idx_buf[:idxA.size] = idxA
    shape = vb.shape_of(N, T, kin, kout, dtype)
    dX = torch.full((R, kin), float("nan"), dtype=torch.bfloat16 if dtype == BF16 else torch.float32, device="cuda")
    vb.vcas_sampled_dgrad(shape, _dev(G, dtype), _dev(W, dtype), _dev(p), _dev(idx_buf),
                          _dev(np.array([idxA.size], np.int32)), dX)
    torch.cuda.synchronize()
    from tests.gpu_util import from_device, rel_l2, rel_l2_rows, rel_l2_tiles
    got = from_device(dX)
    want = oracle.dgrad(G, W, dtype, N, T, p, maskA)
    assert np.isfinite(got).all()
    assert np.all(got[np.repeat(maskA == 0, T)] == 0)
    if idxA.size:
        assert rel_l2_rows(got, want) <= TOL[dtype]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("N,T,kin,kout", [(6, 40, 136, 136), (9, 64, 768, 200), (5, 33, 72, 72)])
def test_dgrad_never_reads_rows_of_dropped_samples(vb, dtype, N, T, kin, kout):
    """Rows of G that belong to dropped samples hold NaN: nothing of them may reach dX, not even through
    the zero-padded tail of a ragged contraction (K_out not a multiple of the step), where a row's last
    pieces are followed in memory by the next row."""
    rng = np.random.default_rng(kin * 7 + kout)
    R = N * T
    g = rng.standard_normal((R, kout)).astype(np.float32)
    w = (rng.standard_normal((kout, kin)) * 0.05).astype(np.float32)
    p = rng.uniform(0.2, 1, N).astype(np.float32)
    maskA = np.array([(i % 2) == 0 for i in range(N)], np.uint8)           # every kept sample has a dropped neighbour
    G, W = (workloads.f32_to_bf16_bits(a) if dtype == BF16 else a for a in (g, w))
    idxA = np.nonzero(maskA)[0].astype(np.int32)
    idx_buf = np.full(N, -1, np.int32)
    idx_buf[:idxA.size] = idxA
    g_dev = _dev(G, dtype).clone()
    g_dev[torch.from_numpy(np.repeat(maskA == 0, T)).cuda()] = float("nan")
    shape = vb.shape_of(N, T, kin, kout, dtype)
    dX = torch.full((R, kin), float("nan"), dtype=torch.bfloat16 if dtype == BF16 else torch.float32, device="cuda")
    vb.vcas_sampled_dgrad(shape, g_dev, _dev(W, dtype), _dev(p), _dev(idx_buf), _dev(np.array([idxA.size], np.int32)), dX)
    torch.cuda.synchronize()
    from tests.gpu_util import from_device, rel_l2, rel_l2_rows, rel_l2_tiles
    got = from_device(dX)
    assert np.isfinite(got).all()
    assert np.all(got[np.repeat(maskA == 0, T)] == 0)
    assert rel_l2_rows(got, oracle.dgrad(G, W, dtype, N, T, p, maskA)) <= TOL[dtype]


@pytest.mark.parametrize("N,T,kin,kout,frac", [(17, 128, 2040, 136, 1.0),     # 128x128 tiles, ragged columns
                                                (17, 128, 2040, 136, 0.6),
                                                (33, 125, 3080, 200, 1.0),     # 256x256 tiles, ragged rows and columns
                                                (33, 125, 3080, 200, 0.5),
                                                (33, 125, 3080, 8, 1.0),       # 256x256 tiles, a single ragged contraction step
                                                (33, 125, 3080, 64, 1.0),      # ... exactly one step
                                                (33, 125, 3080, 72, 0.5),      # ... two steps, the second ragged
                                                (33, 125, 3080, 192, 1.0),     # ... three steps
                                                (17, 128, 1024, 72, 1.0),      # 64x128 tiles, two stages
                                                (1100, 4, 264, 72, 0.7)])     # more kept samples than are staged in LDS
def test_dgrad_bf16_tile_variants(vb, N, T, kin, kout, frac):
    """Every tile shape the bf16 dgrad launcher can choose, against the oracle (Eq. 2, upper line)."""
    rng = np.random.default_rng(N * 1000 + kin)
    R = N * T
    G = workloads.f32_to_bf16_bits(rng.standard_normal((R, kout)).astype(np.float32))
    W = workloads.f32_to_bf16_bits((rng.standard_normal((kout, kin)) * 0.05).astype(np.float32))
    p = rng.uniform(0.2, 1, N).astype(np.float32)
    maskA = (rng.uniform(size=N) < frac).astype(np.uint8)
    idxA = np.nonzero(maskA)[0].astype(np.int32)
    idx_buf = np.full(N, -1, np.int32)
    idx_buf[:idxA.size] = idxA
    shape = vb.shape_of(N, T, kin, kout, BF16)
    dX = torch.full((R, kin), float("nan"), dtype=torch.bfloat16, device="cuda")
    vb.vcas_sampled_dgrad(shape, _dev(G, BF16), _dev(W, BF16), _dev(p), _dev(idx_buf),
                          _dev(np.array([idxA.size], np.int32)), dX)
    torch.cuda.synchronize()
    from tests.gpu_util import from_device, rel_l2, rel_l2_rows, rel_l2_tiles
    got = from_device(dX)
    want = oracle.dgrad(G, W, BF16, N, T, p, maskA)
    assert np.isfinite(got).all()
    assert np.all(got[np.repeat(maskA == 0, T)] == 0)
    # every row on its own, so that a misplaced tile cannot hide in the global norm
    assert rel_l2_rows(got, want) <= TOL[BF16]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("R,kin,kout,frac", [(300, 136, 264, 0.5), (1000, 128, 128, 1.0), (70, 64, 72, 0.0),
                                             (5000, 256, 384, 0.3), (4096, 768, 768, 0.05), (130, 768, 256, 0.7)])
def test_wgrad_with_given_rows(vb, dtype, R, kin, kout, frac):
    rng = np.random.default_rng(R + kin)
    g = rng.standard_normal((R, kout)).astype(np.float32)
    x = rng.standard_normal((R, kin)).astype(np.float32)
    G, X = (workloads.f32_to_bf16_bits(a) if dtype == BF16 else a for a in (g, x))
    keep = rng.random(R) < frac
    scale = np.where(keep, rng.uniform(1, 8, R), 0).astype(np.float32)
    idx = np.nonzero(keep)[0].astype(np.int32)
    idx_buf = np.full(R, -1, np.int32)
    idx_buf[:idx.size] = idx
    shape = vb.shape_of(1, R, kin, kout, dtype)
    ws = vb.make_workspace(shape)
    from tests.gpu_util import from_device, rel_l2, rel_l2_rows, rel_l2_tiles
    want = oracle.wgrad(G, X, dtype, scale)
    for rep in range(2):                                   # second call: counters were left at zero
        dW = torch.full((kout, kin), float("nan"), device="cuda")
        vb.vcas_sampled_wgrad(shape, _dev(G, dtype), _dev(X, dtype), _dev(scale), _dev(idx_buf),
                              _dev(np.array([idx.size], np.int32)), dW, ws)
        torch.cuda.synchronize()
        got = from_device(dW)
        assert np.isfinite(got).all()
        if idx.size == 0:
            assert np.all(got == 0)
        else:
            assert rel_l2_tiles(got, want) <= TOL[dtype]
            assert rel_l2_tiles(got, want, 64) <= 2 * TOL[dtype]      # the small kernel's tile


# ---------------------------------------------------------- the whole path

@pytest.mark.parametrize("spec", workloads.small_cases(), ids=lambda s: f"{s.name}-{'bf16' if s.dtype else 'f32'}")
def test_linear_backward_small_cases(vb, spec):
    from tests.gpu_util import run_layer_gpu, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    G, X, W = workloads.make_layer(spec)
    got_plan, dX, dW = run_layer_gpu(spec, G, X, W, draw=3)
    want_plan, want_dX, want_dW = oracle.linear_backward(G, X, W, spec.dtype, spec.N, spec.T, spec.rho, spec.nu,
                                                         spec.seed, spec.layer, 3)
    compare_plan(got_plan, want_plan)
    assert np.isfinite(dX).all() and np.isfinite(dW).all()
    assert np.all(dX[np.repeat(want_plan.maskA == 0, spec.T)] == 0)
    if want_plan.idxA.size:
        assert rel_l2_rows(dX, want_dX) <= TOL[spec.dtype]
    if want_plan.idxW.size:
        assert rel_l2_tiles(dW, want_dW) <= TOL[spec.dtype]
    else:
        assert np.all(dW == 0)


@pytest.mark.parametrize("N,T", [(20, 1000), (1100, 3), (33, 500)])
def test_linear_backward_long_vectors(vb, N, T):
    # more rows than the register-resident samplers hold (R > 16384) and more samples than 1024
    from tests.gpu_util import run_layer_gpu, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    spec = workloads.LayerSpec("long", BF16, N, T, 64, 72, 0.4, 0.5, layer=2, seed=9, gen_seed=12, token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    got_plan, dX, dW = run_layer_gpu(spec, G, X, W, draw=2)
    want_plan, want_dX, want_dW = oracle.linear_backward(G, X, W, spec.dtype, spec.N, spec.T, spec.rho, spec.nu,
                                                         spec.seed, spec.layer, 2)
    compare_plan(got_plan, want_plan)
    assert rel_l2_rows(dX, want_dX) <= TOL[BF16] and rel_l2_tiles(dW, want_dW) <= TOL[BF16]


def test_linear_backward_long_vectors_with_a_large_x(vb):
    # R > 16384 AND X above 16 MiB: the norms of X are taken after SampleA, on kept samples, by the
    # launch that also writes the SampleW scores, and the long-vector SampleW kernel takes them as given
    from tests.gpu_util import run_layer_gpu, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    spec = workloads.LayerSpec("long_x", BF16, 40, 500, 448, 72, 0.5, 0.5, layer=4, seed=13, gen_seed=3, token_sigma=0.5)
    assert spec.N * spec.T * spec.K_in * 2 > 16 << 20
    G, X, W = workloads.make_layer(spec)
    got_plan, dX, dW = run_layer_gpu(spec, G, X, W, draw=1)
    want_plan, want_dX, want_dW = oracle.linear_backward(G, X, W, spec.dtype, spec.N, spec.T, spec.rho, spec.nu,
                                                         spec.seed, spec.layer, 1)
    compare_plan(got_plan, want_plan)
    assert rel_l2_rows(dX, want_dX) <= TOL[BF16] and rel_l2_tiles(dW, want_dW) <= TOL[BF16]


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_keep_ratio_one_is_the_dense_backward(vb, dtype):
    from tests.gpu_util import run_layer_gpu, rel_l2, rel_l2_rows, rel_l2_tiles
    spec = workloads.LayerSpec("dense", dtype, 7, 45, 200, 136, 1.0, 1.0, layer=9, seed=3, gen_seed=8, token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    plan, dX, dW = run_layer_gpu(spec, G, X, W)
    assert plan["cntA"] == spec.N and plan["cntW"] == spec.R
    assert np.all(plan["p"] == 1) and np.all(plan["q"] == 1) and np.all(plan["scaleW"] == 1)
    g, x, w = (oracle.to_f64(a, dtype) for a in (G, X, W))
    assert rel_l2_rows(dX, g @ w) <= TOL[dtype]
    assert rel_l2_tiles(dW, g.T @ x) <= TOL[dtype]


def test_all_zero_gradient_keeps_nothing(vb):
    from tests.gpu_util import run_layer_gpu
    spec = workloads.LayerSpec("zero", BF16, 4, 20, 64, 72, 0.5, 0.5, layer=1, seed=1, gen_seed=1)
    G, X, W = workloads.make_layer(spec)
    G[:] = 0
    plan, dX, dW = run_layer_gpu(spec, G, X, W)
    assert plan["cntA"] == 0 and plan["cntW"] == 0
    assert np.all(dX == 0) and np.all(dW == 0)


def test_sample_a_only_backward(vb):
    from tests.gpu_util import run_layer_gpu, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    spec = workloads.LayerSpec("aonly", BF16, 9, 33, 136, 200, 0.5, 0.5, layer=6, seed=21, gen_seed=5, token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    got_plan, dX, dW = run_layer_gpu(spec, G, X, W, draw=1, token_sampling=False)
    want_plan, want_dX, want_dW = oracle.linear_backward(G, X, W, spec.dtype, spec.N, spec.T, spec.rho, spec.nu,
                                                         spec.seed, spec.layer, 1, token_sampling=False)
    compare_plan(got_plan, want_plan)
    assert rel_l2_rows(dX, want_dX) <= 1e-2 and rel_l2_tiles(dW, want_dW) <= 1e-2


def test_sample_a_only_siblings_in_a_stack(vb):
    """The SampleA-only backward (Alg. 1: no token sampling) through the shared launches of sibling layers,
    and a run of siblings in which the kind of sampling changes (which ends the shared SampleW launch)."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    kinds = [False, False, False, True]
    entries, outs, host, keep = [], [], [], []
    for k, ts in enumerate(kinds):
        sp = workloads.LayerSpec(f"ao{k}", BF16, 9, 40, 136, 200, 0.4 + 0.1 * k, 0.5, layer=k, seed=22, gen_seed=60 + k,
                                 token_sigma=0.5)
        G, X, W = workloads.make_layer(sp)
        shape = vb.shape_of(sp.N, sp.T, sp.K_in, sp.K_out, sp.dtype)
        g, x, w = (to_device(a, BF16) for a in (G, X, W))
        plan, ws = vb.Plan.allocate(sp.N, sp.T), vb.make_workspace(shape)
        dX = torch.full((sp.R, sp.K_in), float("nan"), dtype=torch.bfloat16, device="cuda")
        dW = torch.full((sp.K_out, sp.K_in), float("nan"), dtype=torch.float32, device="cuda")
        entries.append(vb.layer_args(shape, g, x, w, sp.rho, sp.nu, vb.Rng(sp.seed, sp.layer, 1), ts, plan, dX, dW, ws,
                                     sibling=k > 0))
        outs.append((sp, ts, plan, dX, dW))
        host.append((G, X, W))
        keep.append((g, x, w, ws))
    s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
    vb.vcas_backward_stack(vb.make_stack(entries), 4, s2, s3)
    torch.cuda.synchronize()
    for (sp, ts, plan, dX, dW), (G, X, W) in zip(outs, host):
        want, want_dX, want_dW = oracle.linear_backward(G, X, W, sp.dtype, sp.N, sp.T, sp.rho, sp.nu, sp.seed, sp.layer, 1,
                                                        token_sampling=ts)
        compare_plan(plan_to_numpy(plan), want)
        assert rel_l2_rows(from_device(dX), want_dX) <= 1e-2 and rel_l2_tiles(from_device(dW), want_dW) <= 1e-2


def test_results_are_reproducible(vb):
    from tests.gpu_util import run_layer_gpu
    spec = workloads.LayerSpec("repro", BF16, 8, 128, 768, 768, 0.5, 0.5, layer=2, seed=5, gen_seed=6, token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    a = run_layer_gpu(spec, G, X, W)
    b = run_layer_gpu(spec, G, X, W)
    assert np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    assert np.array_equal(a[0]["idxW"], b[0]["idxW"])


@pytest.mark.parametrize("spec", [
    workloads.LayerSpec("halves_small", BF16, 8, 128, 768, 264, 0.5, 0.5, layer=3, seed=7, gen_seed=8, token_sigma=0.5),
    workloads.LayerSpec("halves_f32", F32, 6, 50, 72, 136, 0.6, 0.4, layer=1, seed=2, gen_seed=3, token_sigma=0.5),
    # rows of X too many bytes for the joint norm launch: the weight half takes the X norms itself
    workloads.LayerSpec("halves_large", BF16, 12, 300, 4096, 64, 0.5, 0.5, layer=5, seed=9, gen_seed=1, token_sigma=0.5),
], ids=lambda s: s.name)
def test_data_and_weight_halves_equal_the_whole(vb, spec):
    """vcas_backward_data + vcas_backward_weight give the bits of vcas_linear_backward (Sec. 4.1, 4.2)."""
    from tests.gpu_util import run_layer_gpu, to_device, plan_to_numpy, from_device
    G, X, W = workloads.make_layer(spec)
    whole_plan, whole_dX, whole_dW = run_layer_gpu(spec, G, X, W, draw=3)
    shape = vb.shape_of(spec.N, spec.T, spec.K_in, spec.K_out, spec.dtype)
    g, x, w = (to_device(a, spec.dtype) for a in (G, X, W))
    plan = vb.Plan.allocate(spec.N, spec.T)
    ws = vb.make_workspace(shape)
    dX = torch.full((spec.R, spec.K_in), float("nan"), dtype=g.dtype, device="cuda")
    dW = torch.full((spec.K_out, spec.K_in), float("nan"), dtype=torch.float32, device="cuda")
    rng = vb.Rng(spec.seed, spec.layer, 3)
    vb.vcas_backward_data(shape, g, x, w, spec.rho, rng, True, plan, dX, ws)
    vb.vcas_backward_weight(shape, g, x, spec.rho, spec.nu, rng, True, plan, dW, ws)
    torch.cuda.synchronize()
    halves = plan_to_numpy(plan)
    for k, v in whole_plan.items():
        assert np.array_equal(np.asarray(v), np.asarray(halves[k])), k
    assert np.array_equal(from_device(dX), whole_dX) and np.array_equal(from_device(dW), whole_dW)


def _to_layer_dtype(a64, dtype):
    """fp64 values -> the layer's storage (fp32, or bf16 bit patterns): how a tensor the oracle computed
    becomes the next layer's input."""
    a32 = np.asarray(a64, np.float64).astype(np.float32)
    return workloads.f32_to_bf16_bits(a32) if dtype == BF16 else a32


def _oracle_chain(dtype, N, T, G_top, layers, nu, seed, draw=0):
    """A chain of layers computed by the oracle alone: layer l's G is the oracle's own dX of layer l-1
    (times the Jacobian, if any), stored in the layer dtype, zero on dropped samples.  layers: list of
    (X, W, J or None, rho).  Returns per layer (G, plan, dX fp64, dW fp64).  Nothing here comes from the GPU:
    the GPU is then fed these G and compared with these results."""
    out = []
    G = G_top
    for l, (X, W, J, rho) in enumerate(layers):
        plan, dX, dW = oracle.linear_backward(G, X, W, dtype, N, T, rho, nu, seed, l, draw)
        if J is not None:
            dX = oracle.dgrad_jacobian(G, W, J, dtype, N, T, plan.p, plan.maskA)
        out.append((G, plan, dX, dW))
        G = _to_layer_dtype(dX, dtype)
    return out


def test_chained_layers_keep_dropped_samples_dropped(vb):
    """Three linears in a row, each layer's dX (kept rows scaled, dropped rows zero) serving as the G of
    the layer below (Sec. 4: the activation gradient grows sparser layer by layer, rho_l monotone).
    The oracle computes the chain on its own; the GPU gets each layer's G from the oracle and must match
    its plan bit for bit.  Then the GPU runs the chain on its own tensors, and the kept sets must nest: a
    sample dropped above has zero norm below, hence p = 0 and no token of it is ever kept."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    N, T, K = 24, 40, 136
    rhos, nu = [0.8, 0.6, 0.4], 0.5                      # top layer first
    rng = np.random.default_rng(7)
    top = workloads.LayerSpec("chain", BF16, N, T, K, K, rhos[0], nu, layer=0, seed=3, gen_seed=21, token_sigma=0.5)
    G_host, _, _ = workloads.make_layer(top)
    shape = vb.shape_of(N, T, K, K, BF16)
    layers = [(workloads.f32_to_bf16_bits(rng.standard_normal((N * T, K)).astype(np.float32)),
               workloads.f32_to_bf16_bits((rng.standard_normal((K, K)) * 0.1).astype(np.float32)), None, rho)
              for rho in rhos]
    chain = _oracle_chain(BF16, N, T, G_host, layers, nu, 3)

    def run(g, l):
        X_host, W_host, _, rho = layers[l]
        plan = vb.Plan.allocate(N, T)
        ws = vb.make_workspace(shape)
        dX = torch.full((N * T, K), float("nan"), dtype=torch.bfloat16, device="cuda")
        dW = torch.full((K, K), float("nan"), dtype=torch.float32, device="cuda")
        vb.vcas_linear_backward(shape, g, to_device(X_host, BF16), to_device(W_host, BF16), rho, nu, vb.Rng(3, l, 0),
                                True, plan, dX, dW, ws)
        torch.cuda.synchronize()
        return plan_to_numpy(plan), dX, dW

    kept_above = np.ones(N, bool)
    for l, (G_l, want, want_dX, want_dW) in enumerate(chain):        # every layer on the oracle's G
        got, dX, dW = run(to_device(G_l, BF16), l)
        compare_plan(got, want)
        assert rel_l2_rows(from_device(dX), want_dX) <= TOL[BF16] and rel_l2_tiles(from_device(dW), want_dW) <= TOL[BF16]
        assert not np.any(want.maskA.astype(bool) & ~kept_above)
        kept_above = want.maskA.astype(bool)
    assert kept_above.sum() < N                                            # something was dropped on the way

    kept_above = np.ones(N, bool)
    g = to_device(G_host, BF16)
    for l in range(len(rhos)):                                             # the GPU's own chain: structure
        got, dX, dW = run(g, l)
        kept = got["maskA"].astype(bool)
        assert not np.any(kept & ~kept_above)                              # nested kept sets
        assert np.all(got["p"][~kept_above] == 0) and np.all(got["gnorm"][~kept_above] == 0)
        assert np.all(got["q"][np.repeat(~kept_above, T)] == 0)
        assert np.all(from_device(dX)[np.repeat(~kept, T)] == 0) and torch.isfinite(dW).all()
        kept_above = kept
        g = dX                                                             # Jacobian of the identity in between
    assert kept_above.sum() < N


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("N,T,kin,kout,frac", [(4, 40, 136, 264, 0.75), (9, 130, 768, 256, 0.5),
                                               (17, 128, 2040, 136, 0.6),      # 128x128 tiles (bf16), ragged columns
                                               (33, 125, 3080, 200, 1.0)])     # 256x256 tiles (bf16)
def test_dgrad_through_an_elementwise_jacobian(vb, dtype, N, T, kin, kout, frac):
    """App. E (proof of unbiasedness): dX = ((1/p) G W) * J on kept rows, zero rows for dropped samples (J holds NaN there:
    it must not be read into the result)."""
    rng = np.random.default_rng(N + kin)
    R = N * T
    g = rng.standard_normal((R, kout)).astype(np.float32)
    w = (rng.standard_normal((kout, kin)) * 0.05).astype(np.float32)
    p = rng.uniform(0.2, 1, N).astype(np.float32)
    maskA = (rng.uniform(size=N) < frac).astype(np.uint8)
    maskA[0] = 1
    j = (rng.uniform(size=(R, kin)) < 0.6).astype(np.float32) * rng.uniform(0.5, 1.5, (R, kin)).astype(np.float32)
    G, W, J = (workloads.f32_to_bf16_bits(a) if dtype == BF16 else a for a in (g, w, j))
    idxA = np.nonzero(maskA)[0].astype(np.int32)
    idx_buf = np.full(N, -1, np.int32)
    idx_buf[:idxA.size] = idxA
    shape = vb.shape_of(N, T, kin, kout, dtype)
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32
    j_dev = _dev(J, dtype).clone()
    j_dev[torch.from_numpy(np.repeat(maskA == 0, T)).cuda()] = float("nan")
    dX = torch.full((R, kin), float("nan"), dtype=tdt, device="cuda")
    vb.vcas_sampled_dgrad_jac(shape, _dev(G, dtype), _dev(W, dtype), _dev(p), _dev(idx_buf),
                              _dev(np.array([idxA.size], np.int32)), j_dev, dX)
    torch.cuda.synchronize()
    from tests.gpu_util import from_device, rel_l2, rel_l2_rows, rel_l2_tiles
    got = from_device(dX)
    want = oracle.dgrad_jacobian(G, W, J, dtype, N, T, p, maskA)
    assert np.isfinite(got).all()
    assert np.all(got[np.repeat(maskA == 0, T)] == 0)
    assert np.all(got[want == 0] == 0)                    # ReLU-like zeros of J stay exact zeros
    assert rel_l2_rows(got, want) <= TOL[dtype]


def test_chained_layers_through_relu_jacobians(vb):
    """Two linears with an elementwise layer between them: the upper layer's data half writes
    (dX * J) (vcas_backward_data_chained), which is the lower layer's G as it stands.  Expectations and
    the lower layer's G come from the oracle's own chain; the GPU's own hand-over is checked for structure."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    N, T, K = 16, 48, 136
    rng = np.random.default_rng(11)
    top = workloads.LayerSpec("chain_j", BF16, N, T, K, K, 0.7, 0.5, layer=0, seed=5, gen_seed=2, token_sigma=0.5)
    G_host, X_host, W_host = workloads.make_layer(top)
    J_host = workloads.f32_to_bf16_bits((rng.uniform(size=(N * T, K)) < 0.5).astype(np.float32))
    X2 = workloads.f32_to_bf16_bits(rng.standard_normal((N * T, K)).astype(np.float32))
    W2 = workloads.f32_to_bf16_bits((rng.standard_normal((K, K)) * 0.1).astype(np.float32))
    (_, want, want_dX, want_dW), (G2, want2, want_dX2, want_dW2) = _oracle_chain(
        BF16, N, T, G_host, [(X_host, W_host, J_host, 0.7), (X2, W2, None, 0.5)], 0.5, 5)
    shape = vb.shape_of(N, T, K, K, BF16)
    g, x, w, jac = (to_device(a, BF16) for a in (G_host, X_host, W_host, J_host))
    plan = vb.Plan.allocate(N, T)
    ws = vb.make_workspace(shape)
    dX = torch.full((N * T, K), float("nan"), dtype=torch.bfloat16, device="cuda")
    dW = torch.full((K, K), float("nan"), dtype=torch.float32, device="cuda")
    vb.vcas_backward_data_chained(shape, g, x, w, jac, None, True, 0.7, vb.Rng(5, 0, 0), True, plan, dX, ws)
    vb.vcas_backward_weight(shape, g, x, 0.7, 0.5, vb.Rng(5, 0, 0), True, plan, dW, ws)
    torch.cuda.synchronize()
    compare_plan(plan_to_numpy(plan), want)
    assert rel_l2_rows(from_device(dX), want_dX) <= TOL[BF16] and rel_l2_tiles(from_device(dW), want_dW) <= TOL[BF16]

    def lower(g2):
        plan2 = vb.Plan.allocate(N, T)
        dX2 = torch.full((N * T, K), float("nan"), dtype=torch.bfloat16, device="cuda")
        dW2 = torch.full((K, K), float("nan"), dtype=torch.float32, device="cuda")
        vb.vcas_linear_backward(shape, g2, to_device(X2, BF16), to_device(W2, BF16), 0.5, 0.5, vb.Rng(5, 1, 0), True,
                                plan2, dX2, dW2, ws)
        torch.cuda.synchronize()
        return plan_to_numpy(plan2), dX2, dW2
    # the layer below on the oracle's version of that tensor ...
    got2, dX2, dW2 = lower(to_device(G2, BF16))
    compare_plan(got2, want2)
    assert rel_l2_rows(from_device(dX2), want_dX2) <= TOL[BF16] and rel_l2_tiles(from_device(dW2), want_dW2) <= TOL[BF16]
    # ... and on the tensor the GPU itself handed over
    got2, dX2, dW2 = lower(dX)
    dropped = want.maskA == 0
    assert np.all(got2["p"][dropped] == 0) and not np.any(got2["maskA"][dropped])
    assert torch.isfinite(dX2).all() and torch.isfinite(dW2).all()


@pytest.mark.parametrize("dtype,K_in", [(BF16, 136), (F32, 72), (BF16, 4096)])
def test_chained_layers_without_zero_fill(vb, dtype, K_in):
    """A stack in its sparse form: no layer writes the rows of samples it drops (they keep the NaN they
    were initialised with) and the layer below is told which samples exist (kept_above = the upper
    layer's maskA), so it never reads them.  The oracle computes the chain on its own, with those rows as
    zeros; the GPU gets each layer's G from the oracle with NaN planted in them.  Then the GPU's own chain,
    as per-layer calls and as ONE vcas_backward_stack call, bit for bit the same.
    K_in = 4096 takes the path that norms X after SampleA (X above 16 MiB)."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    N, T, K = (24, 90, 136) if K_in == 4096 else (24, 40, K_in)
    K_out = K
    rhos, nu = [0.8, 0.6, 0.4], 0.5
    rng = np.random.default_rng(23)
    top = workloads.LayerSpec("sparse_chain", dtype, N, T, K_out, K_out, rhos[0], nu, layer=0, seed=8, gen_seed=31,
                              token_sigma=0.5)
    G_host, _, _ = workloads.make_layer(top)
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32
    conv = (lambda a: workloads.f32_to_bf16_bits(a)) if dtype == BF16 else (lambda a: a)
    layers, shapes = [], []
    for l, rho in enumerate(rhos):
        k_in = K_in if l == 0 else K_out            # only the top layer is wide; its dX feeds a K_in-wide G below
        k_out = K_out if l == 0 else (K_in if l == 1 else K_out)
        shapes.append((k_in, k_out))
        layers.append((conv(rng.standard_normal((N * T, k_in)).astype(np.float32)),
                       conv((rng.standard_normal((k_out, k_in)) * 0.1).astype(np.float32)),
                       conv((rng.uniform(size=(N * T, k_in)) < 0.7).astype(np.float32)), rho))
    chain = _oracle_chain(dtype, N, T, G_host, layers, nu, 8)
    dev = [tuple(to_device(a, dtype) for a in (X, W, J)) for X, W, J, _ in layers]

    def run(l, g, above_dev):
        k_in, k_out = shapes[l]
        shape = vb.shape_of(N, T, k_in, k_out, dtype)
        x, w, jac = dev[l]
        plan = vb.Plan.allocate(N, T)
        ws = vb.make_workspace(shape)
        dX = torch.full((N * T, k_in), float("nan"), dtype=tdt, device="cuda")
        dW = torch.full((k_out, k_in), float("nan"), dtype=torch.float32, device="cuda")
        r = vb.Rng(8, l, 0)
        vb.vcas_backward_data_chained(shape, g, x, w, jac, above_dev, False, layers[l][3], r, True, plan, dX, ws)
        vb.vcas_backward_weight(shape, g, x, layers[l][3], nu, r, True, plan, dW, ws)
        torch.cuda.synchronize()
        return shape, r, plan, dX, dW, ws

    # every layer on the oracle's G, the rows of samples dropped above replaced by NaN
    kept_above = np.ones(N, bool)
    for l, (G_l, want, want_dX, want_dW) in enumerate(chain):
        g = to_device(G_l, dtype)
        g.view(N, T, -1)[torch.from_numpy(~kept_above).cuda()] = float("nan")
        above_dev = None if l == 0 else torch.from_numpy(kept_above.astype(np.uint8)).cuda()
        _, _, plan, dX, dW, _ = run(l, g, above_dev)
        got = plan_to_numpy(plan)
        compare_plan(got, want)
        kept = got["maskA"].astype(bool)
        assert not np.any(kept & ~kept_above)
        got_dX = from_device(dX)
        kept_rows = np.repeat(kept, T)
        assert np.isnan(got_dX[~kept_rows]).all()                          # untouched
        assert np.isfinite(got_dX[kept_rows]).all()
        if kept.any():
            assert rel_l2_rows(got_dX[kept_rows], want_dX[kept_rows]) <= TOL[dtype]
        assert rel_l2_tiles(from_device(dW), want_dW) <= TOL[dtype]
        kept_above = kept
    assert kept_above.sum() < N

    # the GPU's own chain, layer by layer: each dX buffer is the next G, each maskA the next kept_above
    per_layer = []
    g, above_dev, kept_above = to_device(G_host, dtype), None, np.ones(N, bool)
    for l in range(len(rhos)):
        shape, r, plan, dX, dW, ws = run(l, g, above_dev)
        kept = plan.maskA.cpu().numpy().astype(bool)
        assert not np.any(kept & ~kept_above)
        assert torch.isnan(dX.float().view(N, T, -1)[torch.from_numpy(~kept).cuda()]).all()
        assert torch.isfinite(dX.float().view(N, T, -1)[torch.from_numpy(kept).cuda()]).all() and torch.isfinite(dW).all()
        per_layer.append((shape, r, plan_to_numpy(plan), dX, dW, plan, ws))
        g, above_dev, kept_above = dX, plan.maskA, kept

    # the same chain as ONE vcas_backward_stack call
    entries, outs, keep = [], [], []
    g, above = to_device(G_host, dtype), None
    for l, (shape, r, _, dX_ref, dW_ref, _, _) in enumerate(per_layer):
        x, w, jac = dev[l]
        plan = vb.Plan.allocate(N, T)
        ws = vb.make_workspace(shape)
        dX = torch.full_like(dX_ref, float("nan"))
        dW = torch.full_like(dW_ref, float("nan"))
        entries.append(vb.layer_args(shape, g, x, w, layers[l][3], nu, r, True, plan, dX, dW, ws, J=jac, kept_above=above,
                                     leave_dropped_rows=True))
        outs.append((plan, dX, dW))
        keep.append((g, ws))
        g, above = dX, plan.maskA
    s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
    vb.vcas_backward_stack(vb.make_stack(entries), 2, s2, s3)
    torch.cuda.synchronize()

    def bits(t):
        return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)
    for (plan, dX, dW), (_, _, plan_ref, dX_ref, dW_ref, _, _) in zip(outs, per_layer):
        got = plan_to_numpy(plan)
        for key, val in plan_ref.items():
            assert np.array_equal(np.asarray(got[key]), np.asarray(val)), key
        assert torch.equal(bits(dX), bits(dX_ref)) and torch.equal(bits(dW), bits(dW_ref))


@pytest.mark.parametrize("group,streams", [(1, 3), (2, 3), (3, 2), (5, 1)])
def test_stack_of_layers_equals_layer_by_layer_calls(vb, group, streams):
    """vcas_backward_stack lays the launches of several layers out over up to three streams; whatever the
    grouping, every layer must come out bit for bit as from vcas_linear_backward, and as the oracle says."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    specs = [workloads.LayerSpec("st0", BF16, 8, 128, 768, 264, 0.5, 0.5, layer=0, seed=4, gen_seed=1, token_sigma=0.5),
             workloads.LayerSpec("st1", F32, 6, 50, 72, 136, 0.6, 0.4, layer=1, seed=4, gen_seed=2, token_sigma=0.5),
             workloads.LayerSpec("st2", BF16, 12, 300, 4096, 64, 0.5, 0.5, layer=2, seed=4, gen_seed=3, token_sigma=0.5),
             workloads.LayerSpec("st3", BF16, 9, 33, 136, 200, 0.7, 0.5, layer=3, seed=4, gen_seed=4, token_sigma=0.5),
             workloads.LayerSpec("st4", BF16, 16, 64, 256, 768, 1.0, 1.0, layer=4, seed=4, gen_seed=5, token_sigma=0.5),
             # long vectors: sample norms from the tail of the pass over G, SampleA inside dgrad (ragged T, wide rows)
             workloads.LayerSpec("st5", BF16, 33, 131, 136, 264, 0.6, 0.5, layer=5, seed=4, gen_seed=6, token_sigma=0.5),
             workloads.LayerSpec("st6", BF16, 9, 500, 72, 4104, 0.4, 0.5, layer=6, seed=4, gen_seed=7, token_sigma=0.5)]
    host, dev, refs, entries, outs = [], [], [], [], []
    for sp in specs:
        G, X, W = workloads.make_layer(sp)
        shape = vb.shape_of(sp.N, sp.T, sp.K_in, sp.K_out, sp.dtype)
        g, x, w = (to_device(a, sp.dtype) for a in (G, X, W))
        tdt = torch.bfloat16 if sp.dtype == BF16 else torch.float32
        # reference: the per-layer call
        plan_r = vb.Plan.allocate(sp.N, sp.T)
        ws_r = vb.make_workspace(shape)
        dX_r = torch.full((sp.R, sp.K_in), float("nan"), dtype=tdt, device="cuda")
        dW_r = torch.full((sp.K_out, sp.K_in), float("nan"), dtype=torch.float32, device="cuda")
        vb.vcas_linear_backward(shape, g, x, w, sp.rho, sp.nu, vb.Rng(sp.seed, sp.layer, 1), True, plan_r, dX_r, dW_r, ws_r)
        refs.append((plan_to_numpy(plan_r), dX_r, dW_r))
        plan = vb.Plan.allocate(sp.N, sp.T)
        ws = vb.make_workspace(shape)
        dX = torch.full((sp.R, sp.K_in), float("nan"), dtype=tdt, device="cuda")
        dW = torch.full((sp.K_out, sp.K_in), float("nan"), dtype=torch.float32, device="cuda")
        entries.append(vb.layer_args(shape, g, x, w, sp.rho, sp.nu, vb.Rng(sp.seed, sp.layer, 1), True, plan, dX, dW, ws))
        outs.append((plan, dX, dW))
        host.append((G, X, W))
        dev.append((g, x, w, ws))
    torch.cuda.synchronize()
    stack = vb.make_stack(entries)
    s2 = torch.cuda.Stream() if streams >= 2 else None
    s3 = torch.cuda.Stream() if streams >= 3 else None
    for _ in range(2):                                   # twice: the second call re-records the same events
        vb.vcas_backward_stack(stack, group, s2, s3)
    torch.cuda.synchronize()
    for sp, (plan, dX, dW), (plan_r, dX_r, dW_r) in zip(specs, outs, refs):
        got = plan_to_numpy(plan)
        for key, val in plan_r.items():
            assert np.array_equal(np.asarray(got[key]), np.asarray(val)), (sp.name, key)
        assert torch.equal(dX.view(torch.int16) if dX.dtype == torch.bfloat16 else dX.view(torch.int32),
                           dX_r.view(torch.int16) if dX_r.dtype == torch.bfloat16 else dX_r.view(torch.int32)), sp.name
        assert torch.equal(dW.view(torch.int32), dW_r.view(torch.int32)), sp.name
    for k in (2, 5):
        sp = specs[k]
        G, X, W = host[k]
        want, want_dX, want_dW = oracle.linear_backward(G, X, W, sp.dtype, sp.N, sp.T, sp.rho, sp.nu, sp.seed, sp.layer, 1)
        compare_plan(plan_to_numpy(outs[k][0]), want)
        assert rel_l2_rows(from_device(outs[k][1]), want_dX) <= TOL[BF16] and rel_l2_tiles(from_device(outs[k][2]), want_dW) <= TOL[BF16]


@pytest.mark.parametrize("group", [2, 8])
def test_sibling_layers_share_launches_and_keep_their_bits(vb, group):
    """Layers marked as siblings (their G does not depend on the previous entry's dX: Q, K, V of one block) may
    be launched together by vcas_backward_stack.  Each must still come out bit for bit as from a call of its
    own, and as the oracle says: six layers of one shape in a row (split into launches of at most four, and by
    the group boundaries), one of another shape in between, a sibling flag on a layer of another shape or
    dtype (ignored), different keep ratios and Philox layers inside a launch."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    mk = workloads.LayerSpec
    specs = [mk("sb0", BF16, 8, 128, 264, 136, 0.5, 0.5, layer=0, seed=8, gen_seed=1, token_sigma=0.5),
             mk("sb1", BF16, 8, 128, 264, 136, 0.9, 0.5, layer=1, seed=8, gen_seed=2, token_sigma=0.5),
             mk("sb2", BF16, 8, 128, 264, 136, 0.2, 0.7, layer=2, seed=8, gen_seed=3, token_sigma=0.5),
             mk("sb3", BF16, 8, 128, 264, 136, 0.5, 0.5, layer=3, seed=8, gen_seed=4, token_sigma=0.5),
             mk("sb4", BF16, 8, 128, 264, 136, 1.0, 1.0, layer=4, seed=8, gen_seed=5, token_sigma=0.5),
             mk("sb5", BF16, 8, 128, 264, 136, 0.4, 0.5, layer=5, seed=8, gen_seed=6, token_sigma=0.5),
             mk("sb6", BF16, 8, 128, 136, 264, 0.5, 0.5, layer=6, seed=8, gen_seed=7, token_sigma=0.5),   # other shape
             mk("sb7", F32, 8, 128, 136, 264, 0.5, 0.5, layer=7, seed=8, gen_seed=8, token_sigma=0.5),    # other dtype
             mk("sb8", BF16, 32, 128, 768, 768, 0.3, 0.5, layer=8, seed=8, gen_seed=9, token_sigma=0.5),
             mk("sb9", BF16, 32, 128, 768, 768, 0.6, 0.5, layer=9, seed=8, gen_seed=10, token_sigma=0.5),
             mk("sb10", BF16, 32, 128, 768, 768, 1.0, 0.5, layer=10, seed=8, gen_seed=11, token_sigma=0.5),
             # vectors too long for the dgrad workgroups to decide SampleA themselves: one SampleA launch for all
             mk("sb11", BF16, 12, 400, 72, 136, 0.5, 0.5, layer=11, seed=8, gen_seed=12, token_sigma=0.5),
             mk("sb12", BF16, 12, 400, 72, 136, 0.3, 0.5, layer=12, seed=8, gen_seed=13, token_sigma=0.5),
             mk("sb13", BF16, 12, 400, 72, 136, 0.8, 0.5, layer=13, seed=8, gen_seed=14, token_sigma=0.5),
             # more samples than a wavefront
             mk("sb14", BF16, 100, 8, 136, 72, 0.5, 0.5, layer=14, seed=8, gen_seed=15, token_sigma=0.5),
             mk("sb15", BF16, 100, 8, 136, 72, 0.25, 0.5, layer=15, seed=8, gen_seed=16, token_sigma=0.5)]
    flags = [False, True, True, True, True, True, True, True, False, True, True, False, True, True, False, True]
    refs, entries, outs, keep, host = [], [], [], [], []
    for sp, flag in zip(specs, flags):
        G, X, W = workloads.make_layer(sp)
        shape = vb.shape_of(sp.N, sp.T, sp.K_in, sp.K_out, sp.dtype)
        g, x, w = (to_device(a, sp.dtype) for a in (G, X, W))
        tdt = torch.bfloat16 if sp.dtype == BF16 else torch.float32

        def fresh():
            return (vb.Plan.allocate(sp.N, sp.T), vb.make_workspace(shape),
                    torch.full((sp.R, sp.K_in), float("nan"), dtype=tdt, device="cuda"),
                    torch.full((sp.K_out, sp.K_in), float("nan"), dtype=torch.float32, device="cuda"))
        rng = vb.Rng(sp.seed, sp.layer, 4)
        plan_r, ws_r, dX_r, dW_r = fresh()
        vb.vcas_linear_backward(shape, g, x, w, sp.rho, sp.nu, rng, True, plan_r, dX_r, dW_r, ws_r)
        refs.append((plan_to_numpy(plan_r), dX_r, dW_r))
        plan, ws, dX, dW = fresh()
        entries.append(vb.layer_args(shape, g, x, w, sp.rho, sp.nu, rng, True, plan, dX, dW, ws, sibling=flag))
        outs.append((plan, dX, dW))
        keep.append((g, x, w, ws, ws_r))
        host.append((G, X, W))
    torch.cuda.synchronize()
    stack = vb.make_stack(entries)
    s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(2):
        vb.vcas_backward_stack(stack, group, s2, s3)
    torch.cuda.synchronize()

    def bits(t):
        return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)
    for sp, (plan, dX, dW), (plan_r, dX_r, dW_r) in zip(specs, outs, refs):
        got = plan_to_numpy(plan)
        for key, val in plan_r.items():
            assert np.array_equal(np.asarray(got[key]), np.asarray(val)), (sp.name, key)
        assert torch.equal(bits(dX), bits(dX_r)), sp.name
        assert torch.equal(bits(dW), bits(dW_r)), sp.name
    for k in (2, 9, 12, 15):
        sp = specs[k]
        G, X, W = host[k]
        want, want_dX, want_dW = oracle.linear_backward(G, X, W, sp.dtype, sp.N, sp.T, sp.rho, sp.nu, sp.seed, sp.layer, 4)
        compare_plan(plan_to_numpy(outs[k][0]), want)
        assert rel_l2_rows(from_device(outs[k][1]), want_dX) <= TOL[BF16] and rel_l2_tiles(from_device(outs[k][2]), want_dW) <= TOL[BF16]


@pytest.mark.parametrize("N,T", [(20, 64), (37, 117), (64, 70)])
def test_sibling_layers_inside_a_sparse_chain(vb, N, T):
    """Siblings with the additions of the chained data call: a mask of samples dropped above, an elementwise
    Jacobian each, dropped rows left unwritten.  One stack call against per-layer chained calls, bit for bit.
    With more than 4096 rows the stack takes the sample norms in the tail of the pass over G (rows counted per
    sample across workgroups; T = 117 and 70 make workgroups straddle samples) and SampleA inside dgrad."""
    from tests.gpu_util import to_device, plan_to_numpy
    K_in, K_out = 136, 264
    rng_np = np.random.default_rng(41)
    above = torch.from_numpy((rng_np.uniform(size=N) < 0.7).astype(np.uint8)).cuda()
    entries, outs, refs, keep = [], [], [], []
    for k in range(3):
        sp = workloads.LayerSpec(f"sc{k}", BF16, N, T, K_in, K_out, 0.5 + 0.2 * k, 0.5, layer=k, seed=12, gen_seed=50 + k,
                                 token_sigma=0.5)
        G, X, W = workloads.make_layer(sp)
        shape = vb.shape_of(N, T, K_in, K_out, BF16)
        g, x, w = (to_device(a, BF16) for a in (G, X, W))
        g.view(N, T, K_out)[above == 0] = float("nan")                  # rows that must never be read
        jac = to_device(workloads.f32_to_bf16_bits((rng_np.uniform(size=(N * T, K_in)) < 0.6).astype(np.float32)), BF16)
        r = vb.Rng(sp.seed, sp.layer, 1)

        def fresh():
            return (vb.Plan.allocate(N, T), vb.make_workspace(shape),
                    torch.full((N * T, K_in), float("nan"), dtype=torch.bfloat16, device="cuda"),
                    torch.full((K_out, K_in), float("nan"), dtype=torch.float32, device="cuda"))
        plan_r, ws_r, dX_r, dW_r = fresh()
        vb.vcas_backward_data_chained(shape, g, x, w, jac, above, False, sp.rho, r, True, plan_r, dX_r, ws_r)
        vb.vcas_backward_weight(shape, g, x, sp.rho, sp.nu, r, True, plan_r, dW_r, ws_r)
        refs.append((plan_r, dX_r, dW_r))
        plan, ws, dX, dW = fresh()
        entries.append(vb.layer_args(shape, g, x, w, sp.rho, sp.nu, r, True, plan, dX, dW, ws, sibling=k > 0, J=jac,
                                     kept_above=above, leave_dropped_rows=True))
        outs.append((plan, dX, dW))
        keep.append((g, x, w, jac, ws, ws_r))
    s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
    vb.vcas_backward_stack(vb.make_stack(entries), 3, s2, s3)
    torch.cuda.synchronize()
    for (plan, dX, dW), (plan_r, dX_r, dW_r) in zip(outs, refs):
        got, want = plan_to_numpy(plan), plan_to_numpy(plan_r)
        for key, val in want.items():
            assert np.array_equal(np.asarray(got[key]), np.asarray(val)), key
        assert not np.any(got["maskA"].astype(bool) & ~above.cpu().numpy().astype(bool))
        assert torch.equal(dX.view(torch.int16), dX_r.view(torch.int16))
        assert torch.equal(dW.view(torch.int32), dW_r.view(torch.int32))
        assert torch.isfinite(dW).all()


@pytest.mark.parametrize("fill", [1, 128, 384, 100000])
def test_weight_gradient_slices_are_a_choice_of_the_caller(vb, fill):
    """vcas_layer_args.wgrad_fill sets how far the contraction of a weight gradient is cut into split-K slices.
    Whatever it is, the plan is the oracle's bit for bit and dW within tolerance; 384 and anything above are the
    stand-alone call's choice, hence its bits; the same value twice gives the same bits."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    specs = [workloads.LayerSpec("wf0", BF16, 16, 128, 264, 136, 0.8, 0.7, layer=0, seed=14, gen_seed=71, token_sigma=0.5),
             workloads.LayerSpec("wf1", BF16, 16, 128, 264, 136, 0.6, 0.9, layer=1, seed=14, gen_seed=72, token_sigma=0.5),
             workloads.LayerSpec("wf2", F32, 8, 128, 136, 72, 0.7, 0.8, layer=2, seed=14, gen_seed=73, token_sigma=0.5)]
    runs = []
    for rep in range(2):
        entries, outs, keep, host = [], [], [], []
        for k, sp in enumerate(specs):
            G, X, W = workloads.make_layer(sp)
            shape = vb.shape_of(sp.N, sp.T, sp.K_in, sp.K_out, sp.dtype)
            g, x, w = (to_device(a, sp.dtype) for a in (G, X, W))
            plan, ws = vb.Plan.allocate(sp.N, sp.T), vb.make_workspace(shape)
            dX = torch.full((sp.R, sp.K_in), float("nan"), dtype=g.dtype, device="cuda")
            dW = torch.full((sp.K_out, sp.K_in), float("nan"), dtype=torch.float32, device="cuda")
            entries.append(vb.layer_args(shape, g, x, w, sp.rho, sp.nu, vb.Rng(sp.seed, sp.layer, 3), True, plan, dX, dW, ws,
                                         sibling=k == 1, wgrad_fill=fill))
            outs.append((plan, dX, dW))
            keep.append((g, x, w, ws))
            host.append((G, X, W))
        s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
        vb.vcas_backward_stack(vb.make_stack(entries), 3, s2, s3)
        torch.cuda.synchronize()
        runs.append(outs)
    for k, sp in enumerate(specs):
        G, X, W = host[k]
        want, want_dX, want_dW = oracle.linear_backward(G, X, W, sp.dtype, sp.N, sp.T, sp.rho, sp.nu, sp.seed, sp.layer, 3)
        plan, dX, dW = runs[0][k]
        compare_plan(plan_to_numpy(plan), want)
        assert rel_l2_rows(from_device(dX), want_dX) <= TOL[sp.dtype] and rel_l2_tiles(from_device(dW), want_dW) <= TOL[sp.dtype]
        assert torch.equal(dW.view(torch.int32), runs[1][k][2].view(torch.int32))
        if fill >= 384:
            shape = vb.shape_of(sp.N, sp.T, sp.K_in, sp.K_out, sp.dtype)
            g, x, w = (to_device(a, sp.dtype) for a in (G, X, W))
            plan_r, ws_r = vb.Plan.allocate(sp.N, sp.T), vb.make_workspace(shape)
            dW_r = torch.full_like(dW, float("nan"))
            vb.vcas_linear_backward(shape, g, x, w, sp.rho, sp.nu, vb.Rng(sp.seed, sp.layer, 3), True, plan_r, None, dW_r, ws_r)
            torch.cuda.synchronize()
            assert torch.equal(dW.view(torch.int32), dW_r.view(torch.int32))


@pytest.mark.parametrize("streams", [1, 3])
def test_cached_row_norms_of_x_give_the_same_bits(vb, streams):
    """The squared row norms of X can be taken once, when X is produced (vcas_row_norms over every row), and
    handed to the weight half instead of a second sweep over X: every plan field, dX and dW must come out bit
    for bit as without the cache, in the stack launch and in the stand-alone weight call, and as the oracle says."""
    from tests.gpu_util import to_device, from_device, plan_to_numpy, compare_plan, rel_l2, rel_l2_rows, rel_l2_tiles
    specs = [workloads.LayerSpec("cx0", BF16, 8, 128, 768, 264, 0.5, 0.5, layer=0, seed=6, gen_seed=1, token_sigma=0.5),
             workloads.LayerSpec("cx1", F32, 6, 50, 72, 136, 0.6, 0.4, layer=1, seed=6, gen_seed=2, token_sigma=0.5),
             workloads.LayerSpec("cx2", BF16, 12, 300, 2048, 64, 0.4, 0.5, layer=2, seed=6, gen_seed=3, token_sigma=0.5),
             workloads.LayerSpec("cx3", BF16, 16, 64, 256, 768, 1.0, 1.0, layer=3, seed=6, gen_seed=4, token_sigma=0.5)]
    refs, entries, outs, alone, keep, host = [], [], [], [], [], []
    for sp in specs:
        G, X, W = workloads.make_layer(sp)
        shape = vb.shape_of(sp.N, sp.T, sp.K_in, sp.K_out, sp.dtype)
        g, x, w = (to_device(a, sp.dtype) for a in (G, X, W))
        tdt = torch.bfloat16 if sp.dtype == BF16 else torch.float32

        def fresh():
            return (vb.Plan.allocate(sp.N, sp.T), vb.make_workspace(shape),
                    torch.full((sp.R, sp.K_in), float("nan"), dtype=tdt, device="cuda"),
                    torch.full((sp.K_out, sp.K_in), float("nan"), dtype=torch.float32, device="cuda"))
        rng = vb.Rng(sp.seed, sp.layer, 2)
        plan_r, ws_r, dX_r, dW_r = fresh()
        vb.vcas_linear_backward(shape, g, x, w, sp.rho, sp.nu, rng, True, plan_r, dX_r, dW_r, ws_r)
        refs.append((plan_to_numpy(plan_r), dX_r, dW_r))
        # "forward pass": norms of every row of X, nothing masked
        xsq_fwd = torch.full((sp.R,), float("nan"), device="cuda")
        vb.vcas_row_norms(shape, None, x, None, None, xsq_fwd, None)
        xsq_copy = xsq_fwd.clone()
        plan, ws, dX, dW = fresh()
        entries.append(vb.layer_args(shape, g, x, w, sp.rho, sp.nu, rng, True, plan, dX, dW, ws, xsq_forward=xsq_fwd))
        outs.append((plan, dX, dW))
        # stand-alone: data call, then the weight call with the cache
        plan_a, ws_a, dX_a, dW_a = fresh()
        vb.vcas_backward_data(shape, g, x, w, sp.rho, rng, True, plan_a, dX_a, ws_a)
        vb.vcas_backward_weight_cached(shape, g, x, xsq_fwd, sp.rho, sp.nu, rng, True, plan_a, dW_a, ws_a)
        alone.append((plan_a, dX_a, dW_a))
        keep.append((g, x, w, ws, ws_a, ws_r, xsq_fwd, xsq_copy))
        host.append((G, X, W))
    torch.cuda.synchronize()
    stack = vb.make_stack(entries)
    s2 = torch.cuda.Stream() if streams >= 2 else None
    s3 = torch.cuda.Stream() if streams >= 3 else None
    for _ in range(2):                                   # the cache must survive a step: twice
        vb.vcas_backward_stack(stack, 2, s2, s3)
    torch.cuda.synchronize()

    def bits(t):
        return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)
    for k, sp in enumerate(specs):
        plan_r, dX_r, dW_r = refs[k]
        for name, (plan, dX, dW) in (("stack", outs[k]), ("alone", alone[k])):
            got = plan_to_numpy(plan)
            for key, val in plan_r.items():
                assert np.array_equal(np.asarray(got[key]), np.asarray(val)), (sp.name, name, key)
            assert torch.equal(bits(dX), bits(dX_r)), (sp.name, name)
            assert torch.equal(bits(dW), bits(dW_r)), (sp.name, name)
        assert torch.equal(keep[k][6], keep[k][7]), "the cached norms were written to"
    sp = specs[2]
    G, X, W = host[2]
    want, want_dX, want_dW = oracle.linear_backward(G, X, W, sp.dtype, sp.N, sp.T, sp.rho, sp.nu, sp.seed, sp.layer, 2)
    compare_plan(plan_to_numpy(outs[2][0]), want)
    assert rel_l2_tiles(from_device(outs[2][2]), want_dW) <= TOL[BF16]


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_variance_probe_matches_oracle(vb, dtype):
    spec = workloads.LayerSpec("probe", dtype, 8, 24, 72, 64, 0.5, 0.5, layer=4, seed=5, gen_seed=4, token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    M = 4
    shape = vb.shape_of(spec.N, spec.T, spec.K_in, spec.K_out, dtype)
    from tests.gpu_util import to_device
    plan = vb.Plan.allocate(spec.N, spec.T)
    ws = vb.make_workspace(shape)
    out = torch.full((4,), float("nan"), dtype=torch.float64, device="cuda")
    vb.vcas_variance_probe(shape, to_device(G, dtype), to_device(X, dtype), spec.rho, spec.nu,
                           vb.Rng(spec.seed, spec.layer, 10), M, plan, out, ws)
    torch.cuda.synchronize()
    want = oracle.variance_probe(G, X, dtype, spec.N, spec.T, spec.rho, spec.nu, spec.seed, spec.layer, 10, M)
    got = out.cpu().numpy()
    # [0], [1]: same fp32 inputs, fp64 sums.  [2], [3]: squared differences of dW, whose own error is
    # bounded by the GEMM tolerance; the differences are sampling noise, far above rounding.
    np.testing.assert_allclose(got[:2], want[:2], rtol=1e-9)
    np.testing.assert_allclose(got[2:], want[2:], rtol=1e-4 if dtype == F32 else 3e-2)
