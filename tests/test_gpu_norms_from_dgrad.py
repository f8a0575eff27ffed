"""The norms of a layer's incoming gradient from the launch that produced it (Sec. 4: a sampler at every
layer; Sec. 4.1: p_i ~ ||G_i||_F).  Inside a stack a layer's G is the dX the layer above has just written, so
its dgrad epilogue adds up the squares of what it stores, by blocks of 64 columns, and the layer below adds the
block sums instead of sweeping G again (and, inside a stack, takes the sample norms in the same launch and
lets its dgrad decide SampleA).  The summation order (pairwise, neighbours first) makes the two routes
agree bit for bit.

Data flows from the oracle to the GPU only: the consumer is checked against the oracle on the oracle's own
block sums; the producer's dX against the oracle's dX, its block sums against the oracle's within the
tolerance of dX, and bit for bit against a sweep of the very dX buffer it wrote (GPU against GPU)."""
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


def _dev(a, dtype=None):
    from paper_2402_17227_amd import binding
    if dtype is not None:
        return binding.to_device(a, dtype)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("N,T,K", [(5, 37, 8), (6, 50, 136), (32, 128, 768), (7, 64, 1000), (3, 70, 4096), (2, 40, 8184)])
def test_rows_from_blocks_bit_exact(vb, N, T, K):
    rng = np.random.default_rng(K + N)
    a = (rng.standard_normal((N * T, K)) * np.exp(rng.standard_normal((N * T, 1)))).astype(np.float32)
    A = workloads.f32_to_bf16_bits(a)
    from tests.gpu_util import blocks_to_device_layout
    blocks = oracle.block_sumsq(A, BF16)
    keep = (rng.uniform(size=N) < 0.7).astype(np.uint8)
    keep[0] = 1
    poisoned = blocks.copy()
    poisoned[np.repeat(keep == 0, T)] = np.nan          # rows of dropped samples are never read
    for mask, src in ((None, blocks), (keep, poisoned)):
        sq = torch.full((N * T,), float("nan"), device="cuda")
        norm = torch.full((N,), float("nan"), device="cuda")
        vb.vcas_row_norms_from_blocks(N, T, K, _dev(blocks_to_device_layout(src)), None if mask is None else _dev(mask), sq, norm)
        torch.cuda.synchronize()
        want = oracle.row_sumsq(A, BF16, T, mask)
        assert np.array_equal(sq.cpu().numpy().view(np.uint32), want.view(np.uint32))
        assert np.array_equal(norm.cpu().numpy().view(np.uint32), oracle.sample_norms(want, N, T).view(np.uint32))


@pytest.mark.parametrize("N,T,kin,kout,frac,jac", [(17, 128, 2040, 136, 1.0, False),    # 128x128 tiles, ragged columns
                                                    (17, 128, 2040, 136, 0.6, True),
                                                    (33, 125, 3080, 200, 1.0, True),     # 256x256 tiles, ragged rows and columns
                                                    (33, 125, 3080, 200, 0.5, False),
                                                    (17, 128, 1024, 72, 1.0, True),      # 64x128 tiles, two stages
                                                    (6, 50, 264, 136, 0.7, False),       # 64x128 tiles, four stages
                                                    (9, 64, 40, 72, 0.8, True)])         # less than one block of 64 columns
def test_dgrad_block_sums(vb, N, T, kin, kout, frac, jac):
    from tests.gpu_util import from_device, rel_l2_rows, blocks_from_device_layout
    rng = np.random.default_rng(N * 1000 + kin)
    R = N * T
    G = workloads.f32_to_bf16_bits(rng.standard_normal((R, kout)).astype(np.float32))
    W = workloads.f32_to_bf16_bits((rng.standard_normal((kout, kin)) * 0.05).astype(np.float32))
    J = workloads.f32_to_bf16_bits((rng.uniform(size=(R, kin)) < 0.6).astype(np.float32) * 1.5) if jac else None
    p = rng.uniform(0.2, 1, N).astype(np.float32)
    maskA = (rng.uniform(size=N) < frac).astype(np.uint8)
    maskA[0] = 1
    idxA = np.nonzero(maskA)[0].astype(np.int32)
    idx_buf = np.full(N, -1, np.int32)
    idx_buf[:idxA.size] = idxA
    shape = vb.shape_of(N, T, kin, kout, BF16)
    nb = (kin + 63) // 64
    g, w, pd, ix, cn = _dev(G, BF16), _dev(W, BF16), _dev(p), _dev(idx_buf), _dev(np.array([idxA.size], np.int32))
    jd = _dev(J, BF16) if jac else None
    dX = torch.full((R, kin), float("nan"), dtype=torch.bfloat16, device="cuda")
    blocks = vb.make_sq_blocks(R, kin, float("nan"))
    vb.vcas_sampled_dgrad_norms(shape, g, w, pd, ix, cn, jd, dX, blocks)
    # the same dX as the call without the block sums
    ref = torch.full((R, kin), float("nan"), dtype=torch.bfloat16, device="cuda")
    if jac:
        vb.vcas_sampled_dgrad_jac(shape, g, w, pd, ix, cn, jd, ref)
    else:
        vb.vcas_sampled_dgrad(shape, g, w, pd, ix, cn, ref)
    torch.cuda.synchronize()
    assert torch.equal(dX.view(torch.int16), ref.view(torch.int16))
    want_dX = oracle.dgrad_jacobian(G, W, J, BF16, N, T, p, maskA) if jac else oracle.dgrad(G, W, BF16, N, T, p, maskA)
    assert rel_l2_rows(from_device(dX), want_dX) <= 1e-2
    kept_rows = np.repeat(maskA == 1, T)
    got_blocks = blocks_from_device_layout(blocks, nb)
    assert np.isnan(blocks.cpu().numpy().reshape(-1, R, 4)[-1][:, nb - 4 * ((nb - 1) // 4):]).all()   # unused slots untouched
    # rows of dropped samples are not written
    assert np.isnan(got_blocks[~kept_rows]).all() and np.isfinite(got_blocks[kept_rows]).all()
    # within the tolerance of dX of the oracle's block sums of its own dX (squares: twice the relative error)
    want_blocks = oracle.block_sumsq(workloads.f32_to_bf16_bits(want_dX.astype(np.float32)), BF16)
    num = np.abs(got_blocks[kept_rows].astype(np.float64) - want_blocks[kept_rows]).sum(axis=1)
    den = want_blocks[kept_rows].astype(np.float64).sum(axis=1)
    assert (num[den > 0] / den[den > 0]).max() <= 4e-2
    # bit for bit the sweep over the dX buffer this launch wrote (GPU against GPU, same summation tree)
    shape_below = vb.shape_of(N, T, 8, kin, BF16)        # dX is the G [R, kin] of a layer below
    mask_dev = _dev(maskA)
    sq_a = torch.full((R,), float("nan"), device="cuda")
    vb.vcas_row_norms_from_blocks(N, T, kin, blocks, mask_dev, sq_a, None)
    dX_zeroed = dX.clone()                                # a sweep reads every row: dropped rows are zeros there
    sq_b = torch.full((R,), float("nan"), device="cuda")
    vb.vcas_row_norms(shape_below, dX_zeroed, None, None, sq_b, None, None)
    torch.cuda.synchronize()
    assert torch.equal(sq_a.view(torch.int32), sq_b.view(torch.int32))


@pytest.mark.parametrize("N,T", [(24, 64), (5, 300), (3, 1024), (6, 1), (64, 16), (70, 20), (2, 1100)])
def test_stack_takes_norms_from_the_layer_above(vb, N, T):
    """A chain down -> up -> o -> (v, k, q): every entry's dX buffer is the next entry's G, the entries know
    which samples the one above kept and leave dropped rows unwritten.  With the block sums handed down the
    sweeps over G disappear for every entry but the first; plans, dX and dW must be the bits of the same stack
    with the sweeps.  Up to 64 samples of up to 1024 rows the pass over the block sums also leaves the sample
    norms and dgrad decides SampleA (one workgroup per sample, 1 to 16 threads per row); beyond (the last two
    cases) the row sums go through the SampleA launch as before."""
    from tests.gpu_util import to_device, plan_to_numpy
    # G of an entry is [R, K_out]; its dX is [R, K_in] and is the next entry's G: K_in(above) == K_out(below)
    chain = [("down", 264, 136), ("up", 136, 264), ("o", 136, 136), ("v", 200, 136), ("k", 200, 136), ("q", 200, 136)]
    runs = []
    for fused in (False, True):
        entries, outs, keep = [], [], []
        prev, src_of_v = None, None
        for k, (name, kin, kout) in enumerate(chain):
            sp = workloads.LayerSpec(f"nf{k}", BF16, N, T, kin, kout, 0.9 - 0.1 * k, 0.6, layer=k, seed=21, gen_seed=80 + k,
                                     token_sigma=0.5)
            G, X, W = workloads.make_layer(sp)
            shape = vb.shape_of(N, T, kin, kout, BF16)
            x, w = to_device(X, BF16), to_device(W, BF16)
            sib = name in "kq"
            if prev is None:
                src = (to_device(G, BF16), None, None)
            elif sib:
                src = src_of_v                       # a sibling takes what its elder sibling took
            else:
                src = (prev["dX"], prev["plan"].maskA, prev["blocks"] if fused else None)
            if name == "v":
                src_of_v = src
            g, above, gblocks = src
            assert g.shape == (N * T, kout), (name, g.shape)
            plan, ws = vb.Plan.allocate(N, T), vb.make_workspace(shape)
            dX = torch.full((N * T, kin), float("nan"), dtype=torch.bfloat16, device="cuda")
            dW = torch.full((kout, kin), float("nan"), dtype=torch.float32, device="cuda")
            blocks = vb.make_sq_blocks(N * T, kin, float("nan")) if fused else None
            entries.append(vb.layer_args(shape, g, x, w, sp.rho, sp.nu, vb.Rng(sp.seed, sp.layer, 2), True, plan, dX, dW, ws,
                                         sibling=sib, kept_above=above, leave_dropped_rows=True,
                                         dx_sq_blocks=blocks, g_sq_blocks=gblocks))
            prev = dict(dX=dX, plan=plan, blocks=blocks)
            outs.append((plan, dX, dW))
            keep.append((g, x, w, ws, blocks))
        s2, s3 = torch.cuda.Stream(), torch.cuda.Stream()
        vb.vcas_backward_stack(vb.make_stack(entries), 3, s2, s3)
        torch.cuda.synchronize()
        runs.append(outs)
    for (plan_a, dX_a, dW_a), (plan_b, dX_b, dW_b) in zip(*runs):
        a, b = plan_to_numpy(plan_a), plan_to_numpy(plan_b)
        for key, val in a.items():
            assert np.array_equal(np.asarray(val), np.asarray(b[key]), equal_nan=True), key
        assert torch.equal(dX_a.view(torch.int16), dX_b.view(torch.int16))
        assert torch.equal(dW_a.view(torch.int32), dW_b.view(torch.int32))
        assert torch.isfinite(dW_a).all() and a["cntA"] > 0
