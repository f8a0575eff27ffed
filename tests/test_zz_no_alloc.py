"""vcas_sampled_wgrad_static, the weight gradient for callers that cannot allocate (code under graph capture,
serving loops): its split-K partial tiles live in a buffer that is part of the library's device image.  It
runs the kernels of vcas_sampled_wgrad, so dW must come out with the same bits, also on a second call with a
smaller input that finds the first call's partial tiles still in the buffer; and both must agree with the
oracle within the tolerance of the weight gradient (Sec. 4.2)."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import workloads
from workloads import BF16, F32


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


def _problem(R, kin, kout, frac, dtype, seed):
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((R, kout)).astype(np.float32)
    x = rng.standard_normal((R, kin)).astype(np.float32)
    G, X = (workloads.f32_to_bf16_bits(a) if dtype == BF16 else a for a in (g, x))
    keep = rng.random(R) < frac
    scale = np.where(keep, rng.uniform(1, 8, R), 0).astype(np.float32)
    idx = np.nonzero(keep)[0].astype(np.int32)
    idx_buf = np.full(R, -1, np.int32)
    idx_buf[:idx.size] = idx
    return G, X, scale, idx_buf, idx.size


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [BF16, F32])
def test_static_scratch_weight_gradient_matches_the_workspace_one(vb, dtype):
    from tests.gpu_util import from_device, rel_l2_tiles
    tol = 1e-2 if dtype == BF16 else 1e-5
    # two calls in a row on the library's buffer: many split-K slices first, then a smaller problem
    for (R, kin, kout, frac) in [(6000, 768, 384, 0.6), (900, 264, 136, 0.5)]:
        G, X, scale, idx_buf, cnt = _problem(R, kin, kout, frac, dtype, R + kin)
        shape = vb.shape_of(1, R, kin, kout, dtype)
        g, x, sc, ix = _dev(G, dtype), _dev(X, dtype), _dev(scale), _dev(idx_buf)
        cn = _dev(np.array([cnt], np.int32))
        ws = vb.make_workspace(shape)
        want = torch.full((kout, kin), float("nan"), device="cuda")
        vb.vcas_sampled_wgrad(shape, g, x, sc, ix, cn, want, ws)
        got = torch.full((kout, kin), float("nan"), device="cuda")
        before = torch.cuda.memory_allocated()
        vb.vcas_sampled_wgrad_static(shape, g, x, sc, ix, cn, got)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (R, kin, kout)
        assert rel_l2_tiles(from_device(got), oracle.wgrad(G, X, dtype, scale)) <= tol


def test_static_scratch_refuses_what_does_not_fit(vb):
    """Checked on the host before anything touches the GPU: a dW whose partial tiles exceed the buffer."""
    import ctypes as C
    assert vb.vcas_static_scratch_bytes() == 64 << 20
    shape = vb.shape_of(1, 4096, 8184, 8184, BF16)
    one = C.c_void_p(16)
    rc = vb.lib().vcas_sampled_wgrad_static(C.byref(shape), one, one, one, one, one, one, C.c_void_p(0))
    assert rc == 6 and b"static buffer" in vb.lib().vcas_status_string(rc)
