"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- published known answers, closed forms, textbook routines
(numpy fp64 matmul), invariants, and brute-force enumeration over all masks on
tiny inputs.  CPU only."""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import BF16, F32
import workloads

HERE = os.path.dirname(os.path.abspath(__file__))


# ----------------------------------------------------------------- Philox

def _kat_lines():
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        if line.strip() and not line.startswith("#"):
            yield [int(x, 16) for x in line.split()]


def test_philox_known_answers():
    n = 0
    for v in _kat_lines():
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert list(out) == v[6:10]
        n += 1
    assert n == 4


def test_uniform_is_top_24_bits_of_word0():
    for seed, layer, stream, draw, row in [(0, 3, 1, 0, 5), (0xDEADBEEF12345678, 7, 0, 9, 4095), (1, 0, 0, 0, 0)]:
        w = oracle.philox4x32_10([row, layer, stream, draw], [seed & 0xFFFFFFFF, seed >> 32])
        u = oracle.uniform(seed, layer, stream, draw, row)
        assert u == (int(w[0]) >> 8) / 2.0**24
        assert 0.0 <= u < 1.0
    # golden line 4 is exactly (row=5, layer=3, stream=1, draw=0, seed=0)
    assert oracle.uniform(0, 3, 1, 0, 5) == (0xDD3C661D >> 8) / 2.0**24


def test_uniform_looks_uniform():
    u = np.array([oracle.uniform(42, 1, 0, 0, r) for r in range(20000)])
    assert abs(u.mean() - 0.5) < 5 * (1 / 12) ** 0.5 / 20000**0.5
    hist, _ = np.histogram(u, bins=16, range=(0, 1))
    assert np.all(np.abs(hist - 1250) < 6 * 1250**0.5)
    # streams, layers and draws give different sequences
    a = [oracle.uniform(42, 1, 0, 0, r) for r in range(64)]
    for other in [(42, 1, 1, 0), (42, 2, 0, 0), (42, 1, 0, 1), (43, 1, 0, 0)]:
        b = [oracle.uniform(*other, r) for r in range(64)]
        assert sum(x == y for x, y in zip(a, b)) <= 1


# ------------------------------------------------------------------ norms

@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("K", [8, 136, 768, 1024, 4096])
def test_row_sumsq_matches_definition(dtype, K):
    rng = np.random.default_rng(K + dtype)
    a = (rng.standard_normal((19, K)) * np.exp(rng.standard_normal((19, 1)))).astype(np.float32)
    A = workloads.f32_to_bf16_bits(a) if dtype == BF16 else a
    got = oracle.row_sumsq(A, dtype)
    ref = oracle.row_sumsq_f64(A, dtype)
    # independent statement of the definition
    ref2 = (oracle.to_f64(A, dtype) ** 2).sum(axis=1)
    np.testing.assert_allclose(ref, ref2, rtol=1e-13)
    np.testing.assert_allclose(got.astype(np.float64), ref, rtol=1e-6)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_row_sumsq_exact_on_small_integers(dtype):
    # sums of squares of small integers are exact in fp32 in any order
    rng = np.random.default_rng(5)
    a = rng.integers(-15, 16, size=(11, 520)).astype(np.float32)
    A = workloads.f32_to_bf16_bits(a) if dtype == BF16 else a
    got = oracle.row_sumsq(A, dtype)
    assert np.array_equal(got, (a.astype(np.int64) ** 2).sum(axis=1).astype(np.float32))


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_row_sumsq_adds_neighbours_first(dtype):
    """The written-down order of the row sums (pairwise, neighbours first, zero-padded to a power of two),
    on rows worked out by hand where any other order rounds differently.  Squares 2^24, 1, 1, 1: the pair
    (2^24 + 1) rounds back to 2^24 (tie to even), the pair (1 + 1) = 2 survives, 2^24 + 2 is exact; adding one
    element after the other, or one chain per 16-byte group, loses all three ones.  Twelve elements
    (padded to sixteen): 2^24, then eleven ones: pairs 2^24, 2, 2, 2, 2, 2 | fours 2^24 + 2, 4, 4 (+0) |
    eights 2^24 + 6, 4 | 2^24 + 10."""
    def row(vals):
        a = np.zeros((1, 16 if len(vals) > 8 else 8), np.float32)
        a[0, :len(vals)] = vals
        return workloads.f32_to_bf16_bits(a) if dtype == BF16 else a
    assert oracle.row_sumsq(row([4096, 1, 1, 1]), dtype)[0] == np.float32(16777218.0)
    assert oracle.row_sumsq(row([1, 1, 4096, 1]), dtype)[0] == np.float32(16777218.0)
    assert oracle.row_sumsq(row([4096] + [1] * 11), dtype)[0] == np.float32(16777226.0)
    # sixteen elements, the large one in the middle of the second half: 8 + ((2^24 + 2) + 4) = 2^24 + 14
    assert oracle.row_sumsq(row([1] * 9 + [4096] + [1] * 6), dtype)[0] == np.float32(16777230.0)


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("K", [8, 40, 136, 768, 1000, 4096])
@pytest.mark.parametrize("width", [32, 64, 256])
def test_block_sums_are_subtrees_of_the_row_sum(dtype, K, width):
    """Row norms in two stages (sums over blocks of `width` columns, then the blocks pairwise) give the bits of
    the one-stage row sum, ragged last block and non-power-of-two block counts included, whatever the width;
    each block sum is the row sum of the block taken as a row of its own; and the definition in fp64 pins both."""
    rng = np.random.default_rng(K)
    a = (rng.standard_normal((7, K)) * np.exp(rng.standard_normal((7, 1)))).astype(np.float32)
    A = workloads.f32_to_bf16_bits(a) if dtype == BF16 else a
    blocks = oracle.block_sumsq(A, dtype, width)
    assert blocks.shape == (7, (K + width - 1) // width)
    whole = oracle.row_sumsq(A, dtype)
    assert np.array_equal(oracle.rows_from_blocks(blocks).view(np.uint32), whole.view(np.uint32))
    for b in range(blocks.shape[1]):
        piece = np.ascontiguousarray(A[:, width * b:width * b + width])
        assert np.array_equal(oracle.row_sumsq(piece, dtype).view(np.uint32), blocks[:, b].view(np.uint32))
    np.testing.assert_allclose(blocks.astype(np.float64).sum(axis=1), oracle.row_sumsq_f64(A, dtype), rtol=1e-6)
    # dropped samples: zero, whatever their block sums hold
    keep = np.array([1, 0, 1, 1, 0, 1, 1], np.uint8)
    poisoned = blocks.copy()
    poisoned[keep == 0] = np.nan
    got = oracle.rows_from_blocks(poisoned, 1, keep)
    assert np.array_equal(got[keep == 1].view(np.uint32), whole[keep == 1].view(np.uint32)) and np.all(got[keep == 0] == 0)


def test_rows_from_blocks_worked_example():
    """Five block sums (padded to eight): 2^24, 1, 1, 1, 1 -> pairs 2^24 (the 1 is lost to the tie), 2, 1 | fours
    2^24 + 2, 1 | 2^24 + 2 + 1 = 2^24 + 3 -> rounds to 2^24 + 4 (tie to even)."""
    blocks = np.array([[16777216.0, 1, 1, 1, 1]], np.float32)
    assert oracle.rows_from_blocks(blocks)[0] == np.float32(16777220.0)


def test_row_sumsq_sample_mask_zeroes_dropped_samples():
    rng = np.random.default_rng(6)
    a = rng.standard_normal((12, 64)).astype(np.float32)
    keep = np.array([1, 0, 1], np.uint8)
    got = oracle.row_sumsq(a, F32, T=4, sample_keep=keep)
    full = oracle.row_sumsq(a, F32)
    assert np.array_equal(got[0:4], full[0:4]) and np.all(got[4:8] == 0) and np.array_equal(got[8:], full[8:])


def test_sample_norms_are_frobenius_norms():
    rng = np.random.default_rng(7)
    for N, T in [(8, 128), (3, 197), (5, 1), (2, 1024)]:
        g = (rng.standard_normal((N * T, 40)) * np.exp(rng.standard_normal((N * T, 1)))).astype(np.float32)
        gsq = oracle.row_sumsq(g, F32)
        got = oracle.sample_norms(gsq, N, T)
        ref = np.sqrt((g.astype(np.float64) ** 2).reshape(N, -1).sum(axis=1))
        np.testing.assert_allclose(got, ref, rtol=2e-6)


# ------------------------------------------------------ keep probabilities

def _waterfill_by_sorting(a, budget):
    """Independent solver: sort descending, find how many entries sit at 1."""
    a = np.asarray(a, np.float64)
    nz = int((a > 0).sum())
    B = min(budget, nz)
    order = np.argsort(-a, kind="stable")
    s = a[order]
    p = np.zeros_like(a)
    for k in range(0, nz + 1):       # k entries capped at 1
        rest = s[k:nz].sum()
        if rest <= 0:
            c = 0.0
            if k == nz:
                p[order[:k]] = 1.0
                return p
            continue
        c = (B - k) / rest
        if (k == 0 or c * s[k - 1] >= 1.0 - 1e-15) and (k == nz or c * s[k] < 1.0):
            p[order[:k]] = 1.0
            p[order[k:nz]] = c * s[k:nz]
            return p
    raise AssertionError("no solution")


@pytest.mark.parametrize("n,rho,sigma", [(8, 0.5, 1.0), (32, 0.3, 1.0), (64, 0.3, 1.5), (64, 0.9, 2.0),
                                          (4096, 0.25, 1.0), (16384, 0.2, 1.2), (5000, 0.05, 0.5)])
def test_keep_probs_invariants_and_sort_solver(n, rho, sigma):
    rng = np.random.default_rng(n)
    a = np.exp(sigma * rng.standard_normal(n)).astype(np.float32)
    a[rng.random(n) < 0.05] = 0.0
    budget = n * rho
    p, rounds = oracle.keep_probs(a, budget, return_rounds=True)
    nz = int((a > 0).sum())
    Beff = min(budget, nz)
    assert p.dtype == np.float32 and np.all(p >= 0) and np.all(p <= 1)
    assert np.all(p[a == 0] == 0) and np.all(p[a > 0] > 0)
    assert abs(p.astype(np.float64).sum() - Beff) <= 1e-5 * Beff
    un = (p < 1) & (a > 0)
    if un.sum() > 1:
        ratio = p[un].astype(np.float64) / a[un]
        assert ratio.max() / ratio.min() - 1 < 1e-6
        # anything sitting at one would have been pushed past one by that constant
        assert np.all(ratio.mean() * a[p == 1].astype(np.float64) >= 1 - 1e-6)
    ref = _waterfill_by_sorting(a, budget)
    np.testing.assert_allclose(p, ref, rtol=2e-7, atol=0)
    assert 1 <= rounds <= n


def test_keep_probs_special_cases():
    # equal scores -> everyone gets rho
    p = oracle.keep_probs(np.full(40, 3.25, np.float32), 40 * 0.35)
    np.testing.assert_allclose(p, 0.35, rtol=1e-6)
    # keep ratio one -> everyone with a positive score is kept for sure
    a = np.array([5, 0, 1e-3, 7, 0.5], np.float32)
    assert np.array_equal(oracle.keep_probs(a, 5.0), np.array([1, 0, 1, 1, 1], np.float32))
    assert np.array_equal(oracle.keep_probs(a, 4.0), np.array([1, 0, 1, 1, 1], np.float32))
    # one huge score takes 1, the others share budget - 1 in proportion
    a = np.array([1e6, 1, 2, 3, 4], np.float32)
    p = oracle.keep_probs(a, 2.0)
    np.testing.assert_allclose(p, [1, 0.1, 0.2, 0.3, 0.4], rtol=1e-6)
    # all zero -> all zero; empty -> empty
    assert np.all(oracle.keep_probs(np.zeros(9, np.float32), 3.0) == 0)
    assert oracle.keep_probs(np.zeros(0, np.float32), 0.0).size == 0
    # cascade: capping one entry pushes the next one over
    a = np.array([10, 6, 1, 1, 1, 1], np.float32)
    p = oracle.keep_probs(a, 3.0)
    np.testing.assert_allclose(p, [1, 1, 0.25, 0.25, 0.25, 0.25], rtol=1e-6)


def test_keep_probs_minimise_the_variance():
    # p minimises sum a_i^2 / p_i among feasible p (Sec. 4.1): no small budget-preserving
    # move between two coordinates lowers it.
    rng = np.random.default_rng(11)
    for trial in range(20):
        n = int(rng.integers(2, 7))
        a = np.exp(1.5 * rng.standard_normal(n)).astype(np.float32)
        budget = float(rng.uniform(0.3, n - 0.2))
        p = oracle.keep_probs(a, budget).astype(np.float64)
        a64 = a.astype(np.float64)

        def cost(v):
            return float((a64**2 / v).sum())

        base = cost(p)
        for i, j in itertools.permutations(range(n), 2):
            for eps in (1e-3, 1e-2):
                v = p.copy()
                v[i] += eps
                v[j] -= eps
                if v[i] > 1 or v[j] <= 0:
                    continue
                assert cost(v) >= base * (1 - 1e-9)


# ------------------------------------------------------------------ masks

def test_sample_mask_is_the_philox_threshold():
    rng = np.random.default_rng(3)
    prob = rng.random(500).astype(np.float32)
    prob[:10] = 1.0
    prob[10:20] = 0.0
    seed, layer, stream, draw = 0x1234567890ABCDEF, 17, 1, 3
    mask, idx = oracle.sample_mask(prob, seed, layer, stream, draw)
    for r in range(500):
        w = oracle.philox4x32_10([r, layer, stream, draw], [seed & 0xFFFFFFFF, seed >> 32])
        u = np.float32((int(w[0]) >> 8) / 2.0**24)
        assert mask[r] == (1 if u < prob[r] else 0)
    assert np.all(mask[:10] == 1) and np.all(mask[10:20] == 0)
    assert np.array_equal(idx, np.nonzero(mask)[0])
    assert np.all(np.diff(idx) > 0) and idx.size == mask.sum()


def test_sample_mask_keep_frequency_and_expected_count():
    # E[kept] = sum p = N rho (Sec. 4.1); per-row frequency within binomial 5 sigma
    prob = oracle.keep_probs(np.exp(np.random.default_rng(4).standard_normal(48)).astype(np.float32), 48 * 0.4)
    draws = 4000
    hits = np.zeros(48)
    for d in range(draws):
        m, _ = oracle.sample_mask(prob, 7, 2, 0, d)
        hits += m
    sd = np.sqrt(prob * (1 - prob) * draws) + 1e-9
    assert np.all(np.abs(hits - prob * draws) <= 5 * sd + 1)
    assert abs(hits.sum() / draws - 48 * 0.4) < 0.2


def test_leverage_scores_and_row_scale_follow_their_formulas():
    rng = np.random.default_rng(8)
    N, T = 6, 9
    gsq = rng.random(N * T).astype(np.float32) * 10
    xsq = rng.random(N * T).astype(np.float32) * 10
    p = rng.uniform(0.1, 1, N).astype(np.float32)
    maskA = np.array([1, 0, 1, 1, 0, 1], np.uint8)
    s = oracle.leverage_scores(gsq, xsq, p, maskA, N, T)
    ref = np.repeat(maskA / p.astype(np.float64), T) * np.sqrt(gsq.astype(np.float64)) * np.sqrt(xsq.astype(np.float64))
    np.testing.assert_allclose(s, ref, rtol=3e-7)
    assert np.all(s.reshape(N, T)[maskA == 0] == 0)
    q = rng.uniform(0.1, 1, N * T).astype(np.float32)
    maskW = (rng.random(N * T) < 0.5).astype(np.uint8)
    sc = oracle.row_scale(p, q, maskW, N, T)
    ref = maskW / (np.repeat(p.astype(np.float64), T) * q)
    np.testing.assert_allclose(sc, ref, rtol=3e-7)


# ------------------------------------------- keep ratio 1 = exact backward

@pytest.mark.parametrize("dtype", [F32, BF16])
def test_keep_ratio_one_is_the_dense_backward(dtype):
    spec = workloads.LayerSpec("t", dtype, 6, 21, 72, 40, 1.0, 1.0, layer=3, seed=5, gen_seed=1, token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    plan, dX, dW = oracle.linear_backward(G, X, W, dtype, spec.N, spec.T, 1.0, 1.0, 5, 3, 0)
    assert np.all(plan.p == 1) and np.all(plan.q == 1) and np.all(plan.maskA == 1) and np.all(plan.maskW == 1)
    assert np.array_equal(plan.idxW, np.arange(spec.R)) and np.all(plan.scaleW == 1)
    g, x, w = (oracle.to_f64(a, dtype) for a in (G, X, W))
    np.testing.assert_allclose(dX, g @ w, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dW, g.T @ x, rtol=1e-12, atol=1e-11)


def test_gradients_with_given_masks_match_matmul():
    # dX = diag(m/p) G W and dW = G^T diag(scale) X for arbitrary masks (textbook GEMMs)
    rng = np.random.default_rng(12)
    N, T, kin, kout = 4, 5, 24, 16
    G = rng.standard_normal((N * T, kout)).astype(np.float32)
    X = rng.standard_normal((N * T, kin)).astype(np.float32)
    W = rng.standard_normal((kout, kin)).astype(np.float32)
    p = np.array([0.5, 1.0, 0.25, 0.8], np.float32)
    maskA = np.array([1, 0, 1, 1], np.uint8)
    dX = oracle.dgrad(G, W, F32, N, T, p, maskA)
    m = np.repeat(maskA / p.astype(np.float64), T)
    np.testing.assert_allclose(dX, (G.astype(np.float64) * m[:, None]) @ W.astype(np.float64), rtol=1e-12, atol=1e-12)
    scale = (rng.random(N * T) * (rng.random(N * T) < 0.6)).astype(np.float32)
    dW = oracle.wgrad(G, X, F32, scale)
    np.testing.assert_allclose(dW, (G.astype(np.float64) * scale.astype(np.float64)[:, None]).T @ X.astype(np.float64),
                               rtol=1e-12, atol=1e-12)
    rows = np.array([0, 7, 19, 12])
    cols = np.array([0, 23, 5, 11])
    np.testing.assert_allclose(oracle.dgrad_at(G, W, F32, T, p, maskA, rows, cols), dX[rows, cols], rtol=1e-12, atol=1e-13)
    orow = np.array([0, 15, 3])
    kcol = np.array([23, 0, 7])
    np.testing.assert_allclose(oracle.wgrad_at(G, X, F32, scale, orow, kcol), dW[orow, kcol], rtol=1e-12, atol=1e-13)


def test_cast_to_bf16_is_round_to_nearest_even():
    import torch
    rng = np.random.default_rng(13)
    a = (rng.standard_normal(5000) * np.exp(3 * rng.standard_normal(5000)))
    a[:4] = [1.0 + 2**-8, 1.0 + 3 * 2**-8, -(1.0 + 2**-8), 0.0]       # ties
    got = oracle.cast_from_f64(a, BF16)
    ref = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)
    assert np.array_equal(workloads.f32_to_bf16_bits(a.astype(np.float32)), ref)
    assert np.array_equal(oracle.bf16_to_f32(ref), workloads.bf16_bits_to_f32(ref))


# ----------------------- brute force over every mask on a tiny problem

def _tiny(seed=21, N=3, T=2, kin=4, kout=4):
    rng = np.random.default_rng(seed)
    G = (rng.standard_normal((N, T, kout)) * np.exp(rng.standard_normal((N, 1, 1)))).astype(np.float32).reshape(N * T, kout)
    X = rng.standard_normal((N * T, kin)).astype(np.float32)
    return G, X


def _enumerate(N, T, G, X, rho, nu):
    """Yields (probability, maskA, p, q, score, maskW) over every (data mask, token mask)
    pair, with probabilities from the oracle's own p and q but no random numbers."""
    gsq = oracle.row_sumsq(G, F32)
    gnorm = oracle.sample_norms(gsq, N, T)
    p = oracle.keep_probs(gnorm, N * rho)
    for bitsA in itertools.product([0, 1], repeat=N):
        maskA = np.array(bitsA, np.uint8)
        prA = np.prod(np.where(maskA == 1, p.astype(np.float64), 1 - p.astype(np.float64)))
        if prA == 0:
            continue
        xsq = oracle.row_sumsq(X, F32, T, maskA)
        score = oracle.leverage_scores(gsq, xsq, p, maskA, N, T)
        q = oracle.keep_probs(score, N * T * rho * nu)
        live = np.nonzero(q > 0)[0]
        for bitsW in itertools.product([0, 1], repeat=live.size):
            maskW = np.zeros(N * T, np.uint8)
            maskW[live] = bitsW
            q64 = q.astype(np.float64)
            prW = np.prod(np.where(maskW[live] == 1, q64[live], 1 - q64[live]))
            if prW == 0:
                continue
            yield prA, prW, maskA, p, gnorm, q, score, maskW


def test_brute_force_mean_and_variance_of_both_samplers():
    N, T = 3, 2
    G, X = _tiny()
    rho, nu = 0.6, 0.5
    g, x = G.astype(np.float64), X.astype(np.float64)
    exact_dW = g.T @ x
    eye = np.eye(4, dtype=np.float32)

    mean_dW = np.zeros_like(exact_dW)
    mean_Ghat = np.zeros_like(g)
    second_dW = 0.0
    second_Ghat = 0.0
    expected_eq3 = 0.0
    seenA = {}
    for prA, prW, maskA, p, gnorm, q, score, maskW in _enumerate(N, T, G, X, rho, nu):
        keyA = tuple(maskA)
        dW = oracle.wgrad(G, X, F32, oracle.row_scale(p, q, maskW, N, T))
        mean_dW += prA * prW * dW
        second_dW += prA * prW * (dW**2).sum()
        if keyA not in seenA:
            # quantities that depend on the data mask only
            Ghat = oracle.dgrad(G, eye, F32, N, T, p, maskA)          # W = I gives SampleA(G) itself
            dW_A = oracle.wgrad(G, X, F32, oracle.row_scale(p, np.repeat(maskA, T).astype(np.float32),
                                                            np.repeat(maskA, T), N, T))
            seenA[keyA] = dict(pr=prA, dW_A=dW_A, eq3=oracle.var_w_eq3(q, score), cond_mean=np.zeros_like(dW),
                               cond_second=0.0)
            mean_Ghat += prA * Ghat
            second_Ghat += prA * (Ghat**2).sum()
            expected_eq3 += prA * seenA[keyA]["eq3"]
        seenA[keyA]["cond_mean"] += prW * dW
        seenA[keyA]["cond_second"] += prW * (dW**2).sum()

    assert abs(sum(v["pr"] for v in seenA.values()) - 1) < 1e-6
    # unbiased (Sec. 4.1, App. proof)
    np.testing.assert_allclose(mean_Ghat, g, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(mean_dW, exact_dW, rtol=1e-5, atol=1e-5)
    # Var[Ghat] equals the closed form of Sec. 4.1
    p, gnorm = next(_enumerate(N, T, G, X, rho, nu))[3:5]
    var_Ghat = second_Ghat - (g**2).sum()
    np.testing.assert_allclose(var_Ghat, oracle.var_act_closed(p, gnorm), rtol=1e-5)
    # given the data mask: mean of dW is the SampleA-only dW, its variance is Eq. 3
    for v in seenA.values():
        np.testing.assert_allclose(v["cond_mean"], v["dW_A"], rtol=1e-5, atol=1e-5)
        cond_var = v["cond_second"] - (v["dW_A"] ** 2).sum()
        np.testing.assert_allclose(cond_var, v["eq3"], rtol=1e-4, atol=1e-6)
    # law of total variance (Sec. 5): Var = Var_A[E(dW|A)] + E_A[Eq. 3]
    p64 = p.astype(np.float64)
    var_A = sum((1 - p64[i]) / p64[i] * ((g[i * T:(i + 1) * T].T @ x[i * T:(i + 1) * T]) ** 2).sum() for i in range(N))
    total = second_dW - (exact_dW**2).sum()
    np.testing.assert_allclose(total, var_A + expected_eq3, rtol=1e-4)


# ------------------------------------- Monte Carlo with the real Philox

def test_monte_carlo_mean_converges_to_exact_gradients():
    spec = workloads.LayerSpec("mc", F32, 8, 6, 12, 10, 0.5, 0.5, layer=2, seed=77, gen_seed=3, token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    g, x, w = (a.astype(np.float64) for a in (G, X, W))
    S = 600
    mdX = np.zeros((spec.R, spec.K_in))
    mdW = np.zeros((spec.K_out, spec.K_in))
    eq3 = 0.0
    cntA = cntW = 0
    for d in range(S):
        plan, dX, dW = oracle.linear_backward(G, X, W, F32, spec.N, spec.T, spec.rho, spec.nu, spec.seed, spec.layer, d)
        mdX += dX / S
        mdW += dW / S
        eq3 += oracle.var_w_eq3(plan.q, plan.score) / S
        cntA += plan.idxA.size
        cntW += plan.idxW.size
    p = plan.p.astype(np.float64)
    T = spec.T
    var_dX = sum((1 - p[i]) / p[i] * ((g[i * T:(i + 1) * T] @ w) ** 2).sum() for i in range(spec.N))
    var_A = sum((1 - p[i]) / p[i] * ((g[i * T:(i + 1) * T].T @ x[i * T:(i + 1) * T]) ** 2).sum() for i in range(spec.N))
    err_dX = ((mdX - g @ w) ** 2).sum()
    err_dW = ((mdW - g.T @ x) ** 2).sum()
    # E||mean - exact||^2 = Var / S; a biased estimator would sit orders of magnitude above
    assert err_dX < 3 * var_dX / S
    assert err_dW < 3 * (var_A + eq3) / S
    assert err_dX > 0.1 * var_dX / S and err_dW > 0.1 * (var_A + eq3) / S
    # expected kept counts: N rho samples, N T rho nu tokens (Sec. 4.1, 4.2)
    assert abs(cntA / S - spec.N * spec.rho) < 0.25
    assert abs(cntW / S - spec.R * spec.rho * spec.nu) < 0.05 * spec.R * spec.rho * spec.nu + 1


def test_variance_probe_converges_to_closed_forms():
    spec = workloads.LayerSpec("probe", F32, 8, 6, 12, 10, 0.5, 0.5, layer=4, seed=5, gen_seed=4, token_sigma=0.5)
    G, X, W = workloads.make_layer(spec)
    g, x = G.astype(np.float64), X.astype(np.float64)
    M = 400
    out = oracle.variance_probe(G, X, F32, spec.N, spec.T, spec.rho, spec.nu, spec.seed, spec.layer, 0, M)
    plan = oracle.sampling_plan(G, X, F32, spec.N, spec.T, spec.rho, spec.nu, spec.seed, spec.layer, 0)
    p = plan.p.astype(np.float64)
    T = spec.T
    assert out[0] == oracle.var_act_closed(plan.p, plan.gnorm)
    np.testing.assert_allclose(out[0], ((1 - p) / p * (g**2).reshape(spec.N, -1).sum(axis=1)).sum(), rtol=1e-5)
    var_A = sum((1 - p[i]) / p[i] * ((g[i * T:(i + 1) * T].T @ x[i * T:(i + 1) * T]) ** 2).sum() for i in range(spec.N))
    np.testing.assert_allclose(out[2], var_A, rtol=0.2)
    np.testing.assert_allclose(out[3], var_A + out[1], rtol=0.2)


def test_config_one_runs_in_seconds_and_keeps_about_the_stated_fraction():
    spec = workloads.config("single_fp32")[0]
    G, X, W = workloads.make_layer(spec)
    plan, dX, dW = oracle.linear_backward(G, X, W, F32, spec.N, spec.T, spec.rho, spec.nu, spec.seed, spec.layer, 0)
    assert abs(plan.p.astype(np.float64).sum() - spec.N * spec.rho) < 1e-4
    assert abs(plan.q.astype(np.float64).sum() - min(spec.R * spec.rho * spec.nu, (plan.score > 0).sum())) < 1e-2
    dropped = np.repeat(plan.maskA == 0, spec.T)
    assert np.all(dX[dropped] == 0) and np.all(np.abs(dX[~dropped]).sum(axis=1) > 0)
    assert np.all(plan.scaleW[plan.maskW == 0] == 0) and np.all(plan.scaleW[plan.maskW == 1] >= 1)


def test_jacobian_product_is_the_chain_rule_by_finite_differences():
    """App. E (proof of unbiasedness): behind an elementwise layer h = phi(z) the activation gradient is (G W) * phi'(z).
    Checked against central differences of L(z) = sum(G * (phi(z) W^T)) on a tiny case, all samples kept."""
    rng = np.random.default_rng(4)
    N, T, K_in, K_out = 2, 3, 5, 4
    R = N * T
    z = rng.standard_normal((R, K_in))
    W = rng.standard_normal((K_out, K_in)).astype(np.float32)
    G = rng.standard_normal((R, K_out)).astype(np.float32)
    phi = np.tanh
    J = (1.0 - np.tanh(z) ** 2).astype(np.float32)

    def loss(zz):
        return float(np.sum(G.astype(np.float64) * (phi(zz) @ W.astype(np.float64).T)))

    want = np.zeros_like(z)
    h = 1e-5
    for r in range(R):
        for k in range(K_in):
            e = np.zeros_like(z)
            e[r, k] = h
            want[r, k] = (loss(z + e) - loss(z - e)) / (2 * h)
    p = np.ones(N, np.float32)
    got = oracle.dgrad_jacobian(G, W, J, oracle.F32, N, T, p, np.ones(N, np.uint8))
    np.testing.assert_allclose(got, want, rtol=1e-5, atol=1e-7)
    # J = 1 is the plain activation gradient; a dropped sample stays zero whatever J holds
    ones = np.ones((R, K_in), np.float32)
    mask = np.array([1, 0], np.uint8)
    plain = oracle.dgrad(G, W, oracle.F32, N, T, p, mask)
    assert np.array_equal(oracle.dgrad_jacobian(G, W, ones, oracle.F32, N, T, p, mask), plain)
    assert np.all(oracle.dgrad_jacobian(G, W, J, oracle.F32, N, T, p, mask)[T:] == 0)


def test_squared_difference_and_exact_weight_gradient_against_numpy():
    """The two helpers the Monte-Carlo lines of Alg. 1 lean on: ||a - b||_F^2 (exact on small integers, where
    every partial sum is representable, and numpy's fp64 value elsewhere) and the exact weight gradient
    G^T X, the keep-ratio-one state the sampled gradients are compared with (numpy fp64 matmul on the same
    values; a transposed operand or a dropped row shows)."""
    rng = np.random.default_rng(5)
    a = rng.integers(-8, 9, size=(37, 53)).astype(np.float32)
    b = rng.integers(-8, 9, size=(37, 53)).astype(np.float32)
    assert oracle.sq_diff(a, b) == float(((a.astype(np.int64) - b.astype(np.int64)) ** 2).sum())
    assert oracle.sq_diff(a, a) == 0.0
    x = rng.standard_normal((64, 40)).astype(np.float32)
    y = rng.standard_normal((64, 40)).astype(np.float32)
    want = float(((x.astype(np.float64) - y.astype(np.float64)) ** 2).sum())
    assert oracle.sq_diff(x, y) == pytest.approx(want, rel=1e-12)
    assert oracle.sq_diff(x, y) == oracle.sq_diff(y, x)
    for dtype in (F32, BF16):
        R, K_out, K_in = 45, 24, 40                          # nothing square: a transposition changes the shape
        G32 = rng.standard_normal((R, K_out)).astype(np.float32)
        X32 = rng.standard_normal((R, K_in)).astype(np.float32)
        G = workloads.f32_to_bf16_bits(G32) if dtype == BF16 else G32
        X = workloads.f32_to_bf16_bits(X32) if dtype == BF16 else X32
        Gv, Xv = oracle.to_f64(G, dtype), oracle.to_f64(X, dtype)
        got = oracle.exact_wgrad(G, X, dtype)
        assert got.shape == (K_out, K_in)
        np.testing.assert_allclose(got, Gv.T @ Xv, rtol=1e-12, atol=1e-12)
