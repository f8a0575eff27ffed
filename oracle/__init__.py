"""VCAS CPU oracle -- TEST INFRASTRUCTURE ONLY.

numpy front end of ``vcas_oracle.c``: the sampled backward pass of a linear
layer (VCAS paper Sec. 4.1 SampleA, Sec. 4.2 SampleW, Eq. 3; the variance
lines of Alg. 1) taken step by step on the CPU.  Only the tests, the smoke
check and the benchmark's cpu-baseline leg may import this package; the GPU
library and its binding never do, and this package never imports them.

Arrays: fp32 tensors are ``np.float32``; bf16 tensors are ``np.uint16`` bit
patterns; ``dtype`` is ``F32`` or ``BF16``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

F32, BF16 = 0, 1
STREAM_A, STREAM_W = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vcas_oracle.c")
_LIB = os.path.join(_HERE, "libvcas_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no fp contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_uniform.restype = C.c_float
        _lib.orc_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        _lib.orc_var_act_closed.restype = C.c_double
        _lib.orc_var_w_eq3.restype = C.c_double
        _lib.orc_sq_diff.restype = C.c_double
        _lib.orc_keep_probs.restype = C.c_int
        _lib.orc_sample_mask.restype = C.c_int
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _check(a: np.ndarray, dtype: int) -> np.ndarray:
    want = np.uint16 if dtype == BF16 else np.float32
    assert a.dtype == want, (a.dtype, want)
    return np.ascontiguousarray(a)


def num_threads() -> int:
    return int(_L().orc_num_threads())


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, np.float32)
    _L().orc_bf16_to_f32(_p(bits), C.c_int64(bits.size), _p(out))
    return out


def to_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    return (bf16_to_f32(a) if dtype == BF16 else a).astype(np.float64)


def cast_from_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    out = np.empty(a.shape, np.uint16 if dtype == BF16 else np.float32)
    _L().orc_cast_from_f64(_p(a), C.c_int64(a.size), C.c_int(dtype), _p(out))
    return out


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.empty(4, np.uint32)
    _L().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def uniform(seed: int, layer: int, stream: int, draw: int, row: int) -> float:
    return float(_L().orc_uniform(seed, layer, stream, draw, row))


def row_sumsq(A: np.ndarray, dtype: int, T: int = 1, sample_keep: np.ndarray | None = None) -> np.ndarray:
    """fp32 squared row norms of A[R,K] in the written-down order (pairwise, neighbours first)."""
    A = _check(A, dtype)
    R, K = A.shape
    out = np.empty(R, np.float32)
    keep = None if sample_keep is None else np.ascontiguousarray(sample_keep, dtype=np.uint8)
    _L().orc_row_sumsq(_p(A), C.c_int(dtype), C.c_int64(R), C.c_int(K), C.c_int(T),
                       None if keep is None else _p(keep), _p(out))
    return out


def block_sumsq(A: np.ndarray, dtype: int, width: int = 64) -> np.ndarray:
    """Sums of squares of A[R,K] by blocks of `width` columns (a power of two), [R, ceil(K/width)] fp32: subtrees
    of the pairwise order of row_sumsq (what the dgrad of the layer above leaves for a layer inside a stack, Sec. 4)."""
    A = _check(A, dtype)
    R, K = A.shape
    assert width >= 1 and width & (width - 1) == 0
    out = np.empty((R, (K + width - 1) // width), np.float32)
    _L().orc_block_sumsq(_p(A), C.c_int(dtype), C.c_int64(R), C.c_int(K), C.c_int(width), _p(out))
    return out


def rows_from_blocks(blocks: np.ndarray, T: int = 1, sample_keep: np.ndarray | None = None) -> np.ndarray:
    """Row sums from their block sums, pairwise, neighbours first; rows of dropped samples get 0."""
    blocks = np.ascontiguousarray(blocks, dtype=np.float32)
    R, nb = blocks.shape
    out = np.empty(R, np.float32)
    keep = None if sample_keep is None else np.ascontiguousarray(sample_keep, dtype=np.uint8)
    _L().orc_rows_from_blocks(_p(blocks), C.c_int64(R), C.c_int(nb), C.c_int(T), None if keep is None else _p(keep),
                              _p(out))
    return out


def row_sumsq_f64(A: np.ndarray, dtype: int) -> np.ndarray:
    A = _check(A, dtype)
    R, K = A.shape
    out = np.empty(R, np.float64)
    _L().orc_row_sumsq_f64(_p(A), C.c_int(dtype), C.c_int64(R), C.c_int(K), _p(out))
    return out


def sample_norms(gsq: np.ndarray, N: int, T: int) -> np.ndarray:
    gsq = _check(gsq, F32)
    assert gsq.size == N * T
    out = np.empty(N, np.float32)
    _L().orc_sample_norms(_p(gsq), C.c_int(N), C.c_int(T), _p(out))
    return out


def keep_probs(score: np.ndarray, budget: float, return_rounds: bool = False):
    score = _check(score, F32)
    out = np.empty(score.size, np.float32)
    rounds = _L().orc_keep_probs(_p(score), C.c_int(score.size), C.c_double(budget), _p(out))
    return (out, int(rounds)) if return_rounds else out


def sample_mask(prob: np.ndarray, seed: int, layer: int, stream: int, draw: int):
    """Returns (mask u8[n], idx i32[count] ascending)."""
    prob = _check(prob, F32)
    n = prob.size
    mask = np.empty(n, np.uint8)
    idx = np.empty(max(n, 1), np.int32)
    cnt = _L().orc_sample_mask(_p(prob), C.c_int(n), C.c_uint64(seed), C.c_uint32(layer),
                               C.c_uint32(stream), C.c_uint32(draw), _p(mask), _p(idx))
    return mask, idx[:cnt].copy()


def leverage_scores(gsq, xsq, p, maskA, N: int, T: int) -> np.ndarray:
    out = np.empty(N * T, np.float32)
    _L().orc_leverage_scores(_p(_check(gsq, F32)), _p(_check(xsq, F32)), _p(_check(p, F32)),
                             _p(np.ascontiguousarray(maskA, np.uint8)), C.c_int(N), C.c_int(T), _p(out))
    return out


def row_scale(p, q, maskW, N: int, T: int) -> np.ndarray:
    out = np.empty(N * T, np.float32)
    _L().orc_row_scale(_p(_check(p, F32)), _p(_check(q, F32)),
                       _p(np.ascontiguousarray(maskW, np.uint8)), C.c_int(N), C.c_int(T), _p(out))
    return out


def dgrad(G, W, dtype: int, N: int, T: int, p, maskA) -> np.ndarray:
    """fp64 dX[R,K_in] = SampleA(G) W."""
    G, W = _check(G, dtype), _check(W, dtype)
    K_out, K_in = W.shape
    assert G.shape == (N * T, K_out)
    out = np.empty((N * T, K_in), np.float64)
    _L().orc_dgrad(_p(G), _p(W), C.c_int(dtype), C.c_int(N), C.c_int(T), C.c_int(K_in), C.c_int(K_out),
                   _p(_check(p, F32)), _p(np.ascontiguousarray(maskA, np.uint8)), _p(out))
    return out


def dgrad_jacobian(G, W, J, dtype: int, N: int, T: int, p, maskA) -> np.ndarray:
    """fp64 (SampleA(G) W) * J: the activation gradient passed through an elementwise layer whose
    saved Jacobian is J [R, K_in] (App. E, proof of unbiasedness: the Hadamard product for non-linear layers such as ReLU)."""
    J = _check(J, dtype)
    out = dgrad(G, W, dtype, N, T, p, maskA)
    assert J.shape == out.shape
    return out * to_f64(J, dtype)


def wgrad(G, X, dtype: int, scale) -> np.ndarray:
    """fp64 dW[K_out,K_in] = sum_t scale_t g_t x_t^T."""
    G, X = _check(G, dtype), _check(X, dtype)
    R, K_out = G.shape
    K_in = X.shape[1]
    assert X.shape[0] == R
    out = np.empty((K_out, K_in), np.float64)
    _L().orc_wgrad(_p(G), _p(X), C.c_int(dtype), C.c_int64(R), C.c_int(K_in), C.c_int(K_out),
                   _p(_check(scale, F32)), _p(out))
    return out


def dgrad_at(G, W, dtype: int, T: int, p, maskA, rows, cols) -> np.ndarray:
    G, W = _check(G, dtype), _check(W, dtype)
    K_out, K_in = W.shape
    rows = np.ascontiguousarray(rows, np.int64)
    cols = np.ascontiguousarray(cols, np.int32)
    out = np.empty(rows.size, np.float64)
    _L().orc_dgrad_at(_p(G), _p(W), C.c_int(dtype), C.c_int(T), C.c_int(K_in), C.c_int(K_out),
                      _p(_check(p, F32)), _p(np.ascontiguousarray(maskA, np.uint8)), _p(rows), _p(cols),
                      C.c_int64(rows.size), _p(out))
    return out


def wgrad_at(G, X, dtype: int, scale, orow, kcol) -> np.ndarray:
    G, X = _check(G, dtype), _check(X, dtype)
    R, K_out = G.shape
    K_in = X.shape[1]
    orow = np.ascontiguousarray(orow, np.int32)
    kcol = np.ascontiguousarray(kcol, np.int32)
    out = np.empty(orow.size, np.float64)
    _L().orc_wgrad_at(_p(G), _p(X), C.c_int(dtype), C.c_int64(R), C.c_int(K_in), C.c_int(K_out),
                      _p(_check(scale, F32)), _p(orow), _p(kcol), C.c_int64(orow.size), _p(out))
    return out


def var_act_closed(p, gnorm) -> float:
    return float(_L().orc_var_act_closed(_p(_check(p, F32)), _p(_check(gnorm, F32)), C.c_int(p.size)))


def var_w_eq3(q, score) -> float:
    return float(_L().orc_var_w_eq3(_p(_check(q, F32)), _p(_check(score, F32)), C.c_int64(q.size)))


def sq_diff(a, b) -> float:
    a = np.ascontiguousarray(a, np.float64)
    b = np.ascontiguousarray(b, np.float64)
    assert a.shape == b.shape
    return float(_L().orc_sq_diff(_p(a), _p(b), C.c_int64(a.size)))


@dataclass
class Plan:
    """Everything the sampling steps decide for one layer and one draw."""
    gsq: np.ndarray
    gnorm: np.ndarray
    p: np.ndarray
    maskA: np.ndarray
    idxA: np.ndarray
    xsq: np.ndarray
    score: np.ndarray
    q: np.ndarray
    maskW: np.ndarray
    idxW: np.ndarray
    scaleW: np.ndarray
    extra: dict = field(default_factory=dict)


def sampling_plan(G, X, dtype: int, N: int, T: int, rho: float, nu: float,
                  seed: int, layer: int, draw: int, token_sampling: bool = True) -> Plan:
    """Steps of Sec. 4.1 and 4.2 up to the masks, in the paper's order.

    With ``token_sampling=False`` SampleW is skipped (Alg. 1's "SampleA only"
    backward): every token of a kept sample is kept with q = 1.
    """
    R = N * T
    gsq = row_sumsq(G, dtype)
    gnorm = sample_norms(gsq, N, T)
    p = keep_probs(gnorm, N * rho)
    maskA, idxA = sample_mask(p, seed, layer, STREAM_A, draw)
    xsq = row_sumsq(X, dtype, T, maskA)
    score = leverage_scores(gsq, xsq, p, maskA, N, T)
    if token_sampling:
        q = keep_probs(score, R * rho * nu)
        maskW, idxW = sample_mask(q, seed, layer, STREAM_W, draw)
    else:
        q = np.repeat(maskA, T).astype(np.float32)
        maskW = np.repeat(maskA, T).astype(np.uint8)
        idxW = np.nonzero(maskW)[0].astype(np.int32)
    scaleW = row_scale(p, q, maskW, N, T)
    return Plan(gsq, gnorm, p, maskA, idxA, xsq, score, q, maskW, idxW, scaleW)


def linear_backward(G, X, W, dtype: int, N: int, T: int, rho: float, nu: float,
                    seed: int, layer: int, draw: int, token_sampling: bool = True):
    """Returns (plan, dX fp64 [R,K_in], dW fp64 [K_out,K_in])."""
    plan = sampling_plan(G, X, dtype, N, T, rho, nu, seed, layer, draw, token_sampling)
    dX = dgrad(G, W, dtype, N, T, plan.p, plan.maskA)
    dW = wgrad(G, X, dtype, plan.scaleW)
    return plan, dX, dW


def exact_wgrad(G, X, dtype: int) -> np.ndarray:
    """Exact dW = G^T X (every scale one), the keep-ratio-1 state of Alg. 1."""
    return wgrad(G, X, dtype, np.ones(G.shape[0], np.float32))


def variance_probe(G, X, dtype: int, N: int, T: int, rho: float, nu: float,
                   seed: int, layer: int, base_draw: int, M: int) -> np.ndarray:
    """The four scalars of the variance probe, fp64.

    [0] sum_i (1-p_i)/p_i ||G_i||_F^2                      (Sec. 4.1)
    [1] mean over draws of Eq. 3 under that draw's data mask
    [2] mean over draws of ||dW(SampleA only) - dW exact||_F^2   (Alg. 1, V_act line)
    [3] mean over draws of ||dW(SampleA+SampleW) - dW exact||_F^2
    """
    exact = exact_wgrad(G, X, dtype)
    out = np.zeros(4)
    for j in range(M):
        plan = sampling_plan(G, X, dtype, N, T, rho, nu, seed, layer, base_draw + j)
        planA = sampling_plan(G, X, dtype, N, T, rho, nu, seed, layer, base_draw + j, token_sampling=False)
        if j == 0:
            out[0] = var_act_closed(plan.p, plan.gnorm)
        out[1] += var_w_eq3(plan.q, plan.score) / M
        out[2] += sq_diff(wgrad(G, X, dtype, planA.scaleW), exact) / M
        out[3] += sq_diff(wgrad(G, X, dtype, plan.scaleW), exact) / M
    return out


# ---- adaptive keep ratios (Sec. 5, Alg. 1, App. D) ---------------------------------------------

def sparsity_ratio(gnorm, s: float) -> float:
    """Eq. 4: smallest fraction n/N of the largest sample norms that holds the share s of their sum."""
    gnorm = _check(gnorm, F32)
    fn = _L().orc_sparsity_ratio
    fn.restype = C.c_float
    return float(fn(_p(gnorm), C.c_int(gnorm.size), C.c_double(s)))


def grad_stats_update(grad, stride: int, i: int, mean, sqmean) -> None:
    """App. D's running mean / running square mean over every stride-th gradient entry, in place."""
    grad = _check(np.asarray(grad).reshape(-1), F32)
    assert mean.dtype == np.float32 and sqmean.dtype == np.float32 and mean.size == sqmean.size
    assert (mean.size - 1) * stride < grad.size
    _L().orc_grad_stats_update(_p(grad), C.c_int64(mean.size), C.c_int64(stride), C.c_int(i), _p(mean), _p(sqmean))


def grad_stats_variance(mean, sqmean, M: int) -> float:
    fn = _L().orc_grad_stats_variance
    fn.restype = C.c_double
    return float(fn(_p(_check(mean, F32)), _p(_check(sqmean, F32)), C.c_int64(mean.size), C.c_int(M)))


def sq_diff_strided(a, b, m: int, stride: int) -> float:
    fn = _L().orc_sq_diff_strided
    fn.restype = C.c_double
    a = _check(np.asarray(a).reshape(-1), F32)
    b = _check(np.asarray(b).reshape(-1), F32)
    return float(fn(_p(a), _p(b), C.c_int64(m), C.c_int64(stride)))


@dataclass
class ControllerParams:
    """Alg. 1's inputs.  beta < 1 is the paper's setting (0.95)."""
    alpha: float = 0.01
    beta: float = 0.95
    tau_act: float = 0.025
    tau_w: float = 0.025
    nu_min: float = 1.0 / 1024.0


def controller_update(prm: ControllerParams, s: float, nu, V_s: float, V_act: float, V_w, V_s_layer,
                      p_minus, p_plus):
    """One update of Alg. 1 (the lines after the Monte-Carlo loops).  Layers are ordered from the
    input (index 0) to the output; p_minus / p_plus are Eq. 4 evaluated, per layer, at s - alpha and
    s + alpha inside the loops and averaged (App. D).  Returns (s', rho', nu').

    Eq. 5: s' = s + alpha * sign(V_act - tau_act * V_s), sign(0) = +1, kept inside [0, 1].
    Eq. 4: rho'_l = max_{j <= l} p_j(s'), with p_j(s') taken from the side s actually moved to.
    Eq. 7 as printed multiplies nu_l by beta^{sign(.)}, which with beta < 1 lowers the keep ratio when
    the variance is too high; the reading taken here raises it: nu'_l = nu_l * beta^{-sign(V_w,l -
    tau_w V_s,l)}, kept inside [nu_min, 1]."""
    up = (V_act - prm.tau_act * V_s) >= 0.0
    s_new = min(1.0, max(0.0, s + (prm.alpha if up else -prm.alpha)))
    p = np.asarray(p_plus if up else p_minus, np.float64)
    rho = np.maximum.accumulate(p)
    rho = np.minimum(1.0, rho)
    nu = np.asarray(nu, np.float64).copy()
    V_w = np.asarray(V_w, np.float64)
    V_s_layer = np.asarray(V_s_layer, np.float64)
    for l in range(nu.size):
        too_high = (V_w[l] - prm.tau_w * V_s_layer[l]) >= 0.0
        nu[l] = nu[l] / prm.beta if too_high else nu[l] * prm.beta
        nu[l] = min(1.0, max(prm.nu_min, nu[l]))
    return s_new, rho, nu
