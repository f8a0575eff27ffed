"""ctypes binding of libvcas.so: same names as the C ABI (include/vcas.h),
argument marshalling only.  PyTorch supplies device memory and the stream;
every step of the path runs in the library's kernels.  There is no CPU
fallback: a missing library or a failing call raises."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch  # first: libvcas.so then binds to the HIP runtime torch has loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvcas.so")

VCAS_F32, VCAS_BF16 = 0, 1
STATUS = {0: "VCAS_OK", 1: "VCAS_EINVAL", 2: "VCAS_ENULL", 3: "VCAS_EDTYPE", 4: "VCAS_EWORKSPACE", 5: "VCAS_EHIP",
          6: "VCAS_ETOOBIG"}

EXPORTS = [
    "vcas_status_string", "vcas_workspace_bytes", "vcas_workspace_init", "vcas_row_norms", "vcas_keep_probs",
    "vcas_sample_compact", "vcas_leverage_scores", "vcas_row_scale", "vcas_sampled_dgrad", "vcas_sampled_dgrad_jac", "vcas_sampled_wgrad",
    "vcas_static_scratch_bytes", "vcas_sampled_wgrad_static", "vcas_sampled_dgrad_norms", "vcas_row_norms_from_blocks", "vcas_sq_blocks_bytes",
    "vcas_linear_backward", "vcas_backward_stack", "vcas_backward_data", "vcas_backward_data_chained", "vcas_backward_weight", "vcas_backward_weight_cached",
    "vcas_variance_probe", "vcas_sparsity_ratio", "vcas_grad_stats_update", "vcas_grad_stats_variance",
    "vcas_sq_diff_strided", "vcas_controller_update", "vcas_profile_begin", "vcas_profile_end",
]


class VcasError(RuntimeError):
    pass


class Shape(C.Structure):
    _fields_ = [("N", C.c_int32), ("T", C.c_int32), ("K_in", C.c_int32), ("K_out", C.c_int32), ("dtype", C.c_int32)]


class Rng(C.Structure):
    """vcas_rng; draw_offset is the data_ptr() of a device uint32 (or 0 / omitted)."""
    _fields_ = [("seed", C.c_uint64), ("layer", C.c_uint32), ("draw", C.c_uint32), ("draw_offset", C.c_void_p)]


class PlanPtrs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("gsq", "gnorm", "p", "maskA", "idxA", "cntA", "xsq", "score", "q",
                                          "maskW", "idxW", "cntW", "scaleW")]


class LayerArgs(C.Structure):
    """vcas_layer_args"""
    _fields_ = [("shape", Shape), ("G", C.c_void_p), ("X", C.c_void_p), ("W", C.c_void_p), ("rho", C.c_double),
                ("nu", C.c_double), ("rng", Rng), ("token_sampling", C.c_int32), ("plan", PlanPtrs),
                ("dX", C.c_void_p), ("dW", C.c_void_p), ("workspace", C.c_void_p), ("xsq_forward", C.c_void_p), ("sibling", C.c_int32),
                ("J", C.c_void_p), ("kept_above", C.c_void_p), ("leave_dropped_rows", C.c_int32),
                ("wgrad_fill", C.c_int32), ("dx_sq_blocks", C.c_void_p), ("g_sq_blocks", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Loads libvcas.so (build it first with paper_2402_17227_amd.build.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise VcasError(f"{LIB_PATH} is missing: run `python -m paper_2402_17227_amd.build` first")
        _lib = C.CDLL(LIB_PATH)
        _lib.vcas_status_string.restype = C.c_char_p
        _lib.vcas_workspace_bytes.restype = C.c_size_t
        _lib.vcas_workspace_bytes.argtypes = [C.POINTER(Shape)]
    return _lib


def _check(status: int, what: str):
    if status != 0:
        raise VcasError(f"{what}: {STATUS.get(status, status)} ({lib().vcas_status_string(status).decode()})")


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def shape_of(N: int, T: int, K_in: int, K_out: int, dtype: int) -> Shape:
    return Shape(N, T, K_in, K_out, dtype)


def to_device(a, dtype: int) -> torch.Tensor:
    """Host array (numpy fp32, or bf16 bit patterns as uint16) -> device tensor of the layer dtype; a copy,
    no arithmetic."""
    import numpy as np
    if dtype == VCAS_BF16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dtype_of(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return VCAS_BF16
    if t.dtype == torch.float32:
        return VCAS_F32
    raise VcasError(f"unsupported dtype {t.dtype}")


@dataclass
class Plan:
    """Device buffers for everything the sampling steps decide (vcas_plan)."""
    gsq: torch.Tensor
    gnorm: torch.Tensor
    p: torch.Tensor
    maskA: torch.Tensor
    idxA: torch.Tensor
    cntA: torch.Tensor
    xsq: torch.Tensor
    score: torch.Tensor
    q: torch.Tensor
    maskW: torch.Tensor
    idxW: torch.Tensor
    cntW: torch.Tensor
    scaleW: torch.Tensor

    @staticmethod
    def allocate(N: int, T: int, device="cuda") -> "Plan":
        R = N * T
        f = dict(dtype=torch.float32, device=device)
        return Plan(gsq=torch.empty(R, **f), gnorm=torch.empty(N, **f), p=torch.empty(N, **f),
                    maskA=torch.empty(N, dtype=torch.uint8, device=device),
                    idxA=torch.empty(N, dtype=torch.int32, device=device),
                    cntA=torch.zeros(1, dtype=torch.int32, device=device),
                    xsq=torch.empty(R, **f), score=torch.empty(R, **f), q=torch.empty(R, **f),
                    maskW=torch.empty(R, dtype=torch.uint8, device=device),
                    idxW=torch.empty(R, dtype=torch.int32, device=device),
                    cntW=torch.zeros(1, dtype=torch.int32, device=device), scaleW=torch.empty(R, **f))

    def ptrs(self) -> PlanPtrs:
        return PlanPtrs(*[t.data_ptr() for t in (self.gsq, self.gnorm, self.p, self.maskA, self.idxA, self.cntA,
                                                  self.xsq, self.score, self.q, self.maskW, self.idxW, self.cntW,
                                                  self.scaleW)])


def vcas_workspace_bytes(shape: Shape) -> int:
    return int(lib().vcas_workspace_bytes(C.byref(shape)))


def vcas_workspace_init(shape: Shape, workspace):
    _check(lib().vcas_workspace_init(C.byref(shape), _ptr(workspace), _stream()), "vcas_workspace_init")


def make_workspace(shape: Shape, device="cuda") -> torch.Tensor:
    nbytes = vcas_workspace_bytes(shape)
    if nbytes == 0:
        raise VcasError("bad shape")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    _check(lib().vcas_workspace_init(C.byref(shape), _ptr(ws), _stream()), "vcas_workspace_init")
    return ws


def vcas_row_norms(shape: Shape, G, X, sample_mask, gsq, xsq, gnorm):
    _check(lib().vcas_row_norms(C.byref(shape), _ptr(G), _ptr(X), _ptr(sample_mask), _ptr(gsq), _ptr(xsq),
                                _ptr(gnorm), _stream()), "vcas_row_norms")


def vcas_keep_probs(score, n: int, budget: float, prob):
    _check(lib().vcas_keep_probs(_ptr(score), C.c_int32(n), C.c_double(budget), _ptr(prob), _stream()),
           "vcas_keep_probs")


def vcas_sample_compact(prob, n: int, rng: Rng, stream_id: int, mask, idx, count):
    _check(lib().vcas_sample_compact(_ptr(prob), C.c_int32(n), C.byref(rng), C.c_uint32(stream_id), _ptr(mask),
                                     _ptr(idx), _ptr(count), _stream()), "vcas_sample_compact")


def vcas_leverage_scores(shape: Shape, gsq, xsq, p, maskA, score):
    _check(lib().vcas_leverage_scores(C.byref(shape), _ptr(gsq), _ptr(xsq), _ptr(p), _ptr(maskA), _ptr(score),
                                      _stream()), "vcas_leverage_scores")


def vcas_row_scale(shape: Shape, p, q, maskW, scaleW):
    _check(lib().vcas_row_scale(C.byref(shape), _ptr(p), _ptr(q), _ptr(maskW), _ptr(scaleW), _stream()),
           "vcas_row_scale")


def vcas_sampled_dgrad(shape: Shape, G, W, p, idxA, cntA, dX):
    _check(lib().vcas_sampled_dgrad(C.byref(shape), _ptr(G), _ptr(W), _ptr(p), _ptr(idxA), _ptr(cntA), _ptr(dX),
                                    _stream()), "vcas_sampled_dgrad")


def vcas_sampled_dgrad_jac(shape: Shape, G, W, p, idxA, cntA, J, dX):
    _check(lib().vcas_sampled_dgrad_jac(C.byref(shape), _ptr(G), _ptr(W), _ptr(p), _ptr(idxA), _ptr(cntA), _ptr(J),
                                        _ptr(dX), _stream()), "vcas_sampled_dgrad_jac")


def vcas_sampled_dgrad_norms(shape: Shape, G, W, p, idxA, cntA, J, dX, sq_blocks):
    _check(lib().vcas_sampled_dgrad_norms(C.byref(shape), _ptr(G), _ptr(W), _ptr(p), _ptr(idxA), _ptr(cntA), _ptr(J),
                                          _ptr(dX), _ptr(sq_blocks), _stream()), "vcas_sampled_dgrad_norms")


def vcas_sq_blocks_bytes(R: int, K: int) -> int:
    f = lib().vcas_sq_blocks_bytes
    f.restype = C.c_size_t
    return int(f(C.c_int64(R), C.c_int32(K)))


def make_sq_blocks(R: int, K: int, fill=None, device="cuda") -> torch.Tensor:
    """Device buffer for the block sums of squares of an [R, K] matrix, viewed [groups, R, 4] (see include/vcas.h)."""
    n = vcas_sq_blocks_bytes(R, K) // 4
    if n == 0:
        raise VcasError("bad sizes")
    t = torch.empty(n, dtype=torch.float32, device=device) if fill is None else torch.full((n,), fill, dtype=torch.float32, device=device)
    return t.view(-1, R, 4)


def vcas_row_norms_from_blocks(N: int, T: int, K: int, sq_blocks, sample_mask, sq, norm):
    _check(lib().vcas_row_norms_from_blocks(C.c_int32(N), C.c_int32(T), C.c_int32(K), _ptr(sq_blocks),
                                            _ptr(sample_mask), _ptr(sq), _ptr(norm), _stream()),
           "vcas_row_norms_from_blocks")


def vcas_sampled_wgrad(shape: Shape, G, X, row_scale, idxW, cntW, dW, workspace):
    _check(lib().vcas_sampled_wgrad(C.byref(shape), _ptr(G), _ptr(X), _ptr(row_scale), _ptr(idxW), _ptr(cntW),
                                    _ptr(dW), _ptr(workspace), _stream()), "vcas_sampled_wgrad")


def vcas_static_scratch_bytes() -> int:
    f = lib().vcas_static_scratch_bytes
    f.restype = C.c_size_t
    return int(f())


def vcas_sampled_wgrad_static(shape: Shape, G, X, row_scale, idxW, cntW, dW):
    _check(lib().vcas_sampled_wgrad_static(C.byref(shape), _ptr(G), _ptr(X), _ptr(row_scale), _ptr(idxW), _ptr(cntW),
                                           _ptr(dW), _stream()), "vcas_sampled_wgrad_static")


def vcas_linear_backward(shape: Shape, G, X, W, rho: float, nu: float, rng: Rng, token_sampling: bool, plan: Plan,
                         dX, dW, workspace, side_stream=None):
    """side_stream: a torch.cuda.Stream for the weight-gradient half (not joined by the call), or None."""
    ptrs = plan.ptrs()
    side = C.c_void_p(side_stream.cuda_stream if side_stream is not None else 0)
    _check(lib().vcas_linear_backward(C.byref(shape), _ptr(G), _ptr(X), _ptr(W), C.c_double(rho), C.c_double(nu),
                                      C.byref(rng), C.c_int32(1 if token_sampling else 0), C.byref(ptrs), _ptr(dX),
                                      _ptr(dW), _ptr(workspace), _stream(), side), "vcas_linear_backward")


def layer_args(shape: Shape, G, X, W, rho: float, nu: float, rng: Rng, token_sampling: bool, plan: Plan, dX, dW,
               workspace, xsq_forward=None, sibling=False, J=None, kept_above=None,
               leave_dropped_rows=False, wgrad_fill=0, dx_sq_blocks=None, g_sq_blocks=None) -> LayerArgs:
    """One entry of the array vcas_backward_stack takes (the tensors must stay alive while it is used)."""
    a = LayerArgs()
    a.shape = shape
    a.G, a.X, a.W = _ptr(G), _ptr(X), _ptr(W)
    a.rho, a.nu = rho, nu
    a.rng = rng
    a.token_sampling = 1 if token_sampling else 0
    a.plan = plan.ptrs()
    a.dX, a.dW, a.workspace = _ptr(dX), _ptr(dW), _ptr(workspace)
    a.xsq_forward = _ptr(xsq_forward)
    a.sibling = 1 if sibling else 0
    a.J, a.kept_above = _ptr(J), _ptr(kept_above)
    a.leave_dropped_rows = 1 if leave_dropped_rows else 0
    a.wgrad_fill = wgrad_fill
    a.dx_sq_blocks, a.g_sq_blocks = _ptr(dx_sq_blocks), _ptr(g_sq_blocks)
    return a


def make_stack(entries):
    """A C array of LayerArgs from a list of them."""
    return (LayerArgs * len(entries))(*entries)


def vcas_backward_stack(stack, group: int, sampler_stream=None, gemm_stream=None):
    """stack: what make_stack returned; streams: torch.cuda.Stream or None; runs on the current stream."""
    s2 = C.c_void_p(sampler_stream.cuda_stream if sampler_stream is not None else 0)
    s3 = C.c_void_p(gemm_stream.cuda_stream if gemm_stream is not None else 0)
    _check(lib().vcas_backward_stack(stack, C.c_int32(len(stack)), C.c_int32(group), _stream(), s2, s3),
           "vcas_backward_stack")


def vcas_backward_data(shape: Shape, G, X, W, rho: float, rng: Rng, token_sampling: bool, plan: Plan, dX, workspace):
    ptrs = plan.ptrs()
    _check(lib().vcas_backward_data(C.byref(shape), _ptr(G), _ptr(X), _ptr(W), C.c_double(rho), C.byref(rng),
                                    C.c_int32(1 if token_sampling else 0), C.byref(ptrs), _ptr(dX), _ptr(workspace),
                                    _stream()), "vcas_backward_data")


def vcas_backward_data_chained(shape: Shape, G, X, W, J, kept_above, fill_dropped_rows: bool, rho: float, rng: Rng,
                               token_sampling: bool, plan: Plan, dX, workspace):
    """J, kept_above: device tensors or None."""
    ptrs = plan.ptrs()
    _check(lib().vcas_backward_data_chained(C.byref(shape), _ptr(G), _ptr(X), _ptr(W), _ptr(J), _ptr(kept_above),
                                            C.c_int32(1 if fill_dropped_rows else 0), C.c_double(rho), C.byref(rng),
                                            C.c_int32(1 if token_sampling else 0), C.byref(ptrs), _ptr(dX),
                                            _ptr(workspace), _stream()), "vcas_backward_data_chained")


def vcas_backward_weight(shape: Shape, G, X, rho: float, nu: float, rng: Rng, token_sampling: bool, plan: Plan, dW,
                         workspace):
    ptrs = plan.ptrs()
    _check(lib().vcas_backward_weight(C.byref(shape), _ptr(G), _ptr(X), C.c_double(rho), C.c_double(nu),
                                      C.byref(rng), C.c_int32(1 if token_sampling else 0), C.byref(ptrs), _ptr(dW),
                                      _ptr(workspace), _stream()), "vcas_backward_weight")


def vcas_backward_weight_cached(shape: Shape, G, X, xsq_forward, rho: float, nu: float, rng: Rng, token_sampling: bool,
                                plan: Plan, dW, workspace):
    ptrs = plan.ptrs()
    _check(lib().vcas_backward_weight_cached(C.byref(shape), _ptr(G), _ptr(X), _ptr(xsq_forward), C.c_double(rho),
                                             C.c_double(nu), C.byref(rng), C.c_int32(1 if token_sampling else 0),
                                             C.byref(ptrs), _ptr(dW), _ptr(workspace), _stream()),
           "vcas_backward_weight_cached")


def vcas_variance_probe(shape: Shape, G, X, rho: float, nu: float, base: Rng, M: int, plan: Plan, out, workspace):
    ptrs = plan.ptrs()
    _check(lib().vcas_variance_probe(C.byref(shape), _ptr(G), _ptr(X), C.c_double(rho), C.c_double(nu),
                                     C.byref(base), C.c_int32(M), C.byref(ptrs), _ptr(out), _ptr(workspace),
                                     _stream()), "vcas_variance_probe")


def vcas_sparsity_ratio(gnorm, levels, p):
    """levels: host sequence of at most 8 values of s; p: device float tensor of that length."""
    arr = (C.c_double * len(levels))(*[float(v) for v in levels])
    _check(lib().vcas_sparsity_ratio(_ptr(gnorm), C.c_int32(gnorm.numel()), arr, C.c_int32(len(levels)), _ptr(p),
                                     _stream()), "vcas_sparsity_ratio")


def vcas_grad_stats_update(grad, m: int, stride: int, i: int, mean, sqmean):
    _check(lib().vcas_grad_stats_update(_ptr(grad), C.c_int64(m), C.c_int64(stride), C.c_int32(i), _ptr(mean),
                                        _ptr(sqmean), _stream()), "vcas_grad_stats_update")


def vcas_grad_stats_variance(mean, sqmean, M: int, out):
    _check(lib().vcas_grad_stats_variance(_ptr(mean), _ptr(sqmean), C.c_int64(mean.numel()), C.c_int32(M), _ptr(out),
                                          _stream()), "vcas_grad_stats_variance")


def vcas_sq_diff_strided(a, b, m: int, stride: int, weight: float, accumulate: bool, out):
    _check(lib().vcas_sq_diff_strided(_ptr(a), _ptr(b), C.c_int64(m), C.c_int64(stride), C.c_double(weight),
                                      C.c_int32(1 if accumulate else 0), _ptr(out), _stream()), "vcas_sq_diff_strided")


class ControllerParams(C.Structure):
    _fields_ = [("alpha", C.c_double), ("beta", C.c_double), ("tau_act", C.c_double), ("tau_w", C.c_double),
                ("nu_min", C.c_double)]


def vcas_controller_update(prm: ControllerParams, s: float, nu, V_s: float, V_act: float, V_w, V_s_layer, p_minus,
                           p_plus):
    """Host arithmetic only.  Returns (s', rho' list, nu' list)."""
    L = len(nu)
    vec = lambda v: (C.c_double * L)(*[float(x) for x in v])
    s_io = C.c_double(s)
    rho, nu_io = (C.c_double * L)(), vec(nu)
    _check(lib().vcas_controller_update(C.byref(prm), C.c_int32(L), C.byref(s_io), rho, nu_io, C.c_double(V_s),
                                        C.c_double(V_act), vec(V_w), vec(V_s_layer), vec(p_minus), vec(p_plus)),
           "vcas_controller_update")
    return s_io.value, list(rho), list(nu_io)


def vcas_profile_begin():
    _check(lib().vcas_profile_begin(), "vcas_profile_begin")


def vcas_profile_end():
    """Returns ((dgrad_ms, dgrad_launches), (wgrad_ms, wgrad_launches)); synchronises."""
    ms = (C.c_double * 2)()
    n = (C.c_int64 * 2)()
    _check(lib().vcas_profile_end(ms, n), "vcas_profile_end")
    return (ms[0], n[0]), (ms[1], n[1])
