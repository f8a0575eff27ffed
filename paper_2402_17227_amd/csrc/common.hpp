// Shared host/device helpers of the VCAS gfx950 library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <utility>
#include <vector>

#include "vcas.h"

namespace vcas {

constexpr int kWave = 64;

// ---- launch bookkeeping -----------------------------------------------------

inline vcas_status launch_status()
{
    return hipGetLastError() == hipSuccess ? VCAS_OK : VCAS_EHIP;
}

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline vcas_status check_shape(const vcas_shape *s)
{
    if (!s) return VCAS_ENULL;
    if (s->dtype != VCAS_F32 && s->dtype != VCAS_BF16) return VCAS_EDTYPE;
    if (s->N <= 0 || s->T <= 0 || s->K_in <= 0 || s->K_out <= 0) return VCAS_EINVAL;
    if ((s->K_in % 8) != 0 || (s->K_out % 8) != 0) return VCAS_EINVAL;
    if ((int64_t)s->N * s->T > (int64_t)1 << 30) return VCAS_EINVAL;
    return VCAS_OK;
}

// The bf16 GEMM kernels address G, X and W through 32-bit buffer offsets below 2 GiB.
inline vcas_status check_gemm_limits(const vcas_shape *s)
{
    if (s->dtype == VCAS_BF16) {
        const int64_t R = (int64_t)s->N * s->T;
        const int64_t kmax = s->K_in > s->K_out ? s->K_in : s->K_out;
        if (kmax > 8184 || R * kmax * 2 >= (int64_t)1 << 31) return VCAS_EINVAL;
    }
    return VCAS_OK;
}

inline int elem_bytes(int dtype) { return dtype == VCAS_BF16 ? 2 : 4; }

// ---- workspace layout -------------------------------------------------------
// splits * K_out * K_in fp32: split-K partial tiles of the weight gradient,
// then two K_out*K_in fp32 matrices and 32 doubles for the variance probe,
// then R floats: the SampleW uniforms of vcas_linear_backward

struct WorkspaceLayout {
    size_t partials, probe_exact, probe_draw, probe_acc, uniforms, total;
};

int wgrad_split(const vcas_shape *s);   // host: number of split-K slices for this shape

inline WorkspaceLayout workspace_layout(const vcas_shape *s)
{
    WorkspaceLayout w;
    size_t mat = (size_t)s->K_out * s->K_in * sizeof(float);
    w.partials = 0;
    w.probe_exact = w.partials + mat * (size_t)wgrad_split(s);
    w.probe_draw = w.probe_exact + mat;
    w.probe_acc = w.probe_draw + mat;
    w.uniforms = w.probe_acc + 256;
    w.total = w.uniforms + (((size_t)s->N * s->T * sizeof(float) + 255) & ~(size_t)255);
    return w;
}

// ---- optional kernel timer --------------------------------------------------
// When switched on (vcas_profile_begin), every GEMM launch is bracketed by HIP
// events that take their timestamps from the kernel's own dispatch, so the
// durations are the kernels' and not the host's.  0 = dgrad GEMM, 1 = wgrad GEMM.

struct KernelTimer {
    bool on = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pairs[2];
};
KernelTimer &kernel_timer();

template <typename Kern, typename... Args>
inline void launch_timed(int which, Kern kern, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args)
{
    KernelTimer &t = kernel_timer();
    if (!t.on) {
        hipLaunchKernelGGL(kern, grid, block, lds, st, args...);
        return;
    }
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
        hipLaunchKernelGGL(kern, grid, block, lds, st, args...);
        return;
    }
    hipExtLaunchKernelGGL(kern, grid, block, lds, st, a, b, 0, args...);
    t.pairs[which].push_back({a, b});
}

// ---- device helpers ---------------------------------------------------------

// bf16 halves of a packed pair; element k (even) is the low half.
__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

// Sum over the 64 lanes by pairwise exchange at distances 32,16,8,4,2,1.
// Every lane ends with the same value.
__device__ __forceinline__ float wave_exchange_sum(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = v + __shfl_xor(v, d, kWave);
    return v;
}

__device__ __forceinline__ double wave_exchange_sum(double v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = v + __shfl_xor(v, d, kWave);
    return v;
}

// Philox4x32-10 (Salmon et al., SC'11, Sec. 3.3); returns output word 0.
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                        uint32_t k0, uint32_t k1)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t h0 = __umulhi(M0, c0), l0 = M0 * c0;
        uint32_t h1 = __umulhi(M1, c2), l1 = M1 * c2;
        uint32_t n0 = h1 ^ c1 ^ k0;
        uint32_t n2 = h0 ^ c3 ^ k1;
        c0 = n0; c1 = l1; c2 = n2; c3 = l0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c0;
}

// Uniform in [0,1) that decides row `row` of sampler `stream_id`.
__device__ __forceinline__ float philox_uniform(uint64_t seed, uint32_t layer, uint32_t stream_id, uint32_t draw,
                                                uint32_t row)
{
    uint32_t w = philox4x32_10_word0(row, layer, stream_id, draw, (uint32_t)seed, (uint32_t)(seed >> 32));
    return (float)(w >> 8) * 0x1.0p-24f;
}

}  // namespace vcas
