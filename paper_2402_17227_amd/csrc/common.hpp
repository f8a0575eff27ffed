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

// The bf16 GEMM kernels address G, X and W through 32-bit buffer offsets below 2 GiB and form
// row offsets with 24-bit multiplies.
inline vcas_status check_gemm_limits(const vcas_shape *s)
{
    if (s->dtype == VCAS_BF16) {
        const int64_t R = (int64_t)s->N * s->T;
        const int64_t kmax = s->K_in > s->K_out ? s->K_in : s->K_out;
        if (kmax > 8184 || R >= (int64_t)1 << 24 || R * kmax * 2 >= (int64_t)1 << 31) return VCAS_EINVAL;
    }
    return VCAS_OK;
}

inline int elem_bytes(int dtype) { return dtype == VCAS_BF16 ? 2 : 4; }

// ---- workspace layout -------------------------------------------------------
// kPlanTicketBytes of control words (the ticket counters of the fused planning
// kernel), zero between calls; then splits * K_out * K_in fp32: split-K partial tiles of
// the weight gradient, then two K_out*K_in fp32 matrices and 32 doubles for the
// variance probe, then R floats: the SampleW uniforms of vcas_linear_backward, then (bf16) up to
// R rows of min(K_in, K_out) elements: the packed operand of the weight gradient

struct WorkspaceLayout {
    size_t control, partials, probe_exact, probe_draw, probe_acc, uniforms, packed, total;
};

constexpr size_t kPlanTicketBytes = 8192;   // 33 counters, one 128-byte line each, rounded up
int wgrad_split(const vcas_shape *s);   // host: number of split-K slices for this shape

inline WorkspaceLayout workspace_layout(const vcas_shape *s)
{
    WorkspaceLayout w;
    size_t mat = (size_t)s->K_out * s->K_in * sizeof(float);
    w.control = 0;
    w.partials = kPlanTicketBytes;
    w.probe_exact = w.partials + mat * (size_t)wgrad_split(s);
    w.probe_draw = w.probe_exact + mat;
    w.probe_acc = w.probe_draw + mat;
    w.uniforms = w.probe_acc + 256;
    w.packed = w.uniforms + (((size_t)s->N * s->T * sizeof(float) + 255) & ~(size_t)255);
    // bf16: the narrower of G and X over the kept tokens, gathered and multiplied by the token scales
    const size_t packed_bytes = s->dtype == VCAS_BF16 ? (size_t)s->N * s->T * (s->K_in < s->K_out ? s->K_in : s->K_out) * 2 : 0;
    w.total = w.packed + ((packed_bytes + 255) & ~(size_t)255);
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

// Sum over the 64 lanes as a fixed tree: neighbours first (exchange-add at distances
// 1, 2, 4, 8, 16, 32).  Every lane ends with the same value.  The first four levels are DPP
// lane permutes (quad swaps, then mirrors within 8 and within 16 lanes, which pair the same
// groups as distances 4 and 8 once the lanes of a group agree); the last two levels take the
// four 16-lane row values through scalar registers.  No LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

template <int CTRL>
__device__ __forceinline__ double dpp_move(double v)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xF, 0xF, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ float read_lane(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

__device__ __forceinline__ double read_lane(double v, int lane)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), lane);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

template <typename F>
__device__ __forceinline__ F wave_exchange_sum(F v)
{
    v = v + dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]: distance 1
    v = v + dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]: distance 2
    v = v + dpp_move<0x141>(v);   // row_half_mirror: the other quad of each 8 lanes
    v = v + dpp_move<0x140>(v);   // row_mirror: the other 8 lanes of each 16
    const F r0 = read_lane(v, 0), r1 = read_lane(v, 16), r2 = read_lane(v, 32), r3 = read_lane(v, 48);
    return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ int wave_sum_int(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);
    return (__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16)) +
           (__builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}

// The same neighbours-first tree over 16 values (the per-wavefront sums of a 1024-thread block).
template <typename F>
__device__ __forceinline__ F tree16(const F *w)
{
    return (((w[0] + w[1]) + (w[2] + w[3])) + ((w[4] + w[5]) + (w[6] + w[7]))) +
           (((w[8] + w[9]) + (w[10] + w[11])) + ((w[12] + w[13]) + (w[14] + w[15])));
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
