// Device code of the row sums of squares (Eq. 3 factors, Sec. 4.1 sample norms),
// shared by the stand-alone norm kernels and the fused planning kernel.
//
// Summation order (fixed, independent of the launch): 16-byte group j of a row
// belongs to lane j mod 64; a lane folds its elements in ascending k with
// acc = fma(v, v, acc); lanes are combined by the neighbours-first exchange tree.
#pragma once

#include "common.hpp"

namespace vcas {

template <bool BF16>
__device__ __forceinline__ float fold16(const uint4 &c, float acc)
{
    if constexpr (BF16) {
        acc = __builtin_fmaf(bf16_lo(c.x), bf16_lo(c.x), acc);
        acc = __builtin_fmaf(bf16_hi(c.x), bf16_hi(c.x), acc);
        acc = __builtin_fmaf(bf16_lo(c.y), bf16_lo(c.y), acc);
        acc = __builtin_fmaf(bf16_hi(c.y), bf16_hi(c.y), acc);
        acc = __builtin_fmaf(bf16_lo(c.z), bf16_lo(c.z), acc);
        acc = __builtin_fmaf(bf16_hi(c.z), bf16_hi(c.z), acc);
        acc = __builtin_fmaf(bf16_lo(c.w), bf16_lo(c.w), acc);
        acc = __builtin_fmaf(bf16_hi(c.w), bf16_hi(c.w), acc);
    } else {
        float a = __uint_as_float(c.x), b = __uint_as_float(c.y), d = __uint_as_float(c.z), e = __uint_as_float(c.w);
        acc = __builtin_fmaf(a, a, acc);
        acc = __builtin_fmaf(b, b, acc);
        acc = __builtin_fmaf(d, d, acc);
        acc = __builtin_fmaf(e, e, acc);
    }
    return acc;
}

// Sum of squares of one row of `groups` 16-byte groups, computed by one wavefront
// (every lane returns it); CH groups per lane are in flight at once.
template <bool BF16, int CH>
__device__ __forceinline__ float wave_row_sumsq(const uint4 *__restrict__ p, int groups)
{
    const int lane = threadIdx.x & 63;
    float acc = 0.0f;
    for (int base = 0; base < groups; base += 64 * CH) {
        uint4 v[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            int g = base + lane + 64 * j;
            v[j] = g < groups ? p[g] : make_uint4(0u, 0u, 0u, 0u);
        }
        // a zero group leaves acc unchanged (fma(0,0,acc) == acc for acc >= +0)
#pragma unroll
        for (int j = 0; j < CH; ++j) acc = fold16<BF16>(v[j], acc);
    }
    return wave_exchange_sum(acc);
}

// Uniforms of one sampler for every row, drawn alongside a memory-bound pass
// (they do not depend on the data).
struct UniformJob {
    float *uniforms;   // null: no job
    uint64_t seed;
    uint32_t layer, stream_id, draw;
    const uint32_t *draw_offset;
};

// SampleW scores of the rows of X, written by the pass that takes their norms
// once SampleA is done: score_t = ((1/p_i) * sqrt(gsq_t)) * sqrt(xsq_t).
struct ScoreJob {
    const float *gsq;   // row norms of G, squared
    const float *p;     // SampleA keep probabilities, one per sample
    float *score;       // null: no job
};

}  // namespace vcas
