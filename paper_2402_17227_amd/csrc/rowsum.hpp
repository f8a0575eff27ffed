// Device code of the row sums of squares (Eq. 3 factors, Sec. 4.1 sample norms),
// shared by the stand-alone norm kernels and the fused planning kernel.
//
// Summation order (fixed, independent of the launch): pairwise, neighbours first.
// The squares v*v (one rounding each), padded with +0 to a power of two, are added
// as a balanced binary tree in index order.  A wavefront follows it like this: a
// lane adds the squares of its 16-byte group pairwise; the 64 groups of a "pass"
// (512 bf16 or 256 fp32 consecutive elements) are combined by the neighbours-first
// lane tree; passes are paired the same way.  Missing groups and passes count as
// +0, which changes no sum.
#pragma once

#include "common.hpp"

namespace vcas {

// Pairwise sum of the squares of one 16-byte group (8 bf16 or 4 fp32 elements).
template <bool BF16>
__device__ __forceinline__ float group_sumsq(const uint4 &c)
{
    if constexpr (BF16) {
        const float e0 = bf16_lo(c.x), e1 = bf16_hi(c.x), e2 = bf16_lo(c.y), e3 = bf16_hi(c.y);
        const float e4 = bf16_lo(c.z), e5 = bf16_hi(c.z), e6 = bf16_lo(c.w), e7 = bf16_hi(c.w);
        return ((e0 * e0 + e1 * e1) + (e2 * e2 + e3 * e3)) + ((e4 * e4 + e5 * e5) + (e6 * e6 + e7 * e7));
    } else {
        const float a = __uint_as_float(c.x), b = __uint_as_float(c.y), d = __uint_as_float(c.z), e = __uint_as_float(c.w);
        return (a * a + b * b) + (d * d + e * e);
    }
}

// The subtree over CH consecutive passes: v[j] is this lane's group of pass j (zero if the row
// has ended), live = how many of the passes hold any group of the row (wave-uniform).
template <bool BF16, int CH>
__device__ __forceinline__ float chunk_sumsq(const uint4 (&v)[CH], int live)
{
    constexpr int P = CH <= 1 ? 1 : CH <= 2 ? 2 : CH <= 4 ? 4 : CH <= 8 ? 8 : 16;   // CH padded to a power of two
    static_assert(CH <= 16, "at most sixteen passes in flight");
    float q[P];
#pragma unroll
    for (int j = 0; j < P; ++j) q[j] = 0.0f;
#pragma unroll
    for (int j = 0; j < CH; ++j)
        if (j < live) q[j] = wave_exchange_sum(group_sumsq<BF16>(v[j]));
#pragma unroll
    for (int n = P; n > 1; n /= 2)
#pragma unroll
        for (int j = 0; j < n / 2; ++j) q[j] = q[2 * j] + q[2 * j + 1];
    return q[0];
}

// Pairwise summation of a stream of values (the pass sums of a long row, at most 2^LEVELS of them):
// push them in order, then finish.  What a binary counter does: two sums of one level make one of
// the next; at the end the levels that hold a sum are added from the lowest up, which is the
// balanced tree over the stream padded with +0 to a power of two.
template <int LEVELS>
struct PairwiseStream {
    float level[LEVELS];
    int count = 0;
    __device__ __forceinline__ void push(float x)
    {
#pragma unroll
        for (int l = 0; l < LEVELS; ++l) {
            if ((count >> l) & 1) {
                x = level[l] + x;
            } else {
                level[l] = x;
                break;
            }
        }
        ++count;
    }
    __device__ __forceinline__ float finish() const
    {
        float acc = 0.0f;
        bool have = false;
#pragma unroll
        for (int l = 0; l < LEVELS; ++l)
            if ((count >> l) & 1) {
                acc = have ? level[l] + acc : level[l];
                have = true;
            }
        return acc;
    }
};

// Sum of squares of one row of `groups` 16-byte groups, computed by one wavefront
// (every lane returns it); CH groups per lane are in flight at once.
template <bool BF16, int CH>
__device__ __forceinline__ float wave_row_sumsq(const uint4 *__restrict__ p, int groups)
{
    const int lane = threadIdx.x & 63;
    if (groups <= 64 * CH) {
        uint4 v[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int g = lane + 64 * j;
            v[j] = g < groups ? p[g] : make_uint4(0u, 0u, 0u, 0u);
        }
        return chunk_sumsq<BF16, CH>(v, (groups + 63) / 64);
    }
    PairwiseStream<16> passes;   // rows of up to 2^16 * 64 groups; one value per pass, whatever CH is
    for (int base = 0; base < groups; base += 64 * CH) {
        uint4 v[CH];
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int g = base + lane + 64 * j;
            v[j] = g < groups ? p[g] : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int j = 0; j < CH; ++j)
            if (base + 64 * j < groups) passes.push(wave_exchange_sum(group_sumsq<BF16>(v[j])));
    }
    return passes.finish();
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
