// SampleA for at most 64 samples, by one wavefront (Sec. 4.1: p_i ~ ||G_i||_F with sum p = N rho,
// Bernoulli masks, ascending kept list).  With N <= 64 every entry lies in the first 64 of the
// 1024 summation slots, the other fifteen group sums are +0 and x + 0 = x, so one wavefront
// reproduces the sums of the 1024-thread kernels bit for bit, with no LDS and no barriers.
// Shared by the sampler kernel and by the dgrad kernel that decides SampleA for itself.
#pragma once

#include "common.hpp"

namespace vcas {

// ||G_i||_F from the T squared row norms of sample i, by one wavefront (every lane returns it):
// value t belongs to lane t mod 64, plain fp32 adds in ascending t, exchange tree, correctly
// rounded sqrt.  Eight loads are in flight at a time (a lane's values past the end re-read the
// last one and count as +0, which leaves the sum as it is).
__device__ __forceinline__ float sample_norm_wave(const float *__restrict__ row, int T)
{
    const int lane = threadIdx.x & 63;
    float acc = 0.0f;
    for (int t0 = lane; t0 < T; t0 += 512) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = row[min(t0 + 64 * k, T - 1)];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc = acc + (t0 + 64 * k < T ? v[k] : 0.0f);
    }
    return __builtin_sqrtf(wave_exchange_sum(acc));
}

// The same norms for several samples of one wavefront at a time, so that their loads overlap:
// samples first, first + stride, ... (< N), B at a time with K loads per lane and sample in flight;
// out[i] = ||G_i||_F.  Same additions in the same order as sample_norm_wave.
template <int B, int K>
__device__ __forceinline__ void sample_norms_batched(const float *__restrict__ gsq, int first, int stride, int N,
                                                     int T, float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    for (int i0 = first; i0 < N; i0 += stride * B) {
        float acc[B];
#pragma unroll
        for (int b = 0; b < B; ++b) acc[b] = 0.0f;
        for (int t0 = lane; t0 < T; t0 += 64 * K) {
            float v[B][K];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int i = min(i0 + b * stride, N - 1);
#pragma unroll
                for (int k = 0; k < K; ++k) v[b][k] = gsq[(int64_t)i * T + min(t0 + 64 * k, T - 1)];
            }
#pragma unroll
            for (int b = 0; b < B; ++b)
#pragma unroll
                for (int k = 0; k < K; ++k) acc[b] = acc[b] + (t0 + 64 * k < T ? v[b][k] : 0.0f);
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const float norm = __builtin_sqrtf(wave_exchange_sum(acc[b]));
            if (lane == 0 && i0 + b * stride < N) out[i0 + b * stride] = norm;
        }
    }
}

struct SampleADecision {
    float pr;     // keep probability of sample `lane`
    bool keep;    // Bernoulli outcome
    int below;    // kept samples with a smaller index: this sample's place in the kept list
    int count;    // kept samples in all
};

// Lane i (< N) holds a = ||G_i||_F, the other lanes 0.  The whole wavefront must call.
__device__ __forceinline__ SampleADecision sample_a_wave(float a, int N, double budget, uint64_t seed,
                                                         uint32_t layer, uint32_t draw)
{
    const int lane = threadIdx.x & 63;
    const bool pos = a > 0.0f;
    double S = wave_exchange_sum(pos ? (double)a : 0.0);
    const int nonzero = __builtin_popcountll(__ballot(pos));
    float pr = 0.0f;
    if (budget >= (double)nonzero) {
        pr = pos ? 1.0f : 0.0f;
    } else {
        bool fixed = false;
        int ncap = 0;
        double c = 0.0;
        for (;;) {
            const double rem = budget - (double)ncap;
            if (!(S > 0.0) || !(rem > 0.0)) {
                c = 0.0;
                break;
            }
            c = rem / S;
            const bool open = pos && !fixed;
            const bool cap = open && c * (double)a >= 1.0;
            fixed = fixed || cap;
            const int newly = __builtin_popcountll(__ballot(cap));
            const double S_next = wave_exchange_sum(open && !cap ? (double)a : 0.0);
            if (newly == 0) break;
            ncap += newly;
            S = S_next;
        }
        if (fixed) pr = 1.0f;
        else if (pos) {
            pr = (float)(c * (double)a);
            pr = pr < 1.0f ? pr : 1.0f;
        }
    }
    SampleADecision d;
    d.pr = pr;
    d.keep = lane < N && philox_uniform(seed, layer, 0u, draw, (uint32_t)lane) < pr;
    const uint64_t kept = __ballot(d.keep);
    d.below = __builtin_amdgcn_mbcnt_hi((uint32_t)(kept >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)kept, 0u));
    d.count = __builtin_popcountll(kept);
    return d;
}

// SampleA decided inside another kernel: where the row norms of G are, the budget N rho, the
// random stream, and where the plan's SampleA fields go (written by one workgroup).
struct InlineSampleA {
    const float *gsq;     // row sums of squares of G: the sample norms are taken here too
    const float *norms;   // or the sample norms ||G_i||_F themselves; both null: off
    double budget;
    uint64_t seed;
    uint32_t layer, draw;
    const uint32_t *draw_offset;
    float *gnorm, *p;
    uint8_t *maskA;
    int32_t *idxA, *cntA;
};

}  // namespace vcas
