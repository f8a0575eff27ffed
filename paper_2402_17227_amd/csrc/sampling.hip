// Sampling kernels of the VCAS backward pass: capped-proportional keep
// probabilities (Sec. 4.1 p_i ~ ||G_i||_F, Sec. 4.2 q_t ~ leverage score),
// Philox Bernoulli masks, kept-row compaction, and the two small elementwise
// steps (leverage scores, per-row scale).  All vectors are at most R floats,
// so these kernels are latency-bound, not bandwidth-bound.
#include "rowsum.hpp"

namespace vcas {

// ---- block-wide sums over 1024 threads in a fixed order ---------------------
// Thread tid is "slot" tid.  Each 64-slot group (one wavefront) is combined by
// the neighbours-first tree, then the 16 group sums by the same kind of tree.
// Every thread returns the totals.  `bufd` / `bufi` are 16 values of LDS each;
// calls must alternate buffers or be separated by a barrier.
__device__ __forceinline__ void block_sum_pair_1024(double v, int c, double *bufd, int *bufi, double &sum_v, int &sum_c)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = wave_exchange_sum(v);
    c = wave_sum_int(c);
    if (lane == 0) {
        bufd[wave] = v;
        bufi[wave] = c;
    }
    __syncthreads();
    double wd[16];
    int total = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        wd[i] = bufd[i];
        total += bufi[i];
    }
    sum_v = tree16(wd);
    sum_c = total;
}

// prob_i = min(1, c * score_i), sum prob = min(budget, #positive scores).
// c is found by rounds: every not-yet-fixed entry that the current c pushes to
// >= 1 is fixed at one, then c is recomputed from what is left, until a round
// fixes nothing.  Sums in fp64, slot = i mod 1024, ascending i inside a slot.
// While running, prob[i] == 1 marks "fixed at one" (each element is only ever
// touched by its own thread).  Single block of 1024 threads.
__device__ void keep_probs_block(const float *__restrict__ score, int n, double budget, float *__restrict__ prob)
{
    __shared__ double sd[2][16];
    __shared__ int si[2][16];
    const int tid = threadIdx.x;

    double part = 0.0;
    int cnt = 0;
    for (int i = tid; i < n; i += 1024) {
        float a = score[i];
        if (a > 0.0f) {
            part += (double)a;
            ++cnt;
        }
        prob[i] = 0.0f;
    }
    double S;
    int nonzero;
    block_sum_pair_1024(part, cnt, sd[0], si[0], S, nonzero);

    if (budget >= (double)nonzero) {
        for (int i = tid; i < n; i += 1024) prob[i] = score[i] > 0.0f ? 1.0f : 0.0f;
        return;
    }

    int ncap = 0;
    double c = 0.0;
    int flip = 1;
    for (;;) {
        const double rem = budget - (double)ncap;
        if (!(S > 0.0) || !(rem > 0.0)) {
            c = 0.0;
            break;
        }
        c = rem / S;
        part = 0.0;
        cnt = 0;
        for (int i = tid; i < n; i += 1024) {
            float a = score[i];
            if (a > 0.0f && prob[i] != 1.0f) {
                if (c * (double)a >= 1.0) {
                    prob[i] = 1.0f;
                    ++cnt;
                } else {
                    part += (double)a;
                }
            }
        }
        double S_next;
        int newly;
        block_sum_pair_1024(part, cnt, sd[flip], si[flip], S_next, newly);
        flip ^= 1;
        if (newly == 0) break;
        ncap += newly;
        S = S_next;
    }
    for (int i = tid; i < n; i += 1024) {
        float a = score[i];
        if (prob[i] == 1.0f) continue;
        float p = 0.0f;
        if (a > 0.0f) {
            p = (float)(c * (double)a);
            p = p < 1.0f ? p : 1.0f;
        }
        prob[i] = p;
    }
}

__global__ __launch_bounds__(1024) void keep_probs_kernel(const float *__restrict__ score, int n, double budget,
                                                          float *__restrict__ prob)
{
    keep_probs_block(score, n, budget, prob);
}

// mask[r] = [u_r < prob[r]]
__global__ __launch_bounds__(256) void bernoulli_mask_kernel(const float *__restrict__ prob, int n, uint64_t seed,
                                                             uint32_t layer, uint32_t stream_id, uint32_t draw,
                                                             const uint32_t *__restrict__ draw_offset,
                                                             uint8_t *__restrict__ mask)
{
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= n) return;
    if (draw_offset) draw += *draw_offset;
    const float u = philox_uniform(seed, layer, stream_id, draw, (uint32_t)r);
    mask[r] = u < prob[r] ? 1 : 0;
}

// Ascending list of the r with mask[r] != 0, and their count.  Single block of
// 1024 threads; thread tid owns the contiguous slice [tid*per, (tid+1)*per).
// Slice counts are scanned across the block (wave scan, then the 16 wave
// totals through LDS).
__device__ void compact_block(const uint8_t *__restrict__ mask, int n, int32_t *__restrict__ idx,
                              int32_t *__restrict__ count)
{
    __shared__ int wave_total[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (n + 1023) / 1024;
    const int lo = min(n, tid * per), hi = min(n, lo + per);
    int mine = 0;
    for (int r = lo; r < hi; ++r) mine += mask[r] != 0;
    int incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    if (lane == 63) wave_total[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        int t = wave_total[w];
        if (w < wave) before += t;
        total += t;
    }
    int pos = before + incl - mine;
    for (int r = lo; r < hi; ++r)
        if (mask[r] != 0) idx[pos++] = r;
    if (tid == 0) *count = total;
}

__global__ __launch_bounds__(1024) void compact_kernel(const uint8_t *__restrict__ mask, int n,
                                                       int32_t *__restrict__ idx, int32_t *__restrict__ count)
{
    compact_block(mask, n, idx, count);
}

// score[t] = maskA[i] * ((1/p[i]) * sqrt(gsq[t])) * sqrt(xsq[t])
__global__ __launch_bounds__(256) void leverage_kernel(const float *__restrict__ gsq, const float *__restrict__ xsq,
                                                       const float *__restrict__ p, const uint8_t *__restrict__ maskA,
                                                       int64_t R, int T, float *__restrict__ score)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= R) return;
    const int i = (int)(t / T);
    float s = 0.0f;
    if (maskA[i]) {
        const float inv = 1.0f / (p[i]);
        const float a = inv * __builtin_sqrtf(gsq[t]);
        s = a * __builtin_sqrtf(xsq[t]);
    }
    score[t] = s;
}

// scaleW[t] = maskW[t] ? 1/(p[i] q[t]) : 0
__global__ __launch_bounds__(256) void row_scale_kernel(const float *__restrict__ p, const float *__restrict__ q,
                                                        const uint8_t *__restrict__ maskW, int64_t R, int T,
                                                        float *__restrict__ scale)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= R) return;
    const int i = (int)(t / T);
    scale[t] = maskW[t] ? 1.0f / (p[i] * q[t]) : 0.0f;
}

// "SampleA only" token plan: every token of a kept sample is kept with q = 1.
__global__ __launch_bounds__(256) void broadcast_data_mask_kernel(const uint8_t *__restrict__ maskA, int64_t R, int T,
                                                                  float *__restrict__ q, uint8_t *__restrict__ maskW)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= R) return;
    const uint8_t m = maskA[t / T] ? 1 : 0;
    q[t] = m ? 1.0f : 0.0f;
    maskW[t] = m;
}

// ---- fused single-workgroup samplers (used by vcas_linear_backward) -----------
// The vectors are at most R floats, so one workgroup of 1024 threads does the
// whole decision chain of a sampler in one launch instead of five.

// keep_probs_block with the scores held in registers: thread tid owns elements
// tid + 1024*j, j < E (zero past the end).  Same sums in the same order, but a
// round costs one barrier and no memory traffic.
template <int E>
__device__ void keep_probs_regs(const float (&a)[E], double budget, float (&prob)[E])
{
    __shared__ double sd[2][16];
    __shared__ int si[2][16];
    double part = 0.0;
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < E; ++j)
        if (a[j] > 0.0f) {
            part += (double)a[j];
            ++cnt;
        }
    double S;
    int nonzero;
    block_sum_pair_1024(part, cnt, sd[0], si[0], S, nonzero);
    if (budget >= (double)nonzero) {
#pragma unroll
        for (int j = 0; j < E; ++j) prob[j] = a[j] > 0.0f ? 1.0f : 0.0f;
        return;
    }
    uint32_t fixed = 0;   // bit j: element j is fixed at one
    int ncap = 0;
    double c = 0.0;
    int flip = 1;
    for (;;) {
        const double rem = budget - (double)ncap;
        if (!(S > 0.0) || !(rem > 0.0)) {
            c = 0.0;
            break;
        }
        c = rem / S;
        part = 0.0;
        cnt = 0;
#pragma unroll
        for (int j = 0; j < E; ++j)
            if (a[j] > 0.0f && !((fixed >> j) & 1u)) {
                if (c * (double)a[j] >= 1.0) {
                    fixed |= 1u << j;
                    ++cnt;
                } else {
                    part += (double)a[j];
                }
            }
        double S_next;
        int newly;
        block_sum_pair_1024(part, cnt, sd[flip], si[flip], S_next, newly);
        flip ^= 1;
        if (newly == 0) break;
        ncap += newly;
        S = S_next;
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
        float p = 0.0f;
        if ((fixed >> j) & 1u) p = 1.0f;
        else if (a[j] > 0.0f) {
            p = (float)(c * (double)a[j]);
            p = p < 1.0f ? p : 1.0f;
        }
        prob[j] = p;
    }
}

// SampleA for N <= 1024 with every intermediate in LDS or registers (one workgroup of 1024).
__device__ __forceinline__ void sampler_a_fast_body(const float *__restrict__ gsq, int N, int T, double budget,
                                                    uint64_t seed, uint32_t layer, uint32_t draw,
                                                    const uint32_t *__restrict__ draw_offset,
                                                    float *__restrict__ gnorm, float *__restrict__ p,
                                                    uint8_t *__restrict__ maskA, int32_t *__restrict__ idxA,
                                                    int32_t *__restrict__ cntA)
{
    __shared__ float gn[1024];
    __shared__ uint8_t mk[1024];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (draw_offset) draw += *draw_offset;
    for (int i = wave; i < N; i += 16) {
        const float *row = gsq + (int64_t)i * T;
        float acc = 0.0f;
        for (int t = lane; t < T; t += 64) acc = acc + row[t];
        acc = wave_exchange_sum(acc);
        if (lane == 0) gn[i] = __builtin_sqrtf(acc);
    }
    __syncthreads();
    float a[1], pr[1];
    a[0] = tid < N ? gn[tid] : 0.0f;
    keep_probs_regs<1>(a, budget, pr);
    uint8_t m = 0;
    if (tid < N) {
        m = philox_uniform(seed, layer, 0u, draw, (uint32_t)tid) < pr[0] ? 1 : 0;
        gnorm[tid] = a[0];
        p[tid] = pr[0];
        maskA[tid] = m;
    }
    mk[tid] = m;
    __syncthreads();
    compact_block(mk, N, idxA, cntA);
}

__global__ __launch_bounds__(1024) void sampler_a_fast_kernel(const float *__restrict__ gsq, int N, int T,
                                                              double budget, uint64_t seed, uint32_t layer,
                                                              uint32_t draw, const uint32_t *__restrict__ draw_offset,
                                                              float *__restrict__ gnorm, float *__restrict__ p,
                                                              uint8_t *__restrict__ maskA, int32_t *__restrict__ idxA,
                                                              int32_t *__restrict__ cntA)
{
    sampler_a_fast_body(gsq, N, T, budget, seed, layer, draw, draw_offset, gnorm, p, maskA, idxA, cntA);
}

// SampleW for R <= 1024*E (one workgroup of 1024).
template <int E>
__device__ __forceinline__ void sampler_w_fast_body(const float *__restrict__ gsq, float *__restrict__ xsq,
                                                    int zero_dropped_xsq, const float *__restrict__ p,
                                                    const uint8_t *__restrict__ maskA, const float *__restrict__ u,
                                                    int N, int T, double budget, int token_sampling,
                                                    float *__restrict__ score, float *__restrict__ q,
                                                    uint8_t *__restrict__ maskW, float *__restrict__ scaleW,
                                                    int32_t *__restrict__ idxW, int32_t *__restrict__ cntW)
{
    __shared__ uint8_t mk[1024 * E];
    const int tid = threadIdx.x;
    const int R = N * T;
    float a[E], qv[E], pinv_src[E], uu[E];
    uint8_t keepA[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int t = tid + 1024 * j;
        a[j] = 0.0f;
        pinv_src[j] = 1.0f;
        uu[j] = 2.0f;
        keepA[j] = 0;
        if (t < R) {
            const int i = t / T;
            keepA[j] = maskA[i];
            pinv_src[j] = p[i];
            const float g = gsq[t], x = xsq[t];
            if (token_sampling) uu[j] = u[t];
            if (keepA[j]) {
                const float inv = 1.0f / pinv_src[j];
                const float s1 = inv * __builtin_sqrtf(g);
                a[j] = s1 * __builtin_sqrtf(x);
            } else if (zero_dropped_xsq) {
                xsq[t] = 0.0f;
            }
            score[t] = a[j];
        }
    }
    if (token_sampling) {
        keep_probs_regs<E>(a, budget, qv);
    } else {
#pragma unroll
        for (int j = 0; j < E; ++j) qv[j] = keepA[j] ? 1.0f : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int t = tid + 1024 * j;
        uint8_t m = 0;
        if (t < R) {
            m = token_sampling ? (uu[j] < qv[j] ? 1 : 0) : (keepA[j] ? 1 : 0);
            q[t] = qv[j];
            maskW[t] = m;
            scaleW[t] = m ? 1.0f / (pinv_src[j] * qv[j]) : 0.0f;
        }
        mk[t] = m;
    }
    __syncthreads();
    compact_block(mk, R, idxW, cntW);
}

template <int E>
__global__ __launch_bounds__(1024) void sampler_w_fast_kernel(const float *__restrict__ gsq,
                                                              float *__restrict__ xsq, int zero_dropped_xsq,
                                                              const float *__restrict__ p,
                                                              const uint8_t *__restrict__ maskA,
                                                              const float *__restrict__ u, int N, int T, double budget,
                                                              int token_sampling, float *__restrict__ score,
                                                              float *__restrict__ q, uint8_t *__restrict__ maskW,
                                                              float *__restrict__ scaleW, int32_t *__restrict__ idxW,
                                                              int32_t *__restrict__ cntW)
{
    sampler_w_fast_body<E>(gsq, xsq, zero_dropped_xsq, p, maskA, u, N, T, budget, token_sampling, score, q, maskW,
                           scaleW, idxW, cntW);
}

// SampleA: ||G_i||_F from gsq, p, Bernoulli mask over samples, kept list.
__global__ __launch_bounds__(1024) void sampler_a_kernel(const float *__restrict__ gsq, int N, int T, double budget,
                                                         uint64_t seed, uint32_t layer, uint32_t draw,
                                                         const uint32_t *__restrict__ draw_offset,
                                                         float *__restrict__ gnorm, float *__restrict__ p,
                                                         uint8_t *__restrict__ maskA, int32_t *__restrict__ idxA,
                                                         int32_t *__restrict__ cntA)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (draw_offset) draw += *draw_offset;
    for (int i = wave; i < N; i += 16) {
        const float *row = gsq + (int64_t)i * T;
        float acc = 0.0f;
        for (int t = lane; t < T; t += 64) acc = acc + row[t];
        acc = wave_exchange_sum(acc);
        if (lane == 0) gnorm[i] = __builtin_sqrtf(acc);
    }
    __syncthreads();
    keep_probs_block(gnorm, N, budget, p);
    __syncthreads();
    for (int i = tid; i < N; i += 1024) maskA[i] = philox_uniform(seed, layer, 0u, draw, (uint32_t)i) < p[i] ? 1 : 0;
    __syncthreads();
    compact_block(maskA, N, idxA, cntA);
}

// Uniforms of SampleW for every row (independent of the data, so they are
// drawn by many workgroups while the row norms stream).
__global__ __launch_bounds__(256) void uniforms_kernel(int64_t R, uint64_t seed, uint32_t layer, uint32_t stream_id,
                                                       uint32_t draw, const uint32_t *__restrict__ draw_offset,
                                                       float *__restrict__ u)
{
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (draw_offset) draw += *draw_offset;
    if (r < R) u[r] = philox_uniform(seed, layer, stream_id, draw, (uint32_t)r);
}

// SampleW: leverage scores, q, Bernoulli mask over tokens (uniforms given),
// per-token scale, kept list.  With token_sampling == 0 every token of a kept
// sample is kept with q = 1.
__global__ __launch_bounds__(1024) void sampler_w_kernel(const float *__restrict__ gsq, float *__restrict__ xsq,
                                                         int zero_dropped_xsq, const float *__restrict__ p,
                                                         const uint8_t *__restrict__ maskA,
                                                         const float *__restrict__ u, int N, int T, double budget,
                                                         int token_sampling, float *__restrict__ score,
                                                         float *__restrict__ q, uint8_t *__restrict__ maskW,
                                                         float *__restrict__ scaleW, int32_t *__restrict__ idxW,
                                                         int32_t *__restrict__ cntW)
{
    const int tid = threadIdx.x;
    const int R = N * T;
    for (int t = tid; t < R; t += 1024) {
        const int i = t / T;
        float s = 0.0f;
        if (maskA[i]) {
            const float inv = 1.0f / p[i];
            const float a = inv * __builtin_sqrtf(gsq[t]);
            s = a * __builtin_sqrtf(xsq[t]);
        } else if (zero_dropped_xsq) {
            xsq[t] = 0.0f;
        }
        score[t] = s;
    }
    __syncthreads();
    if (token_sampling) {
        keep_probs_block(score, R, budget, q);
        __syncthreads();
    }
    for (int t = tid; t < R; t += 1024) {
        const int i = t / T;
        uint8_t m;
        float qt;
        if (token_sampling) {
            qt = q[t];
            m = u[t] < qt ? 1 : 0;
        } else {
            m = maskA[i] ? 1 : 0;
            qt = m ? 1.0f : 0.0f;
            q[t] = qt;
        }
        maskW[t] = m;
        scaleW[t] = m ? 1.0f / (p[i] * qt) : 0.0f;
    }
    __syncthreads();
    compact_block(maskW, R, idxW, cntW);
}

// ---- host launchers ---------------------------------------------------------

vcas_status keep_probs(const float *score, int n, double budget, float *prob, hipStream_t st)
{
    hipLaunchKernelGGL(keep_probs_kernel, dim3(1), dim3(1024), 0, st, score, n, budget, prob);
    return launch_status();
}

vcas_status sample_compact(const float *prob, int n, const vcas_rng &rng, uint32_t stream_id, uint8_t *mask,
                           int32_t *idx, int32_t *count, hipStream_t st)
{
    if (n > 0) {
        hipLaunchKernelGGL(bernoulli_mask_kernel, dim3((n + 255) / 256), dim3(256), 0, st, prob, n, rng.seed,
                           rng.layer, stream_id, rng.draw, rng.draw_offset, mask);
        if (hipGetLastError() != hipSuccess) return VCAS_EHIP;
    }
    hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(1024), 0, st, mask, n, idx, count);
    return launch_status();
}

vcas_status compact_only(const uint8_t *mask, int n, int32_t *idx, int32_t *count, hipStream_t st)
{
    hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(1024), 0, st, mask, n, idx, count);
    return launch_status();
}

vcas_status leverage_scores(const float *gsq, const float *xsq, const float *p, const uint8_t *maskA, int64_t R,
                            int T, float *score, hipStream_t st)
{
    hipLaunchKernelGGL(leverage_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, gsq, xsq, p, maskA, R, T,
                       score);
    return launch_status();
}

vcas_status row_scale(const float *p, const float *q, const uint8_t *maskW, int64_t R, int T, float *scale,
                      hipStream_t st)
{
    hipLaunchKernelGGL(row_scale_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, p, q, maskW, R, T,
                       scale);
    return launch_status();
}

vcas_status broadcast_data_mask(const uint8_t *maskA, int64_t R, int T, float *q, uint8_t *maskW, hipStream_t st)
{
    hipLaunchKernelGGL(broadcast_data_mask_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, maskA, R, T,
                       q, maskW);
    return launch_status();
}

vcas_status sampler_a(const float *gsq, int N, int T, double budget, const vcas_rng &rng, float *gnorm, float *p,
                      uint8_t *maskA, int32_t *idxA, int32_t *cntA, hipStream_t st)
{
    if (N <= 1024)
        hipLaunchKernelGGL(sampler_a_fast_kernel, dim3(1), dim3(1024), 0, st, gsq, N, T, budget, rng.seed, rng.layer,
                           rng.draw, rng.draw_offset, gnorm, p, maskA, idxA, cntA);
    else
        hipLaunchKernelGGL(sampler_a_kernel, dim3(1), dim3(1024), 0, st, gsq, N, T, budget, rng.seed, rng.layer,
                           rng.draw, rng.draw_offset, gnorm, p, maskA, idxA, cntA);
    return launch_status();
}

vcas_status uniforms(int64_t R, const vcas_rng &rng, uint32_t stream_id, float *u, hipStream_t st)
{
    hipLaunchKernelGGL(uniforms_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, R, rng.seed, rng.layer,
                       stream_id, rng.draw, rng.draw_offset, u);
    return launch_status();
}

vcas_status sampler_w(const float *gsq, float *xsq, int zero_dropped_xsq, const float *p, const uint8_t *maskA,
                      const float *u, int N, int T, double budget, int token_sampling, float *score, float *q,
                      uint8_t *maskW, float *scaleW, int32_t *idxW, int32_t *cntW, hipStream_t st)
{
    const int64_t R = (int64_t)N * T;
#define VCAS_SAMPLER_W_ARGS \
    gsq, xsq, zero_dropped_xsq, p, maskA, u, N, T, budget, token_sampling, score, q, maskW, scaleW, idxW, cntW
    if (R <= 4096)
        hipLaunchKernelGGL(sampler_w_fast_kernel<4>, dim3(1), dim3(1024), 0, st, VCAS_SAMPLER_W_ARGS);
    else if (R <= 16384)
        hipLaunchKernelGGL(sampler_w_fast_kernel<16>, dim3(1), dim3(1024), 0, st, VCAS_SAMPLER_W_ARGS);
    else
        hipLaunchKernelGGL(sampler_w_kernel, dim3(1), dim3(1024), 0, st, VCAS_SAMPLER_W_ARGS);
#undef VCAS_SAMPLER_W_ARGS
    return launch_status();
}

}  // namespace vcas
