// Sampling kernels of the VCAS backward pass: capped-proportional keep
// probabilities (Sec. 4.1 p_i ~ ||G_i||_F, Sec. 4.2 q_t ~ leverage score),
// Philox Bernoulli masks, kept-row compaction, and the two small elementwise
// steps (leverage scores, per-row scale).  All vectors are at most R floats,
// so these kernels are latency-bound, not bandwidth-bound.
#include "rowsum.hpp"
#include "groups.hpp"

namespace vcas {

// ---- block-wide sums over 1024 threads in a fixed order ---------------------
// Thread tid is "slot" tid.  Each 64-slot group (one wavefront) is combined by
// the neighbours-first tree, then the 16 group sums by the same kind of tree.
// Every thread returns the totals.  `bufd` / `bufi` are 16 values of LDS each;
// calls must alternate buffers or be separated by a barrier.
// `c_wave` is the wavefront's count, already the same in all its lanes.
__device__ __forceinline__ void block_totals_1024(double v, int c_wave, double *bufd, int *bufi, double &sum_v,
                                                  int &sum_c)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = wave_exchange_sum(v);
    if (lane == 0) {
        bufd[wave] = v;
        bufi[wave] = c_wave;
    }
    __syncthreads();
    // every 16-lane row holds the 16 partials, one per lane, and adds them by the same tree
    // (quad swaps, then the two mirrors) instead of every lane reading and adding all 16
    double w = bufd[lane & 15];
    int c = bufi[lane & 15];
    w = w + dpp_move<0xB1>(w);
    w = w + dpp_move<0x4E>(w);
    w = w + dpp_move<0x141>(w);
    w = w + dpp_move<0x140>(w);
    c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);
    c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);
    c += __builtin_amdgcn_update_dpp(0, c, 0x141, 0xF, 0xF, true);
    c += __builtin_amdgcn_update_dpp(0, c, 0x140, 0xF, 0xF, true);
    sum_v = read_lane(w, 0);
    sum_c = __builtin_amdgcn_readlane(c, 0);
}

__device__ __forceinline__ void block_sum_pair_1024(double v, int c, double *bufd, int *bufi, double &sum_v, int &sum_c)
{
    block_totals_1024(v, wave_sum_int(c), bufd, bufi, sum_v, sum_c);
}

__device__ __forceinline__ int ballot_count(bool c) { return __builtin_popcountll(__ballot(c)); }

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
    // w[j]: the score, as the fp64 summand it is, while element j is open (positive and not yet
    // fixed at one), +0 otherwise.  Adding +0 leaves a sum of non-negative terms as it is and
    // c * 0 never reaches one, so a round is one multiply, compare, select and add per element.
    double w[E];
    double part = 0.0;
    int cnt = 0;   // per wavefront, from ballots (scalar work, beside the vector sums)
    float open_max = 0.0f;   // largest score of this thread that is still open
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const bool pos = a[j] > 0.0f;
        w[j] = pos ? (double)a[j] : 0.0;
        part += w[j];
        cnt += ballot_count(pos);
        open_max = pos && a[j] > open_max ? a[j] : open_max;
    }
    double S;
    int nonzero;
    block_totals_1024(part, cnt, sd[0], si[0], S, nonzero);
    if (budget >= (double)nonzero) {
#pragma unroll
        for (int j = 0; j < E; ++j) prob[j] = a[j] > 0.0f ? 1.0f : 0.0f;
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
        cnt = 0;
        // The product is monotone in the score, rounding included: a thread whose largest open score
        // stays below one has nothing to fix, and its partial sum, the same additions over the same
        // values, is the one it already holds.  A wavefront without any thread that fixes something
        // skips the round's arithmetic (in the later rounds that is most of them).
        if (__ballot(c * (double)open_max >= 1.0) != 0ull) {
            part = 0.0;
            open_max = 0.0f;
#pragma unroll
            for (int j = 0; j < E; ++j) {
                const bool cap = c * w[j] >= 1.0;
                w[j] = cap ? 0.0 : w[j];
                part += w[j];
                cnt += ballot_count(cap);
                const float still = (float)w[j];   // exact: a score, or zero
                open_max = still > open_max ? still : open_max;
            }
        }
        double S_next;
        int newly;
        block_totals_1024(part, cnt, sd[flip], si[flip], S_next, newly);
        flip ^= 1;
        if (newly == 0) break;
        ncap += newly;
        S = S_next;
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
        float p = 0.0f;
        if (a[j] > 0.0f) {
            if (w[j] == 0.0) {
                p = 1.0f;   // fixed at one in some round
            } else {
                p = (float)(c * w[j]);
                p = p < 1.0f ? p : 1.0f;
            }
        }
        prob[j] = p;
    }
}

// Ascending list of the kept indices and their count for the register layout of the fused
// samplers: element j of thread tid is index tid + 1024 j, so ascending order is j, then
// wavefront, then lane.  Every wavefront counts its kept lanes per j with a ballot; the first
// wavefront turns the 16 E counts into bases; a lane's position is its base plus the kept lanes
// below it.
template <int E>
__device__ __forceinline__ void compact_regs(const bool (&m)[E], int32_t *__restrict__ idx,
                                             int32_t *__restrict__ count)
{
    constexpr int CNT = 16 * E, PER = (CNT + 63) / 64;
    __shared__ int counts[CNT + 1];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint64_t b[E];
#pragma unroll
    for (int j = 0; j < E; ++j) b[j] = __ballot(m[j]);
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < E; ++j) counts[j * 16 + wave] = __builtin_popcountll(b[j]);
    }
    __syncthreads();
    if (wave == 0) {
        // lane L owns counts PER*L .. PER*L+PER-1; exclusive prefix of all of them, in place
        int c[PER], mine = 0;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            c[q] = PER * lane + q < CNT ? counts[PER * lane + q] : 0;
            mine += c[q];
        }
        int incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += up;
        }
        int run = incl - mine;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            if (PER * lane + q < CNT) counts[PER * lane + q] = run;
            run += c[q];
        }
        if (lane == 63) counts[CNT] = incl;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int base = counts[j * 16 + wave];
        const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(b[j] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b[j], 0u));
        if (m[j]) idx[base + below] = (int)threadIdx.x + 1024 * j;
    }
    if (threadIdx.x == 0) *count = counts[CNT];
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
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (draw_offset) draw += *draw_offset;
    for (int i = wave; i < N; i += 16) {
        const float norm = sample_norm_wave(gsq + (int64_t)i * T, T);
        if (lane == 0) gn[i] = norm;
    }
    __syncthreads();
    if (N <= 64) {
        // one wavefront decides (see sample_a_small.hpp)
        if (wave != 0) return;
        const float a = lane < N ? gn[lane] : 0.0f;
        const SampleADecision d = sample_a_wave(a, N, budget, seed, layer, draw);
        if (lane < N) {
            gnorm[lane] = a;
            p[lane] = d.pr;
            maskA[lane] = d.keep ? 1 : 0;
        }
        if (d.keep) idxA[d.below] = lane;
        if (lane == 0) *cntA = d.count;
        return;
    }
    float a[1], pr[1];
    a[0] = tid < N ? gn[tid] : 0.0f;
    keep_probs_regs<1>(a, budget, pr);
    bool m[1] = {false};
    if (tid < N) {
        m[0] = philox_uniform(seed, layer, 0u, draw, (uint32_t)tid) < pr[0];
        gnorm[tid] = a[0];
        p[tid] = pr[0];
        maskA[tid] = m[0] ? 1 : 0;
    }
    compact_regs<1>(m, idxA, cntA);
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

// SampleA of up to kMaxSiblings layers with the same N and T, one workgroup per layer.
__global__ __launch_bounds__(1024) void sampler_a_group_kernel(SampleAGroup grp, int N, int T)
{
    const InlineSampleA &q = grp.prob[blockIdx.x];
    sampler_a_fast_body(q.gsq, N, T, q.budget, q.seed, q.layer, q.draw, q.draw_offset, q.gnorm, q.p, q.maskA, q.idxA,
                        q.cntA);
}

// What the caller has already left in the score and q arrays when SampleW starts.
enum : int {
    kFromSquares = 0,   // nothing: scores come from gsq, xsq and p
    kRootsGiven = 1,    // score[t] = sqrt(gsq[t]), q[t] = sqrt(xsq[t]) for every row
    kScoresGiven = 2,   // score[t] is final (0 on dropped samples, whose xsq is 0 already)
};

// t / T for t * T < 2^32 with a multiplier the wavefront computes once (T > 1):
// t * (floor(2^32 / T) + 1) / 2^32 = t / T + t * e / 2^32 with 0 < e <= 1, and
// t / 2^32 < 1 / T keeps the sum below the next integer.
__device__ __forceinline__ int sample_of(int t, int T, uint32_t magic)
{
    return T > 1 ? (int)__umulhi((uint32_t)t, magic) : t;
}

// SampleW for R <= 1024*E (one workgroup of 1024).  The whole vector is this one
// workgroup's arithmetic, so everything per sample (1/p_i, the keep byte) is
// computed once into LDS when N <= 1024, and the square roots come from the
// many-workgroup norm pass when the caller says so (`prepared`).
template <int E>
__device__ __forceinline__ void sampler_w_fast_body(const float *__restrict__ gsq, float *__restrict__ xsq,
                                                    int zero_dropped_xsq, const float *__restrict__ p,
                                                    const uint8_t *__restrict__ maskA, const float *__restrict__ u,
                                                    int N, int T, double budget, int token_sampling, int prepared,
                                                    float *__restrict__ score, float *__restrict__ q,
                                                    uint8_t *__restrict__ maskW, float *__restrict__ scaleW,
                                                    int32_t *__restrict__ idxW, int32_t *__restrict__ cntW)
{
    __shared__ float p_of[1024], pinv_of[1024];
    __shared__ uint8_t keep_of[1024];
    const int tid = threadIdx.x;
    const int R = N * T;
    const bool table = N <= 1024;
    const uint32_t magic = T > 1 ? (uint32_t)(0x100000000ull / (uint32_t)T) + 1u : 0u;
    // Every load of the vectors first, with no condition on a loaded value in between, so that
    // they are all in flight together (rows past the end re-read the last row and are ignored).
    float a[E], rx[E], qv[E], uu[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int t = min(tid + 1024 * j, R - 1);
        uu[j] = token_sampling ? u[t] : 0.0f;
        if (prepared == kFromSquares) {
            a[j] = gsq[t];
            rx[j] = xsq[t];
        } else {
            a[j] = score[t];
            rx[j] = prepared == kRootsGiven ? q[t] : 0.0f;
        }
    }
    if (table) {
        if (tid < N) {
            const float pi = p[tid];
            const uint8_t k = maskA[tid];
            p_of[tid] = pi;
            keep_of[tid] = k;
            pinv_of[tid] = k ? 1.0f / pi : 0.0f;
        }
        __syncthreads();
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int t = tid + 1024 * j;
        if (t >= R) {
            a[j] = 0.0f;
            uu[j] = 2.0f;
        } else if (prepared != kScoresGiven) {
            const int i = sample_of(t, T, magic);
            const bool keep = table ? keep_of[i] != 0 : maskA[i] != 0;
            const float rg = prepared == kRootsGiven ? a[j] : __builtin_sqrtf(a[j]);
            const float rxx = prepared == kRootsGiven ? rx[j] : __builtin_sqrtf(rx[j]);
            a[j] = 0.0f;
            if (keep) {
                const float inv = table ? pinv_of[i] : 1.0f / p[i];
                const float s1 = inv * rg;
                a[j] = s1 * rxx;
            } else if (zero_dropped_xsq) {
                xsq[t] = 0.0f;
            }
            score[t] = a[j];
        }
    }
    if (token_sampling) keep_probs_regs<E>(a, budget, qv);
    bool m[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
        const int t = tid + 1024 * j;
        m[j] = false;
        if (t < R) {
            const int i = sample_of(t, T, magic);
            const float pi = table ? p_of[i] : p[i];
            if (token_sampling) {
                m[j] = uu[j] < qv[j];
            } else {
                m[j] = table ? keep_of[i] != 0 : maskA[i] != 0;
                qv[j] = m[j] ? 1.0f : 0.0f;
            }
            q[t] = qv[j];
            maskW[t] = m[j] ? 1 : 0;
            scaleW[t] = m[j] ? 1.0f / (pi * qv[j]) : 0.0f;
        }
    }
    compact_regs<E>(m, idxW, cntW);
}

template <int E>
__global__ __launch_bounds__(1024) void sampler_w_fast_kernel(const float *__restrict__ gsq,
                                                              float *__restrict__ xsq, int zero_dropped_xsq,
                                                              const float *__restrict__ p,
                                                              const uint8_t *__restrict__ maskA,
                                                              const float *__restrict__ u, int N, int T, double budget,
                                                              int token_sampling, int prepared,
                                                              float *__restrict__ score, float *__restrict__ q,
                                                              uint8_t *__restrict__ maskW, float *__restrict__ scaleW,
                                                              int32_t *__restrict__ idxW, int32_t *__restrict__ cntW)
{
    sampler_w_fast_body<E>(gsq, xsq, zero_dropped_xsq, p, maskA, u, N, T, budget, token_sampling, prepared, score, q,
                           maskW, scaleW, idxW, cntW);
}

// SampleW of up to kMaxSiblings layers of one shape, one workgroup per layer.
template <int E>
__global__ __launch_bounds__(1024) void sampler_w_group_kernel(SampleWGroup grp, int zero_dropped_xsq, int N, int T,
                                                               int token_sampling, int prepared)
{
    const SampleWProblem &w = grp.prob[blockIdx.x];
    sampler_w_fast_body<E>(w.gsq, w.xsq, zero_dropped_xsq, w.p, w.maskA, w.u, N, T, w.budget, token_sampling, prepared,
                           w.score, w.q, w.maskW, w.scaleW, w.idxW, w.cntW);
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
                                                         int token_sampling, int prepared,
                                                         float *__restrict__ score, float *__restrict__ q,
                                                         uint8_t *__restrict__ maskW, float *__restrict__ scaleW,
                                                         int32_t *__restrict__ idxW, int32_t *__restrict__ cntW)
{
    const int tid = threadIdx.x;
    const int R = N * T;
    for (int t = tid; t < R && prepared != kScoresGiven; t += 1024) {
        const int i = t / T;
        float s = 0.0f;
        if (maskA[i]) {
            const float inv = 1.0f / p[i];
            const float a = inv * (prepared == kRootsGiven ? score[t] : __builtin_sqrtf(gsq[t]));
            s = a * (prepared == kRootsGiven ? q[t] : __builtin_sqrtf(xsq[t]));
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

// sampler_a for n <= kMaxSiblings layers of N <= 1024 samples in one launch
vcas_status sampler_a_group(const SampleAGroup &grp, int n, int N, int T, hipStream_t st)
{
    if (n < 1 || n > kMaxSiblings || N > 1024) return VCAS_EINVAL;
    hipLaunchKernelGGL(sampler_a_group_kernel, dim3(n), dim3(1024), 0, st, grp, N, T);
    return launch_status();
}

vcas_status uniforms(int64_t R, const vcas_rng &rng, uint32_t stream_id, float *u, hipStream_t st)
{
    hipLaunchKernelGGL(uniforms_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, R, rng.seed, rng.layer,
                       stream_id, rng.draw, rng.draw_offset, u);
    return launch_status();
}

vcas_status sampler_w(const float *gsq, float *xsq, int zero_dropped_xsq, const float *p, const uint8_t *maskA,
                      const float *u, int N, int T, double budget, int token_sampling, int prepared, float *score,
                      float *q, uint8_t *maskW, float *scaleW, int32_t *idxW, int32_t *cntW, hipStream_t st)
{
    const int64_t R = (int64_t)N * T;
#define VCAS_SAMPLER_W_ARGS                                                                                      \
    gsq, xsq, zero_dropped_xsq, p, maskA, u, N, T, budget, token_sampling, prepared, score, q, maskW, scaleW, idxW, \
        cntW
    if (R <= 4096)
        hipLaunchKernelGGL(sampler_w_fast_kernel<4>, dim3(1), dim3(1024), 0, st, VCAS_SAMPLER_W_ARGS);
    else if (R <= 16384)
        hipLaunchKernelGGL(sampler_w_fast_kernel<16>, dim3(1), dim3(1024), 0, st, VCAS_SAMPLER_W_ARGS);
    else
        hipLaunchKernelGGL(sampler_w_kernel, dim3(1), dim3(1024), 0, st, VCAS_SAMPLER_W_ARGS);
#undef VCAS_SAMPLER_W_ARGS
    return launch_status();
}

// sampler_w for n <= kMaxSiblings layers with at most 16384 rows each in one launch
vcas_status sampler_w_group(const SampleWGroup &grp, int n, int zero_dropped_xsq, int N, int T, int token_sampling,
                            int prepared, hipStream_t st)
{
    const int64_t R = (int64_t)N * T;
    if (n < 1 || n > kMaxSiblings || R > 16384) return VCAS_EINVAL;
    if (R <= 4096)
        hipLaunchKernelGGL(sampler_w_group_kernel<4>, dim3(n), dim3(1024), 0, st, grp, zero_dropped_xsq, N, T,
                           token_sampling, prepared);
    else
        hipLaunchKernelGGL(sampler_w_group_kernel<16>, dim3(n), dim3(1024), 0, st, grp, zero_dropped_xsq, N, T,
                           token_sampling, prepared);
    return launch_status();
}

}  // namespace vcas
