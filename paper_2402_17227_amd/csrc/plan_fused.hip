// The whole sampling plan of a small layer in ONE launch (Sec. 4.1 SampleA,
// Sec. 4.2 SampleW): every workgroup takes rows of G and X and writes their sums
// of squares (and the SampleW uniforms); the workgroup that finishes last then
// runs both samplers on the vectors the others left in memory.  A layer of
// BERT-base size needs seven launches otherwise, and the command processor
// starts only about one kernel every 2.5 us.
//
// The samplers here are written for 256 threads (so that the norm phase keeps
// small workgroups) and compute bit for bit what the 1024-thread kernels of
// sampling.hip compute: the same 1024 summation slots (slot = index mod 1024,
// ascending index inside a slot), the same 64-slot group trees and the same tree
// over the 16 group sums.  Thread tid owns slots tid + 256 k, k < 4, i.e. groups
// wave + 4 k.
#include "rowsum.hpp"

namespace vcas {

namespace {

constexpr int kThreads = 256;
constexpr int kSub = 32;       // first-level ticket counters
constexpr int kLine = 32;      // words between counters: every counter has a 128-byte line to itself

struct PlanLds {
    float gn[1024];      // ||G_i||_F
    float p[1024];       // keep probability of sample i
    float pinv[1024];    // 1 / p_i
    uint8_t m[1024];     // SampleA mask
    double sd[2][16];    // group sums of a round (double buffered: one barrier per round)
    int si[2][4];        // per-wavefront counts of a round
    int counts[64];      // kept elements per (j, k, wavefront), compaction
    int last;
};

struct PlanArgs {
    const uint4 *G, *X;
    int groups_g, groups_x;       // 16-byte groups per row
    int N, T;
    double budget_a, budget_w;
    int token_sampling;
    UniformJob job;               // SampleW uniforms (stream 1); seed, layer, draw also serve SampleA
    uint32_t *tickets;            // kSub + 1 zeroed counters, kLine words apart
    float *gsq, *gnorm, *p;
    uint8_t *maskA;
    int32_t *idxA, *cntA;
    float *xsq, *score, *q;
    uint8_t *maskW;
    float *scaleW;
    int32_t *idxW, *cntW;
};

// Store that is written through to device-coherent memory (no dirty line stays in this XCD's L2).
__device__ __forceinline__ void store_through(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ int ballot_count(bool c) { return __builtin_popcountll(__ballot(c)); }

// prob = min(1, c * a) with sum prob = min(budget, #positive a): the rounds of keep_probs_regs
// in sampling.hip, for 256 threads.  SINGLE: every positive entry lies in slots 0..63, so the
// first wavefront does it alone (the other 15 group sums are +0 and x + 0 = x) without LDS or
// barriers; the other wavefronts' entries are all zero.
template <int E, bool SINGLE>
__device__ __forceinline__ void keep_probs_256(const float (&a)[4][E], double budget, float (&prob)[4][E],
                                               PlanLds &L)
{
    constexpr int KK = SINGLE ? 1 : 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < E; ++j) prob[k][j] = 0.0f;
    if (SINGLE && wave != 0) return;
    int flip = 0;
    auto totals = [&](const double (&part)[4], int cnt_wave, double &S, int &C) {
        if (SINGLE) {
            S = wave_exchange_sum(part[0]);
            C = cnt_wave;
            return;
        }
        double g[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) g[k] = wave_exchange_sum(part[k]);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) L.sd[flip][4 * k + wave] = g[k];
            L.si[flip][wave] = cnt_wave;
        }
        __syncthreads();
        double wd[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) wd[i] = L.sd[flip][i];
        S = tree16(wd);
        C = (L.si[flip][0] + L.si[flip][1]) + (L.si[flip][2] + L.si[flip][3]);
        flip ^= 1;
    };
    double part[4] = {0.0, 0.0, 0.0, 0.0};
    int cnt = 0;
#pragma unroll
    for (int k = 0; k < KK; ++k)
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const bool pos = a[k][j] > 0.0f;
            if (pos) part[k] += (double)a[k][j];
            cnt += ballot_count(pos);
        }
    double S;
    int nonzero;
    totals(part, cnt, S, nonzero);
    if (budget >= (double)nonzero) {
#pragma unroll
        for (int k = 0; k < KK; ++k)
#pragma unroll
            for (int j = 0; j < E; ++j) prob[k][j] = a[k][j] > 0.0f ? 1.0f : 0.0f;
        return;
    }
    uint32_t fixed = 0;   // bit k*E+j: element fixed at one
    int ncap = 0;
    double c = 0.0;
    for (;;) {
        const double rem = budget - (double)ncap;
        if (!(S > 0.0) || !(rem > 0.0)) {
            c = 0.0;
            break;
        }
        c = rem / S;
        cnt = 0;
#pragma unroll
        for (int k = 0; k < KK; ++k) {
            part[k] = 0.0;
#pragma unroll
            for (int j = 0; j < E; ++j) {
                const uint32_t bit = 1u << (k * E + j);
                const bool open = a[k][j] > 0.0f && !(fixed & bit);
                const bool cap = open && c * (double)a[k][j] >= 1.0;
                if (cap) fixed |= bit;
                if (open && !cap) part[k] += (double)a[k][j];
                cnt += ballot_count(cap);
            }
        }
        double S_next;
        int newly;
        totals(part, cnt, S_next, newly);
        if (newly == 0) break;
        ncap += newly;
        S = S_next;
    }
#pragma unroll
    for (int k = 0; k < KK; ++k)
#pragma unroll
        for (int j = 0; j < E; ++j) {
            float pr = 0.0f;
            if (fixed & (1u << (k * E + j))) pr = 1.0f;
            else if (a[k][j] > 0.0f) {
                pr = (float)(c * (double)a[k][j]);
                pr = pr < 1.0f ? pr : 1.0f;
            }
            prob[k][j] = pr;
        }
}

template <int E>
__device__ __forceinline__ void keep_probs_256(const float (&a)[4][E], double budget, int used_slots,
                                               float (&prob)[4][E], PlanLds &L)
{
    if (used_slots <= 64) keep_probs_256<E, true>(a, budget, prob, L);
    else keep_probs_256<E, false>(a, budget, prob, L);
}

// Ascending list of the kept indices and their count.  Element (k, j) of thread tid is index
// tid + 256 k + 1024 j, so ascending order is j, then k, then wavefront, then lane: each
// wavefront counts its kept lanes per (j, k) with a ballot, one 64-lane scan turns the
// 16 E counts into bases, and a lane's position is its base plus the kept lanes below it.
template <int E>
__device__ __forceinline__ void compact_256(const bool (&m)[4][E], int32_t *__restrict__ idx,
                                            int32_t *__restrict__ count, PlanLds &L)
{
    static_assert(16 * E <= 64, "one wavefront scans all counts");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint64_t b[4][E];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < E; ++j) b[k][j] = __ballot(m[k][j]);
    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int j = 0; j < E; ++j) L.counts[(j * 4 + k) * 4 + wave] = __builtin_popcountll(b[k][j]);
    }
    __syncthreads();
    const int c = lane < 16 * E ? L.counts[lane] : 0;
    int incl = c;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    const int excl = incl - c;
    const int total = __builtin_amdgcn_readlane(incl, 63);
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int base = __builtin_amdgcn_readlane(excl, (j * 4 + k) * 4 + wave);
            const int below = __builtin_amdgcn_mbcnt_hi((uint32_t)(b[k][j] >> 32),
                                                        __builtin_amdgcn_mbcnt_lo((uint32_t)b[k][j], 0u));
            if (m[k][j]) idx[base + below] = (int)threadIdx.x + 256 * k + 1024 * j;
        }
    if (threadIdx.x == 0) *count = total;
}

// SampleA then SampleW by one workgroup of 256 threads; N <= 1024, R <= 4096.
__device__ __forceinline__ void samplers_256(const PlanArgs &a, PlanLds &L)
{
    constexpr int E = 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = a.N, T = a.T, R = N * T;
    const uint32_t draw = a.job.draw + (a.job.draw_offset ? *a.job.draw_offset : 0u);
    // ||G_i||_F: value t of a sample belongs to lane t mod 64, fp32 adds in ascending t, lane tree.
    // These loads are the first to be needed, so they go out before the thread's own tokens, and
    // for eight samples at a time (adding +0 for t >= T changes nothing: the sums are >= +0).
    if (T <= 256) {
        for (int i0 = wave; i0 < N; i0 += 32) {
            float v[8][4];
#pragma unroll
            for (int s = 0; s < 8; ++s)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int i = i0 + 4 * s, t = lane + 64 * c;
                    v[s][c] = (i < N && t < T) ? a.gsq[(int64_t)i * T + t] : 0.0f;
                }
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                float acc = 0.0f;
#pragma unroll
                for (int c = 0; c < 4; ++c) acc = acc + v[s][c];
                acc = wave_exchange_sum(acc);
                if (lane == 0 && i0 + 4 * s < N) L.gn[i0 + 4 * s] = __builtin_sqrtf(acc);
            }
        }
    } else {
        for (int i = wave; i < N; i += 4) {
            const float *row = a.gsq + (int64_t)i * T;
            float acc = 0.0f;
            for (int t = lane; t < T; t += 64) acc = acc + row[t];
            acc = wave_exchange_sum(acc);
            if (lane == 0) L.gn[i] = __builtin_sqrtf(acc);
        }
    }
    // this thread's tokens: issued now, needed after SampleA
    float g[4][E], x[4][E], uu[4][E];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int t = tid + 256 * k + 1024 * j;
            g[k][j] = x[k][j] = 0.0f;
            uu[k][j] = 2.0f;
            if (t < R) {
                g[k][j] = a.gsq[t];
                x[k][j] = a.xsq[t];
                if (a.token_sampling) uu[k][j] = a.job.uniforms[t];
            }
        }
    __syncthreads();

    float a1[4][1], p1[4][1];
#pragma unroll
    for (int k = 0; k < 4; ++k) a1[k][0] = tid + 256 * k < N ? L.gn[tid + 256 * k] : 0.0f;
    keep_probs_256<1>(a1, a.budget_a, N, p1, L);
    bool mA[4][1];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int i = tid + 256 * k;
        mA[k][0] = false;
        if (i < N) {
            mA[k][0] = philox_uniform(a.job.seed, a.job.layer, 0u, draw, (uint32_t)i) < p1[k][0];
            a.gnorm[i] = a1[k][0];
            a.p[i] = p1[k][0];
            a.maskA[i] = mA[k][0] ? 1 : 0;
            L.p[i] = p1[k][0];
            L.pinv[i] = 1.0f / p1[k][0];
            L.m[i] = mA[k][0] ? 1 : 0;
        }
    }
    compact_256<1>(mA, a.idxA, a.cntA, L);   // its barrier also publishes L.p and L.m

    // t / T by a multiply: exact for t * T < 2^32 (t < 4096 here)
    const uint32_t magic = (uint32_t)((((uint64_t)1 << 32) + (uint32_t)T - 1) / (uint32_t)T);
    float sc[4][E], qv[4][E], pi[4][E];
    bool keep[4][E];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int t = tid + 256 * k + 1024 * j;
            sc[k][j] = 0.0f;
            pi[k][j] = 1.0f;
            keep[k][j] = false;
            if (t < R) {
                const int i = T == 1 ? t : (int)__umulhi((uint32_t)t, magic);
                keep[k][j] = L.m[i] != 0;
                pi[k][j] = L.p[i];
                if (keep[k][j]) {
                    const float s1 = L.pinv[i] * __builtin_sqrtf(g[k][j]);
                    sc[k][j] = s1 * __builtin_sqrtf(x[k][j]);
                } else {
                    a.xsq[t] = 0.0f;
                }
                a.score[t] = sc[k][j];
            }
        }
    if (a.token_sampling) {
        keep_probs_256<E>(sc, a.budget_w, R < 1024 ? R : 1024, qv, L);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int j = 0; j < E; ++j) qv[k][j] = keep[k][j] ? 1.0f : 0.0f;
    }
    bool mW[4][E];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int t = tid + 256 * k + 1024 * j;
            mW[k][j] = false;
            if (t < R) {
                mW[k][j] = a.token_sampling ? uu[k][j] < qv[k][j] : keep[k][j];
                a.q[t] = qv[k][j];
                a.maskW[t] = mW[k][j] ? 1 : 0;
                a.scaleW[t] = mW[k][j] ? 1.0f / (pi[k][j] * qv[k][j]) : 0.0f;
            }
        }
    __syncthreads();   // the first compaction's counts have been read by every wavefront
    compact_256<E>(mW, a.idxW, a.cntW, L);
}

template <bool BF16, int CH>
__global__ __launch_bounds__(kThreads) void plan_fused_kernel(PlanArgs a)
{
    __shared__ PlanLds L;
    const int R = a.N * a.T;
    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t draw = a.job.draw + (a.job.draw_offset ? *a.job.draw_offset : 0u);
    if (a.job.uniforms)
        for (int r = blockIdx.x * kThreads + tid; r < R; r += gridDim.x * kThreads)
            store_through(a.job.uniforms + r,
                          philox_uniform(a.job.seed, a.job.layer, a.job.stream_id, draw, (uint32_t)r));
    // rows [0, R) are G's, [R, 2R) are X's; a wavefront takes two rows at a time so that the
    // loads of both are in flight together
    const int wave = blockIdx.x * (kThreads / 64) + (tid >> 6), nwaves = gridDim.x * (kThreads / 64);
    for (int w = wave; w < 2 * R; w += 2 * nwaves) {
        const int w2 = w + nwaves;
        const bool two = w2 < 2 * R;
        const bool sx0 = w >= R, sx1 = w2 >= R;
        const int row0 = sx0 ? w - R : w, row1 = sx1 ? w2 - R : w2;
        const int gr0 = sx0 ? a.groups_x : a.groups_g, gr1 = sx1 ? a.groups_x : a.groups_g;
        const uint4 *p0 = (sx0 ? a.X : a.G) + (int64_t)row0 * gr0;
        const uint4 *p1 = (sx1 ? a.X : a.G) + (int64_t)row1 * gr1;
        float acc0, acc1 = 0.0f;
        if (gr0 <= 64 * CH && gr1 <= 64 * CH) {
            uint4 v0[CH], v1[CH];
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                const int gidx = lane + 64 * j;
                v0[j] = gidx < gr0 ? p0[gidx] : make_uint4(0u, 0u, 0u, 0u);
                v1[j] = two && gidx < gr1 ? p1[gidx] : make_uint4(0u, 0u, 0u, 0u);
            }
            acc0 = chunk_sumsq<BF16, CH>(v0, (gr0 + 63) / 64);
            if (two) acc1 = chunk_sumsq<BF16, CH>(v1, (gr1 + 63) / 64);
        } else {
            acc0 = wave_row_sumsq<BF16, CH>(p0, gr0);
            if (two) acc1 = wave_row_sumsq<BF16, CH>(p1, gr1);
        }
        if (lane == 0) {
            store_through((sx0 ? a.xsq : a.gsq) + row0, acc0);
            if (two) store_through((sx1 ? a.xsq : a.gsq) + row1, acc1);
        }
    }
    // The results went out as write-through stores, so releasing them needs no L2 write-back
    // (which costs every workgroup microseconds): wait until this workgroup's stores are
    // acknowledged, then take a ticket.  Two levels of counters keep the atomics on one address
    // few: a workgroup that completes its first-level counter takes a ticket of the top one.
    // Only the workgroup that completes the top counter stays; it zeroes the counters for the
    // next launch and drops whatever stale lines its caches hold before it reads the vectors.
    __builtin_amdgcn_s_waitcnt(0);   // vmcnt = expcnt = lgkmcnt = 0
    __syncthreads();
    if (tid == 0) {
        const uint32_t sub = blockIdx.x % kSub;
        const uint32_t members = (gridDim.x - sub + kSub - 1) / kSub;
        const uint32_t used = gridDim.x < (uint32_t)kSub ? gridDim.x : (uint32_t)kSub;
        int last = 0;
        if (__hip_atomic_fetch_add(a.tickets + sub * kLine, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
            members - 1)
            last = __hip_atomic_fetch_add(a.tickets + kSub * kLine, 1u, __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT) == used - 1;
        if (last)
            for (int i = 0; i <= kSub; ++i)
                __hip_atomic_store(a.tickets + i * kLine, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        L.last = last;
    }
    __syncthreads();
    if (!L.last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    samplers_256(a, L);
}

}  // namespace

// True when plan_fused handles this layer.
bool plan_fused_fits(int N, int T) { return N <= 1024 && (int64_t)N * T <= 4096; }

// Row norms of G and X, SampleA and SampleW of one layer in a single launch.  `tickets` are
// kPlanTicketBytes zeroed bytes of device memory that no other launch in flight uses; they are
// zero again when the launch has finished.
vcas_status plan_fused(const void *G, int K_out, const void *X, int K_in, int dtype, int N, int T, double budget_a,
                       double budget_w, int token_sampling, const vcas_rng &rng, float *uniforms, uint32_t *tickets,
                       const vcas_plan &pl, hipStream_t st)
{
    if (!plan_fused_fits(N, T)) return VCAS_EINVAL;
    const int per = dtype == VCAS_BF16 ? 8 : 4;
    PlanArgs a;
    a.G = static_cast<const uint4 *>(G);
    a.X = static_cast<const uint4 *>(X);
    a.groups_g = K_out / per;
    a.groups_x = K_in / per;
    a.N = N;
    a.T = T;
    a.budget_a = budget_a;
    a.budget_w = budget_w;
    a.token_sampling = token_sampling;
    a.job = {token_sampling ? uniforms : nullptr, rng.seed, rng.layer, 1u, rng.draw, rng.draw_offset};
    a.tickets = tickets;
    a.gsq = pl.gsq; a.gnorm = pl.gnorm; a.p = pl.p; a.maskA = pl.maskA; a.idxA = pl.idxA; a.cntA = pl.cntA;
    a.xsq = pl.xsq; a.score = pl.score; a.q = pl.q; a.maskW = pl.maskW; a.scaleW = pl.scaleW;
    a.idxW = pl.idxW; a.cntW = pl.cntW;
    const int R = N * T;
    const int need = ((a.groups_g > a.groups_x ? a.groups_g : a.groups_x) + 63) / 64;
    // four rows (two pairs) per wavefront, four wavefronts per workgroup
    const int blocks = (2 * R + 15) / 16;
#define VCAS_PLAN(B, C) hipLaunchKernelGGL((plan_fused_kernel<B, C>), dim3(blocks), dim3(kThreads), 0, st, a)
    if (dtype == VCAS_BF16) {
        if (need <= 2) VCAS_PLAN(true, 2);
        else if (need <= 4) VCAS_PLAN(true, 4);
        else VCAS_PLAN(true, 8);
    } else {
        if (need <= 2) VCAS_PLAN(false, 2);
        else if (need <= 4) VCAS_PLAN(false, 4);
        else VCAS_PLAN(false, 8);
    }
#undef VCAS_PLAN
    return launch_status();
}

}  // namespace vcas
