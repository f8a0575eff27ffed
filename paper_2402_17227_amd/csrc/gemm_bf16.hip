// bf16 MFMA gather-GEMM of the VCAS activation gradient (gfx950):
//   dgrad  dX[rows of kept samples] = (1/p_i) * G[row,:] W          (Eq. 2, upper line)
// A dense contraction over the kept rows only, on the matrix cores:
// v_mfma_f32_32x32x16_bf16, fp32 accumulation.  (The weight gradient is in wgrad_bf16.hip.)
//
// Tiling: a workgroup of WM x WN wavefronts owns a BM x BN output tile and walks the contraction
// in steps of 64, operand tiles double buffered in LDS.  The operand tiles never pass through
// registers: buffer loads write straight into LDS; W, which lies "the wrong way" for an MFMA
// lane (the contraction index is its slow dimension), stays as it is in memory, [64 k][columns],
// and ds_read_b64_tr_b16 transposes it on the way out.  The per-row 1/p goes into the epilogue.
#include <type_traits>

#include "mfma_bf16.hpp"

namespace vcas {

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 7); }
// byte offset of 16-byte slot `slot` (0..7) of tile row `row`
__device__ __forceinline__ int lds_off(int row, int slot) { return row * 128 + ((slot ^ swz(row)) << 4); }

// The j-th sample (0-based) that is NOT in the ascending list idx[0..cnt).
__device__ __forceinline__ int nth_missing(const int32_t *idx, int cnt, int j)
{
    int lo = 0, hi = cnt;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (idx[mid] - mid > j) hi = mid;
        else lo = mid + 1;
    }
    return j + lo;
}

// ------------------------------------------------------------------ dgrad
//
// The operand tiles of dgrad never pass through registers: buffer loads write
// straight into LDS (16 bytes per lane, a wavefront fills 1 KiB of consecutive
// LDS per instruction).  G lands as [row][64 k] rows with the XOR slot swizzle
// realised by WHICH 16-byte piece of the row each lane fetches; W lands as it
// lies in memory, [64 k][BN n], its slots swizzled the same way, and is
// transposed on the way out of LDS by ds_read_b64_tr_b16 (a block of 16 lanes
// reads 4 k-rows x 16 columns and each lane receives one column's 4 k values).
// NS stages; the loads of step s+NS-1 are issued while step s is computed.  One
// barrier per step: before it every wavefront waits until its own loads of the
// step have landed (s_waitcnt vmcnt, the counter is in order), after it the
// stage computed in the previous step is free.
template <int N>
__device__ __forceinline__ void wait_loads_outstanding()
{
    // s_waitcnt vmcnt(N) only: expcnt and lgkmcnt fields left at "no wait"
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

constexpr int kIdxStaged = 1024;   // kept-sample indices a workgroup stages in LDS ahead of the count

// grid: 1-D, tiles_n * (ceil(R/BM) + 1) + 8 workgroups.  The first ceil8(compute
// tiles) ids compute (spread over the XCDs in contiguous runs), the following
// ones write the zero rows of dropped samples, the rest exit.
// SPQ >= 0: one barrier at the top of every step; the loads of the next step are spread over the
// MFMAs of the first SPQ quarters of the current one (0: all issued right after the barrier).
// SPQ < 0 (two stages only): the barrier sits ahead of the step's LAST k-slice, the loads of the
// step after next go out one per -SPQ MFMAs from there, and the next step's first fragments are
// read under the last slice's MFMAs (256x256, one workgroup per CU: nothing else covers the
// wait for LDS behind a barrier there).
template <int BM, int BN, int WM, int WN, int NS, int SPQ>
__device__ __forceinline__ void dgrad_bf16_body(const uint16_t *__restrict__ G, const uint16_t *__restrict__ W,
                                                const float *__restrict__ p, const int32_t *__restrict__ idxA,
                                                const int32_t *__restrict__ cntA, uint16_t *__restrict__ dX, int N,
                                                int T, int K_in, int K_out, int tiles_n,
                                                const uint16_t *__restrict__ J, int fill_dropped,
                                                const InlineSampleA &sa, float *__restrict__ sq_blocks)
{
    constexpr int NW = WM * WN, NT = NW * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int AI = BM / (8 * NW), BI = BN / (8 * NW);     // LDS-direct loads per wavefront and step
    constexpr int B_ROWS = 512 / BN, B_SLOTS = BN / 8;         // k rows per W load, 16-byte slots per W row
    constexpr int STAGE = (BM + BN) * 128, B_AT = BM * 128, B_PITCH = BN * 2;
    constexpr int LOADS = AI + BI;
    static_assert(AI >= 1 && BI >= 1 && BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile/wave mismatch");
    static_assert(STAGE >= kIdxStaged * 4, "index staging area does not fit a stage");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int32_t *row_of = reinterpret_cast<int32_t *>(smem + NS * STAGE);
    float *scale_of = reinterpret_cast<float *>(row_of + BM);
    // The last stage is not loaded before the first barrier of the main loop; until then it
    // holds the kept-sample list, fetched together with the count instead of after it.
    int32_t *idx_staged = reinterpret_cast<int32_t *>(smem + (NS - 1) * STAGE);
    const int staged = min(N, kIdxStaged);
    __shared__ float sa_norm[64], sa_p[64];
    __shared__ int sa_count;
    int cnt;
    if (sa.gsq != nullptr || sa.norms != nullptr) {
        // SampleA decided here, by every workgroup for itself (N <= 64: a few microseconds of one
        // wavefront's work), instead of by a launch of its own in front of this one; the first
        // workgroup writes the plan's fields for everybody else.  The sample norms are either given
        // or taken here from the row sums (4 N T bytes that sit in L2: short vectors only).
        const int lane_ = threadIdx.x & 63, wave_ = threadIdx.x >> 6;
        const uint32_t draw = sa.draw + (sa.draw_offset ? *sa.draw_offset : 0u);   // fetched beside the norms
        const bool given = sa.norms != nullptr;
        if (!given) {
            if (T <= 128) sample_norms_batched<8, 2>(sa.gsq, wave_, NW, N, T, sa_norm);
            else sample_norms_batched<4, 8>(sa.gsq, wave_, NW, N, T, sa_norm);
            __syncthreads();
        }
        if (wave_ == 0) {
            const float a = lane_ < N ? (given ? sa.norms[lane_] : sa_norm[lane_]) : 0.0f;
            const SampleADecision d = sample_a_wave(a, N, sa.budget, sa.seed, sa.layer, draw);
            if (lane_ < N) sa_p[lane_] = d.pr;
            if (d.keep) idx_staged[d.below] = lane_;
            if (lane_ == 0) sa_count = d.count;
            if (blockIdx.x == 0) {
                if (lane_ < N) {
                    if (!given) sa.gnorm[lane_] = a;
                    sa.p[lane_] = d.pr;
                    sa.maskA[lane_] = d.keep ? 1 : 0;
                }
                if (d.keep) sa.idxA[d.below] = lane_;
                if (lane_ == 0) *sa.cntA = d.count;
            }
        }
        __syncthreads();
        cnt = sa_count;
        idxA = idx_staged;   // the kept list lives in LDS from here on (N <= 64 entries)
        p = sa_p;
    } else {
        for (int j = threadIdx.x; j < staged; j += NT) idx_staged[j] = idxA[j];
        cnt = min(max(*cntA, 0), N);
    }
    const int64_t M = (int64_t)cnt * T;
    const int64_t R = (int64_t)N * T;
    const int compute = (int)((M + BM - 1) / BM) * tiles_n;
    const int compute8 = (compute + 7) / 8 * 8;

    if ((int)blockIdx.x >= compute8) {
        // zero-fill duty: rows of the samples that are not in the kept list
        if (!fill_dropped) return;
        const int z = blockIdx.x - compute8;
        const int64_t d0 = (int64_t)(z / tiles_n) * BM;
        const int n0 = (z % tiles_n) * BN;
        if (d0 >= R - M) return;
        for (int r = threadIdx.x; r < BM; r += NT) {
            const int64_t d = d0 + r;
            int32_t dst = -1;
            if (d < R - M) dst = nth_missing(idxA, cnt, (int)(d / T)) * T + (int)(d % T);
            row_of[r] = dst;
        }
        __syncthreads();
        constexpr int CH = BN / 8;
        for (int u = threadIdx.x; u < BM * CH; u += NT) {
            const int r = u / CH, col = n0 + (u % CH) * 8;
            if (row_of[r] >= 0 && col < K_in)
                *reinterpret_cast<uint4 *>(dX + (int64_t)row_of[r] * K_in + col) = make_uint4(0u, 0u, 0u, 0u);
        }
        return;
    }
    const int tile = xcd_remap(blockIdx.x, compute);
    if (tile >= compute) return;
    int tile_m, tile_n;
    // An XCD gets a contiguous run of tile ids and has an L2 of its own: a run that spans all
    // column tiles reads its rows of G once and W whole (W eight times in all); with the
    // columns in `a` panels an XCD reads 1/a of W and every row of G is read by `a` XCDs.
    // a*|G kept| + (8/a)*|W|, i.e. a*M + (8/a)*K_in, is least at a = 1, 2, 4 for M >= 4 K_in, >= K_in, below.
    const int a_panels = M >= 4 * (int64_t)K_in ? 1 : M >= K_in ? 2 : 4;
    const int panel = min(8, max(1, (tiles_n + a_panels - 1) / a_panels));
    panel_order_rt(tile, compute / tiles_n, tiles_n, panel, tile_m, tile_n);
    const int n0 = tile_n * BN;
    const int64_t m0 = (int64_t)tile_m * BM;
    __syncthreads();   // idx_staged complete
    for (int r = threadIdx.x; r < BM; r += NT) {
        const int64_t m = m0 + r;
        int32_t dst = -1;
        if (m < M) {
            const int j = (int)(m / T);
            const int s = j < staged ? idx_staged[j] : idxA[j];
            if (s >= 0 && s < N) dst = s * T + (int)(m % T);
        }
        row_of[r] = dst;
    }
    __syncthreads();

    const i32x4 descG = raw_descriptor(G, (uint32_t)(R * K_out * 2));
    const i32x4 descW = raw_descriptor(W, (uint32_t)((int64_t)K_out * K_in * 2));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    // G load j: rows (wave*AI + j)*8 + lane/8, LDS slot lane%8 <- the row's 16-byte piece (slot ^ swz)
    // W load j: k rows (wave*BI + j)*B_ROWS + lane/B_SLOTS, LDS slot lane%B_SLOTS <- column chunk (slot ^ wswz)
    uint32_t a_off[AI], b_off[BI];
#pragma unroll
    for (int j = 0; j < AI; ++j) {
        const int row = (wave * AI + j) * 8 + (lane >> 3);
        const int32_t src = row_of[row];
        a_off[j] = src >= 0 ? (uint32_t)src * (uint32_t)K_out * 2u + (uint32_t)(((lane & 7) ^ swz(row)) * 16) : kOutside;
    }
#pragma unroll
    for (int j = 0; j < BI; ++j) {
        const int krow = (wave * BI + j) * B_ROWS + lane / B_SLOTS;
        const int col = n0 + ((lane % B_SLOTS) ^ wswz(krow)) * 8;
        b_off[j] = col < K_in ? ((uint32_t)krow * (uint32_t)K_in + (uint32_t)col) * 2u : kOutside;
    }
    const int steps = (K_out + BK - 1) / BK;
    // 16-byte pieces of a G row that the last step still owns (8 unless K_out is ragged).  The
    // pieces behind them lie in the NEXT row of G: they meet zero rows of W, but zero times
    // whatever that row holds (a NaN, an Inf, a row nobody has written) is not zero, so they are
    // not fetched.
    const int tail_pieces = (K_out - (steps - 1) * BK + 7) / 8;
    // the d-th of the LOADS loads of contraction step `step` into stage `stage`: G and W pieces alternate
    auto issue_nth = [&](int d, int stage, int step) {
        const uint32_t a_dst = __builtin_amdgcn_readfirstlane(lds0 + stage * STAGE + wave * AI * 1024);
        const uint32_t b_dst = __builtin_amdgcn_readfirstlane(lds0 + stage * STAGE + B_AT + wave * BI * 1024);
        const uint32_t kb = __builtin_amdgcn_readfirstlane(step * BK * 2);
        const uint32_t wb = __builtin_amdgcn_readfirstlane(step * BK * K_in * 2);
        const int pieces = step == steps - 1 ? tail_pieces : 8;
        int seen = 0;
#pragma unroll
        for (int j = 0; j < (AI > BI ? AI : BI); ++j) {
            if (j < AI) {
                if (seen == d) {
                    const int piece = (lane & 7) ^ swz((wave * AI + j) * 8 + (lane >> 3));
                    lds_direct_load16(descG, a_dst + j * 1024, piece < pieces ? a_off[j] : kOutside, kb);
                }
                ++seen;
            }
            if (j < BI) {
                if (seen == d) lds_direct_load16(descW, b_dst + j * 1024, b_off[j], wb);
                ++seen;
            }
        }
    };
    // prologue: steps 0 .. NS-2 in flight (a step past the end fills a stage nobody reads and keeps the counts uniform)
#pragma unroll
    for (int d = 0; d < NS - 1; ++d)
#pragma unroll
        for (int q = 0; q < LOADS; ++q) issue_nth(q, d, d < steps ? d : steps + 64);
    // 1/p of the tile's rows is needed in the epilogue only: fetched behind the first tile loads
    for (int r = threadIdx.x; r < BM; r += NT) {
        const int32_t dst = row_of[r];
        scale_of[r] = dst >= 0 ? 1.0f / p[dst / T] : 0.0f;
    }

    const int wm0 = (wave / WN) * (BM / WM), wn0 = (wave % WN) * (BN / WN);
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int r32 = lane & 31, h = lane >> 5;
    const int blk = lane >> 4, sl = lane & 15;    // 16-lane block and lane within it
    constexpr int KS = BK / 16, MM = TM * TN, SPAN = KS * MM * (SPQ > 0 ? SPQ : 0) / 4;
    // One contraction step on stage `stage`; the loads of step `nstep` go to stage `nstage`.
    // Fragments of two k-slices are read ahead; load d goes out after MFMA number d*SPAN/LOADS.
    auto step_body = [&](int stage, int nstage, int nstep) {
        const unsigned char *tileA = smem + stage * STAGE;
        const unsigned char *tileB = tileA + B_AT;
        bf16x8 a[2][TM], b[2][TN];
        auto read_frags = [&](int ks, bf16x8(&fa)[TM], bf16x8(&fb)[TN]) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const bf16x8 *>(tileA + lds_off(wm0 + i * 32 + r32, ks * 2 + h));
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                bf16x4 half[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int k = ks * 16 + (blk >> 1) * 8 + e * 4 + (sl >> 2);
                    const int col = wn0 + i * 32 + (blk & 1) * 16 + (sl & 3) * 4;
                    const unsigned char *src = tileB + k * B_PITCH + (((col >> 3) ^ wswz(k)) << 4) + (col & 7) * 2;
                    half[e] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (__attribute__((address_space(3))) bf16x4 *)(src));
                }
                fb[i] = __builtin_shufflevector(half[0], half[1], 0, 1, 2, 3, 4, 5, 6, 7);
            }
        };
        if (SPQ == 0) {
#pragma unroll
            for (int d = 0; d < LOADS; ++d) issue_nth(d, nstage, nstep);
            __builtin_amdgcn_sched_barrier(0);
        }
        read_frags(0, a[0], b[0]);
        if (KS > 1) read_frags(1, a[1], b[1]);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][i], b[ks & 1][j], acc[i][j], 0, 0, 0);
                    if (SPQ > 0) {
                        const int m = ks * MM + i * TN + j;
#pragma unroll
                        for (int d = 0; d < LOADS; ++d)
                            if (d * SPAN / LOADS == m) {
                                __builtin_amdgcn_sched_barrier(0);
                                issue_nth(d, nstage, nstep);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                    }
                }
            if (ks + 2 < KS) read_frags(ks + 2, a[ks & 1], b[ks & 1]);
        }
    };

    if constexpr (SPQ < 0) {
        // Two stages, the barrier ahead of the step's LAST k-slice.  By then every wavefront holds that
        // slice's fragments in registers, so the stage is free: the loads of step s+2 start there (one
        // per -SPQ MFMAs, running on into the next step's slices), and the first fragments of step s+1
        // are read under the last slice's MFMAs, so that no wavefront sits behind the barrier waiting for LDS.
        constexpr int EVERY = -SPQ;
        static_assert(NS == 2 && KS >= 2 && KS % 2 == 0, "two fragment sets alternate over an even number of slices");
        static_assert(LOADS * EVERY <= KS * MM, "a step's loads are all issued before its barrier");
        constexpr int AT_ONCE = MM / EVERY < LOADS ? MM / EVERY : LOADS;   // loads that go out during a last slice
        bf16x8 a[2][TM], b[2][TN];
        auto read_frags = [&](int stage, int ks, bf16x8(&fa)[TM], bf16x8(&fb)[TN]) {
            const unsigned char *tileA = smem + stage * STAGE;
            const unsigned char *tileB = tileA + B_AT;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const bf16x8 *>(tileA + lds_off(wm0 + i * 32 + r32, ks * 2 + h));
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                bf16x4 half[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int k = ks * 16 + (blk >> 1) * 8 + e * 4 + (sl >> 2);
                    const int col = wn0 + i * 32 + (blk & 1) * 16 + (sl & 3) * 4;
                    const unsigned char *src = tileB + k * B_PITCH + (((col >> 3) ^ wswz(k)) << 4) + (col & 7) * 2;
                    half[e] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (__attribute__((address_space(3))) bf16x4 *)(src));
                }
                fb[i] = __builtin_shufflevector(half[0], half[1], 0, 1, 2, 3, 4, 5, 6, 7);
            }
        };
        wait_loads_outstanding<0>();
        __syncthreads();                           // step 0 has landed
#pragma unroll
        for (int d = 0; d < AT_ONCE; ++d) issue_nth(d, 1, 1 < steps ? 1 : steps + 64);
        read_frags(0, 0, a[0], b[0]);
        for (int s = 0; s < steps; ++s) {
            const int cur = s & 1;
            const int after = s + 1 < steps ? s + 1 : steps + 64, after2 = s + 2 < steps ? s + 2 : steps + 64;
            __builtin_amdgcn_sched_barrier(0);
            read_frags(cur, 1, a[1], b[1]);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks == KS - 1) {
                    __builtin_amdgcn_sched_barrier(0);
                    wait_loads_outstanding<0>();   // step s+1: all of its loads have been issued by now
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // ... and this stage has been read
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_sched_barrier(0);
                    read_frags(cur ^ 1, 0, a[0], b[0]);
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][i], b[ks & 1][j], acc[i][j], 0, 0, 0);
                        // MFMAs counted from the start of a last slice: that slice, then the slices of the next step
                        const int m = (ks == KS - 1 ? 0 : (ks + 1) * MM) + i * TN + j;
                        if (m % EVERY == 0 && m / EVERY < LOADS) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (ks == KS - 1) issue_nth(m / EVERY, cur, after2);
                            else issue_nth(m / EVERY, cur ^ 1, after);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                if (ks + 2 < KS) read_frags(cur, ks + 2, a[ks & 1], b[ks & 1]);
            }
        }
    } else {
        for (int s = 0; s < steps; ++s) {
            // the NS-2 younger steps may stay in flight; step s must have landed
            wait_loads_outstanding<(NS - 2) * LOADS>();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const int nxt = s + NS - 1;
            __builtin_amdgcn_sched_barrier(0);
            step_body(s % NS, nxt % NS, nxt < steps ? nxt : steps + 64);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    wait_loads_outstanding<0>();

    // Epilogue.  An MFMA lane holds one column of 16 rows, so stores straight from the
    // accumulators would be 64-byte pieces, 64 instructions per wavefront.  Instead every wavefront
    // passes its (TM*32) x 64 sub-tile through LDS (the operand stages are free by now): rounded
    // values in, 128-byte rows (whole cache lines) out, 16 bytes per lane.  Row `row` of the strip
    // keeps logical 16-byte slot s at slot s ^ esw(row), so that the two rows a write instruction
    // touches per half-wavefront fall into different banks.
    static_assert(TN == 2, "a staged row is 64 columns = 128 bytes");
    static_assert(NW * TM * 4096 <= NS * STAGE, "the output strips are staged in the operand stages");
    __syncthreads();   // every wavefront is done with the stages
    unsigned char *strip = smem + wave * (TM * 4096);
    auto esw = [](int row) { return (row & 1) << 2; };
    if (J) {
        // Elementwise Jacobian of the layer below (App. E, proof of unbiasedness), same layout as
        // dX: its sub-tile is fetched into the strip first (zeros for rows and columns that are not
        // stored), in the layout the results will have; each lane then picks up the values at its
        // own column and multiplies before the one rounding.
        const i32x4 descJ = raw_descriptor(J, (uint32_t)(R * K_in * 2));
        const uint32_t strip_lds = __builtin_amdgcn_readfirstlane(lds0 + wave * (TM * 4096));
#pragma unroll
        for (int q = 0; q < TM * 4; ++q) {
            const int row = q * 8 + (lane >> 3);
            const int32_t dst = row_of[wm0 + row];
            const int col = n0 + wn0 + (((lane & 7) ^ esw(row)) << 3);
            const uint32_t off = dst >= 0 && col < K_in ? ((uint32_t)dst * (uint32_t)K_in + (uint32_t)col) * 2u : kOutside;
            lds_direct_load16(descJ, strip_lds + q * 1024, off, 0u);
        }
        wait_loads_outstanding<0>();
        asm volatile("" ::: "memory");
    }
    // A lane rounds its column's values of two neighbouring rows into one dword; neighbouring lanes
    // then trade halves (one DPP move, one byte permute) so that each owns two adjacent columns of
    // one row.  A dropped row has scale 0 and a column past K_in met zero columns of W, so what is
    // not stored arrives as zero and counts as zero in the block sums.  All LDS reads of a group
    // of cells come before its writes: the compiler cannot tell the strip from the row tables.
    const bool odd = lane & 1;
    const uint32_t halves = odd ? 0x03020706u : 0x05040100u;   // even: (mine.lo, other.lo); odd: (other.hi, mine.hi)
    auto fill_strip = [&](auto with_jacobian) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            float4 sc[4];
#pragma unroll
            for (int g = 0; g < 4; ++g)
                sc[g] = *reinterpret_cast<const float4 *>(scale_of + wm0 + i * 32 + g * 8 + (lane >> 5) * 4);
            uint16_t jw[16][TN];
            if (with_jacobian) {
                // the Jacobian's values at this lane's own column, rows acc_row(v)
#pragma unroll
                for (int v = 0; v < 16; ++v)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int row = i * 32 + acc_row(v);
                        const int slot = j * 4 + ((lane & 31) >> 3);
                        jw[v][j] = *reinterpret_cast<const uint16_t *>(strip + row * 128 + ((slot ^ esw(row)) << 4) +
                                                                      (lane & 7) * 2);
                    }
            }
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                const int row = i * 32 + acc_row(v) + (odd ? 1 : 0);
                const float sc_e = (v & 2) ? sc[v >> 2].z : sc[v >> 2].x, sc_o = (v & 2) ? sc[v >> 2].w : sc[v >> 2].y;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    float mine_e = acc[i][j][v] * sc_e, mine_o = acc[i][j][v + 1] * sc_o;
                    if (with_jacobian) {
                        mine_e = mine_e * __uint_as_float((uint32_t)jw[v][j] << 16);
                        mine_o = mine_o * __uint_as_float((uint32_t)jw[v + 1][j] << 16);
                    }
                    const uint32_t mine = pack_bf16(mine_e, mine_o);
                    const uint32_t other = __float_as_uint(dpp_move<0xB1>(__uint_as_float(mine)));
                    const int slot = j * 4 + ((lane & 31) >> 3);
                    *reinterpret_cast<uint32_t *>(strip + row * 128 + ((slot ^ esw(row)) << 4) + ((lane >> 1) & 3) * 4) =
                        __builtin_amdgcn_perm(other, mine, halves);
                }
            }
        }
    };
    if (J) fill_strip(std::true_type{});
    else fill_strip(std::false_type{});
    __builtin_amdgcn_wave_barrier();   // the strip is this wavefront's own: its LDS accesses execute in order
    int32_t dst_of[TM * 4];
    uint4 val[TM * 4];
#pragma unroll
    for (int q = 0; q < TM * 4; ++q) {
        const int row = q * 8 + (lane >> 3);
        dst_of[q] = row_of[wm0 + row];
        val[q] = *reinterpret_cast<const uint4 *>(strip + row * 128 + ((lane & 7) << 4));
    }
#pragma unroll
    for (int q = 0; q < TM * 4; ++q) {
        const int row = q * 8 + (lane >> 3);
        const int col = n0 + wn0 + (((lane & 7) ^ esw(row)) << 3);
        if (dst_of[q] >= 0 && col < K_in) *reinterpret_cast<uint4 *>(dX + (int64_t)dst_of[q] * K_in + col) = val[q];
    }
    if (sq_blocks) {
        // Sums of squares of the stored values by blocks of 64 columns (this wavefront's strip is
        // exactly one), pairwise with neighbours first: a lane adds its eight columns (three levels),
        // the eight lanes of a row the rest.  Four neighbouring blocks of a row lie side by side:
        // sq_blocks[((blk / 4) * R + row) * 4 + blk % 4].
        const int blk = (n0 + wn0) >> 6;
        const int nb = (K_in + 63) >> 6;
#pragma unroll
        for (int q = 0; q < TM * 4; ++q) {
            const uint4 w = val[q];
            const float q0 = bf16_lo(w.x) * bf16_lo(w.x), q1 = bf16_hi(w.x) * bf16_hi(w.x);
            const float q2 = bf16_lo(w.y) * bf16_lo(w.y), q3 = bf16_hi(w.y) * bf16_hi(w.y);
            const float q4 = bf16_lo(w.z) * bf16_lo(w.z), q5 = bf16_hi(w.z) * bf16_hi(w.z);
            const float q6 = bf16_lo(w.w) * bf16_lo(w.w), q7 = bf16_hi(w.w) * bf16_hi(w.w);
            float t = ((q0 + q1) + (q2 + q3)) + ((q4 + q5) + (q6 + q7));
            t = t + dpp_move<0xB1>(t);    // slots (0,1), (2,3), (4,5), (6,7)
            t = t + dpp_move<0x4E>(t);    // the two halves of each 32 columns
            t = t + dpp_move<0x141>(t);   // the two 32-column halves (the other quad of the row's eight lanes)
            if ((lane & 7) == 0 && dst_of[q] >= 0 && blk < nb)
                sq_blocks[((int64_t)(blk >> 2) * R + dst_of[q]) * 4 + (blk & 3)] = t;
        }
    }
}

template <int BM, int BN, int WM, int WN, int NS, int OCC, int SPQ>
__global__ __launch_bounds__(WM *WN * 64, OCC) void dgrad_bf16_kernel(const uint16_t *__restrict__ G,
                                                                  const uint16_t *__restrict__ W,
                                                                  const float *__restrict__ p,
                                                                  const int32_t *__restrict__ idxA,
                                                                  const int32_t *__restrict__ cntA,
                                                                  uint16_t *__restrict__ dX, int N, int T, int K_in,
                                                                  int K_out, int tiles_n,
                                                                  const uint16_t *__restrict__ J, int fill_dropped,
                                                                  InlineSampleA sa, float *__restrict__ sq_blocks)
{
    dgrad_bf16_body<BM, BN, WM, WN, NS, SPQ>(G, W, p, idxA, cntA, dX, N, T, K_in, K_out, tiles_n, J, fill_dropped, sa,
                                             sq_blocks);
}

// Several layers of one shape whose upstream gradients do not depend on each other (the Q, K and V
// projections of an attention block) in one launch: blockIdx.y picks the layer, everything else
// is the kernel above.
template <int BM, int BN, int WM, int WN, int NS, int OCC, int SPQ>
__global__ __launch_bounds__(WM *WN * 64, OCC) void dgrad_bf16_group_kernel(DgradGroup grp, int N, int T, int K_in,
                                                                        int K_out, int tiles_n, int fill_dropped)
{
    const DgradProblem &q = grp.prob[blockIdx.y];
    dgrad_bf16_body<BM, BN, WM, WN, NS, SPQ>(q.G, q.W, q.p, q.idxA, q.cntA, q.dX, N, T, K_in, K_out, tiles_n, q.J,
                                             fill_dropped, q.sa, q.sq_blocks);
}

// ---------------------------------------------------------- host launchers

template <int BM, int BN, int WM, int WN, int NS, int OCC, int SPQ>
static vcas_status launch_dgrad(const vcas_shape &s, const void *G, const void *W, const float *p,
                                const int32_t *idxA, const int32_t *cntA, void *dX, const void *J, bool fill,
                                const InlineSampleA &sa, float *sq_blocks, hipStream_t st)
{
    const int64_t R = (int64_t)s.N * s.T;
    const int tiles_n = (s.K_in + BN - 1) / BN;
    // without zero-fill duty the ids past the compute tiles have nothing to do
    const int64_t grid = tiles_n * ((R + BM - 1) / BM + (fill ? 1 : 0)) + 8;
    if (grid > (int64_t)1 << 30) return VCAS_EINVAL;
    const size_t lds = NS * (BM + BN) * 128 + BM * 8;
    auto kern = dgrad_bf16_kernel<BM, BN, WM, WN, NS, OCC, SPQ>;
    static bool allowed = false;
    if (!allowed) {
        if (!allow_lds(kern, lds)) return VCAS_EHIP;
        allowed = true;
    }
    launch_timed(0, kern, dim3((unsigned)grid), dim3(WM * WN * 64), lds, st, static_cast<const uint16_t *>(G),
                 static_cast<const uint16_t *>(W), p, idxA, cntA, static_cast<uint16_t *>(dX), s.N, s.T, s.K_in,
                 s.K_out, tiles_n, static_cast<const uint16_t *>(J), fill ? 1 : 0, sa, sq_blocks);
    return launch_status();
}

template <int BM, int BN, int WM, int WN, int NS, int OCC, int SPQ>
static vcas_status launch_dgrad_group(const vcas_shape &s, const DgradGroup &grp, int n, bool fill, hipStream_t st)
{
    const int64_t R = (int64_t)s.N * s.T;
    const int tiles_n = (s.K_in + BN - 1) / BN;
    // a multiple of 8 per layer, so that a workgroup's XCD is the same function of blockIdx.x in every layer
    const int64_t grid = (tiles_n * ((R + BM - 1) / BM + (fill ? 1 : 0)) + 8 + 7) / 8 * 8;
    if (grid > (int64_t)1 << 30) return VCAS_EINVAL;
    const size_t lds = NS * (BM + BN) * 128 + BM * 8;
    auto kern = dgrad_bf16_group_kernel<BM, BN, WM, WN, NS, OCC, SPQ>;
    static bool allowed = false;
    if (!allowed) {
        if (!allow_lds(kern, lds)) return VCAS_EHIP;
        allowed = true;
    }
    launch_timed(0, kern, dim3((unsigned)grid, (unsigned)n), dim3(WM * WN * 64), lds, st, grp, s.N, s.T, s.K_in,
                 s.K_out, tiles_n, fill ? 1 : 0);
    return launch_status();
}

// dgrad of n <= kMaxSiblings layers of shape s in one launch (see dgrad_bf16_group_kernel); the
// tile choice looks at the tiles of all of them together.
vcas_status dgrad_bf16_group(const vcas_shape &s, const DgradProblem *probs, int n, bool fill, int64_t expected_rows,
                             hipStream_t st)
{
    if (n < 1 || n > kMaxSiblings) return VCAS_EINVAL;
    DgradGroup grp = {};
    for (int i = 0; i < n; ++i) {
        if ((probs[i].sa.gsq || probs[i].sa.norms) && s.N > 64) return VCAS_EINVAL;
        grp.prob[i] = probs[i];
    }
    const int64_t R = (int64_t)s.N * s.T;
    const int64_t rows = expected_rows > 0 && expected_rows < R ? expected_rows : R;
    const int64_t tiles256 = n * ((rows + 255) / 256) * ((s.K_in + 255) / 256);
    const int64_t tiles128 = n * ((rows + 127) / 128) * ((s.K_in + 127) / 128);
    if (tiles256 >= 128) return launch_dgrad_group<256, 256, 2, 4, 2, 1, -1>(s, grp, n, fill, st);
    if (tiles128 > 256) return launch_dgrad_group<128, 128, 2, 2, 2, 2, 4>(s, grp, n, fill, st);
    const int64_t tiles64 = n * ((rows + 63) / 64) * ((s.K_in + 127) / 128);
    if (tiles64 > 256) return launch_dgrad_group<64, 128, 2, 2, 2, 2, 0>(s, grp, n, fill, st);
    return launch_dgrad_group<64, 128, 2, 2, 4, 1, 0>(s, grp, n, fill, st);
}

// expected_rows: how many of the R rows the caller expects to be kept (R if unknown); it only
// steers the tile choice, any count is computed correctly by every variant.
// J: elementwise Jacobian [R, K_in] multiplied into dX, or null.  fill: write the zero rows of
// dropped samples (false: leave them as they are).
// sample_a (null: SampleA has been decided, p / idxA / cntA hold its outcome): the kernel decides
// it itself from the row sums or the sample norms and writes the plan's SampleA fields; N <= 64 only.
vcas_status dgrad_bf16(const vcas_shape &s, const void *G, const void *W, const float *p, const int32_t *idxA,
                       const int32_t *cntA, void *dX, const void *J, bool fill, int64_t expected_rows,
                       const InlineSampleA *sample_a, float *sq_blocks, hipStream_t st)
{
    InlineSampleA sa = {};
    sa.gsq = nullptr;
    if (sample_a) {
        if (s.N > 64) return VCAS_EINVAL;
        sa = *sample_a;
    }
    // The loads into LDS run at about 40 bytes per clock and CU, so the largest tile that still
    // fills the chip wins: 256x256 (one 8-wave workgroup per CU) from 128 tiles up (half the CUs:
    // inside a stack other kernels take the rest; 192 made a step 1-3 % longer); else 128x128
    // (two per CU) while more than 256 of them exist; else 64x128, twice as many workgroups with
    // half the serial work each.  Measured, R=16384, 1024->4096: 123 / 137 / 191 us; R=4096,
    // 768->3072: 68 / 37 / 33 us.  When even the 64x128 tiles leave CUs with a single workgroup,
    // nothing overlaps a tile's own load latency, so the pipeline goes four stages deep instead
    // (2048 kept rows, 768->3072: 22 vs 29 us).
    const int64_t R = (int64_t)s.N * s.T;
    const int64_t rows = expected_rows > 0 && expected_rows < R ? expected_rows : R;
    const int64_t tiles256 = ((rows + 255) / 256) * ((s.K_in + 255) / 256);
    const int64_t tiles128 = ((rows + 127) / 128) * ((s.K_in + 127) / 128);
    // without an expectation (the kept count is known on the device only) the tiles of ALL rows are counted, and a
    // kernel picked for them may find half of them empty: the larger tile then needs more of them to pay
    if (tiles256 >= (expected_rows > 0 ? 128 : 192))
        return launch_dgrad<256, 256, 2, 4, 2, 1, -1>(s, G, W, p, idxA, cntA, dX, J, fill, sa, sq_blocks, st);
    if (tiles128 > 256) return launch_dgrad<128, 128, 2, 2, 2, 2, 4>(s, G, W, p, idxA, cntA, dX, J, fill, sa, sq_blocks, st);
    const int64_t tiles64 = ((rows + 63) / 64) * ((s.K_in + 127) / 128);
    if (tiles64 > 256) return launch_dgrad<64, 128, 2, 2, 2, 2, 0>(s, G, W, p, idxA, cntA, dX, J, fill, sa, sq_blocks, st);
    return launch_dgrad<64, 128, 2, 2, 4, 1, 0>(s, G, W, p, idxA, cntA, dX, J, fill, sa, sq_blocks, st);
}

}  // namespace vcas
