// bf16 MFMA gather-GEMMs of the VCAS backward pass (gfx950):
//   dgrad  dX[rows of kept samples] = (1/p_i) * G[row,:] W          (Eq. 2, upper line)
//   wgrad  dW = sum over kept tokens t of scale_t * g_t x_t^T        (Sec. 4.2)
// Both are dense contractions over the kept rows only, so they run on the
// matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
// Tiling: a workgroup of WM x WN wavefronts owns a BM x BN output tile and
// walks the contraction in steps of 64, operand tiles double (or deeper)
// buffered in LDS.  An MFMA lane needs 8 consecutive contraction values of one
// row/column, but W (for dgrad) and both G and X (for wgrad) are stored with
// the contraction index as the slow dimension.  Two ways of getting them there:
//
//  * LDS-direct (dgrad, and the 128x128 wgrad): buffer loads write straight
//    into LDS; an operand that lies "the wrong way" stays as it is in memory,
//    [64 k][columns], and ds_read_b64_tr_b16 transposes it on the way out.
//  * register-staged (the 64x64 wgrad for small dW): 4 rows x 8 columns per
//    thread with coalesced 16-byte loads, transposed in registers (v_perm_b32)
//    and written as 8-byte pieces to a [column][64 k] tile whose 16-byte slots
//    are XOR-swizzled so that fragment reads and transposing writes spread
//    over all banks.
//
// wgrad multiplies G by the per-token scale before it reaches LDS (the scale
// lies on the contraction axis and cannot go into the epilogue); dgrad's
// per-row 1/p goes into the epilogue.
#include <type_traits>

#include "groups.hpp"

namespace vcas {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2v;
typedef __attribute__((ext_vector_type(2))) float f32x2v;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BK = 64;  // contraction elements per step (one 128-byte LDS row)

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 7); }
// byte offset of 16-byte slot `slot` (0..7) of tile row `row`
__device__ __forceinline__ int lds_off(int row, int slot) { return row * 128 + ((slot ^ swz(row)) << 4); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2v v = {lo, hi};
    bf16x2v r = __builtin_convertvector(v, bf16x2v);
    return *reinterpret_cast<uint32_t *>(&r);
}

// ---------------------------------------------------------------- loaders
//
// All global reads are raw buffer loads: a 128-bit resource descriptor in
// SGPRs (base, size), a per-thread byte offset in one VGPR that does not change
// over the contraction loop, and the loop's advance in an SGPR.  Reads past the
// end of the tensor return zero, so a masked-out row is just an offset beyond
// the end (kOutside) and ragged tails need no branches or address arithmetic.

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr uint32_t kOutside = 0x80000000u;   // tensors are < 2 GiB (checked on the host)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voffset, uint32_t soffset)
{
    // soffset is wave-uniform by construction; say so, or the compiler loops over its values
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voffset, __builtin_amdgcn_readfirstlane((int)soffset), 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Operand stored [k][col] (col contiguous).  64 x COLS tile; unit u = 4 k-rows
// x 8 columns.
template <int COLS, int NT>
struct TransLoader {
    static constexpr int CH = COLS / 8;
    static constexpr int PER = 16 * CH / NT;
    static_assert(16 * CH % NT == 0 && PER >= 1, "tile/thread mismatch");
    typedef uint4 Regs[PER][4];

    // Neighbouring lanes take the two k-quads that share a 16-byte LDS slot, so that their 8-byte
    // writes fill whole slots and 16 lanes cover 8 distinct slots (no bank conflicts).
    __device__ __forceinline__ static int chunk(int j) { return ((threadIdx.x + j * NT) >> 1) % CH; }
    __device__ __forceinline__ static int kquad(int j)
    {
        const int u = threadIdx.x + j * NT;
        return ((u >> 1) / CH) * 2 + (u & 1);
    }

    // voff(j, i) -> byte offset of the 8 columns of k-row kquad(j)*4+i (or kOutside)
    template <typename Off>
    __device__ __forceinline__ static void load(Regs &regs, __amdgpu_buffer_rsrc_t rsrc, Off voff, uint32_t soffset)
    {
#pragma unroll
        for (int j = 0; j < PER; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) regs[j][i] = buffer_load16(rsrc, voff(j, i), soffset);
    }

    __device__ __forceinline__ static void put(unsigned char *tile, int j, int c, uint32_t d0, uint32_t d1)
    {
        const int row = chunk(j) * 8 + c;
        const int kq = kquad(j);
        *reinterpret_cast<uint2 *>(tile + lds_off(row, kq >> 1) + (kq & 1) * 8) = make_uint2(d0, d1);
    }

    // plain transpose
    __device__ __forceinline__ static void store(const Regs &regs, unsigned char *tile)
    {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const uint32_t *r0 = reinterpret_cast<const uint32_t *>(&regs[j][0]);
            const uint32_t *r1 = reinterpret_cast<const uint32_t *>(&regs[j][1]);
            const uint32_t *r2 = reinterpret_cast<const uint32_t *>(&regs[j][2]);
            const uint32_t *r3 = reinterpret_cast<const uint32_t *>(&regs[j][3]);
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                // even column: low halves; odd column: high halves
                put(tile, j, 2 * d, __builtin_amdgcn_perm(r1[d], r0[d], 0x05040100u),
                    __builtin_amdgcn_perm(r3[d], r2[d], 0x05040100u));
                put(tile, j, 2 * d + 1, __builtin_amdgcn_perm(r1[d], r0[d], 0x07060302u),
                    __builtin_amdgcn_perm(r3[d], r2[d], 0x07060302u));
            }
        }
    }

    // transpose with k-row i multiplied by s[i] (fp32 multiply, one bf16 rounding); PER == 1
    __device__ __forceinline__ static void store_scaled(const Regs &regs, unsigned char *tile, const float (&s)[4])
    {
        static_assert(PER == 1, "scaled store handles one unit per thread");
        const uint32_t *r0 = reinterpret_cast<const uint32_t *>(&regs[0][0]);
        const uint32_t *r1 = reinterpret_cast<const uint32_t *>(&regs[0][1]);
        const uint32_t *r2 = reinterpret_cast<const uint32_t *>(&regs[0][2]);
        const uint32_t *r3 = reinterpret_cast<const uint32_t *>(&regs[0][3]);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            put(tile, 0, 2 * d, pack_bf16(bf16_lo(r0[d]) * s[0], bf16_lo(r1[d]) * s[1]),
                pack_bf16(bf16_lo(r2[d]) * s[2], bf16_lo(r3[d]) * s[3]));
            put(tile, 0, 2 * d + 1, pack_bf16(bf16_hi(r0[d]) * s[0], bf16_hi(r1[d]) * s[1]),
                pack_bf16(bf16_hi(r2[d]) * s[2], bf16_hi(r3[d]) * s[3]));
        }
    }
};

// ------------------------------------------------------------ MFMA core

template <int TM, int TN>
__device__ __forceinline__ void mma_tile(const unsigned char *tileA, const unsigned char *tileB, int rowA0,
                                         int rowB0, f32x16 (&acc)[TM][TN])
{
    const int lane = threadIdx.x & 63;
    const int r = lane & 31, h = lane >> 5;
    constexpr int KS = BK / 16;
    // all fragment reads of the step are issued before the first MFMA, so only the first one's
    // LDS latency is exposed
    bf16x8 a[KS][TM], b[KS][TN];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            a[ks][i] = *reinterpret_cast<const bf16x8 *>(tileA + lds_off(rowA0 + i * 32 + r, ks * 2 + h));
#pragma unroll
        for (int i = 0; i < TN; ++i)
            b[ks][i] = *reinterpret_cast<const bf16x8 *>(tileB + lds_off(rowB0 + i * 32 + r, ks * 2 + h));
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][i], b[ks][j], acc[i][j], 0, 0, 0);
}

// The instruction mix of one pipeline phase, spelled out for the scheduler (it
// would otherwise sink every LDS read next to its MFMA and run global loads,
// matrix work and LDS staging one after the other): global loads first, the
// fragment reads of two k-slices, then each MFMA followed by one instruction of
// the staging work (transposing VALU op or LDS write), with the fragment reads
// of the slice after next in each slice's shadow.  Counts that exceed what the
// region holds are harmless.
template <int TM, int TN, int VMEM, int VALU, int DSW, int ID>
__device__ __forceinline__ void schedule_phase()
{
    constexpr int KS = BK / 16, RD = TM + TN, MM = TM * TN, TOTAL = KS * MM;
    constexpr int VALU_PER = (VALU + TOTAL - 1) / TOTAL, DSW_PER = (DSW + TOTAL - 1) / TOTAL;
    __builtin_amdgcn_sched_group_barrier(0x020, VMEM, ID);
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * RD, ID);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int m = 0; m < MM; ++m) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, ID);
            if (VALU_PER > 0) __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, ID);
            if (DSW_PER > 0) __builtin_amdgcn_sched_group_barrier(0x200, DSW_PER, ID);
        }
        if (ks + 2 < KS) __builtin_amdgcn_sched_group_barrier(0x100, RD, ID);
    }
}

// Row of the 32x32 accumulator block that register v of this lane holds;
// the column is lane % 32.
__device__ __forceinline__ int acc_row(int v) { return (v >> 2) * 8 + ((threadIdx.x & 63) >> 5) * 4 + (v & 3); }

// XCD-aware tile order: consecutive workgroup ids land on different XCDs
// (id mod 8), so hand each XCD one contiguous run of tiles; neighbours in the
// run share operand rows through that XCD's L2.
__device__ __forceinline__ int xcd_remap(int id, int total)
{
    const int per = (total + 7) / 8;
    return (id & 7) * per + (id >> 3);
}

// The same with the panel width chosen at run time.
__device__ __forceinline__ void panel_order_rt(int tile, int tiles_m, int tiles_n, int panel_w, int &tile_m,
                                               int &tile_n)
{
    const int panel = tile / (tiles_m * panel_w);
    const int in_panel = tile - panel * tiles_m * panel_w;
    const int width = min(panel_w, tiles_n - panel * panel_w);
    tile_m = in_panel / width;
    tile_n = panel * panel_w + in_panel % width;
}

// Tile number -> (row tile, column tile), column panels of PANEL tiles, row-major inside a panel.
template <int PANEL>
__device__ __forceinline__ void panel_order(int tile, int tiles_m, int tiles_n, int &tile_m, int &tile_n)
{
    const int panel = tile / (tiles_m * PANEL);
    const int in_panel = tile - panel * tiles_m * PANEL;
    const int width = min(PANEL, tiles_n - panel * PANEL);
    tile_m = in_panel / width;
    tile_n = panel * PANEL + in_panel % width;
}

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

// ------------------------------------------------- register-staged pipeline

// Software pipeline of the weight-gradient kernel.  Two register sets and two LDS
// buffers: while step s is on the matrix cores, the loads of step s+1 are
// landing in one register set and the loads of step s+2 are being issued into
// the other, so a global load has about one and a half steps to arrive.
//   load(set, s)   issue the global loads of step s into register set `set`
//   stage(set, b)  write register set `set` (transposed / scaled) to LDS buffer b
//   compute(b)     MFMA over LDS buffer b
template <typename Load, typename Stage, typename Compute, typename Schedule>
__device__ __forceinline__ void pipeline(int steps, Load load, Stage stage, Compute compute, Schedule schedule)
{
    if (steps <= 0) return;
    load(0, 0);
    if (steps > 1) load(1, 1);
    stage(0, 0);
    __syncthreads();
    // Steady state without conditions inside: LDS buffer 0 holds step s, register set 1 holds
    // step s+1 (landed or about to).  One phase = issue the loads of step s+2 into the free
    // set, run the MFMAs of step s and, interleaved with them, move step s+1 from its register
    // set into the other LDS buffer.
    int s = 0;
    for (; s + 3 < steps; s += 2) {
        load(0, s + 2);
        compute(0);
        stage(1, 1);
        schedule(std::integral_constant<int, 0>());
        __builtin_amdgcn_sched_barrier(0);   // nothing moves across the phase boundary
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
        load(1, s + 3);
        compute(1);
        stage(0, 0);
        schedule(std::integral_constant<int, 1>());
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
    }
    const int left = steps - s;   // 1, 2 or 3
    if (left == 3) load(0, s + 2);
    compute(0);
    if (left >= 2) {
        stage(1, 1);
        __syncthreads();
        compute(1);
        if (left == 3) {
            stage(0, 0);
            __syncthreads();
            compute(0);
        }
    }
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
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

// slot XOR of W-tile row k: the four k rows that a half-wave transposes at once land in four
// different 64-byte bank groups
__device__ __forceinline__ int wswz(int k) { return (k & 3) * 4; }

// 128-bit buffer descriptor built by hand (base, stride 0, size in bytes, raw dword format) for
// use in inline assembly.
__device__ __forceinline__ i32x4 raw_descriptor(const void *base, uint32_t bytes)
{
    const uint64_t b = reinterpret_cast<uint64_t>(base);
    i32x4 d;
    d[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    d[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((b >> 32) & 0xffffu));
    d[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    d[3] = 0x00020000;
    return d;
}

// One LDS-direct load: every lane fetches 16 bytes at buffer offset voffset + soffset, the
// wavefront's 1 KiB lands at LDS byte address lds_base (wave-uniform) in lane order.  Written as
// assembly so that the compiler does not track it: it would otherwise make every later LDS read
// wait for ALL loads in flight (it cannot tell the stages apart), and the waits are placed by
// hand before the barrier anyway.
__device__ __forceinline__ void lds_direct_load16(i32x4 desc, uint32_t lds_base, uint32_t voffset, uint32_t soffset)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(desc), "s"(soffset)
                 : "memory", "m0");
}

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
// SPQ: the loads of the next step are spread over the MFMAs of the first SPQ
// quarters of the current one (0: all issued right after the barrier).
template <int BM, int BN, int WM, int WN, int NS, int SPQ>
__device__ __forceinline__ void dgrad_bf16_body(const uint16_t *__restrict__ G, const uint16_t *__restrict__ W,
                                                const float *__restrict__ p, const int32_t *__restrict__ idxA,
                                                const int32_t *__restrict__ cntA, uint16_t *__restrict__ dX, int N,
                                                int T, int K_in, int K_out, int tiles_n,
                                                const uint16_t *__restrict__ J, int fill_dropped,
                                                const InlineSampleA &sa)
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
    if (sa.gsq != nullptr) {
        // SampleA decided here, by every workgroup for itself (N <= 64: a few microseconds of one
        // wavefront's work on 4 N T bytes that sit in L2), instead of by a launch of its own in
        // front of this one; the first workgroup writes the plan's fields for everybody else.
        const int lane_ = threadIdx.x & 63, wave_ = threadIdx.x >> 6;
        const uint32_t draw = sa.draw + (sa.draw_offset ? *sa.draw_offset : 0u);   // fetched beside the norms
        if (T <= 128) sample_norms_batched<8, 2>(sa.gsq, wave_, NW, N, T, sa_norm);
        else sample_norms_batched<4, 8>(sa.gsq, wave_, NW, N, T, sa_norm);
        __syncthreads();
        if (wave_ == 0) {
            const float a = lane_ < N ? sa_norm[lane_] : 0.0f;
            const SampleADecision d = sample_a_wave(a, N, sa.budget, sa.seed, sa.layer, draw);
            if (lane_ < N) sa_p[lane_] = d.pr;
            if (d.keep) idx_staged[d.below] = lane_;
            if (lane_ == 0) sa_count = d.count;
            if (blockIdx.x == 0) {
                if (lane_ < N) {
                    sa.gnorm[lane_] = a;
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
    constexpr int KS = BK / 16, MM = TM * TN, SPAN = KS * MM * SPQ / 4;
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
    wait_loads_outstanding<0>();

    // Each MFMA lane holds one column of 16 rows; neighbouring lanes swap every second value so
    // that a lane owns two adjacent columns of one row and stores them as one dword.
    const bool odd = lane & 1;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
            const int r_even = wm0 + i * 32 + acc_row(v);
            const int r = r_even + (odd ? 1 : 0);
            const int32_t dst = row_of[r];
            const float sc_e = scale_of[r_even], sc_o = scale_of[r_even + 1];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const float mine_e = acc[i][j][v] * sc_e, mine_o = acc[i][j][v + 1] * sc_o;
                const float send = odd ? mine_e : mine_o;
                const float recv = dpp_move<0xB1>(send);
                float lo = odd ? recv : mine_e, hi = odd ? mine_o : recv;
                const int col = n0 + wn0 + j * 32 + (lane & 30);
                if (dst >= 0 && col < K_in) {
                    if (J) {   // elementwise Jacobian of the layer below (App. E, proof of unbiasedness), same layout as dX
                        const uint32_t jw = *reinterpret_cast<const uint32_t *>(J + (int64_t)dst * K_in + col);
                        lo = lo * bf16_lo(jw);
                        hi = hi * bf16_hi(jw);
                    }
                    *reinterpret_cast<uint32_t *>(dX + (int64_t)dst * K_in + col) = pack_bf16(lo, hi);
                }
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
                                                                  InlineSampleA sa)
{
    dgrad_bf16_body<BM, BN, WM, WN, NS, SPQ>(G, W, p, idxA, cntA, dX, N, T, K_in, K_out, tiles_n, J, fill_dropped, sa);
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
                                             fill_dropped, q.sa);
}

// ------------------------------------------------------------------ wgrad

// How many of the launched split-K slices do work for a given number of
// contraction steps, and how many steps each takes.  Used by the GEMM and by
// the reduction so that both agree.
__host__ __device__ inline int wgrad_active_splits(int steps_all, int splits, int min_steps, int &per)
{
    int active = splits < steps_all / min_steps ? splits : steps_all / min_steps;
    if (active < 1) active = 1;
    per = (steps_all + active - 1) / active;
    if (per < 1) per = 1;
    active = (steps_all + per - 1) / per;
    return active < 1 ? 1 : active;
}

// dW = partial[0] + partial[1] + ... in that order; does nothing when only one
// split was active (the GEMM wrote dW itself).  `step` is the GEMM's
// contraction step in tokens.
__device__ __forceinline__ void splitk_reduce_body(const float *__restrict__ partials,
                                                   const int32_t *__restrict__ cntW, float *__restrict__ dW,
                                                   int64_t R, int64_t elems, int splits, int min_steps, int step)
{
    const int64_t cnt = min((int64_t)max(*cntW, 0), R);
    int per;
    const int active = wgrad_active_splits((int)((cnt + step - 1) / step), splits, min_steps, per);
    if (active == 1) return;
    for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4; i < elems; i += (int64_t)gridDim.x * 1024) {
        float4 t[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            t[s] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (s < active) t[s] = *reinterpret_cast<const float4 *>(partials + s * elems + i);
        }
        float4 sum = t[0];
#pragma unroll
        for (int s = 1; s < 8; ++s) {
            sum.x += t[s].x;
            sum.y += t[s].y;
            sum.z += t[s].z;
            sum.w += t[s].w;
        }
        *reinterpret_cast<float4 *>(dW + i) = sum;
    }
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partials,
                                                            const int32_t *__restrict__ cntW, float *__restrict__ dW,
                                                            int64_t R, int64_t elems, int splits, int min_steps,
                                                            int step)
{
    splitk_reduce_body(partials, cntW, dW, R, elems, splits, min_steps, step);
}

// the same for several layers of one shape: blockIdx.y picks the layer
__global__ __launch_bounds__(256) void splitk_reduce_group_kernel(WgradGroup grp, int64_t R, int64_t elems, int splits,
                                                                  int min_steps, int step)
{
    const WgradProblem &q = grp.prob[blockIdx.y];
    splitk_reduce_body(q.partials, q.cntW, q.dW, R, elems, splits, min_steps, step);
}

static vcas_status splitk_reduce_group(const WgradGroup &grp, int n, int64_t R, int64_t elems, int splits,
                                       int min_steps, int step, hipStream_t st)
{
    if (splits <= 1) return VCAS_OK;
    int64_t blocks = (elems / 4 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(splitk_reduce_group_kernel, dim3((unsigned)blocks, (unsigned)n), dim3(256), 0, st, grp, R, elems,
                       splits, min_steps, step);
    return launch_status();
}

vcas_status splitk_reduce(const float *partials, const int32_t *cntW, float *dW, int64_t R, int64_t elems, int splits,
                          int min_steps, int step, hipStream_t st)
{
    if (splits <= 1) return VCAS_OK;
    int64_t blocks = (elems / 4 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, st, partials, cntW, dW, R, elems,
                       splits, min_steps, step);
    return launch_status();
}

// grid: 1-D, splits * tiles workgroups (rounded up to a multiple of 8), split-
// major, so that the workgroups one XCD gets (a contiguous run after the remap)
// contract the same tokens and share those G and X rows in its L2.  Split s of
// a tile contracts a contiguous run of 64-token steps.  The number of active
// splits is derived from the device-side count (wgrad_active_splits).  With one
// active split the tile goes straight to dW; otherwise the partial tiles go to
// `partials` [split][K_out][K_in] and splitk_reduce_kernel adds them in split
// order, so the sum order is fixed.  (An in-kernel "last workgroup reduces"
// scheme was measured first: its device-scope fences write back the XCD's L2
// and cost more than the second launch.)
template <int BM, int BN, int WM, int WN>
__device__ __forceinline__ void wgrad_bf16_body(const uint16_t *__restrict__ G, const uint16_t *__restrict__ X,
                                                const float *__restrict__ row_scale,
                                                const int32_t *__restrict__ idxW, const int32_t *__restrict__ cntW,
                                                float *__restrict__ dW, float *__restrict__ partials, int64_t R,
                                                int K_in, int K_out, int tiles_n, int tiles, int splits,
                                                int min_steps)
{
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    auto tA = [&](int buf) { return smem + buf * (BM * 128); };
    auto tB = [&](int buf) { return smem + 2 * BM * 128 + buf * (BN * 128); };
    const int total = tiles * splits;
    const int id = xcd_remap(blockIdx.x, total);
    if (id >= total) return;
    const int split = id / tiles, tile = id % tiles;
    int tile_o, tile_c;   // panels of 4 column tiles: an XCD's ~32-64 workgroups cover a squarish patch of dW
    panel_order<4>(tile, tiles / tiles_n, tiles_n, tile_o, tile_c);
    const int o0 = tile_o * BM, c0 = tile_c * BN;

    const int64_t cnt = min((int64_t)max(*cntW, 0), R);
    const int steps_all = (int)((cnt + BK - 1) / BK);
    int per;
    const int active = wgrad_active_splits(steps_all, splits, min_steps, per);
    if (split >= active) return;
    const int s_begin = split * per, s_end = min(steps_all, s_begin + per);

    typedef TransLoader<BM, NT> LA;
    typedef TransLoader<BN, NT> LB;
    static_assert(LA::PER == 1 && LB::PER == 1 && BM == BN, "one unit per thread, square tile assumed");
    const int kq = LA::kquad(0);
    const int cola = o0 + LA::chunk(0) * 8, colb = c0 + LB::chunk(0) * 8;
    const __amdgpu_buffer_rsrc_t rsrcG = make_rsrc(G, (uint32_t)(R * K_out * 2));
    const __amdgpu_buffer_rsrc_t rsrcX = make_rsrc(X, (uint32_t)(R * K_in * 2));
    typename LA::Regs ra[2];
    typename LB::Regs rb[2];
    float scale_of_set[2][4];   // per-token scales of the step held in the register set of the same index

    // Token indices and scales run two resp. one step ahead of the tile loads, and each small
    // load is issued BEFORE the 16 tile loads of its phase: the memory counter is in-order, so
    // waiting for an index then leaves the younger tile loads in flight.
    const __amdgpu_buffer_rsrc_t rsrcI = make_rsrc(idxW, (uint32_t)(R * 4));
    const __amdgpu_buffer_rsrc_t rsrcS = make_rsrc(row_scale, (uint32_t)(R * 4));
    const int64_t k_end = min(cnt, (int64_t)s_end * BK);
    struct Tokens {
        int32_t tok[4];   // row of G / X, or -1
    };
    // this thread's column chunk lies inside G resp. X (only ragged edge tiles have chunks outside)
    const bool a_inside = cola < K_out, b_inside = colb < K_in;
    const uint32_t g_pitch = (uint32_t)K_out * 2u, x_pitch = (uint32_t)K_in * 2u;   // row bytes, < 2^15
    auto fetch_tokens = [&](int step) {
        const int64_t k0 = (int64_t)(s_begin + step) * BK + kq * 4;
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrcI, k0 < k_end ? (int)(k0 * 4) : (int)kOutside, 0, 0);
        Tokens t;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int32_t r = (int32_t)v[i];
            t.tok[i] = (k0 + i < k_end && (uint32_t)r < (uint32_t)R) ? r : -1;
        }
        return t;
    };
    auto fetch_scales = [&](const Tokens &t, float (&sc)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            sc[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                  rsrcS, t.tok[i] >= 0 ? t.tok[i] * 4 : (int)kOutside, 0, 0));
    };

    const int wave = threadIdx.x >> 6;
    const int wm0 = (wave / WN) * (BM / WM), wn0 = (wave % WN) * (BN / WN);
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    Tokens tok_cur = fetch_tokens(0), tok_next = fetch_tokens(1);
    float sc_cur[4];
    fetch_scales(tok_cur, sc_cur);
    auto load = [&](int set, int s) {
        // steps are loaded in order: tok_cur / sc_cur belong to step s, tok_next to step s + 1
        float sc_next[4];
        fetch_scales(tok_next, sc_next);
        const Tokens tok_after = fetch_tokens(s + 2);
        const Tokens q = tok_cur;
        // rows < 2^24 and row bytes < 2^15 (checked on the host): 24-bit multiplies are exact and full rate
        auto g_voff = [&](int, int i) {
            return (q.tok[i] >= 0 && a_inside) ? __umul24((uint32_t)q.tok[i], g_pitch) + (uint32_t)cola * 2u : kOutside;
        };
        auto x_voff = [&](int, int i) {
            return (q.tok[i] >= 0 && b_inside) ? __umul24((uint32_t)q.tok[i], x_pitch) + (uint32_t)colb * 2u : kOutside;
        };
        if (set == 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) scale_of_set[0][i] = sc_cur[i];
            LA::load(ra[0], rsrcG, g_voff, 0u);
            LB::load(rb[0], rsrcX, x_voff, 0u);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) scale_of_set[1][i] = sc_cur[i];
            LA::load(ra[1], rsrcG, g_voff, 0u);
            LB::load(rb[1], rsrcX, x_voff, 0u);
        }
        tok_cur = tok_next;
        tok_next = tok_after;
#pragma unroll
        for (int i = 0; i < 4; ++i) sc_cur[i] = sc_next[i];
    };
    auto stage = [&](int set, int buf) {
        if (set == 0) {
            LA::store_scaled(ra[0], tA(buf), scale_of_set[0]);
            LB::store(rb[0], tB(buf));
        } else {
            LA::store_scaled(ra[1], tA(buf), scale_of_set[1]);
            LB::store(rb[1], tB(buf));
        }
    };
    auto compute_step = [&](int buf) { mma_tile<TM, TN>(tA(buf), tB(buf), wm0, wn0, acc); };
    // staging VALU per thread: G unit 40 (unpack, scale, pack), X unit 16 (byte permutes), a few for the token fetch
    auto schedule = [&](auto id) { schedule_phase<TM, TN, 8 + 5, 64, 16, decltype(id)::value>(); };
    pipeline(s_end - s_begin, load, stage, compute_step, schedule);

    const int lane = threadIdx.x & 63;
    float *dst = active == 1 ? dW : partials + (int64_t)split * K_out * K_in;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int o = o0 + wm0 + i * 32 + acc_row(v);
            if (o >= K_out) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int c = c0 + wn0 + j * 32 + (lane & 31);
                if (c < K_in) dst[(int64_t)o * K_in + c] = acc[i][j][v];
            }
        }
}

template <int BM, int BN, int WM, int WN, int OCC>
__global__ __launch_bounds__(WM *WN * 64, OCC) void wgrad_bf16_kernel(const uint16_t *__restrict__ G,
                                                                  const uint16_t *__restrict__ X,
                                                                  const float *__restrict__ row_scale,
                                                                  const int32_t *__restrict__ idxW,
                                                                  const int32_t *__restrict__ cntW, float *__restrict__ dW,
                                                                  float *__restrict__ partials, int64_t R, int K_in,
                                                                  int K_out, int tiles_n, int tiles, int splits,
                                                                  int min_steps)
{
    wgrad_bf16_body<BM, BN, WM, WN>(G, X, row_scale, idxW, cntW, dW, partials, R, K_in, K_out, tiles_n, tiles, splits,
                                    min_steps);
}

// Several layers of one shape (siblings) in one launch: blockIdx.y picks the layer.
template <int BM, int BN, int WM, int WN, int OCC>
__global__ __launch_bounds__(WM *WN * 64, OCC) void wgrad_bf16_group_kernel(WgradGroup grp, int64_t R, int K_in,
                                                                        int K_out, int tiles_n, int tiles,
                                                                        int splits, int min_steps)
{
    const WgradProblem &q = grp.prob[blockIdx.y];
    wgrad_bf16_body<BM, BN, WM, WN>(q.G, q.X, q.row_scale, q.idxW, q.cntW, q.dW, q.partials, R, K_in, K_out, tiles_n,
                                    tiles, splits, min_steps);
}

// The 128x128 weight-gradient kernel for layers with many kept tokens.  Same split-K protocol
// and epilogue as above, different data path: X goes straight into LDS (LDS-direct loads, as in
// dgrad), G passes through registers only to be multiplied by the per-token scale and is written
// as it came, 16 bytes per lane; both tiles lie in LDS as [64 tokens][128 columns] with the
// 16-byte slots swizzled by wswz, and both MFMA operands are transposed on the way out by
// ds_read_b64_tr_b16.  No v_perm transposes, half the staging registers.  A thread handles four
// consecutive kept tokens (one 16-byte index load); they occupy LDS rows 4 apart, which is fine
// because both tiles use the same row order and the contraction does not care about it.
template <int BM, int BN, int WM, int WN>
__device__ __forceinline__ void wgrad_bf16_dma_body(
    const uint16_t *__restrict__ G, const uint16_t *__restrict__ X, const float *__restrict__ row_scale,
    const int32_t *__restrict__ idxW, const int32_t *__restrict__ cntW, float *__restrict__ dW,
    float *__restrict__ partials, int64_t R, int K_in, int K_out, int tiles_n, int tiles, int splits, int min_steps)
{
    static_assert(BM == 128 && BN == 128 && WM * WN == 4, "four wavefronts, 16 slots per tile row");
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int A_TILE = BK * BM * 2, STAGE = A_TILE + BK * BN * 2, PITCH = 256;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int total = tiles * splits;
    const int id = xcd_remap(blockIdx.x, total);
    if (id >= total) return;
    const int split = id / tiles, tile = id % tiles;
    int tile_o, tile_c;
    panel_order<4>(tile, tiles / tiles_n, tiles_n, tile_o, tile_c);
    const int o0 = tile_o * BM, c0 = tile_c * BN;

    const int64_t cnt = min((int64_t)max(*cntW, 0), R);
    const int steps_all = (int)((cnt + BK - 1) / BK);
    int per;
    const int active = wgrad_active_splits(steps_all, splits, min_steps, per);
    if (split >= active) return;
    const int s_begin = split * per, s_end = min(steps_all, s_begin + per);
    const int steps = s_end - s_begin;
    const int64_t k_end = min(cnt, (int64_t)s_end * BK);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, slot = lane & 15;        // row within a 4-row load, 16-byte slot
    const int k_first = 16 * wave + 4 * grp;            // this thread's tokens of a step: k_first + j, j < 4
    // token k_first + j lives in LDS row 16*wave + 4*j + grp
    const __amdgpu_buffer_rsrc_t rsrcG = make_rsrc(G, (uint32_t)(R * K_out * 2));
    const __amdgpu_buffer_rsrc_t rsrcI = make_rsrc(idxW, (uint32_t)(R * 4));
    const __amdgpu_buffer_rsrc_t rsrcS = make_rsrc(row_scale, (uint32_t)(R * 4));
    const i32x4 descX = raw_descriptor(X, (uint32_t)(R * K_in * 2));
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const uint32_t g_pitch = (uint32_t)K_out * 2u, x_pitch = (uint32_t)K_in * 2u;
    const int g_col = o0 + slot * 8;
    const bool g_inside = g_col < K_out;
    // column piece of X that lands in LDS slot `slot` of row r: slot ^ wswz(r); r & 3 == grp for all four rows
    const int x_col = c0 + ((slot ^ wswz(grp)) * 8);
    const bool x_inside = x_col < K_in;

    struct Tokens {
        int32_t tok[4];
    };
    auto fetch_tokens = [&](int step) {
        const int64_t k0 = (int64_t)(s_begin + step) * BK + k_first;
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrcI, k0 < k_end ? (int)(k0 * 4) : (int)kOutside, 0, 0);
        Tokens t;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int32_t r = (int32_t)v[j];
            t.tok[j] = (k0 + j < k_end && (uint32_t)r < (uint32_t)R) ? r : -1;
        }
        return t;
    };
    auto fetch_scales = [&](const Tokens &t, float (&sc)[4]) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            sc[j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                  rsrcS, t.tok[j] >= 0 ? t.tok[j] * 4 : (int)kOutside, 0, 0));
    };
    uint4 g_regs[4];
    auto load_g = [&](const Tokens &t) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            g_regs[j] = buffer_load16(rsrcG, (t.tok[j] >= 0 && g_inside)
                                                 ? __umul24((uint32_t)t.tok[j], g_pitch) + (uint32_t)g_col * 2u
                                                 : kOutside, 0u);
    };
    auto issue_x = [&](int stage, const Tokens &t) {
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds0 + stage * STAGE + A_TILE + wave * 16 * PITCH);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            lds_direct_load16(descX, dst + j * 4 * PITCH,
                              (t.tok[j] >= 0 && x_inside) ? __umul24((uint32_t)t.tok[j], x_pitch) + (uint32_t)x_col * 2u
                                                          : kOutside, 0u);
    };
    auto stage_g = [&](int stage, const float (&sc)[4]) {
        unsigned char *tileA = smem + stage * STAGE;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = 16 * wave + 4 * j + grp;
            const uint32_t *r = reinterpret_cast<const uint32_t *>(&g_regs[j]);
            uint4 o;
            o.x = pack_bf16(bf16_lo(r[0]) * sc[j], bf16_hi(r[0]) * sc[j]);
            o.y = pack_bf16(bf16_lo(r[1]) * sc[j], bf16_hi(r[1]) * sc[j]);
            o.z = pack_bf16(bf16_lo(r[2]) * sc[j], bf16_hi(r[2]) * sc[j]);
            o.w = pack_bf16(bf16_lo(r[3]) * sc[j], bf16_hi(r[3]) * sc[j]);
            *reinterpret_cast<uint4 *>(tileA + row * PITCH + ((slot ^ wswz(row)) << 4)) = o;
        }
    };

    const int wm0 = (wave / WN) * (BM / WM), wn0 = (wave % WN) * (BN / WN);
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    const int blk = lane >> 4, sl = lane & 15;
    // fragment of 32 columns x 16 tokens of a [64][128] tile: two transposing reads
    auto frag = [&](const unsigned char *t, int col0, int ks) {
        bf16x4 half[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int k = ks * 16 + (blk >> 1) * 8 + e * 4 + (sl >> 2);
            const int col = col0 + (blk & 1) * 16 + (sl & 3) * 4;
            const unsigned char *src = t + k * PITCH + (((col >> 3) ^ wswz(k)) << 4) + (col & 7) * 2;
            half[e] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4 *)(src));
        }
        return __builtin_shufflevector(half[0], half[1], 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto compute = [&](int stage) {
        const unsigned char *tileA = smem + stage * STAGE;
        const unsigned char *tileB = tileA + A_TILE;
        constexpr int KS = BK / 16;
        bf16x8 a[KS][TM], b[KS][TN];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int i = 0; i < TM; ++i) a[ks][i] = frag(tileA, wm0 + i * 32, ks);
#pragma unroll
            for (int i = 0; i < TN; ++i) b[ks][i] = frag(tileB, wn0 + i * 32, ks);
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks][i], b[ks][j], acc[i][j], 0, 0, 0);
        // fragment reads of two k-slices, then each slice's MFMAs with the reads of the slice after next
        constexpr int RD = 2 * (TM + TN), MM = TM * TN;
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * RD, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            __builtin_amdgcn_sched_group_barrier(0x008, MM, 0);
            if (ks + 2 < KS) __builtin_amdgcn_sched_group_barrier(0x100, RD, 0);
        }
    };

    // prologue: step 0 into stage 0, tokens of step 1 known
    Tokens tok_cur = fetch_tokens(0), tok_next = fetch_tokens(1);
    float sc_cur[4];
    fetch_scales(tok_cur, sc_cur);
    load_g(tok_cur);
    issue_x(0, tok_cur);
    stage_g(0, sc_cur);
    for (int s = 0; s < steps; ++s) {
        wait_loads_outstanding<0>();          // this wavefront's part of X(s) has landed
        asm volatile("" ::: "memory");
        __syncthreads();                       // tile s complete; tile s-1 no longer read
        __builtin_amdgcn_sched_barrier(0);
        // step s+1 on its way while step s is on the matrix cores (past the end: zeros); the
        // scaled G(s+1) goes to LDS once the MFMAs of the step are issued
        const Tokens tok_after = fetch_tokens(s + 2);
        float sc_next[4];
        fetch_scales(tok_next, sc_next);
        load_g(tok_next);
        issue_x((s + 1) & 1, tok_next);
        __builtin_amdgcn_sched_barrier(0);
        compute(s & 1);
        __builtin_amdgcn_sched_barrier(0);
        stage_g((s + 1) & 1, sc_next);
        tok_next = tok_after;
    }
    wait_loads_outstanding<0>();

    const int lane32 = lane & 31;
    float *dst = active == 1 ? dW : partials + (int64_t)split * K_out * K_in;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int o = o0 + wm0 + i * 32 + acc_row(v);
            if (o >= K_out) continue;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int c = c0 + wn0 + j * 32 + lane32;
                if (c < K_in) dst[(int64_t)o * K_in + c] = acc[i][j][v];
            }
        }
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64, 2) void wgrad_bf16_dma_kernel(
    const uint16_t *__restrict__ G, const uint16_t *__restrict__ X, const float *__restrict__ row_scale,
    const int32_t *__restrict__ idxW, const int32_t *__restrict__ cntW, float *__restrict__ dW,
    float *__restrict__ partials, int64_t R, int K_in, int K_out, int tiles_n, int tiles, int splits, int min_steps)
{
    wgrad_bf16_dma_body<BM, BN, WM, WN>(G, X, row_scale, idxW, cntW, dW, partials, R, K_in, K_out, tiles_n, tiles,
                                        splits, min_steps);
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64, 2) void wgrad_bf16_dma_group_kernel(WgradGroup grp, int64_t R, int K_in,
                                                                          int K_out, int tiles_n, int tiles,
                                                                          int splits, int min_steps)
{
    const WgradProblem &q = grp.prob[blockIdx.y];
    wgrad_bf16_dma_body<BM, BN, WM, WN>(q.G, q.X, q.row_scale, q.idxW, q.cntW, q.dW, q.partials, R, K_in, K_out,
                                        tiles_n, tiles, splits, min_steps);
}

// ---------------------------------------------------------- host launchers

// Tile edge of the bf16 weight-gradient GEMM: 128, unless dW has so few 128x128 tiles that filling
// the chip takes many split-K slices, whose fp32 partial tiles then cost more HBM traffic than
// the operands (BERT-base: 3 to 8 slices, partials 2 to 4 times dW), and few enough tokens are
// expected that the matrix cores are not the limit: then 64x64 tiles, four times as many, with a
// quarter of the slices (1000 kept tokens, 768x3072: 24 vs 28 us and no partials at all).  Up to
// 1024 expected tokens: at 1900 (ViT-B/16) the 128x128 kernel is ahead again (step 3.67 -> 3.53 ms).
int wgrad_tile_bf16(int K_out, int K_in, int64_t expected_tokens)
{
    const int tiles128 = ((K_out + 127) / 128) * ((K_in + 127) / 128);
    return tiles128 <= 160 && expected_tokens <= 1024 ? 64 : 128;
}

int wgrad_tiles_bf16(int K_out, int K_in, int tile) { return ((K_out + tile - 1) / tile) * ((K_in + tile - 1) / tile); }

template <typename Kern>
static bool allow_lds(Kern kern, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes) == hipSuccess;
}

template <int BM, int BN, int WM, int WN, int NS, int OCC, int SPQ>
static vcas_status launch_dgrad(const vcas_shape &s, const void *G, const void *W, const float *p,
                                const int32_t *idxA, const int32_t *cntA, void *dX, const void *J, bool fill,
                                const InlineSampleA &sa, hipStream_t st)
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
                 s.K_out, tiles_n, static_cast<const uint16_t *>(J), fill ? 1 : 0, sa);
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
        if (probs[i].sa.gsq && s.N > 64) return VCAS_EINVAL;
        grp.prob[i] = probs[i];
    }
    const int64_t R = (int64_t)s.N * s.T;
    const int64_t rows = expected_rows > 0 && expected_rows < R ? expected_rows : R;
    const int64_t tiles256 = n * ((rows + 255) / 256) * ((s.K_in + 255) / 256);
    const int64_t tiles128 = n * ((rows + 127) / 128) * ((s.K_in + 127) / 128);
    if (tiles256 >= 128) return launch_dgrad_group<256, 256, 2, 4, 2, 1, 2>(s, grp, n, fill, st);
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
// it itself from the row norms and writes the plan's SampleA fields; N <= 64 only.
vcas_status dgrad_bf16(const vcas_shape &s, const void *G, const void *W, const float *p, const int32_t *idxA,
                       const int32_t *cntA, void *dX, const void *J, bool fill, int64_t expected_rows,
                       const InlineSampleA *sample_a, hipStream_t st)
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
        return launch_dgrad<256, 256, 2, 4, 2, 1, 2>(s, G, W, p, idxA, cntA, dX, J, fill, sa, st);
    if (tiles128 > 256) return launch_dgrad<128, 128, 2, 2, 2, 2, 4>(s, G, W, p, idxA, cntA, dX, J, fill, sa, st);
    const int64_t tiles64 = ((rows + 63) / 64) * ((s.K_in + 127) / 128);
    if (tiles64 > 256) return launch_dgrad<64, 128, 2, 2, 2, 2, 0>(s, G, W, p, idxA, cntA, dX, J, fill, sa, st);
    return launch_dgrad<64, 128, 2, 2, 4, 1, 0>(s, G, W, p, idxA, cntA, dX, J, fill, sa, st);
}

template <int BM, int BN, int WM, int WN, int OCC>
static vcas_status launch_wgrad(const vcas_shape &s, const void *G, const void *X, const float *row_scale,
                                const int32_t *idxW, const int32_t *cntW, float *dW, float *partials, int splits,
                                hipStream_t st)
{
    constexpr int MIN_STEPS = 2;
    const int64_t R = (int64_t)s.N * s.T;
    const int tiles_n = (s.K_in + BN - 1) / BN;
    const int tiles = ((s.K_out + BM - 1) / BM) * tiles_n;
    if (splits > 8) splits = 8;
    const size_t lds = 2 * (BM + BN) * 128;
    auto kern = wgrad_bf16_kernel<BM, BN, WM, WN, OCC>;
    static bool allowed = false;
    if (!allowed) {
        if (!allow_lds(kern, lds)) return VCAS_EHIP;
        allowed = true;
    }
    const int grid = (tiles * splits + 7) / 8 * 8;
    launch_timed(1, kern, dim3(grid), dim3(WM * WN * 64), lds, st, static_cast<const uint16_t *>(G),
                 static_cast<const uint16_t *>(X), row_scale, idxW, cntW, dW, partials, R, s.K_in, s.K_out, tiles_n,
                 tiles, splits, MIN_STEPS);
    if (hipGetLastError() != hipSuccess) return VCAS_EHIP;
    return splitk_reduce(partials, cntW, dW, R, (int64_t)s.K_out * s.K_in, splits, MIN_STEPS, BK, st);
}

static vcas_status launch_wgrad_dma(const vcas_shape &s, const void *G, const void *X, const float *row_scale,
                                    const int32_t *idxW, const int32_t *cntW, float *dW, float *partials,
                                    int splits, hipStream_t st)
{
    constexpr int BM = 128, BN = 128, MIN_STEPS = 2;
    const int64_t R = (int64_t)s.N * s.T;
    const int tiles_n = (s.K_in + BN - 1) / BN;
    const int tiles = ((s.K_out + BM - 1) / BM) * tiles_n;
    if (splits > 8) splits = 8;
    const size_t lds = 2 * (BM + BN) * 128;
    auto kern = wgrad_bf16_dma_kernel<BM, BN, 2, 2>;
    static bool allowed = false;
    if (!allowed) {
        if (!allow_lds(kern, lds)) return VCAS_EHIP;
        allowed = true;
    }
    const int grid = (tiles * splits + 7) / 8 * 8;
    launch_timed(1, kern, dim3(grid), dim3(256), lds, st, static_cast<const uint16_t *>(G),
                 static_cast<const uint16_t *>(X), row_scale, idxW, cntW, dW, partials, R, s.K_in, s.K_out, tiles_n,
                 tiles, splits, MIN_STEPS);
    if (hipGetLastError() != hipSuccess) return VCAS_EHIP;
    return splitk_reduce(partials, cntW, dW, R, (int64_t)s.K_out * s.K_in, splits, MIN_STEPS, BK, st);
}

// wgrad of n <= kMaxSiblings layers of shape s in one launch, and one launch for their reductions:
// tile and splits as for a layer on its own, so that every dW keeps its bits.
vcas_status wgrad_bf16_group(const vcas_shape &s, const WgradProblem *probs, int n, int tile, int splits, hipStream_t st)
{
    if (n < 1 || n > kMaxSiblings) return VCAS_EINVAL;
    WgradGroup grp = {};
    for (int i = 0; i < n; ++i) grp.prob[i] = probs[i];
    constexpr int MIN_STEPS = 2;
    const int64_t R = (int64_t)s.N * s.T;
    const int tiles_n = (s.K_in + tile - 1) / tile;
    const int tiles = ((s.K_out + tile - 1) / tile) * tiles_n;
    if (splits > 8) splits = 8;
    const size_t lds = 2 * (size_t)(tile + tile) * 128;
    const int grid = (tiles * splits + 7) / 8 * 8;
    if (tile == 64) {
        auto kern = wgrad_bf16_group_kernel<64, 64, 2, 1, 2>;
        static bool allowed = false;
        if (!allowed) {
            if (!allow_lds(kern, lds)) return VCAS_EHIP;
            allowed = true;
        }
        launch_timed(1, kern, dim3(grid, n), dim3(128), lds, st, grp, R, s.K_in, s.K_out, tiles_n, tiles, splits, MIN_STEPS);
    } else {
        auto kern = wgrad_bf16_dma_group_kernel<128, 128, 2, 2>;
        static bool allowed = false;
        if (!allowed) {
            if (!allow_lds(kern, lds)) return VCAS_EHIP;
            allowed = true;
        }
        launch_timed(1, kern, dim3(grid, n), dim3(256), lds, st, grp, R, s.K_in, s.K_out, tiles_n, tiles, splits, MIN_STEPS);
    }
    if (hipGetLastError() != hipSuccess) return VCAS_EHIP;
    return splitk_reduce_group(grp, n, R, (int64_t)s.K_out * s.K_in, splits, MIN_STEPS, BK, st);
}

// tile: 64 or 128 (wgrad_tile_bf16); splits: as sized by the caller for that tile
vcas_status wgrad_bf16(const vcas_shape &s, const void *G, const void *X, const float *row_scale,
                       const int32_t *idxW, const int32_t *cntW, float *dW, float *partials, int tile, int splits,
                       hipStream_t st)
{
    if (tile == 64)
        return launch_wgrad<64, 64, 2, 1, 2>(s, G, X, row_scale, idxW, cntW, dW, partials, splits, st);
    return launch_wgrad_dma(s, G, X, row_scale, idxW, cntW, dW, partials, splits, st);
}

}  // namespace vcas
