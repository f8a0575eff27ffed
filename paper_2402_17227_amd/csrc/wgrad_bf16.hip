// bf16 MFMA gather-GEMM of the VCAS weight gradient (gfx950):
//   dW = sum over kept tokens t of scale_t * g_t x_t^T,  scale_t = 1/(p_i q_t)      (Sec. 4.2)
// A dense contraction over the kept tokens only: v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
// Both operands have the contraction index (tokens) as their slow dimension, so both MFMA
// operands lie "the wrong way": their tiles stay as they are in memory, [64 tokens][columns],
// and ds_read_b64_tr_b16 transposes them on the way out of LDS.
//
// The per-token scale lies on the contraction axis, so it has to be multiplied into one of the two
// operands before the MFMAs.  Doing that inside the GEMM costs five vector instructions per pair
// of elements, more issue slots than the matrix instructions leave free (the earlier kernels of
// this file did, and were bound by exactly that).  Here a small memory-bound launch does it once,
// ahead of the GEMM, for the NARROWER operand:
//   packed[j, :] = bf16(scale[t] * src[t, :]),  t = idx[j],  j < count
// (rows in kept-list order; fp32 multiply, one rounding).  The GEMM then moves both operands
// straight into LDS and its wavefronts issue little besides LDS reads and MFMAs: the packed
// operand's rows are consecutive (offsets fixed, the step advances a scalar), only the other
// operand is gathered through the kept list.
//
// A launch covers a BATCH of up to kWgradBatch layers of any shapes (the weight gradients of a
// block of layers do not depend on each other): workgroup ids are cut into per-layer ranges, so
// small weight gradients fill the chip together instead of being cut into split-K slices one by
// one.
#include "mfma_bf16.hpp"

namespace vcas {

// ------------------------------------------------------------------ split-K

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

// also used by the fp32 kernels
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

// Slot XOR of row k of a [64 tokens][columns] tile with SL 16-byte slots per row.  A half-wave's
// transposing read takes 32 bytes from each of four consecutive rows; the XOR puts them into four
// different 64-byte bank groups.  Rows of 256 bytes or more all start at bank 0: shift row k by
// (k mod 4) * 64 bytes.  Rows of 128 bytes alternate between the two halves of the banks already:
// shift every second pair of rows by 64 bytes.
template <int SL>
__device__ __forceinline__ int tile_swz(int k)
{
    return SL >= 16 ? (k & 3) * 4 : ((k >> 1) & 1) * 4;
}

// ------------------------------------------------------------------ batch

// One layer of a batched launch (device view).
struct WgradTask {
    const uint16_t *gathered;   // G [R,K_out] (X side packed) or X [R,K_in] (G side packed)
    const uint16_t *src;        // the operand the pre-pass rewrites: the other one of G, X
    uint16_t *packed;           // [count rows][K_p] written by the pre-pass, read by the GEMM
    const float *row_scale;
    const int32_t *idxW, *cntW;
    float *dW, *partials;
    int32_t R, K_in, K_out;
    int32_t packed_a;           // nonzero: the G side is the packed operand
    int32_t tiles_n, tiles, splits;
    int32_t first_wg;           // first workgroup id of this layer's range (a multiple of 8)
};
struct WgradBatch {
    WgradTask task[kWgradBatch];
    int32_t n;
};

// Pre-pass: one wavefront per kept token, blockIdx.y = layer.
__global__ __launch_bounds__(256) void pack_scaled_rows_kernel(WgradBatch batch)
{
    const WgradTask &q = batch.task[blockIdx.y];
    const int R = q.R;
    const int c = min(max(*q.cntW, 0), R);
    const int groups = (q.packed_a ? q.K_out : q.K_in) / 8;
    const uint4 *src = reinterpret_cast<const uint4 *>(q.src);
    uint4 *dst = reinterpret_cast<uint4 *>(q.packed);
    const int lane = threadIdx.x & 63;
    for (int j = blockIdx.x * 4 + (threadIdx.x >> 6); j < c; j += gridDim.x * 4) {
        const uint32_t t = (uint32_t)q.idxW[j];
        const bool inside = t < (uint32_t)R;
        const float sc = inside ? q.row_scale[t] : 0.0f;
        const uint4 *row = src + (int64_t)(inside ? t : 0u) * groups;
        uint4 *out = dst + (int64_t)j * groups;
        for (int g = lane; g < groups; g += 64) {
            uint4 o = make_uint4(0u, 0u, 0u, 0u);
            if (inside) {
                const uint4 v = row[g];
                o.x = pack_bf16(bf16_lo(v.x) * sc, bf16_hi(v.x) * sc);
                o.y = pack_bf16(bf16_lo(v.y) * sc, bf16_hi(v.y) * sc);
                o.z = pack_bf16(bf16_lo(v.z) * sc, bf16_hi(v.z) * sc);
                o.w = pack_bf16(bf16_lo(v.w) * sc, bf16_hi(v.w) * sc);
            }
            out[g] = o;
        }
    }
}

__global__ __launch_bounds__(256) void splitk_reduce_batch_kernel(WgradBatch batch, int min_steps, int step)
{
    const WgradTask &q = batch.task[blockIdx.y];
    splitk_reduce_body(q.partials, q.cntW, q.dW, q.R, (int64_t)q.K_out * q.K_in, q.splits, min_steps, step);
}

// 16 bytes of the kept list into registers, by hand like every other load of the GEMM.
__device__ __forceinline__ u32x4 asm_load_b128(i32x4 desc, uint32_t voffset)
{
    u32x4 v;
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(v) : "v"(voffset), "s"(desc) : "memory");
    return v;
}

// The GEMM.  BM x BM output tile, WM x WN wavefronts (BM = 32 * WM * WN, so that a wavefront
// fills its rows of a tile with four loads), NS (2 or 3) stages of [64 tokens][BM columns] tile
// pairs, slots swizzled by tile_swz.  Every load is inline assembly and counted by hand: per step and
// thread one 16-byte read of the kept list (four tokens, issued two steps before they are turned
// into offsets) followed by eight LDS-direct tile loads for the step NS-1 ahead; one barrier per
// step, in front of it ONE s_waitcnt that leaves the loads of the NS-2 younger steps in flight.
//
// grid: 1-D; a layer's range holds splits * tiles workgroups (rounded up to a multiple of 8),
// split-major, so that the workgroups one XCD gets (a contiguous run after the remap) contract
// the same tokens and share those rows in its L2.  Split s of a tile contracts a contiguous run
// of 64-token steps; the number of active splits is derived from the device-side count
// (wgrad_active_splits).  With one active split the tile goes straight to dW; otherwise the
// partial tiles go to `partials` [split][K_out][K_in] and the reduction kernel adds them in split
// order, so the sum order is fixed.
template <int BM, int WM, int WN, int NS>
__device__ __forceinline__ void wgrad_bf16_packed_body(const WgradTask &q, int local_id)
{
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM / 32, TN = BM / WN / 32;
    constexpr int PITCH = BM * 2, SL = BM / 8, RPI = 1024 / PITCH, BLOCK = BK / NW;
    constexpr int A_TILE = BK * PITCH, STAGE = 2 * A_TILE;
    static_assert(BLOCK == 4 * RPI, "a wavefront fills its rows of a tile with four loads");
    static_assert(NS == 2 || NS == 3, "the kept-list reads run two steps ahead");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tiles = q.tiles, tiles_n = q.tiles_n, splits = q.splits;
    const int K_in = q.K_in, K_out = q.K_out, R = q.R;
    const int total = tiles * splits;
    const int id = xcd_remap(local_id, total);
    if (id >= total) return;
    const int split = id / tiles, tile = id % tiles;
    int tile_o, tile_c;   // panels of 4 column tiles: an XCD's run of workgroups covers a squarish patch of dW
    panel_order_rt(tile, tiles / tiles_n, tiles_n, 4, tile_o, tile_c);
    const int o0 = tile_o * BM, c0 = tile_c * BM;

    const int cnt = min(max(*q.cntW, 0), R);
    const int steps_all = (cnt + BK - 1) / BK;
    int per;
    const int active = wgrad_active_splits(steps_all, splits, 2, per);
    if (split >= active) return;
    const int s_begin = split * per, s_end = min(steps_all, s_begin + per);
    const int steps = s_end - s_begin;
    const int k_end = min(cnt, s_end * BK);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane / SL, slot = lane % SL;
    const int k_first = BLOCK * wave + 4 * sub;   // this thread's tokens of a step: k_first + j, j < 4
    // token k_first + j lives in LDS row BLOCK * wave + RPI * j + sub (the same in both tiles)
    const bool packed_a = q.packed_a != 0;        // wave-uniform
    const int K_g = packed_a ? K_in : K_out, K_p = packed_a ? K_out : K_in;     // row lengths
    const int g0 = packed_a ? c0 : o0, p0 = packed_a ? o0 : c0;                 // the tile's first column in each
    const i32x4 descG = raw_descriptor(q.gathered, (uint32_t)((int64_t)R * K_g * 2));
    const i32x4 descP = raw_descriptor(q.packed, (uint32_t)((int64_t)cnt * K_p * 2));   // rows past the count read as zeros
    const i32x4 descI = raw_descriptor(q.idxW, (uint32_t)((int64_t)R * 4));
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const uint32_t g_pitch = (uint32_t)K_g * 2u, p_pitch = (uint32_t)K_p * 2u;
    const int g_at = packed_a ? A_TILE : 0, p_at = packed_a ? 0 : A_TILE;       // each operand's tile within a stage
    // offset of gathered token r's piece = r * pitch + column bytes: one multiply-add; a thread
    // whose columns lie outside the matrix multiplies by zero and adds the out-of-range offset
    uint32_t g_mul[4], g_add[4], p_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = BLOCK * wave + RPI * j + sub;
        const int piece = slot ^ tile_swz<SL>(row);
        const int gcol = g0 + piece * 8, pcol = p0 + piece * 8;
        g_mul[j] = gcol < K_g ? g_pitch : 0u;
        g_add[j] = gcol < K_g ? (uint32_t)gcol * 2u : kOutside;
        p_off[j] = pcol < K_p ? (uint32_t)(k_first + j) * p_pitch + (uint32_t)pcol * 2u : kOutside;
    }
    auto idx_offset = [&](int st) {
        const int k0 = (s_begin + st) * BK + k_first;
        return k0 < k_end ? (uint32_t)k0 * 4u : kOutside;
    };
    // Byte offsets of the gathered operand's four rows of step st.  Every step but a slice's last
    // holds 64 kept tokens: no per-token checks there (the branch is wave-uniform); list entries
    // are rows < 2^24 (checked on the host), and one that is not a row of the matrix can at worst
    // read zeros through the bounded descriptor.
    auto gather_offsets = [&](const u32x4 &t, int st, uint32_t (&off)[4]) {
        if ((s_begin + st + 1) * BK <= k_end) {
#pragma unroll
            for (int j = 0; j < 4; ++j) off[j] = __umul24(t[j], g_mul[j]) + g_add[j];
        } else {
            const int k0 = (s_begin + st) * BK + k_first;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                off[j] = (k0 + j < k_end && t[j] < (uint32_t)R) ? __umul24(t[j], g_mul[j]) + g_add[j] : kOutside;
        }
    };
    auto issue_tiles = [&](int st, const uint32_t (&goff)[4]) {
        const uint32_t base = __builtin_amdgcn_readfirstlane(lds0 + (st % NS) * STAGE + wave * BLOCK * PITCH);
        // rows of the packed operand advance with the step; past the slice's end nothing is fetched
        const bool live = st < steps;
        const uint32_t adv = __builtin_amdgcn_readfirstlane(live ? (uint32_t)((s_begin + st) * BK) * p_pitch : 0u);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            lds_direct_load16(descG, base + g_at + j * 1024, goff[j], 0u);
            lds_direct_load16(descP, base + p_at + j * 1024, live ? p_off[j] : kOutside, adv);
        }
    };

    const int wm0 = (wave / WN) * (BM / WM), wn0 = (wave % WN) * (BM / WN);
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    const int blk = lane >> 4, sl = lane & 15;
    // fragment of 32 columns x 16 tokens of a [64][BM] tile: two transposing reads
    auto frag = [&](const unsigned char *t, int col0, int ks) {
        bf16x4 half[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int k = ks * 16 + (blk >> 1) * 8 + e * 4 + (sl >> 2);
            const int col = col0 + (blk & 1) * 16 + (sl & 3) * 4;
            const unsigned char *src = t + k * PITCH + (((col >> 3) ^ tile_swz<SL>(k)) << 4) + (col & 7) * 2;
            half[e] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((__attribute__((address_space(3))) bf16x4 *)(src));
        }
        return __builtin_shufflevector(half[0], half[1], 0, 1, 2, 3, 4, 5, 6, 7);
    };

    // Two register sets for the kept-list reads: the read issued in step s (for the tiles of step
    // s + NS + 1) lands in set s & 1 and is turned into offsets at the top of step s + 2.  A
    // register that a load is still filling is never copied: it is written by one asm statement
    // and passes through the wait statement as a read-write operand before its first use.
    u32x4 tokset[2];
    {
        // prologue = the steps -2 and -1 of that schedule: tokens of steps 0 .. NS-2 first (used
        // here), then per step one kept-list read and, from step -(NS-1) on, the tile loads
        u32x4 t0 = asm_load_b128(descI, idx_offset(0));
        u32x4 t1 = asm_load_b128(descI, idx_offset(1));
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(t0), "+v"(t1) : : "memory");
        uint32_t off[4];
        tokset[0] = asm_load_b128(descI, idx_offset(NS - 1));
        if (NS == 3) {
            gather_offsets(t0, 0, off);
            issue_tiles(0, off);
        }
        tokset[1] = asm_load_b128(descI, idx_offset(NS));
        gather_offsets(NS == 3 ? t1 : t0, NS - 2, off);
        issue_tiles(NS - 2, off);
    }

    // One contraction step; E = parity of s.
    auto step = [&](int s, auto e_) {
        constexpr int E = decltype(e_)::value;
        // the tiles of step s have landed once at most the loads of the NS-2 steps behind it
        // (nine each: the kept-list read, then eight tile loads) are in flight
        if (NS == 2) asm volatile("s_waitcnt vmcnt(0)" : "+v"(tokset[E]) : : "memory");
        else asm volatile("s_waitcnt vmcnt(9)" : "+v"(tokset[E]) : : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        const int u = s + NS - 1;
        uint32_t off[4];
        gather_offsets(tokset[E], u, off);
        __builtin_amdgcn_sched_barrier(0);
        tokset[E] = asm_load_b128(descI, idx_offset(u + 2));
        issue_tiles(u, off);
        __builtin_amdgcn_sched_barrier(0);
        const unsigned char *tileA = smem + (s % NS) * STAGE;
        const unsigned char *tileB = tileA + A_TILE;
        constexpr int KS = BK / 16;
        bf16x8 a[2][TM], b[2][TN];
        auto read_frags = [&](int ks, bf16x8(&fa)[TM], bf16x8(&fb)[TN]) {
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = frag(tileA, wm0 + i * 32, ks);
#pragma unroll
            for (int i = 0; i < TN; ++i) fb[i] = frag(tileB, wn0 + i * 32, ks);
        };
        read_frags(0, a[0], b[0]);
        read_frags(1, a[1], b[1]);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][i], b[ks & 1][j], acc[i][j], 0, 0, 0);
            if (ks + 2 < KS) read_frags(ks + 2, a[ks & 1], b[ks & 1]);
        }
        // fragment reads of two k-slices, then each slice's MFMAs with the reads of the slice after next
        constexpr int RD = 2 * (TM + TN), MM = TM * TN;
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * RD, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            __builtin_amdgcn_sched_group_barrier(0x008, MM, 0);
            if (ks + 2 < KS) __builtin_amdgcn_sched_group_barrier(0x100, RD, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    for (int s = 0; s < steps; s += 2) {
        step(s, std::integral_constant<int, 0>());
        if (s + 1 < steps) step(s + 1, std::integral_constant<int, 1>());
    }
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(tokset[0]), "+v"(tokset[1]) : : "memory");

    const int lane32 = lane & 31;
    float *dst = active == 1 ? q.dW : q.partials + (int64_t)split * K_out * K_in;
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

template <int BM, int WM, int WN, int NS, int OCC>
__global__ __launch_bounds__(WM *WN * 64, OCC) void wgrad_bf16_batch_kernel(WgradBatch batch)
{
    // the layer whose range holds this workgroup (ranges ascend; at most kWgradBatch of them)
    int p = 0;
    for (int i = 1; i < batch.n; ++i)
        if ((int)blockIdx.x >= batch.task[i].first_wg) p = i;
    const WgradTask &q = batch.task[p];
    wgrad_bf16_packed_body<BM, WM, WN, NS>(q, (int)blockIdx.x - q.first_wg);
}

// ---------------------------------------------------------- host launchers

int wgrad_tiles_bf16(int K_out, int K_in, int tile) { return ((K_out + tile - 1) / tile) * ((K_in + tile - 1) / tile); }

template <int BM, int WM, int WN, int NS, int OCC>
static vcas_status launch_batch(const WgradBatch &batch, int grid, hipStream_t st)
{
    const size_t lds = (size_t)NS * 2 * BK * BM * 2;
    auto kern = wgrad_bf16_batch_kernel<BM, WM, WN, NS, OCC>;
    static bool allowed = false;
    if (!allowed) {
        if (!allow_lds(kern, lds)) return VCAS_EHIP;
        allowed = true;
    }
    launch_timed(1, kern, dim3((unsigned)grid), dim3(WM * WN * 64), lds, st, batch);
    return launch_status();
}

// Weight gradients of n <= kWgradBatch bf16 layers: the pre-pass over every layer's narrower
// operand, ONE GEMM launch with `tile`-edged output tiles (256, 128 or 64), one launch for the
// split-K reductions where any layer has more than one slice.  items[i].splits slices per tile
// (at most 8; the caller sized `partials` for them).
vcas_status wgrad_bf16_batch(const WgradItem *items, int n, int tile, hipStream_t st)
{
    if (n < 1 || n > kWgradBatch || (tile != 256 && tile != 128 && tile != 64)) return VCAS_EINVAL;
    WgradBatch batch = {};
    batch.n = n;
    int64_t grid = 0, rows_max = 0, elems_max = 0;
    bool reduce = false;
    for (int i = 0; i < n; ++i) {
        const WgradItem &it = items[i];
        const vcas_shape &s = it.shape;
        WgradTask &q = batch.task[i];
        const int64_t R = (int64_t)s.N * s.T;
        q.packed_a = s.K_out < s.K_in ? 1 : 0;      // the narrower operand is the one rewritten
        q.gathered = static_cast<const uint16_t *>(q.packed_a ? it.X : it.G);
        q.src = static_cast<const uint16_t *>(q.packed_a ? it.G : it.X);
        q.packed = it.packed;
        q.row_scale = it.row_scale;
        q.idxW = it.idxW;
        q.cntW = it.cntW;
        q.dW = it.dW;
        q.partials = it.partials;
        q.R = (int32_t)R;
        q.K_in = s.K_in;
        q.K_out = s.K_out;
        q.tiles_n = (s.K_in + tile - 1) / tile;
        q.tiles = ((s.K_out + tile - 1) / tile) * q.tiles_n;
        q.splits = it.splits < 1 ? 1 : it.splits > 8 ? 8 : it.splits;
        q.first_wg = (int32_t)grid;
        grid += ((int64_t)q.tiles * q.splits + 7) / 8 * 8;
        if (q.splits > 1) reduce = true;
        if (R > rows_max) rows_max = R;
        if ((int64_t)s.K_out * s.K_in > elems_max) elems_max = (int64_t)s.K_out * s.K_in;
    }
    if (grid > (int64_t)1 << 30) return VCAS_EINVAL;
    int64_t pack_blocks = (rows_max + 3) / 4;
    if (pack_blocks > 2048) pack_blocks = 2048;
    hipLaunchKernelGGL(pack_scaled_rows_kernel, dim3((unsigned)pack_blocks, (unsigned)n), dim3(256), 0, st, batch);
    if (hipGetLastError() != hipSuccess) return VCAS_EHIP;
    vcas_status rc;
    if (tile == 256) rc = launch_batch<256, 2, 4, 2, 1>(batch, (int)grid, st);
    else if (tile == 128) rc = launch_batch<128, 2, 2, 2, 2>(batch, (int)grid, st);
    else rc = launch_batch<64, 2, 1, 2, 4>(batch, (int)grid, st);
    if (rc != VCAS_OK) return rc;
    if (reduce) {
        int64_t blocks = (elems_max / 4 + 255) / 256;
        if (blocks > 2048) blocks = 2048;
        hipLaunchKernelGGL(splitk_reduce_batch_kernel, dim3((unsigned)blocks, (unsigned)n), dim3(256), 0, st, batch, 2, BK);
        return launch_status();
    }
    return VCAS_OK;
}

}  // namespace vcas
