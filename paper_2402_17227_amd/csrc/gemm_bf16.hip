// bf16 MFMA gather-GEMMs of the VCAS backward pass (gfx950):
//   dgrad  dX[rows of kept samples] = (1/p_i) * G[row,:] W          (Eq. 1, upper line)
//   wgrad  dW = sum over kept tokens t of scale_t * g_t x_t^T        (Sec. 4.2)
// Both are dense contractions over the kept rows only, so they run on the
// matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
// Tiling: a workgroup of WM x WN wavefronts owns a BM x BN output tile and
// walks the contraction in steps of 64.  Operand tiles live in LDS as
// [row][64 k] bf16 (128 bytes per row, 16-byte slots XOR-swizzled so that both
// the fragment reads and the transposing writes spread over all banks), double
// buffered: the global loads of step i+1 are in flight while step i is on the
// matrix cores.
//
// W (for dgrad) and both G and X (for wgrad) are stored with the contraction
// index as the slow dimension, while an MFMA lane needs 8 consecutive
// contraction values of one row/column.  The loaders therefore read 4 rows x 8
// columns per thread with coalesced 16-byte loads, transpose the 4x8 block in
// registers (v_perm_b32) and write 8-byte pieces to the [column][k] LDS tile.
// wgrad multiplies the G block by the per-token scale on the way (the scale
// lies on the contraction axis and cannot go into the epilogue); dgrad's
// per-row 1/p goes into the epilogue.
#include "common.hpp"

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

// Operand whose rows are contiguous along the contraction (G in dgrad).
// ROWS x 64 tile; thread owns 16-byte slot (tid % 8) of rows tid/8 + j*NT/8.
template <int ROWS, int NT>
struct DirectLoader {
    static constexpr int PER = ROWS * 8 / NT;
    static_assert(ROWS * 8 % NT == 0 && NT % 8 == 0, "tile/thread mismatch");
    const uint16_t *row_ptr[PER];  // null: row outside the problem
    uint4 regs[PER];

    __device__ __forceinline__ void load(int k0, int K)
    {
        const int k = k0 + (threadIdx.x & 7) * 8;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            regs[j] = make_uint4(0u, 0u, 0u, 0u);
            if (row_ptr[j] != nullptr && k < K) regs[j] = *reinterpret_cast<const uint4 *>(row_ptr[j] + k);
        }
    }
    __device__ __forceinline__ void store(unsigned char *tile) const
    {
        const int slot = threadIdx.x & 7;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int row = (threadIdx.x >> 3) + j * (NT / 8);
            *reinterpret_cast<uint4 *>(tile + lds_off(row, slot)) = regs[j];
        }
    }
};

// Operand stored [k][col] (col contiguous).  64 x COLS tile; unit u = 4 k-rows
// x 8 columns: column chunk u % (COLS/8), k-quad u / (COLS/8).
template <int COLS, int NT>
struct TransLoader {
    static constexpr int CH = COLS / 8;
    static constexpr int PER = 16 * CH / NT;
    static_assert(16 * CH % NT == 0 && PER >= 1, "tile/thread mismatch");
    uint4 regs[PER][4];

    __device__ __forceinline__ static int chunk(int j) { return (threadIdx.x + j * NT) % CH; }
    __device__ __forceinline__ static int kquad(int j) { return (threadIdx.x + j * NT) / CH; }

    // addr(j, i) -> pointer to the 8 columns of k-row kquad(j)*4+i, or null
    template <typename Addr>
    __device__ __forceinline__ void load(Addr addr)
    {
#pragma unroll
        for (int j = 0; j < PER; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint16_t *p = addr(j, i);
                regs[j][i] = make_uint4(0u, 0u, 0u, 0u);
                if (p != nullptr) regs[j][i] = *reinterpret_cast<const uint4 *>(p);
            }
    }

    __device__ __forceinline__ static void put(unsigned char *tile, int j, int c, uint32_t d0, uint32_t d1)
    {
        const int row = chunk(j) * 8 + c;
        const int kq = kquad(j);
        *reinterpret_cast<uint2 *>(tile + lds_off(row, kq >> 1) + (kq & 1) * 8) = make_uint2(d0, d1);
    }

    // plain transpose
    __device__ __forceinline__ void store(unsigned char *tile) const
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

    // transpose with k-row i multiplied by s[j][i] (fp32 multiply, one bf16 rounding)
    __device__ __forceinline__ void store_scaled(unsigned char *tile, const float (*s)[4]) const
    {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const uint32_t *r0 = reinterpret_cast<const uint32_t *>(&regs[j][0]);
            const uint32_t *r1 = reinterpret_cast<const uint32_t *>(&regs[j][1]);
            const uint32_t *r2 = reinterpret_cast<const uint32_t *>(&regs[j][2]);
            const uint32_t *r3 = reinterpret_cast<const uint32_t *>(&regs[j][3]);
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                put(tile, j, 2 * d, pack_bf16(bf16_lo(r0[d]) * s[j][0], bf16_lo(r1[d]) * s[j][1]),
                    pack_bf16(bf16_lo(r2[d]) * s[j][2], bf16_lo(r3[d]) * s[j][3]));
                put(tile, j, 2 * d + 1, pack_bf16(bf16_hi(r0[d]) * s[j][0], bf16_hi(r1[d]) * s[j][1]),
                    pack_bf16(bf16_hi(r2[d]) * s[j][2], bf16_hi(r3[d]) * s[j][3]));
            }
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
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 a[TM], b[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
            a[i] = *reinterpret_cast<const bf16x8 *>(tileA + lds_off(rowA0 + i * 32 + r, ks * 2 + h));
#pragma unroll
        for (int i = 0; i < TN; ++i)
            b[i] = *reinterpret_cast<const bf16x8 *>(tileB + lds_off(rowB0 + i * 32 + r, ks * 2 + h));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
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

// grid: 1-D, tiles_n * (ceil(R/BM) + 1) + 8 workgroups.  The first ceil8(compute
// tiles) ids compute (spread over the XCDs in contiguous runs), the following
// ones write the zero rows of dropped samples, the rest exit.
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64) void dgrad_bf16_kernel(const uint16_t *__restrict__ G,
                                                                  const uint16_t *__restrict__ W,
                                                                  const float *__restrict__ p,
                                                                  const int32_t *__restrict__ idxA,
                                                                  const int32_t *__restrict__ cntA,
                                                                  uint16_t *__restrict__ dX, int N, int T, int K_in,
                                                                  int K_out, int tiles_n)
{
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    auto tA = [&](int buf) { return smem + buf * (BM * 128); };
    auto tB = [&](int buf) { return smem + 2 * BM * 128 + buf * (BN * 128); };
    int32_t *row_of = reinterpret_cast<int32_t *>(smem + 2 * (BM + BN) * 128);  // [BM] destination row or -1
    float *scale_of = reinterpret_cast<float *>(row_of + BM);                  // [BM] 1/p of the row's sample

    const int cnt = min(max(*cntA, 0), N);
    const int64_t M = (int64_t)cnt * T;
    const int64_t R = (int64_t)N * T;
    const int compute = (int)((M + BM - 1) / BM) * tiles_n;
    const int compute8 = (compute + 7) / 8 * 8;

    if ((int)blockIdx.x >= compute8) {
        // zero rows of dropped samples
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
    const int tile_m = tile / tiles_n, tile_n = tile % tiles_n;
    const int n0 = tile_n * BN;

    const int64_t m0 = (int64_t)tile_m * BM;
    for (int r = threadIdx.x; r < BM; r += NT) {
        const int64_t m = m0 + r;
        int32_t dst = -1;
        float sc = 0.0f;
        if (m < M) {
            const int s = idxA[m / T];
            dst = s * T + (int)(m % T);
            sc = 1.0f / (p[s]);
        }
        row_of[r] = dst;
        scale_of[r] = sc;
    }
    __syncthreads();

    DirectLoader<BM, NT> la;
#pragma unroll
    for (int j = 0; j < la.PER; ++j) {
        const int32_t src = row_of[(threadIdx.x >> 3) + j * (NT / 8)];
        la.row_ptr[j] = src >= 0 ? G + (int64_t)src * K_out : nullptr;
    }
    TransLoader<BN, NT> lb;
    auto w_addr = [&](int k0) {
        return [=](int j, int i) -> const uint16_t * {
            const int k = k0 + lb.kquad(j) * 4 + i;
            const int col = n0 + lb.chunk(j) * 8;
            return (k < K_out && col < K_in) ? W + (int64_t)k * K_in + col : nullptr;
        };
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

    const int steps = (K_out + BK - 1) / BK;
    la.load(0, K_out);
    lb.load(w_addr(0));
    la.store(tA(0));
    lb.store(tB(0));
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
        const int cur = s & 1;
        if (s + 1 < steps) {
            la.load((s + 1) * BK, K_out);
            lb.load(w_addr((s + 1) * BK));
        }
        mma_tile<TM, TN>(tA(cur), tB(cur), wm0, wn0, acc);
        if (s + 1 < steps) {
            la.store(tA(cur ^ 1));
            lb.store(tB(cur ^ 1));
        }
        __syncthreads();
    }

    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = wm0 + i * 32 + acc_row(v);
            const int32_t dst = row_of[r];
            if (dst < 0) continue;
            const float sc = scale_of[r];
            uint16_t *out = dX + (int64_t)dst * K_in;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = n0 + wn0 + j * 32 + (lane & 31);
                if (col < K_in) {
                    __bf16 b = (__bf16)(acc[i][j][v] * sc);
                    out[col] = *reinterpret_cast<uint16_t *>(&b);
                }
            }
        }
}

// ------------------------------------------------------------------ wgrad

struct TokenQuad {
    int32_t tok[4];
    float sc[4];
};

// grid: 1-D, splits * tiles workgroups (rounded up to a multiple of 8), split-
// major, so that the workgroups one XCD gets (a contiguous run after the remap)
// contract the same tokens and share those G and X rows in its L2.  Split s of
// a tile contracts a contiguous run of 64-token steps.  With more than
// one active split the partial tiles go to `partials` [split][K_out][K_in] and
// the workgroup that arrives last at the tile's counter adds them up in split
// order and writes dW, so the sum order is fixed.
template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM *WN * 64) void wgrad_bf16_kernel(const uint16_t *__restrict__ G,
                                                                  const uint16_t *__restrict__ X,
                                                                  const float *__restrict__ row_scale,
                                                                  const int32_t *__restrict__ idxW,
                                                                  const int32_t *__restrict__ cntW, float *__restrict__ dW,
                                                                  float *__restrict__ partials,
                                                                  int32_t *__restrict__ counters, int64_t R, int K_in,
                                                                  int K_out, int tiles_n, int tiles, int splits,
                                                                  int min_steps)
{
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    auto tA = [&](int buf) { return smem + buf * (BM * 128); };
    auto tB = [&](int buf) { return smem + 2 * BM * 128 + buf * (BN * 128); };
    __shared__ int last_flag;

    const int total = tiles * splits;
    const int id = xcd_remap(blockIdx.x, total);
    if (id >= total) return;
    const int split = id / tiles, tile = id % tiles;
    const int o0 = (tile / tiles_n) * BM, c0 = (tile % tiles_n) * BN;

    const int64_t cnt = min((int64_t)max(*cntW, 0), R);
    const int steps_all = (int)((cnt + BK - 1) / BK);
    int active = min(splits, max(1, steps_all / min_steps));
    const int per = max(1, (steps_all + active - 1) / active);
    active = max(1, (steps_all + per - 1) / per);
    if (split >= active) return;
    const int s_begin = split * per, s_end = min(steps_all, s_begin + per);

    TransLoader<BM, NT> la;
    TransLoader<BN, NT> lb;
    static_assert(TransLoader<BM, NT>::PER == 1 && TransLoader<BN, NT>::PER == 1, "one unit per thread assumed");
    const int kqa = la.kquad(0), kqb = lb.kquad(0);
    const int cola = o0 + la.chunk(0) * 8, colb = c0 + lb.chunk(0) * 8;

    auto fetch_quad = [&](int step, int kq) {
        TokenQuad t;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t k = (int64_t)step * BK + kq * 4 + i;
            t.tok[i] = -1;
            t.sc[i] = 0.0f;
            if (step < s_end && k < cnt) {
                const int32_t r = idxW[k];
                if (r >= 0 && r < R) {
                    t.tok[i] = r;
                    t.sc[i] = row_scale[r];
                }
            }
        }
        return t;
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

    if (s_begin < s_end) {
        TokenQuad qa = fetch_quad(s_begin, kqa), qb = fetch_quad(s_begin, kqb);
        TokenQuad na, nb;
        auto load_both = [&]() {
            la.load([&](int, int i) -> const uint16_t * {
                return (qa.tok[i] >= 0 && cola < K_out) ? G + (int64_t)qa.tok[i] * K_out + cola : nullptr;
            });
            lb.load([&](int, int i) -> const uint16_t * {
                return (qb.tok[i] >= 0 && colb < K_in) ? X + (int64_t)qb.tok[i] * K_in + colb : nullptr;
            });
        };
        load_both();
        na = fetch_quad(s_begin + 1, kqa);
        nb = fetch_quad(s_begin + 1, kqb);
        {
            const float sc[1][4] = {{qa.sc[0], qa.sc[1], qa.sc[2], qa.sc[3]}};
            la.store_scaled(tA(0), sc);
            lb.store(tB(0));
        }
        __syncthreads();
        for (int s = s_begin; s < s_end; ++s) {
            const int cur = (s - s_begin) & 1;
            const bool more = s + 1 < s_end;
            if (more) {
                qa = na;
                qb = nb;
                load_both();
                na = fetch_quad(s + 2, kqa);
                nb = fetch_quad(s + 2, kqb);
            }
            mma_tile<TM, TN>(tA(cur), tB(cur), wm0, wn0, acc);
            if (more) {
                const float sc[1][4] = {{qa.sc[0], qa.sc[1], qa.sc[2], qa.sc[3]}};
                la.store_scaled(tA(cur ^ 1), sc);
                lb.store(tB(cur ^ 1));
            }
            __syncthreads();
        }
    }

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
    if (active == 1) return;

    // arrival: the last split of this tile reduces
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
        const int prev = atomicAdd(&counters[tile], 1);
        const int last = prev == active - 1;
        if (last) counters[tile] = 0;
        last_flag = last;
    }
    __syncthreads();
    if (!last_flag) return;
    __threadfence();
    constexpr int CH = BN / 4;
    for (int u = threadIdx.x; u < BM * CH; u += NT) {
        const int o = o0 + u / CH, c = c0 + (u % CH) * 4;
        if (o >= K_out || c >= K_in) continue;
        const int64_t off = (int64_t)o * K_in + c;
        float4 sum = *reinterpret_cast<const float4 *>(partials + off);
        for (int s = 1; s < active; ++s) {
            const float4 t = *reinterpret_cast<const float4 *>(partials + (int64_t)s * K_out * K_in + off);
            sum.x += t.x;
            sum.y += t.y;
            sum.z += t.z;
            sum.w += t.w;
        }
        *reinterpret_cast<float4 *>(dW + off) = sum;
    }
}

// ---------------------------------------------------------- host launchers

int wgrad_tiles_bf16(int K_out, int K_in) { return ((K_out + 127) / 128) * ((K_in + 127) / 128); }

template <typename Kern>
static bool allow_lds(Kern kern, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes) == hipSuccess;
}

vcas_status dgrad_bf16(const vcas_shape &s, const void *G, const void *W, const float *p, const int32_t *idxA,
                       const int32_t *cntA, void *dX, hipStream_t st)
{
    constexpr int BM = 128, BN = 128, WM = 2, WN = 2;
    const int64_t R = (int64_t)s.N * s.T;
    const int tiles_n = (s.K_in + BN - 1) / BN;
    const int64_t grid = tiles_n * ((R + BM - 1) / BM + 1) + 8;
    if (grid > (int64_t)1 << 30) return VCAS_EINVAL;
    const size_t lds = 2 * (BM + BN) * 128 + BM * 8;
    auto kern = dgrad_bf16_kernel<BM, BN, WM, WN>;
    if (!allow_lds(kern, lds)) return VCAS_EHIP;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(WM * WN * 64), lds, st, static_cast<const uint16_t *>(G),
                       static_cast<const uint16_t *>(W), p, idxA, cntA, static_cast<uint16_t *>(dX), s.N, s.T, s.K_in,
                       s.K_out, tiles_n);
    return launch_status();
}

vcas_status wgrad_bf16(const vcas_shape &s, const void *G, const void *X, const float *row_scale,
                       const int32_t *idxW, const int32_t *cntW, float *dW, float *partials, int32_t *counters,
                       int splits, hipStream_t st)
{
    constexpr int BM = 128, BN = 128, WM = 2, WN = 2;
    const int64_t R = (int64_t)s.N * s.T;
    const int tiles_n = (s.K_in + BN - 1) / BN;
    const int tiles = ((s.K_out + BM - 1) / BM) * tiles_n;
    if (tiles > (int)kCounterInts) splits = 1;
    const size_t lds = 2 * (BM + BN) * 128;
    auto kern = wgrad_bf16_kernel<BM, BN, WM, WN>;
    if (!allow_lds(kern, lds)) return VCAS_EHIP;
    const int grid = (tiles * splits + 7) / 8 * 8;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), lds, st, static_cast<const uint16_t *>(G),
                       static_cast<const uint16_t *>(X), row_scale, idxW, cntW, dW, partials, counters, R, s.K_in,
                       s.K_out, tiles_n, tiles, splits, 4);
    return launch_status();
}

}  // namespace vcas
