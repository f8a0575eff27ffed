// fp32 gather-GEMMs of the VCAS backward pass (the fp32 configuration):
// dgrad (Eq. 2, upper line) and wgrad (Sec. 4.2) on v_mfma_f32_32x32x2_f32.
// 64x64 output tile per workgroup of 4 wavefronts (2x2, one 32x32 MFMA block
// each), contraction in steps of 16.  LDS tiles are k-major ([k][row], pitch
// 68 floats) so that fragment reads are 32 consecutive floats; only dgrad's G
// operand (contiguous along the contraction) is transposed on its way in.
#include "common.hpp"

namespace vcas {

typedef __attribute__((ext_vector_type(16))) float f32x16;

// gemm_bf16.hip
vcas_status splitk_reduce(const float *partials, const int32_t *cntW, float *dW, int64_t R, int64_t elems, int splits,
                          int min_steps, int step, hipStream_t st);

// same rule as the bf16 kernels use (kept in step with it by the shared reduction kernel's tests)
__host__ __device__ inline int wgrad_active_splits(int steps_all, int splits, int min_steps, int &per)
{
    int active = splits < steps_all / min_steps ? splits : steps_all / min_steps;
    if (active < 1) active = 1;
    per = (steps_all + active - 1) / active;
    if (per < 1) per = 1;
    active = (steps_all + per - 1) / per;
    return active < 1 ? 1 : active;
}

namespace f32gemm {

constexpr int BM = 64, BN = 64, BKF = 16, PITCH = 68, NT = 256;
constexpr int TILE_FLOATS = BKF * PITCH;

__device__ __forceinline__ int acc_row(int v) { return (v >> 2) * 8 + ((threadIdx.x & 63) >> 5) * 4 + (v & 3); }

__device__ __forceinline__ int xcd_remap(int id, int total)
{
    const int per = (total + 7) / 8;
    return (id & 7) * per + (id >> 3);
}

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

__device__ __forceinline__ void mma_step(const float *As, const float *Bs, int wm0, int wn0, f32x16 &acc)
{
    const int lane = threadIdx.x & 63;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int kk = 0; kk < BKF; kk += 2) {
        const float a = As[(kk + h) * PITCH + wm0 + r];
        const float b = Bs[(kk + h) * PITCH + wn0 + r];
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
}

}  // namespace f32gemm

// grid: tiles_n * (ceil(R/64) + 1) + 8 workgroups.  The first ceil8(compute
// tiles) ids compute (spread over the XCDs), the next ones zero the rows of
// dropped samples, the rest exit.
__global__ __launch_bounds__(256) void dgrad_f32_kernel(const float *__restrict__ G, const float *__restrict__ W,
                                                        const float *__restrict__ p,
                                                        const int32_t *__restrict__ idxA,
                                                        const int32_t *__restrict__ cntA, float *__restrict__ dX,
                                                        int N, int T, int K_in, int K_out, int tiles_n,
                                                        const float *__restrict__ J, int fill_dropped)
{
    using namespace f32gemm;
    __shared__ __attribute__((aligned(16))) float As[2][TILE_FLOATS];
    __shared__ __attribute__((aligned(16))) float Bs[2][TILE_FLOATS];
    __shared__ int32_t row_of[BM];
    __shared__ float scale_of[BM];

    const int cnt = min(max(*cntA, 0), N);
    const int64_t M = (int64_t)cnt * T, R = (int64_t)N * T;
    const int compute = (int)((M + BM - 1) / BM) * tiles_n;
    const int compute8 = (compute + 7) / 8 * 8;
    const int tid = threadIdx.x;

    if ((int)blockIdx.x >= compute8) {
        if (!fill_dropped) return;
        const int z = blockIdx.x - compute8;
        const int64_t d0 = (int64_t)(z / tiles_n) * BM;
        const int n0 = (z % tiles_n) * BN;
        if (d0 >= R - M) return;
        if (tid < BM) {
            const int64_t d = d0 + tid;
            row_of[tid] = d < R - M ? nth_missing(idxA, cnt, (int)(d / T)) * T + (int)(d % T) : -1;
        }
        __syncthreads();
        for (int u = tid; u < BM * (BN / 4); u += NT) {
            const int r = u / (BN / 4), col = n0 + (u % (BN / 4)) * 4;
            if (row_of[r] >= 0 && col < K_in)
                *reinterpret_cast<float4 *>(dX + (int64_t)row_of[r] * K_in + col) = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        return;
    }
    const int tile = xcd_remap(blockIdx.x, compute);
    if (tile >= compute) return;
    const int64_t m0 = (int64_t)(tile / tiles_n) * BM;
    const int n0 = (tile % tiles_n) * BN;
    if (tid < BM) {
        const int64_t m = m0 + tid;
        int32_t dst = -1;
        float sc = 0.0f;
        if (m < M) {
            const int s = idxA[m / T];
            dst = s * T + (int)(m % T);
            sc = 1.0f / (p[s]);
        }
        row_of[tid] = dst;
        scale_of[tid] = sc;
    }
    __syncthreads();

    // G tile: 64 rows x 16 k, thread = (row tid/4, k-quad tid%4); W tile: 16 k x 64 cols, thread = (k tid/16, col-quad tid%16)
    const int a_row = tid >> 2, a_kq = tid & 3;
    const float *a_ptr = row_of[a_row] >= 0 ? G + (int64_t)row_of[a_row] * K_out : nullptr;
    const int b_k = tid >> 4, b_col = n0 + (tid & 15) * 4;
    // A step's MFMAs take a fifth of a microsecond and a workgroup often has its CU to itself, so the
    // global loads run DEPTH steps ahead of the step on the matrix cores, each step in a register set
    // of its own: set d holds step s = d (mod DEPTH) until the step before s has put it into LDS.
    constexpr int DEPTH = 4;
    float4 ra[DEPTH], rb[DEPTH];
    auto load = [&](int k0, float4 &qa, float4 &qb) {   // a step past the end loads zeros
        qa = make_float4(0.f, 0.f, 0.f, 0.f);
        qb = make_float4(0.f, 0.f, 0.f, 0.f);
        const int ka = k0 + a_kq * 4;
        if (a_ptr != nullptr && ka < K_out) qa = *reinterpret_cast<const float4 *>(a_ptr + ka);
        const int kb = k0 + b_k;
        if (kb < K_out && b_col < K_in) qb = *reinterpret_cast<const float4 *>(W + (int64_t)kb * K_in + b_col);
    };
    auto store = [&](int buf, const float4 &qa, const float4 &qb) {
        float *a = As[buf] + (a_kq * 4) * PITCH + a_row;
        a[0] = qa.x;
        a[PITCH] = qa.y;
        a[2 * PITCH] = qa.z;
        a[3 * PITCH] = qa.w;
        *reinterpret_cast<float4 *>(Bs[buf] + b_k * PITCH + (tid & 15) * 4) = qb;
    };

    const int wave = tid >> 6;
    const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    const int steps = (K_out + BKF - 1) / BKF;
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) load(d * BKF, ra[d], rb[d]);
    store(0, ra[0], rb[0]);
    __syncthreads();
    for (int s0 = 0; s0 < steps; s0 += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int s = s0 + d;
            if (s < steps) {   // the same for every thread
                const int cur = s & 1;
                load((s + DEPTH) * BKF, ra[d], rb[d]);   // set d (step s) went to LDS one step ago
                mma_step(As[cur], Bs[cur], wm0, wn0, acc);
                if (s + 1 < steps) store(cur ^ 1, ra[(d + 1) % DEPTH], rb[(d + 1) % DEPTH]);
                __syncthreads();
            }
        }
    }

    const int col = n0 + wn0 + (tid & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int r = wm0 + acc_row(v);
        if (row_of[r] >= 0 && col < K_in) {
            const int64_t at = (int64_t)row_of[r] * K_in + col;
            float val = acc[v] * scale_of[r];
            if (J) val = val * J[at];   // elementwise Jacobian of the layer below (App. E, proof of unbiasedness)
            dX[at] = val;
        }
    }
}

// grid: splits * tiles workgroups rounded up to 8, split-major; see the bf16
// kernel for the split-K protocol (same partial buffers and reduction kernel).
__global__ __launch_bounds__(256) void wgrad_f32_kernel(const float *__restrict__ G, const float *__restrict__ X,
                                                        const float *__restrict__ row_scale,
                                                        const int32_t *__restrict__ idxW,
                                                        const int32_t *__restrict__ cntW, float *__restrict__ dW,
                                                        float *__restrict__ partials, int64_t R, int K_in, int K_out, int tiles_n, int tiles,
                                                        int splits, int min_steps)
{
    using namespace f32gemm;
    __shared__ __attribute__((aligned(16))) float As[2][TILE_FLOATS];
    __shared__ __attribute__((aligned(16))) float Bs[2][TILE_FLOATS];

    const int total = tiles * splits;
    const int id = xcd_remap(blockIdx.x, total);
    if (id >= total) return;
    const int split = id / tiles, tile = id % tiles;
    const int o0 = (tile / tiles_n) * BM, c0 = (tile % tiles_n) * BN;
    const int tid = threadIdx.x;

    const int64_t cnt = min((int64_t)max(*cntW, 0), R);
    const int steps_all = (int)((cnt + BKF - 1) / BKF);
    int per;
    const int active = wgrad_active_splits(steps_all, splits, min_steps, per);
    if (split >= active) return;
    const int s_begin = split * per, s_end = min(steps_all, s_begin + per);

    // both tiles: 16 tokens x 64 cols, thread = (token tid/16, col-quad tid%16)
    const int kk = tid >> 4, cq = (tid & 15) * 4;
    // Token indices and scales of CHUNK steps at a time go to LDS first (two dependent loads that
    // nothing else could hide); inside a chunk the row loads run DEPTH steps ahead of the MFMAs,
    // each step in a register set of its own, as in dgrad.
    constexpr int DEPTH = 4, CHUNK = 64;
    __shared__ int32_t tok_of[CHUNK * BKF];
    __shared__ float scale_of[CHUNK * BKF];
    float4 ra[DEPTH], rb[DEPTH];
    auto load = [&](int local_step, int local_steps, float4 &qa, float4 &qb) {   // past the chunk: zeros
        qa = make_float4(0.f, 0.f, 0.f, 0.f);
        qb = make_float4(0.f, 0.f, 0.f, 0.f);
        const int32_t t = local_step < local_steps ? tok_of[local_step * BKF + kk] : -1;
        if (t >= 0 && o0 + cq < K_out) qa = *reinterpret_cast<const float4 *>(G + (int64_t)t * K_out + o0 + cq);
        if (t >= 0 && c0 + cq < K_in) qb = *reinterpret_cast<const float4 *>(X + (int64_t)t * K_in + c0 + cq);
    };
    auto store = [&](int buf, int local_step, const float4 &qa, const float4 &qb) {
        const float sc = scale_of[local_step * BKF + kk];
        const float4 a = make_float4(qa.x * sc, qa.y * sc, qa.z * sc, qa.w * sc);
        *reinterpret_cast<float4 *>(As[buf] + kk * PITCH + cq) = a;
        *reinterpret_cast<float4 *>(Bs[buf] + kk * PITCH + cq) = qb;
    };

    const int wave = tid >> 6;
    const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    for (int chunk0 = s_begin; chunk0 < s_end; chunk0 += CHUNK) {
        const int local_steps = min(CHUNK, s_end - chunk0);
        __syncthreads();   // the previous chunk's table and tiles are no longer read
        for (int i = tid; i < local_steps * BKF; i += NT) {
            const int64_t k = (int64_t)chunk0 * BKF + i;
            int32_t t = -1;
            float sc = 0.0f;
            if (k < cnt) {
                const int32_t r = idxW[k];
                if (r >= 0 && r < R) {
                    t = r;
                    sc = row_scale[r];
                }
            }
            tok_of[i] = t;
            scale_of[i] = sc;
        }
        __syncthreads();
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) load(d, local_steps, ra[d], rb[d]);
        store(0, 0, ra[0], rb[0]);
        __syncthreads();
        for (int s0 = 0; s0 < local_steps; s0 += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                const int s = s0 + d;
                if (s < local_steps) {   // the same for every thread
                    const int cur = s & 1;
                    load(s + DEPTH, local_steps, ra[d], rb[d]);
                    mma_step(As[cur], Bs[cur], wm0, wn0, acc);
                    if (s + 1 < local_steps) store(cur ^ 1, s + 1, ra[(d + 1) % DEPTH], rb[(d + 1) % DEPTH]);
                    __syncthreads();
                }
            }
        }
    }

    float *dst = active == 1 ? dW : partials + (int64_t)split * K_out * K_in;
    const int c = c0 + wn0 + (tid & 31);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int o = o0 + wm0 + acc_row(v);
        if (o < K_out && c < K_in) dst[(int64_t)o * K_in + c] = acc[v];
    }
}

int wgrad_tiles_f32(int K_out, int K_in) { return ((K_out + 63) / 64) * ((K_in + 63) / 64); }

vcas_status dgrad_f32(const vcas_shape &s, const void *G, const void *W, const float *p, const int32_t *idxA,
                      const int32_t *cntA, void *dX, const void *J, bool fill, hipStream_t st)
{
    const int64_t R = (int64_t)s.N * s.T;
    const int tiles_n = (s.K_in + 63) / 64;
    const int64_t grid = tiles_n * ((R + 63) / 64 + 1) + 8;
    if (grid > (int64_t)1 << 30) return VCAS_EINVAL;
    launch_timed(0, dgrad_f32_kernel, dim3((unsigned)grid), dim3(256), 0, st, static_cast<const float *>(G),
                       static_cast<const float *>(W), p, idxA, cntA, static_cast<float *>(dX), s.N, s.T, s.K_in,
                       s.K_out, tiles_n, static_cast<const float *>(J), fill ? 1 : 0);
    return launch_status();
}

vcas_status wgrad_f32(const vcas_shape &s, const void *G, const void *X, const float *row_scale, const int32_t *idxW,
                      const int32_t *cntW, float *dW, float *partials, int splits, hipStream_t st)
{
    constexpr int MIN_STEPS = 8;
    const int64_t R = (int64_t)s.N * s.T;
    const int tiles_n = (s.K_in + 63) / 64;
    const int tiles = ((s.K_out + 63) / 64) * tiles_n;
    if (splits > 8) splits = 8;
    const int grid = (tiles * splits + 7) / 8 * 8;
    launch_timed(1, wgrad_f32_kernel, dim3(grid), dim3(256), 0, st, static_cast<const float *>(G),
                       static_cast<const float *>(X), row_scale, idxW, cntW, dW, partials, R, s.K_in, s.K_out, tiles_n,
                       tiles, splits, MIN_STEPS);
    if (hipGetLastError() != hipSuccess) return VCAS_EHIP;
    return splitk_reduce(partials, cntW, dW, R, (int64_t)s.K_out * s.K_in, splits, MIN_STEPS, f32gemm::BKF, st);
}

}  // namespace vcas
