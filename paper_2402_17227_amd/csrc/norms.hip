// Row-norm kernels: squared 2-norms of the rows of G and X (the factors of
// Eq. 3 and the per-sample Frobenius norms of Sec. 4.1 of the VCAS paper).
// HBM-bound: every element is read once, one fp32 per row is written.
#include "rowsum.hpp"
#include "groups.hpp"

namespace vcas {

// One wavefront per row; CH 16-byte groups per lane are in flight at once.
// Rows of samples whose sample_keep byte is 0 are not read and get 0.
// If a UniformJob is given, the launch also draws the Philox uniform of every
// row for that sampler (the arithmetic hides under the memory stream).
// If a ScoreJob is given (A is X, SampleA is done), the row's SampleW score
// ((1/p_i) * sqrt(gsq_t)) * sqrt(xsq_t) is written as well, 0 on dropped samples:
// the square roots and the division then run on every CU instead of in the one
// workgroup of the sampler.
template <bool BF16, int CH>
__device__ __forceinline__ void row_sumsq_body(const uint4 *__restrict__ A, int64_t R, int groups_per_row, int T,
                                               const uint8_t *__restrict__ sample_keep, float *__restrict__ out,
                                               const UniformJob &job, const ScoreJob &sj)
{
    if (job.uniforms) {
        const uint32_t draw = job.draw + (job.draw_offset ? *job.draw_offset : 0u);
        for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < R; r += (int64_t)gridDim.x * 256)
            job.uniforms[r] = philox_uniform(job.seed, job.layer, job.stream_id, draw, (uint32_t)r);
    }
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t row = wave; row < R; row += nwaves) {
        const int64_t i = row / T;
        if (sample_keep && sample_keep[i] == 0) {
            if (lane == 0) {
                out[row] = 0.0f;
                if (sj.score) sj.score[row] = 0.0f;
            }
            continue;
        }
        float s1 = 0.0f;
        if (sj.score) {
            const float inv = 1.0f / sj.p[i];
            s1 = inv * __builtin_sqrtf(sj.gsq[row]);
        }
        const float acc = wave_row_sumsq<BF16, CH>(A + row * groups_per_row, groups_per_row);
        if (lane == 0) {
            out[row] = acc;
            if (sj.score) sj.score[row] = s1 * __builtin_sqrtf(acc);
        }
    }
}

// The pass over X replaced by a pass over its cached row norms: xsq_forward holds sum_k X[t,k]^2
// of EVERY row (taken when X was produced, e.g. in the forward pass, by the kernel above).  Writes
// what row_sumsq_kernel with a ScoreJob writes, bit for bit: xsq (0 on dropped samples), the
// SampleW score ((1/p_i) * sqrt(gsq_t)) * sqrt(xsq_t) (0 on dropped samples), and the uniforms.
__global__ __launch_bounds__(256) void cached_xsq_scores_kernel(const float *__restrict__ xsq_forward, int64_t R, int T,
                                                                const uint8_t *__restrict__ sample_keep,
                                                                float *__restrict__ xsq, UniformJob job, ScoreJob sj)
{
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= R) return;
    if (job.uniforms) {
        const uint32_t draw = job.draw + (job.draw_offset ? *job.draw_offset : 0u);
        job.uniforms[r] = philox_uniform(job.seed, job.layer, job.stream_id, draw, (uint32_t)r);
    }
    const int64_t i = r / T;
    if (sample_keep[i] == 0) {
        xsq[r] = 0.0f;
        sj.score[r] = 0.0f;
        return;
    }
    const float inv = 1.0f / sj.p[i];
    const float s1 = inv * __builtin_sqrtf(sj.gsq[r]);
    const float acc = xsq_forward[r];
    xsq[r] = acc;
    sj.score[r] = s1 * __builtin_sqrtf(acc);
}

template <bool BF16, int CH>
__global__ __launch_bounds__(256) void row_sumsq_kernel(const uint4 *__restrict__ A, int64_t R, int groups_per_row,
                                                        int T, const uint8_t *__restrict__ sample_keep,
                                                        float *__restrict__ out, UniformJob job, ScoreJob sj)
{
    row_sumsq_body<BF16, CH>(A, R, groups_per_row, T, sample_keep, out, job, sj);
}

// The same, side jobs included, for several matrices of one shape: blockIdx.y picks the matrix.
template <bool BF16, int CH>
__global__ __launch_bounds__(256) void row_sumsq_jobs_group_kernel(RowJobGroup grp, int64_t R, int groups_per_row,
                                                                   int T)
{
    const int z = blockIdx.y;
    row_sumsq_body<BF16, CH>(grp.A[z], R, groups_per_row, T, grp.keep[z], grp.out[z], grp.job[z], grp.sj[z]);
}

// row_sumsq_kernel (without the side jobs) for several matrices of one shape in one launch:
// blockIdx.y picks the matrix.
template <bool BF16, int CH>
__global__ __launch_bounds__(256) void row_sumsq_group_kernel(RowNormGroup grp, int64_t R, int groups_per_row, int T)
{
    const uint4 *__restrict__ A = grp.A[blockIdx.y];
    float *__restrict__ out = grp.out[blockIdx.y];
    const uint8_t *__restrict__ sample_keep = grp.keep[blockIdx.y];
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t row = wave; row < R; row += nwaves) {
        const bool skip = sample_keep && sample_keep[row / T] == 0;
        const float acc = skip ? 0.0f : wave_row_sumsq<BF16, CH>(A + row * groups_per_row, groups_per_row);
        if (lane == 0) out[row] = acc;
    }
}

// (keep_a, T: as sample_keep above, for the rows of A only.)
// Row norms of two matrices with the same number of rows in one launch (G and X
// of a layer when both are small enough that a second launch would cost more
// than reading the rows of X that SampleA is about to drop): wavefronts
// [0, R) take the rows of A, [R, 2R) the rows of B.
template <bool BF16, int CH>
__global__ __launch_bounds__(256) void row_sumsq_pair_kernel(const uint4 *__restrict__ A, int groups_a,
                                                             float *__restrict__ out_a, const uint4 *__restrict__ B,
                                                             int groups_b, float *__restrict__ out_b, int64_t R,
                                                             UniformJob job, float *__restrict__ root_a,
                                                             float *__restrict__ root_b, int T,
                                                             const uint8_t *__restrict__ keep_a)
{
    if (job.uniforms) {
        const uint32_t draw = job.draw + (job.draw_offset ? *job.draw_offset : 0u);
        for (int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x; r < R; r += (int64_t)gridDim.x * 256)
            job.uniforms[r] = philox_uniform(job.seed, job.layer, job.stream_id, draw, (uint32_t)r);
    }
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t w = wave; w < 2 * R; w += nwaves) {
        const bool second = w >= R;
        const int64_t row = second ? w - R : w;
        const int groups = second ? groups_b : groups_a;
        // rows of A that belong to samples with keep_a == 0 are not read and count as zero
        const bool skip = !second && keep_a && keep_a[row / T] == 0;
        const float acc = skip ? 0.0f : wave_row_sumsq<BF16, CH>((second ? B : A) + row * groups, groups);
        if (lane == 0) {
            (second ? out_b : out_a)[row] = acc;
            // the square roots SampleW multiplies, taken here by many workgroups (null: not wanted)
            float *root = second ? root_b : root_a;
            if (root) root[row] = __builtin_sqrtf(acc);
        }
    }
}

// Row sums of squares from the sums of squares of their 64-column blocks (what the dgrad epilogue
// emits for the dX it has just written), added pairwise, neighbours first: the upper levels of the
// same tree a sweep over the row forms.  Layout: four neighbouring blocks of a row lie side by
// side, blocks[((b / 4) * R + row) * 4 + b % 4], b < nb = ceil(K/64), so that a thread fetches
// 16 bytes at a time and neighbouring threads (neighbouring rows) fetch neighbouring 16 bytes; the
// slots b >= nb of the last group are never written and never used.  Rows of samples whose
// sample_keep byte is 0 are not read and get 0.  Up to kMaxSiblings outputs receive the same values
// (sibling layers share their G).
struct RowsFromBlocks {
    float *out[kMaxSiblings];
    float *gnorm[kMaxSiblings];   // sample norms too (sample_norms_from_blocks_kernel only)
};

// The leaves first + 4 * g0 .. of one row, groups g0 <= g < g1, pushed in order (eight loads in flight).
__device__ __forceinline__ float block_subtree(const float4 *__restrict__ blocks4, int64_t R, int64_t row, int g0, int g1,
                                               int nb)
{
    PairwiseStream<12> leaves;
    for (int g = g0; g < g1; g += 8) {
        float4 v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            v[k] = g + k < g1 ? blocks4[(int64_t)(g + k) * R + row] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int b = 4 * (g + k);
            if (g + k < g1) {
                leaves.push(v[k].x);
                if (b + 1 < nb) leaves.push(v[k].y);
                if (b + 2 < nb) leaves.push(v[k].z);
                if (b + 3 < nb) leaves.push(v[k].w);
            }
        }
    }
    return leaves.finish();
}

__global__ __launch_bounds__(256) void rows_from_blocks_kernel(const float4 *__restrict__ blocks4, int64_t R, int nb,
                                                               int T, const uint8_t *__restrict__ sample_keep,
                                                               RowsFromBlocks outs, int n_out)
{
    // 32 rows per workgroup, eight threads per row: thread (row, part) adds an aligned run of
    // groups (a power of two of them), i.e. one subtree of the row's tree; the eight subtree sums
    // meet in LDS and are added as the top three levels.
    __shared__ float part_sum[8][32];
    const int r_local = threadIdx.x & 31, part = threadIdx.x >> 5;
    const int64_t row = (int64_t)blockIdx.x * 32 + r_local;
    const int groups = (nb + 3) >> 2;
    int Gp = 1;
    while (Gp < groups) Gp *= 2;
    const int chunk = Gp >= 8 ? Gp / 8 : 1;
    const bool live = row < R && (!sample_keep || sample_keep[row / T] != 0);
    float acc = 0.0f;
    if (live && part * chunk < groups) acc = block_subtree(blocks4, R, row, part * chunk, min(groups, (part + 1) * chunk), nb);
    part_sum[part][r_local] = acc;
    __syncthreads();
    if (part == 0 && row < R) {
        const float total = ((part_sum[0][r_local] + part_sum[1][r_local]) + (part_sum[2][r_local] + part_sum[3][r_local])) +
                            ((part_sum[4][r_local] + part_sum[5][r_local]) + (part_sum[6][r_local] + part_sum[7][r_local]));
        for (int k = 0; k < n_out; ++k) outs.out[k][row] = live ? total : 0.0f;
    }
}

// The same, and the sample norms ||G_i||_F = sqrt(sum of the sample's row sums) (Sec. 4.1) behind
// them: one workgroup of 1024 threads per sample (T <= 1024 rows), `parts` threads per row.  The
// row sums stay in LDS for the norm, which one wavefront adds in the order of sample_norm_wave
// (value t on lane t mod 64, ascending t, exchange tree).  The chain row norms -> SampleA -> dX of
// a layer inside a stack is then this launch and a dgrad that decides SampleA itself.
__global__ __launch_bounds__(1024) void sample_norms_from_blocks_kernel(const float4 *__restrict__ blocks4, int64_t R, int nb,
                                                                        int T, const uint8_t *__restrict__ sample_keep,
                                                                        RowsFromBlocks outs, int n_out)
{
    __shared__ float part_sum[1024];
    __shared__ float row_total[1024];
    const int i = blockIdx.x, tid = threadIdx.x;
    const bool live = !sample_keep || sample_keep[i] != 0;
    const int groups = (nb + 3) >> 2;
    int Gp = 1;
    while (Gp < groups) Gp *= 2;
    int parts = 1;
    while (parts < 16 && parts * 2 * T <= 1024 && parts * 2 <= Gp) parts *= 2;
    const int chunk = Gp / parts;
    const int r = tid % T, part = tid / T;
    const int64_t row = (int64_t)i * T + r;
    float acc = 0.0f;
    if (live && part < parts && part * chunk < groups)
        acc = block_subtree(blocks4, R, row, part * chunk, min(groups, (part + 1) * chunk), nb);
    part_sum[tid] = acc;
    __syncthreads();
    if (part == 0) {
        // the parts of a row, pairwise (parts is a power of two, at most 16 with Gp >= parts)
        float v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = k < parts ? part_sum[r + k * T] : 0.0f;
#pragma unroll
        for (int n = 16; n > 1; n /= 2)
#pragma unroll
            for (int k = 0; k < n / 2; ++k) v[k] = v[2 * k] + v[2 * k + 1];
        const float total = live ? v[0] : 0.0f;
        row_total[r] = total;
        for (int k = 0; k < n_out; ++k) outs.out[k][row] = total;
    }
    __syncthreads();
    if (tid < 64) {
        float sum = 0.0f;
        for (int t = tid; t < T; t += 64) sum = sum + row_total[t];
        const float norm = __builtin_sqrtf(wave_exchange_sum(sum));
        if (tid == 0)
            for (int k = 0; k < n_out; ++k) outs.gnorm[k][i] = norm;
    }
}

// outs: n_out <= kMaxSiblings arrays of R floats
vcas_status rows_from_blocks(const float *blocks, int64_t R, int K, int T, const uint8_t *keep, float *const *outs,
                             int n_out, hipStream_t st)
{
    if (n_out < 1 || n_out > kMaxSiblings) return VCAS_EINVAL;
    RowsFromBlocks o = {};
    for (int k = 0; k < n_out; ++k) o.out[k] = outs[k];
    hipLaunchKernelGGL(rows_from_blocks_kernel, dim3((unsigned)((R + 31) / 32)), dim3(256), 0, st,
                       reinterpret_cast<const float4 *>(blocks), R, (K + 63) / 64, T, keep, o, n_out);
    return launch_status();
}

// True where sample_norms_from_blocks applies.
bool sample_norms_from_blocks_fits(int N, int T) { return T <= 1024 && N >= 1; }

// Row sums (outs) and sample norms (gnorms) of N samples of T <= 1024 rows from the block sums.
vcas_status sample_norms_from_blocks(const float *blocks, int N, int T, int K, const uint8_t *keep, float *const *outs,
                                     float *const *gnorms, int n_out, hipStream_t st)
{
    if (n_out < 1 || n_out > kMaxSiblings || !sample_norms_from_blocks_fits(N, T)) return VCAS_EINVAL;
    RowsFromBlocks o = {};
    for (int k = 0; k < n_out; ++k) {
        o.out[k] = outs[k];
        o.gnorm[k] = gnorms[k];
    }
    hipLaunchKernelGGL(sample_norms_from_blocks_kernel, dim3((unsigned)N), dim3(1024), 0, st,
                       reinterpret_cast<const float4 *>(blocks), (int64_t)N * T, (K + 63) / 64, T, keep, o, n_out);
    return launch_status();
}

// ||G_i||_F: value t of a sample belongs to lane t mod 64, plain fp32 adds in
// ascending t, exchange steps, correctly rounded sqrt.  One wavefront per sample.
__global__ __launch_bounds__(256) void sample_norm_kernel(const float *__restrict__ gsq, int N, int T,
                                                          float *__restrict__ gnorm)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= N) return;
    const float *p = gsq + (int64_t)i * T;
    float acc = 0.0f;
    for (int t = lane; t < T; t += 64) acc = acc + p[t];
    acc = wave_exchange_sum(acc);
    if (lane == 0) gnorm[i] = __builtin_sqrtf(acc);
}

template <bool BF16>
static vcas_status launch_row_sumsq(const void *A, int64_t R, int K, int T, const uint8_t *keep, float *out,
                                    const UniformJob &job, const ScoreJob &sj, hipStream_t st)
{
    const int groups = K / (BF16 ? 8 : 4);
    const int need = (groups + 63) / 64;
    int64_t blocks64 = (R + 3) / 4;
    const int blocks = (int)(blocks64 < 4096 ? blocks64 : 4096);
    const uint4 *a = static_cast<const uint4 *>(A);
#define VCAS_LAUNCH_CH(C) \
    hipLaunchKernelGGL((row_sumsq_kernel<BF16, C>), dim3(blocks), dim3(256), 0, st, a, R, groups, T, keep, out, job, sj)
    if (need <= 1) VCAS_LAUNCH_CH(1);
    else if (need <= 2) VCAS_LAUNCH_CH(2);
    else if (need <= 3) VCAS_LAUNCH_CH(3);
    else if (need <= 4) VCAS_LAUNCH_CH(4);
    else if (need <= 6) VCAS_LAUNCH_CH(6);
    else VCAS_LAUNCH_CH(8);
#undef VCAS_LAUNCH_CH
    return launch_status();
}

template <bool BF16>
static vcas_status launch_row_sumsq_group(const RowNormGroup &grp, int n, int64_t R, int K, int T, hipStream_t st)
{
    const int groups = K / (BF16 ? 8 : 4);
    const int need = (groups + 63) / 64;
    int64_t blocks64 = (R + 3) / 4;
    const int blocks = (int)(blocks64 < 4096 ? blocks64 : 4096);
#define VCAS_LAUNCH_CH(C) \
    hipLaunchKernelGGL((row_sumsq_group_kernel<BF16, C>), dim3(blocks, n), dim3(256), 0, st, grp, R, groups, T)
    if (need <= 1) VCAS_LAUNCH_CH(1);
    else if (need <= 2) VCAS_LAUNCH_CH(2);
    else if (need <= 3) VCAS_LAUNCH_CH(3);
    else if (need <= 4) VCAS_LAUNCH_CH(4);
    else if (need <= 6) VCAS_LAUNCH_CH(6);
    else VCAS_LAUNCH_CH(8);
#undef VCAS_LAUNCH_CH
    return launch_status();
}

// row_sumsq_scores_uniforms for n <= kMaxSiblings layers of one shape in one launch
vcas_status row_sumsq_scores_uniforms_group(const RowJobGroup &grp, int n, int dtype, int64_t R, int K, int T,
                                            hipStream_t st)
{
    if (n < 1 || n > kMaxSiblings) return VCAS_EINVAL;
    const bool bf = dtype == VCAS_BF16;
    const int groups = K / (bf ? 8 : 4);
    const int need = (groups + 63) / 64;
    int64_t blocks64 = (R + 3) / 4;
    const int blocks = (int)(blocks64 < 4096 ? blocks64 : 4096);
#define VCAS_LAUNCH_CH(B, C) \
    hipLaunchKernelGGL((row_sumsq_jobs_group_kernel<B, C>), dim3(blocks, n), dim3(256), 0, st, grp, R, groups, T)
#define VCAS_LAUNCH_DT(C)          \
    do {                           \
        if (bf) VCAS_LAUNCH_CH(true, C); \
        else VCAS_LAUNCH_CH(false, C);   \
    } while (0)
    if (need <= 1) VCAS_LAUNCH_DT(1);
    else if (need <= 2) VCAS_LAUNCH_DT(2);
    else if (need <= 3) VCAS_LAUNCH_DT(3);
    else if (need <= 4) VCAS_LAUNCH_DT(4);
    else if (need <= 6) VCAS_LAUNCH_DT(6);
    else VCAS_LAUNCH_DT(8);
#undef VCAS_LAUNCH_DT
#undef VCAS_LAUNCH_CH
    return launch_status();
}

// row_sumsq for n <= kMaxSiblings matrices [R, K] in one launch
vcas_status row_sumsq_group(const RowNormGroup &grp, int n, int dtype, int64_t R, int K, int T, hipStream_t st)
{
    if (n < 1 || n > kMaxSiblings) return VCAS_EINVAL;
    return dtype == VCAS_BF16 ? launch_row_sumsq_group<true>(grp, n, R, K, T, st)
                              : launch_row_sumsq_group<false>(grp, n, R, K, T, st);
}

vcas_status row_sumsq(const void *A, int dtype, int64_t R, int K, int T, const uint8_t *keep, float *out,
                      hipStream_t st)
{
    const UniformJob none = {nullptr, 0, 0, 0, 0, nullptr};
    const ScoreJob no_score = {nullptr, nullptr, nullptr};
    return dtype == VCAS_BF16 ? launch_row_sumsq<true>(A, R, K, T, keep, out, none, no_score, st)
                              : launch_row_sumsq<false>(A, R, K, T, keep, out, none, no_score, st);
}

// row norms of X on kept samples, the SampleW scores and the uniforms of sampler `stream_id`
// (null: none) in one launch
vcas_status row_sumsq_scores_uniforms(const void *X, int dtype, int64_t R, int K, int T, const uint8_t *keep,
                                      float *xsq, const float *gsq, const float *p, float *score, const vcas_rng &rng,
                                      uint32_t stream_id, float *uniforms, hipStream_t st)
{
    const UniformJob job = {uniforms, rng.seed, rng.layer, stream_id, rng.draw, rng.draw_offset};
    const ScoreJob sj = {gsq, p, score};
    return dtype == VCAS_BF16 ? launch_row_sumsq<true>(X, R, K, T, keep, xsq, job, sj, st)
                              : launch_row_sumsq<false>(X, R, K, T, keep, xsq, job, sj, st);
}

// row_sumsq_scores_uniforms without the sweep over X: its row norms come from xsq_forward
vcas_status cached_xsq_scores_uniforms(const float *xsq_forward, int64_t R, int T, const uint8_t *keep, float *xsq,
                                       const float *gsq, const float *p, float *score, const vcas_rng &rng,
                                       uint32_t stream_id, float *uniforms, hipStream_t st)
{
    const UniformJob job = {uniforms, rng.seed, rng.layer, stream_id, rng.draw, rng.draw_offset};
    const ScoreJob sj = {gsq, p, score};
    hipLaunchKernelGGL(cached_xsq_scores_kernel, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, xsq_forward, R, T,
                       keep, xsq, job, sj);
    return launch_status();
}

template <bool BF16>
static vcas_status launch_pair(const void *A, int K_a, float *out_a, const void *B, int K_b, float *out_b, int64_t R,
                               const UniformJob &job, float *root_a, float *root_b, int T, const uint8_t *keep_a,
                               hipStream_t st)
{
    const int ga = K_a / (BF16 ? 8 : 4), gb = K_b / (BF16 ? 8 : 4);
    const int need = ((ga > gb ? ga : gb) + 63) / 64;
    int64_t blocks64 = (2 * R + 3) / 4;
    const int blocks = (int)(blocks64 < 4096 ? blocks64 : 4096);
    const uint4 *a = static_cast<const uint4 *>(A), *b = static_cast<const uint4 *>(B);
#define VCAS_LAUNCH_CH(C)                                                                                         \
    hipLaunchKernelGGL((row_sumsq_pair_kernel<BF16, C>), dim3(blocks), dim3(256), 0, st, a, ga, out_a, b, gb, out_b, \
                       R, job, root_a, root_b, T, keep_a)
    if (need <= 2) VCAS_LAUNCH_CH(2);
    else if (need <= 4) VCAS_LAUNCH_CH(4);
    else VCAS_LAUNCH_CH(8);
#undef VCAS_LAUNCH_CH
    return launch_status();
}

// gsq of every row of G, xsq of EVERY row of X (the caller zeroes the rows of dropped samples
// later), their square roots (root_g, root_x; null: not wanted) and the uniforms of sampler
// `stream_id`, one launch; keep_g (null: all): samples whose rows of G are read at all
vcas_status row_sumsq_pair(const void *G, int K_out, float *gsq, const void *X, int K_in, float *xsq, int dtype,
                           int64_t R, const vcas_rng &rng, uint32_t stream_id, float *uniforms, float *root_g,
                           float *root_x, int T, const uint8_t *keep_g, hipStream_t st)
{
    const UniformJob job = {uniforms, rng.seed, rng.layer, stream_id, rng.draw, rng.draw_offset};
    return dtype == VCAS_BF16
               ? launch_pair<true>(G, K_out, gsq, X, K_in, xsq, R, job, root_g, root_x, T, keep_g, st)
               : launch_pair<false>(G, K_out, gsq, X, K_in, xsq, R, job, root_g, root_x, T, keep_g, st);
}

vcas_status sample_norms(const float *gsq, int N, int T, float *gnorm, hipStream_t st)
{
    hipLaunchKernelGGL(sample_norm_kernel, dim3((N + 3) / 4), dim3(256), 0, st, gsq, N, T, gnorm);
    return launch_status();
}

}  // namespace vcas
