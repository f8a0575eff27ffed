/*
 * VCAS CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step CPU statement of the sampled backward pass of a
 * linear layer Z = X W^T as the VCAS paper defines it (Sec. 4.1 SampleA,
 * Sec. 4.2 SampleW and Eq. 3).  It exists so that the GPU library can be
 * checked against something that can be read next to the paper.  It shares no
 * code with the GPU library, and nothing in the product path may call it:
 * only the tests, the smoke check and the benchmark's cpu-baseline leg do.
 *
 * Precision: the paper fixes none.  Everything that later decides an integer
 * (a kept / dropped bit) is evaluated in fp32 in one written-down order, the
 * same the GPU kernels follow, so that masks and index lists can be compared
 * bit for bit.  Both gradient contractions accumulate in fp64.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1 };

/* ------------------------------------------------------------------ dtypes */

static float bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* round-to-nearest-even fp32 -> bf16; NaN stays NaN */
static uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

static inline float elem(const void *base, int dtype, size_t i)
{
    if (dtype == ORC_BF16)
        return bf16_bits_to_f32(((const uint16_t *)base)[i]);
    return ((const float *)base)[i];
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Casts an fp64 result to the layer's storage type (fp32, or bf16 bits). */
void orc_cast_from_f64(const double *src, int64_t n, int dtype, void *dst)
{
    for (int64_t i = 0; i < n; ++i) {
        float f = (float)src[i];
        if (dtype == ORC_BF16)
            ((uint16_t *)dst)[i] = f32_to_bf16_bits(f);
        else
            ((float *)dst)[i] = f;
    }
}

void orc_bf16_to_f32(const uint16_t *src, int64_t n, float *dst)
{
    for (int64_t i = 0; i < n; ++i)
        dst[i] = bf16_bits_to_f32(src[i]);
}

/* ------------------------------------------------------------------ Philox */

/*
 * Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11, Sec. 3.3):
 * each round maps (c0,c1,c2,c3) to
 *   (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2), hi(M0*c0) ^ c3 ^ k1, lo(M0*c0))
 * and the key is bumped by the Weyl constants between rounds.
 */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * c0;
        uint64_t p1 = M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * The uniform that decides row `row`: 24 top bits of output word 0, scaled to
 * [0,1).  Counter = (row, layer, stream, draw); key = the 64-bit seed's halves.
 * The paper only says Bern(p; eps) (Sec. 4.1); this is the fixed reading.
 */
float orc_uniform(uint64_t seed, uint32_t layer, uint32_t stream, uint32_t draw, uint32_t row)
{
    uint32_t ctr[4] = { row, layer, stream, draw };
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return (float)(out[0] >> 8) * 0x1.0p-24f;
}

/* ------------------------------------------------- norms (Sec. 4.1 / 4.2) */

/*
 * fp32 sum in the written-down "64-lane" order (the per-sample sums): value j
 * of the sequence goes to accumulator j mod 64, accumulators add their values
 * in ascending j, then six pairwise exchange steps (distance 1,2,4,...,32) add
 * accumulator l and l^distance, i.e. neighbours first.
 */
static float lane_sum(const float *v, int count)
{
    float acc[64];
    for (int l = 0; l < 64; ++l)
        acc[l] = 0.0f;
    for (int j = 0; j < count; ++j)
        acc[j % 64] = acc[j % 64] + v[j];
    for (int dist = 1; dist <= 32; dist <<= 1) {
        float nxt[64];
        for (int l = 0; l < 64; ++l)
            nxt[l] = acc[l] + acc[l ^ dist];
        memcpy(acc, nxt, sizeof acc);
    }
    return acc[0];
}

/*
 * Pairwise summation, neighbours first: the n values, padded with +0 to the
 * next power of two, are added as a balanced binary tree in index order.
 * v is overwritten; room for the padded length.
 */
static float pairwise_sum_f32(float *v, int n)
{
    int len = 1;
    while (len < n)
        len *= 2;
    for (int j = n; j < len; ++j)
        v[j] = 0.0f;
    for (; len > 1; len /= 2)
        for (int j = 0; j < len / 2; ++j)
            v[j] = v[2 * j] + v[2 * j + 1];
    return v[0];
}

/*
 * Squared 2-norm of every row t of A[R,K] (the ||g_t||^2 and ||x_t||^2 of
 * Eq. 3, the row sums behind the ||G_i||_F of Sec. 4.1), fp32: the squares
 * v*v (one rounding each) summed pairwise, neighbours first.  The paper fixes
 * no order; this is the written-down one.  If sample_keep is given (one byte
 * per sample of T rows), rows of dropped samples get 0.
 */
void orc_row_sumsq(const void *A, int dtype, int64_t R, int K, int T,
                   const uint8_t *sample_keep, float *out)
{
    int len = 1;
    while (len < K)
        len *= 2;
    float *sq = (float *)malloc((size_t)len * sizeof(float));
    for (int64_t t = 0; t < R; ++t) {
        if (sample_keep && !sample_keep[t / T]) {
            out[t] = 0.0f;
            continue;
        }
        for (int k = 0; k < K; ++k) {
            float v = elem(A, dtype, (size_t)t * K + k);
            sq[k] = v * v;
        }
        out[t] = pairwise_sum_f32(sq, K);
    }
    free(sq);
}

/*
 * The same row sums in two stages, the way a layer inside a stack gets them
 * from the launch that wrote the matrix (Sec. 4: a sampler at every layer needs
 * the norms of the gradient the layer above has just produced): first the sum of
 * squares of every block of `width` consecutive columns (width a power of two;
 * pairwise, neighbours first; a last, shorter block is padded with +0),
 * blocks[t * nb + b], nb = ceil(K/width); then, per row, the nb block sums
 * pairwise, neighbours first.  Both stages are subtrees of the one tree
 * orc_row_sumsq forms, so the results are its bits, whatever the width.
 */
void orc_block_sumsq(const void *A, int dtype, int64_t R, int K, int width, float *blocks)
{
    int nb = (K + width - 1) / width;
    float *sq = (float *)malloc((size_t)width * sizeof(float));
    for (int64_t t = 0; t < R; ++t)
        for (int b = 0; b < nb; ++b) {
            int n = K - width * b < width ? K - width * b : width;
            for (int k = 0; k < n; ++k) {
                float v = elem(A, dtype, (size_t)t * K + (size_t)width * b + k);
                sq[k] = v * v;
            }
            blocks[t * nb + b] = pairwise_sum_f32(sq, n);
        }
    free(sq);
}

void orc_rows_from_blocks(const float *blocks, int64_t R, int nb, int T, const uint8_t *sample_keep, float *out)
{
    int len = 1;
    while (len < nb)
        len *= 2;
    float *v = (float *)malloc((size_t)len * sizeof(float));
    for (int64_t t = 0; t < R; ++t) {
        if (sample_keep && !sample_keep[t / T]) {
            out[t] = 0.0f;
            continue;
        }
        memcpy(v, blocks + t * nb, (size_t)nb * sizeof(float));
        out[t] = pairwise_sum_f32(v, nb);
    }
    free(v);
}

/* The same quantity by its plain definition in fp64 (used to pin the above). */
void orc_row_sumsq_f64(const void *A, int dtype, int64_t R, int K, double *out)
{
    for (int64_t t = 0; t < R; ++t) {
        double s = 0.0;
        for (int k = 0; k < K; ++k) {
            double v = elem(A, dtype, (size_t)t * K + k);
            s += v * v;
        }
        out[t] = s;
    }
}

/* ||G_i||_F of every sample i from its T row sums (Sec. 4.1). */
void orc_sample_norms(const float *gsq, int N, int T, float *gnorm)
{
    for (int i = 0; i < N; ++i)
        gnorm[i] = sqrtf(lane_sum(gsq + (size_t)i * T, T));
}

/* --------------------------- keep probabilities (Sec. 4.1, Sec. 4.2) */

/* fp64 sum in the written-down "1024-slot" order: slot = i mod 1024, ascending
 * inside a slot; each run of 64 consecutive slots is reduced by adding
 * neighbours pairwise, (0,1), (2,3), ..., then the pair sums pairwise, and so
 * on; the 16 run sums are then reduced the same way. */
static double pairwise_tree(double *v, int n)
{
    for (; n > 1; n /= 2)
        for (int j = 0; j < n / 2; ++j)
            v[j] = v[2 * j] + v[2 * j + 1];
    return v[0];
}

static double slot_sum(const double *v, int n)
{
    double part[1024], run[16];
    for (int s = 0; s < 1024; ++s)
        part[s] = 0.0;
    for (int i = 0; i < n; ++i)
        part[i % 1024] += v[i];
    for (int r = 0; r < 16; ++r)
        run[r] = pairwise_tree(part + 64 * r, 64);
    return pairwise_tree(run, 16);
}

/*
 * Keep probabilities proportional to `score`, summing to `budget`, none above
 * one: p_i = min(1, c * score_i).  The paper states p_i proportional to the
 * norm with sum N*rho (Sec. 4.1) resp. q_i proportional to the leverage score
 * with sum N*T*rho*nu (Sec. 4.2) and is silent on p > 1; minimising
 * sum score_i^2 / p_i under 0 < p_i <= 1 gives this capped form.  c is found
 * by repeatedly fixing at one every entry that the current c pushes to >= 1.
 * Zero scores get probability zero and the budget is clipped to the number of
 * positive scores.  Returns the number of rounds taken.
 */
int orc_keep_probs(const float *score, int n, double budget, float *prob)
{
    double *live = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    uint8_t *capped = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);
    int nonzero = 0;
    for (int i = 0; i < n; ++i)
        if (score[i] > 0.0f)
            ++nonzero;
    int rounds = 0;
    double c = 0.0;
    if (budget >= (double)nonzero) {
        for (int i = 0; i < n; ++i)
            capped[i] = score[i] > 0.0f;
    } else {
        int ncap = 0;
        for (;;) {
            ++rounds;
            for (int i = 0; i < n; ++i)
                live[i] = (!capped[i] && score[i] > 0.0f) ? (double)score[i] : 0.0;
            double S = slot_sum(live, n);
            double rem = budget - (double)ncap;
            if (!(S > 0.0) || !(rem > 0.0)) {
                c = 0.0;
                break;
            }
            c = rem / S;
            int newly = 0;
            for (int i = 0; i < n; ++i)
                if (!capped[i] && score[i] > 0.0f && c * (double)score[i] >= 1.0) {
                    capped[i] = 1;
                    ++newly;
                }
            if (newly == 0)
                break;
            ncap += newly;
        }
    }
    for (int i = 0; i < n; ++i) {
        if (capped[i])
            prob[i] = 1.0f;
        else if (score[i] > 0.0f) {
            float p = (float)(c * (double)score[i]);
            prob[i] = p < 1.0f ? p : 1.0f;
        } else
            prob[i] = 0.0f;
    }
    free(live);
    free(capped);
    return rounds;
}

/* ------------------------------------------------- Bernoulli masks + lists */

/*
 * keep_r = [u_r < prob_r] with u_r the Philox uniform of row r; idx lists the
 * kept rows in ascending order.  Returns the kept count.
 */
int orc_sample_mask(const float *prob, int n, uint64_t seed, uint32_t layer, uint32_t stream,
                    uint32_t draw, uint8_t *mask, int32_t *idx)
{
    int count = 0;
    for (int r = 0; r < n; ++r) {
        float u = orc_uniform(seed, layer, stream, draw, (uint32_t)r);
        mask[r] = u < prob[r] ? 1 : 0;
        if (mask[r])
            idx[count++] = r;
    }
    return count;
}

/*
 * Leverage score of token t of sample i (Sec. 4.2): ||ghat_t|| * ||x_t|| where
 * ghat = SampleA(G) already carries m_i / p_i.  fp32, in this association.
 */
void orc_leverage_scores(const float *gsq, const float *xsq, const float *p, const uint8_t *maskA,
                         int N, int T, float *score)
{
    for (int i = 0; i < N; ++i)
        for (int t = 0; t < T; ++t) {
            size_t r = (size_t)i * T + t;
            if (!maskA[i]) {
                score[r] = 0.0f;
                continue;
            }
            float inv = 1.0f / p[i];
            float a = inv * sqrtf(gsq[r]);
            score[r] = a * sqrtf(xsq[r]);
        }
}

/* Factor m_i m_t = 1 / (p_i q_t) that a kept token's outer product carries
 * in the weight gradient (Sec. 4.1 and 4.2 masks multiplied); 0 if dropped. */
void orc_row_scale(const float *p, const float *q, const uint8_t *maskW, int N, int T, float *scale)
{
    for (int i = 0; i < N; ++i)
        for (int t = 0; t < T; ++t) {
            size_t r = (size_t)i * T + t;
            scale[r] = maskW[r] ? 1.0f / (p[i] * q[r]) : 0.0f;
        }
}

/* --------------------------------------------------------------- gradients */

/*
 * Activation gradient (Eq. 2 upper line with h = multiplication by W):
 * dX[r,:] = (m_i / p_i) * sum_o G[r,o] W[o,:] for r in sample i; fp64.
 */
void orc_dgrad(const void *G, const void *W, int dtype, int N, int T, int K_in, int K_out,
               const float *p, const uint8_t *maskA, double *dX)
{
    int64_t R = (int64_t)N * T;
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t r = 0; r < R; ++r) {
        double *row = dX + (size_t)r * K_in;
        for (int k = 0; k < K_in; ++k)
            row[k] = 0.0;
        int i = (int)(r / T);
        if (!maskA[i])
            continue;
        for (int o = 0; o < K_out; ++o) {
            double g = elem(G, dtype, (size_t)r * K_out + o);
            for (int k = 0; k < K_in; ++k)
                row[k] += g * (double)elem(W, dtype, (size_t)o * K_in + k);
        }
        double m = 1.0 / (double)p[i];
        for (int k = 0; k < K_in; ++k)
            row[k] *= m;
    }
}

/*
 * Weight gradient (Sec. 4.2): dW = Gtilde^T X = sum_t scale_t g_t x_t^T over
 * rows with scale_t != 0, taken in ascending t; fp64.
 */
void orc_wgrad(const void *G, const void *X, int dtype, int64_t R, int K_in, int K_out,
               const float *scale, double *dW)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int o = 0; o < K_out; ++o) {
        double *row = dW + (size_t)o * K_in;
        for (int k = 0; k < K_in; ++k)
            row[k] = 0.0;
        for (int64_t t = 0; t < R; ++t) {
            if (scale[t] == 0.0f)
                continue;
            double g = (double)scale[t] * (double)elem(G, dtype, (size_t)t * K_out + o);
            for (int k = 0; k < K_in; ++k)
                row[k] += g * (double)elem(X, dtype, (size_t)t * K_in + k);
        }
    }
}

/* Single entries of the two gradients, for spot checks at sizes where the
 * full contraction is too slow: coordinates are (row, col) pairs. */
void orc_dgrad_at(const void *G, const void *W, int dtype, int T, int K_in, int K_out,
                  const float *p, const uint8_t *maskA, const int64_t *rows, const int32_t *cols,
                  int64_t count, double *out)
{
    for (int64_t j = 0; j < count; ++j) {
        int64_t r = rows[j];
        int i = (int)(r / T);
        double s = 0.0;
        if (maskA[i]) {
            for (int o = 0; o < K_out; ++o)
                s += (double)elem(G, dtype, (size_t)r * K_out + o) *
                     (double)elem(W, dtype, (size_t)o * K_in + cols[j]);
            s *= 1.0 / (double)p[i];
        }
        out[j] = s;
    }
}

void orc_wgrad_at(const void *G, const void *X, int dtype, int64_t R, int K_in, int K_out,
                  const float *scale, const int32_t *orow, const int32_t *kcol, int64_t count,
                  double *out)
{
#pragma omp parallel for
    for (int64_t j = 0; j < count; ++j) {
        double s = 0.0;
        for (int64_t t = 0; t < R; ++t) {
            if (scale[t] == 0.0f)
                continue;
            s += (double)scale[t] * (double)elem(G, dtype, (size_t)t * K_out + orow[j]) *
                 (double)elem(X, dtype, (size_t)t * K_in + kcol[j]);
        }
        out[j] = s;
    }
}

/* --------------------------------------------------------------- variances */

/* Var[Ghat] = sum_i (1 - p_i)/p_i ||G_i||_F^2 (Sec. 4.1), over p_i > 0. */
double orc_var_act_closed(const float *p, const float *gnorm, int N)
{
    double v = 0.0;
    for (int i = 0; i < N; ++i)
        if (p[i] > 0.0f) {
            double pi = p[i], ni = gnorm[i];
            v += (1.0 - pi) / pi * ni * ni;
        }
    return v;
}

/* Eq. 3: Var[dW | data mask] = sum_t (1 - q_t)/q_t ||ghat_t||^2 ||x_t||^2,
 * with score_t = ||ghat_t|| ||x_t||, over q_t > 0. */
double orc_var_w_eq3(const float *q, const float *score, int64_t R)
{
    double v = 0.0;
    for (int64_t t = 0; t < R; ++t)
        if (q[t] > 0.0f) {
            double qt = q[t], st = score[t];
            v += (1.0 - qt) / qt * st * st;
        }
    return v;
}

/* ||a - b||_F^2 in fp64 (the squared differences of Alg. 1's V_act line). */
double orc_sq_diff(const double *a, const double *b, int64_t n)
{
    double v = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double d = a[i] - b[i];
        v += d * d;
    }
    return v;
}

/* ------------------------------------------- adaptive keep ratios (Sec. 5) */

static int cmp_desc(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x < y) - (x > y);
}

/* Eq. 4: the gradient-norm sparsity of a layer at level s,
 *   p(s) = min { n/N : sum of the n LARGEST norms >= s * sum of all norms },  n >= 1.
 * The paper does not say "largest"; a sparsity measure needs the norms in
 * descending order.  Sums run in fp64 over the sorted sequence, one after the
 * other, so the last prefix equals the total and n = N always qualifies. */
float orc_sparsity_ratio(const float *gnorm, int N, double s)
{
    float *v = (float *)malloc(sizeof(float) * (size_t)N);
    memcpy(v, gnorm, sizeof(float) * (size_t)N);
    qsort(v, (size_t)N, sizeof(float), cmp_desc);
    double total = 0.0;
    for (int i = 0; i < N; ++i) total += (double)v[i];
    const double target = s * total;
    double prefix = 0.0;
    int n = N;
    for (int i = 0; i < N; ++i) {
        prefix += (double)v[i];
        if (prefix >= target) {
            n = i + 1;
            break;
        }
    }
    free(v);
    return (float)n / (float)N;
}

/* Running mean and running mean of squares of a strided subset of a gradient
 * (App. D keeps exactly these two tensors for the SGD variance V_s): after the
 * call with 1-based index i they hold the statistics of gradients 1..i.
 *   mean   <- mean   + (x   - mean)   / i
 *   sqmean <- sqmean + (x*x - sqmean) / i        (fp32, each operation rounded) */
void orc_grad_stats_update(const float *grad, int64_t m, int64_t stride, int i, float *mean, float *sqmean)
{
    const float fi = (float)i;
    for (int64_t j = 0; j < m; ++j) {
        const float x = grad[j * stride];
        const float d = x - mean[j];
        mean[j] = mean[j] + d / fi;
        const float xx = x * x;
        const float e = xx - sqmean[j];
        sqmean[j] = sqmean[j] + e / fi;
    }
}

/* Alg. 1's V_s from the two running tensors of M gradients:
 *   1/(M-1) sum_i ||g_i - gbar||^2 = M/(M-1) sum_j (sqmean_j - mean_j^2),  fp64. */
double orc_grad_stats_variance(const float *mean, const float *sqmean, int64_t m, int M)
{
    double v = 0.0;
    for (int64_t j = 0; j < m; ++j) v += (double)sqmean[j] - (double)mean[j] * (double)mean[j];
    return v * (double)M / (double)(M - 1);
}

/* ||a - b||^2 over the same strided subset (Alg. 1's V_act line on the kept parameters). */
double orc_sq_diff_strided(const float *a, const float *b, int64_t m, int64_t stride)
{
    double v = 0.0;
    for (int64_t j = 0; j < m; ++j) {
        const double d = (double)a[j * stride] - (double)b[j * stride];
        v += d * d;
    }
    return v;
}
