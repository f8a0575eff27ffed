// Adaptive keep ratios (Sec. 5 of the VCAS paper): the device pieces of one
// update of Alg. 1 -- Eq. 4's gradient-norm sparsity, the running statistics of
// the SGD gradient that App. D keeps for V_s, the squared difference of V_act on
// a parameter subset -- and the host-side update rules (Eq. 5, Eq. 4's running
// maximum, Eq. 7).  These run once every F iterations on vectors of N floats and
// on about 1 % of a layer's parameters: latency, not bandwidth.
#include <math.h>

#include "common.hpp"

namespace vcas {

constexpr int kMaxLevels = 8;

struct Levels {
    double s[kMaxLevels];
    int n;
};

// p(s) = min { n/N : sum of the n largest norms >= s * sum of all }, n >= 1, for up to
// kMaxLevels values of s.  One workgroup: bitonic sort (descending) of the norms in LDS, then
// thread j walks the sorted norms for level j, adding them in fp64 one after the other (first
// for the total, then for the prefixes: the last prefix IS the total, so n = N always
// qualifies).  Equal norms may come out in any order; the sums do not depend on it.
__global__ __launch_bounds__(1024) void sparsity_kernel(const float *__restrict__ gnorm, int N, Levels lv,
                                                        float *__restrict__ out)
{
    __shared__ float v[1024];
    const int tid = threadIdx.x;
    v[tid] = tid < N ? gnorm[tid] : -1.0f;   // padding sorts behind every norm (they are >= 0)
    __syncthreads();
    int P = 1;                               // the sort network only spans the next power of two
    while (P < N) P <<= 1;
    for (int k = 2; k <= P; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            const int other = tid ^ j;
            if (other > tid && other < P) {
                const float a = v[tid], b = v[other];
                const bool descending = (tid & k) == 0 || k == P;
                if (descending ? a < b : a > b) {
                    v[tid] = b;
                    v[other] = a;
                }
            }
            __syncthreads();
        }
    if (tid < lv.n) {
        double total = 0.0;
        for (int i = 0; i < N; ++i) total += (double)v[i];
        const double target = lv.s[tid] * total;
        double prefix = 0.0;
        int n = N;
        for (int i = 0; i < N; ++i) {
            prefix += (double)v[i];
            if (prefix >= target) {
                n = i + 1;
                break;
            }
        }
        out[tid] = (float)n / (float)N;
    }
}

// mean <- mean + (x - mean)/i, sqmean <- sqmean + (x*x - sqmean)/i over every stride-th entry
__global__ __launch_bounds__(256) void grad_stats_update_kernel(const float *__restrict__ grad, int64_t m,
                                                                int64_t stride, float fi, float *__restrict__ mean,
                                                                float *__restrict__ sqmean)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= m) return;
    const float x = grad[j * stride];
    const float mu = mean[j], sq = sqmean[j];
    const float d = x - mu;
    mean[j] = mu + d / fi;
    const float xx = x * x;
    const float e = xx - sq;
    sqmean[j] = sq + e / fi;
}

// One workgroup; out = (accumulate ? out : 0) + weight * sum_j term(j), fp64.
// MODE 0: term = sqmean_j - mean_j^2 (a = mean, b = sqmean); MODE 1: term = (a - b)^2 at j*stride.
template <int MODE>
__global__ __launch_bounds__(1024) void subset_sum_kernel(const float *__restrict__ a, const float *__restrict__ b,
                                                          int64_t m, int64_t stride, double weight, int accumulate,
                                                          double *__restrict__ out)
{
    __shared__ double sh[1024];
    double acc = 0.0;
    for (int64_t j = threadIdx.x; j < m; j += 1024) {
        if (MODE == 0) {
            acc += (double)b[j] - (double)a[j] * (double)a[j];
        } else {
            const double d = (double)a[j * stride] - (double)b[j * stride];
            acc += d * d;
        }
    }
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int h = 512; h >= 1; h >>= 1) {
        if ((int)threadIdx.x < h) sh[threadIdx.x] += sh[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = (accumulate ? *out : 0.0) + weight * sh[0];
}

}  // namespace vcas

using namespace vcas;

extern "C" {

vcas_status vcas_sparsity_ratio(const float *gnorm, int32_t N, const double *s, int32_t ns, float *p, void *stream)
{
    if (!gnorm || !s || !p) return VCAS_ENULL;
    if (N <= 0 || N > 1024 || ns <= 0 || ns > kMaxLevels) return VCAS_EINVAL;
    Levels lv;
    lv.n = ns;
    for (int i = 0; i < ns; ++i) {
        if (!(s[i] >= 0.0 && s[i] <= 1.0)) return VCAS_EINVAL;
        lv.s[i] = s[i];
    }
    hipLaunchKernelGGL(sparsity_kernel, dim3(1), dim3(1024), 0, as_stream(stream), gnorm, (int)N, lv, p);
    return launch_status();
}

vcas_status vcas_grad_stats_update(const float *grad, int64_t m, int64_t stride, int32_t i, float *mean,
                                   float *sqmean, void *stream)
{
    if (!grad || !mean || !sqmean) return VCAS_ENULL;
    if (m <= 0 || stride <= 0 || i <= 0 || m > ((int64_t)1 << 40)) return VCAS_EINVAL;
    hipLaunchKernelGGL(grad_stats_update_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, as_stream(stream),
                       grad, m, stride, (float)i, mean, sqmean);
    return launch_status();
}

vcas_status vcas_grad_stats_variance(const float *mean, const float *sqmean, int64_t m, int32_t M, double *out,
                                     void *stream)
{
    if (!mean || !sqmean || !out) return VCAS_ENULL;
    if (m <= 0 || M < 2) return VCAS_EINVAL;
    hipLaunchKernelGGL(subset_sum_kernel<0>, dim3(1), dim3(1024), 0, as_stream(stream), mean, sqmean, m, (int64_t)1,
                       (double)M / (double)(M - 1), 0, out);
    return launch_status();
}

vcas_status vcas_sq_diff_strided(const float *a, const float *b, int64_t m, int64_t stride, double weight,
                                 int32_t accumulate, double *out, void *stream)
{
    if (!a || !b || !out) return VCAS_ENULL;
    if (m <= 0 || stride <= 0) return VCAS_EINVAL;
    hipLaunchKernelGGL(subset_sum_kernel<1>, dim3(1), dim3(1024), 0, as_stream(stream), a, b, m, stride, weight,
                       accumulate ? 1 : 0, out);
    return launch_status();
}

vcas_status vcas_controller_update(const vcas_controller_params *prm, int32_t L, double *s, double *rho, double *nu,
                                   double V_s, double V_act, const double *V_w, const double *V_s_layer,
                                   const double *p_minus, const double *p_plus)
{
    if (!prm || !s || !rho || !nu || !V_w || !V_s_layer || !p_minus || !p_plus) return VCAS_ENULL;
    if (L <= 0 || !(prm->alpha > 0.0) || !(prm->beta > 0.0 && prm->beta < 1.0) || !(prm->nu_min > 0.0 && prm->nu_min <= 1.0))
        return VCAS_EINVAL;
    // Eq. 5; sign(0) = +1
    const bool up = V_act - prm->tau_act * V_s >= 0.0;
    double sn = *s + (up ? prm->alpha : -prm->alpha);
    sn = sn > 1.0 ? 1.0 : (sn < 0.0 ? 0.0 : sn);
    *s = sn;
    // Eq. 4, right-hand part: running maximum from the input layer upwards, of the sparsities measured
    // on the side s moved to
    const double *pl = up ? p_plus : p_minus;
    double run = 0.0;
    for (int l = 0; l < L; ++l) {
        run = pl[l] > run ? pl[l] : run;
        rho[l] = run > 1.0 ? 1.0 : run;
    }
    // Eq. 7, read so that too much variance raises the keep ratio (beta < 1)
    for (int l = 0; l < L; ++l) {
        const bool high = V_w[l] - prm->tau_w * V_s_layer[l] >= 0.0;
        double v = high ? nu[l] / prm->beta : nu[l] * prm->beta;
        v = v > 1.0 ? 1.0 : (v < prm->nu_min ? prm->nu_min : v);
        nu[l] = v;
    }
    return VCAS_OK;
}

}  // extern "C"
