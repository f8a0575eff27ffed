// C ABI of the VCAS gfx950 library: argument checks on the host, then kernel
// launches on the caller's stream.  See include/vcas.h for the contract.
#include "groups.hpp"

namespace vcas {

KernelTimer &kernel_timer()
{
    static KernelTimer t;
    return t;
}

// norms.hip
vcas_status row_sumsq(const void *A, int dtype, int64_t R, int K, int T, const uint8_t *keep, float *out,
                      hipStream_t st);
vcas_status sample_norms(const float *gsq, int N, int T, float *gnorm, hipStream_t st);
vcas_status row_sumsq_group(const RowNormGroup &grp, int n, int dtype, int64_t R, int K, int T, hipStream_t st);
vcas_status row_sumsq_scores_uniforms(const void *X, int dtype, int64_t R, int K, int T, const uint8_t *keep,
                                      float *xsq, const float *gsq, const float *p, float *score, const vcas_rng &rng,
                                      uint32_t stream_id, float *uniforms, hipStream_t st);
vcas_status cached_xsq_scores_uniforms(const float *xsq_forward, int64_t R, int T, const uint8_t *keep, float *xsq,
                                       const float *gsq, const float *p, float *score, const vcas_rng &rng,
                                       uint32_t stream_id, float *uniforms, hipStream_t st);
// sampling.hip
vcas_status keep_probs(const float *score, int n, double budget, float *prob, hipStream_t st);
vcas_status sample_compact(const float *prob, int n, const vcas_rng &rng, uint32_t stream_id, uint8_t *mask,
                           int32_t *idx, int32_t *count, hipStream_t st);
vcas_status compact_only(const uint8_t *mask, int n, int32_t *idx, int32_t *count, hipStream_t st);
vcas_status leverage_scores(const float *gsq, const float *xsq, const float *p, const uint8_t *maskA, int64_t R,
                            int T, float *score, hipStream_t st);
vcas_status row_scale(const float *p, const float *q, const uint8_t *maskW, int64_t R, int T, float *scale,
                      hipStream_t st);
vcas_status broadcast_data_mask(const uint8_t *maskA, int64_t R, int T, float *q, uint8_t *maskW, hipStream_t st);
vcas_status sampler_a(const float *gsq, int N, int T, double budget, const vcas_rng &rng, float *gnorm, float *p,
                      uint8_t *maskA, int32_t *idxA, int32_t *cntA, hipStream_t st);
vcas_status sampler_a_group(const SampleAGroup &grp, int n, int N, int T, hipStream_t st);
vcas_status sampler_w_group(const SampleWGroup &grp, int n, int zero_dropped_xsq, int N, int T, int token_sampling,
                            int prepared, hipStream_t st);
vcas_status row_sumsq_scores_uniforms_group(const RowJobGroup &grp, int n, int dtype, int64_t R, int K, int T,
                                            hipStream_t st);
vcas_status uniforms(int64_t R, const vcas_rng &rng, uint32_t stream_id, float *u, hipStream_t st);
vcas_status sampler_w(const float *gsq, float *xsq, int zero_dropped_xsq, const float *p, const uint8_t *maskA,
                      const float *u, int N, int T, double budget, int token_sampling, int prepared, float *score,
                      float *q, uint8_t *maskW, float *scaleW, int32_t *idxW, int32_t *cntW, hipStream_t st);
vcas_status row_sumsq_pair(const void *G, int K_out, float *gsq, const void *X, int K_in, float *xsq, int dtype,
                           int64_t R, const vcas_rng &rng, uint32_t stream_id, float *uniforms, float *root_g,
                           float *root_x, int T, const uint8_t *keep_g, hipStream_t st);
bool plan_fused_fits(int N, int T);
vcas_status plan_fused(const void *G, int K_out, const void *X, int K_in, int dtype, int N, int T, double budget_a,
                       double budget_w, int token_sampling, const vcas_rng &rng, float *uniforms, uint32_t *ticket,
                       const vcas_plan &pl, hipStream_t st);
// gemm_bf16.hip / wgrad_bf16.hip / gemm_f32.hip
int wgrad_tiles_bf16(int K_out, int K_in, int tile);
int wgrad_tiles_f32(int K_out, int K_in);
vcas_status dgrad_bf16(const vcas_shape &s, const void *G, const void *W, const float *p, const int32_t *idxA,
                       const int32_t *cntA, void *dX, const void *J, bool fill, int64_t expected_rows,
                       const InlineSampleA *sample_a, float *sq_blocks, hipStream_t st);
vcas_status rows_from_blocks(const float *blocks, int64_t R, int K, int T, const uint8_t *keep, float *const *outs,
                             int n_out, hipStream_t st);
bool sample_norms_from_blocks_fits(int N, int T);
vcas_status sample_norms_from_blocks(const float *blocks, int N, int T, int K, const uint8_t *keep, float *const *outs,
                                     float *const *gnorms, int n_out, hipStream_t st);
vcas_status dgrad_bf16_group(const vcas_shape &s, const DgradProblem *probs, int n, bool fill, int64_t expected_rows,
                             hipStream_t st);
vcas_status wgrad_bf16_batch(const WgradItem *items, int n, int tile, hipStream_t st);
vcas_status dgrad_f32(const vcas_shape &s, const void *G, const void *W, const float *p, const int32_t *idxA,
                      const int32_t *cntA, void *dX, const void *J, bool fill, hipStream_t st);
vcas_status wgrad_f32(const vcas_shape &s, const void *G, const void *X, const float *row_scale, const int32_t *idxW,
                      const int32_t *cntW, float *dW, float *partials, int splits, hipStream_t st);

// Split-K slices of the weight gradient: about one and a half workgroups per CU (a second one
// hides the first one's waits; more splits cost reduction traffic), at most 8, and never so many
// that a slice at full length R would have fewer than 2 (bf16) or 8 (fp32) contraction steps.
constexpr int kWgradFill = 384;   // workgroups a weight-gradient launch wants when it has the chip to itself

static int wgrad_split_for(const vcas_shape *s, int tiles, int fill = kWgradFill)
{
    const bool bf = s->dtype == VCAS_BF16;
    const int64_t R = (int64_t)s->N * s->T;
    const int64_t steps = (R + (bf ? 63 : 15)) / (bf ? 64 : 16);
    if (fill <= 0 || fill > kWgradFill) fill = kWgradFill;   // the workspace is sized for kWgradFill
    int64_t want = (fill + tiles - 1) / tiles;
    int64_t cap = steps / (bf ? 2 : 8);
    if (want > cap) want = cap;
    if (want > 8) want = 8;
    if (want < 1) want = 1;
    return (int)want;
}

// The most slices any tile choice for this shape uses: sizes the partial-tile area of the workspace.
int wgrad_split(const vcas_shape *s)
{
    return wgrad_split_for(s, s->dtype == VCAS_BF16 ? wgrad_tiles_bf16(s->K_out, s->K_in, 128)
                                                    : wgrad_tiles_f32(s->K_out, s->K_in));
}

__global__ void fill_zero_kernel(uint32_t *p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// ---- variance probe reductions (fp64) ---------------------------------------

// out[slot] (+)= weight * sum_i (1-p_i)/p_i * n_i^2 over p_i > 0; one block.
__global__ __launch_bounds__(256) void var_closed_kernel(const float *__restrict__ prob, const float *__restrict__ val,
                                                         int64_t n, int square_val, double weight, int accumulate,
                                                         double *__restrict__ out)
{
    __shared__ double sh[256];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 256) {
        const double pr = prob[i];
        if (pr > 0.0) {
            const double v = val[i];
            acc += (1.0 - pr) / pr * (square_val ? v * v : v);
        }
    }
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int h = 128; h >= 1; h >>= 1) {
        if ((int)threadIdx.x < h) sh[threadIdx.x] += sh[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = (accumulate ? *out : 0.0) + weight * sh[0];
}

// per-block partial sums of (a-b)^2, then a one-block pass adds them in order
__global__ __launch_bounds__(256) void sq_diff_partial_kernel(const float *__restrict__ a, const float *__restrict__ b,
                                                              int64_t n, double *__restrict__ partial)
{
    __shared__ double sh[256];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const double d = (double)a[i] - (double)b[i];
        acc += d * d;
    }
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int h = 128; h >= 1; h >>= 1) {
        if ((int)threadIdx.x < h) sh[threadIdx.x] += sh[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = sh[0];
}

__global__ __launch_bounds__(64) void sq_diff_final_kernel(const double *__restrict__ partial, int blocks,
                                                           double weight, double *__restrict__ out)
{
    if (threadIdx.x != 0) return;
    double s = 0.0;
    for (int i = 0; i < blocks; ++i) s += partial[i];
    *out += weight * s;
}

// J: elementwise Jacobian [R, K_in] in the layer dtype, multiplied into dX (null: none);
// fill: write zero rows for the samples that are not kept
// sq_blocks (bf16 only, else null): also write the sums of squares of dX by blocks of 32 columns
static vcas_status dispatch_dgrad(const vcas_shape &s, const void *G, const void *W, const float *p,
                                  const int32_t *idxA, const int32_t *cntA, void *dX, const void *J, bool fill,
                                  int64_t expected_rows, hipStream_t st, float *sq_blocks = nullptr)
{
    if (s.dtype == VCAS_BF16) return dgrad_bf16(s, G, W, p, idxA, cntA, dX, J, fill, expected_rows, nullptr, sq_blocks, st);
    return sq_blocks ? VCAS_EDTYPE : dgrad_f32(s, G, W, p, idxA, cntA, dX, J, fill, st);
}

// Tile edge and split-K slices of bf16 weight gradients.  `fill` = the workgroups a launch should
// have before the contraction stops being cut into slices; tiles256 / tiles128 = output tiles of
// everything the launch covers (one layer, or a batch of layers).  The largest tile that fills the
// launch without slicing wins (a 256x256 tile moves half the operand bytes per flop of a 128x128
// one, and a CU pulls operand tiles in at a fixed rate); else 128x128 with slices; 64x64 for
// weight gradients of a few tiles only.
static int wgrad_tile_choice(int tiles256, int tiles128, int fill)
{
    if (tiles256 >= fill) return 256;
    return tiles128 >= 16 ? 128 : 64;
}

// Slices for one layer of a launch whose tiles (of every layer it covers) number `launch_tiles`:
// enough to reach `fill` workgroups, at most 8, never so many that a slice at full length R would
// have fewer than 2 contraction steps, never more than the workspace has room for.
static int wgrad_slices_bf16(const vcas_shape &s, int launch_tiles, int fill)
{
    const int64_t R = (int64_t)s.N * s.T;
    int64_t want = (fill + launch_tiles - 1) / launch_tiles;
    const int64_t cap = ((R + 63) / 64) / 2;
    if (want > cap) want = cap;
    if (want > wgrad_split(&s)) want = wgrad_split(&s);
    if (want > 8) want = 8;
    return want < 1 ? 1 : (int)want;
}

static int fill_or_default(int fill) { return fill <= 0 || fill > kWgradFill ? kWgradFill : fill; }

static WgradItem wgrad_item(const vcas_shape &s, const void *G, const void *X, const float *scale, const int32_t *idxW,
                            const int32_t *cntW, float *dW, float *partials, uint16_t *packed)
{
    WgradItem it;
    it.shape = s;
    it.G = G;
    it.X = X;
    it.row_scale = scale;
    it.idxW = idxW;
    it.cntW = cntW;
    it.dW = dW;
    it.partials = partials;
    it.packed = packed;
    it.splits = 1;
    return it;
}

// One layer on its own.  partials: room for wgrad_split(s) partial tiles; packed (bf16): room for
// R rows of the narrower operand.
static vcas_status dispatch_wgrad_into(const vcas_shape &s, const void *G, const void *X, const float *scale,
                                       const int32_t *idxW, const int32_t *cntW, float *dW, float *partials,
                                       uint16_t *packed, hipStream_t st, int fill = kWgradFill)
{
    if (s.dtype != VCAS_BF16)
        return wgrad_f32(s, G, X, scale, idxW, cntW, dW, partials, wgrad_split_for(&s, wgrad_tiles_f32(s.K_out, s.K_in), fill),
                         st);
    fill = fill_or_default(fill);
    const int tile = wgrad_tile_choice(wgrad_tiles_bf16(s.K_out, s.K_in, 256), wgrad_tiles_bf16(s.K_out, s.K_in, 128), fill);
    WgradItem it = wgrad_item(s, G, X, scale, idxW, cntW, dW, partials, packed);
    it.splits = wgrad_slices_bf16(s, wgrad_tiles_bf16(s.K_out, s.K_in, tile), fill);
    return wgrad_bf16_batch(&it, 1, tile, st);
}

static vcas_status dispatch_wgrad(const vcas_shape &s, const void *G, const void *X, const float *scale,
                                  const int32_t *idxW, const int32_t *cntW, float *dW, void *workspace,
                                  hipStream_t st, int fill = kWgradFill)
{
    const WorkspaceLayout w = workspace_layout(&s);
    unsigned char *base = static_cast<unsigned char *>(workspace);
    return dispatch_wgrad_into(s, G, X, scale, idxW, cntW, dW, reinterpret_cast<float *>(base + w.partials),
                               reinterpret_cast<uint16_t *>(base + w.packed), st, fill);
}

// ---- the library's own scratch, for the entry point that takes no workspace --------------------
// One array per GPU the library runs on, held until the process ends.  In host code the array's name
// is only a handle: its device address comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void *scratch_of_device[kMaxDevices];   // zero until first use on that device

static vcas_status static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VCAS_EHIP;
    if (!scratch_of_device[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return VCAS_EHIP;
        scratch_of_device[dev] = ptr;
    }
    *out = scratch_of_device[dev];
    return VCAS_OK;
}

// Bytes of scratch vcas_sampled_wgrad's kernels use for this shape: the split-K partial tiles, then
// (bf16) the packed operand.
static size_t wgrad_partial_bytes(const vcas_shape &s)
{
    return (((size_t)s.K_out * s.K_in * sizeof(float) * (size_t)wgrad_split(&s)) + 255) & ~(size_t)255;
}

static size_t wgrad_scratch_bytes(const vcas_shape &s)
{
    const WorkspaceLayout w = workspace_layout(&s);
    return wgrad_partial_bytes(s) + (w.total - w.packed);
}

static bool plan_complete(const vcas_plan *pl)
{
    return pl && pl->gsq && pl->gnorm && pl->p && pl->maskA && pl->idxA && pl->cntA && pl->xsq && pl->score &&
           pl->q && pl->maskW && pl->idxW && pl->cntW && pl->scaleW;
}

static bool ratio_ok(double r) { return r > 0.0 && r <= 1.0; }

#define VCAS_TRY(expr)                      \
    do {                                    \
        vcas_status st__ = (expr);          \
        if (st__ != VCAS_OK) return st__;   \
    } while (0)

// One event, created on first use and kept: orders the side stream after SampleA.
static hipEvent_t fork_event()
{
    static hipEvent_t ev = nullptr;
    if (!ev && hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) ev = nullptr;
    return ev;
}

// Small layers: the row norms of X do not wait for SampleA; they are taken for every row in the
// same launch as those of G (one launch and one dependency fewer; rows of dropped samples are
// zeroed afterwards).  Large layers: a second launch that skips dropped samples' rows.
static bool norms_together(const vcas_shape &s)
{
    return (int64_t)s.N * s.T * s.K_in * elem_bytes(s.dtype) <= ((int64_t)16 << 20);
}

static float *uniforms_of(const vcas_shape &s, void *workspace)
{
    return reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + workspace_layout(&s).uniforms);
}

// Data half: row norms of G (and of X, with the SampleW uniforms, on small layers), SampleA, dX.
// What a layer inside a stack adds to the data half (all optional).
struct ChainArgs {
    const void *J = nullptr;              // elementwise Jacobian multiplied into dX
    const uint8_t *kept_above = nullptr;  // samples whose rows of G exist at all (the others count as zero)
    bool fill = true;                     // write zero rows of dX for the samples that are not kept
    const float *g_sq_blocks = nullptr;   // block sums of squares of G from the dgrad that wrote it: no sweep over G
    float *dx_sq_blocks = nullptr;        // where this layer's dgrad leaves the block sums of squares of its dX
};

// Where the norms of X are taken: with those of G, before SampleA (one launch fewer, every row
// read), or by the weight half, after SampleA (kept samples only; the norms of X then stay off the
// stream that carries the dX chain).  Both give the same bits.
enum XNorms { kXNormsByShape, kXNormsWithG, kXNormsAfterSampleA };

static bool together_for(const vcas_shape &s, XNorms x)
{
    return x == kXNormsByShape ? norms_together(s) : x == kXNormsWithG;
}

static vcas_status data_half(const vcas_shape &s, const void *G, const void *X, const void *W, double rho,
                             const vcas_rng &rng, int token_sampling, const vcas_plan &pl, void *dX,
                             const ChainArgs &chain, void *workspace, hipStream_t st, XNorms xnorms = kXNormsByShape,
                             bool sample_a_in_dgrad = false)
{
    const int64_t R = (int64_t)s.N * s.T;
    float *uw = token_sampling ? uniforms_of(s, workspace) : nullptr;
    // together: the square roots SampleW needs travel in the plan's score and q arrays until
    // SampleW overwrites them with their final contents
    // Inside a stack, with the block sums of G at hand: one workgroup per sample adds them to row
    // sums and the sample's norm, and the dgrad workgroups decide SampleA themselves from the N
    // norms, so that the chain row norms -> SampleA -> dX is two launches instead of three.
    const bool norms_for_dgrad = sample_a_in_dgrad && chain.g_sq_blocks && dX && s.dtype == VCAS_BF16 && s.N <= 64 &&
                                 sample_norms_from_blocks_fits(s.N, s.T);
    if (norms_for_dgrad) {
        float *outs[1] = {pl.gsq}, *gnorms[1] = {pl.gnorm};
        VCAS_TRY(sample_norms_from_blocks(chain.g_sq_blocks, s.N, s.T, s.K_out, chain.kept_above, outs, gnorms, 1, st));
    } else if (chain.g_sq_blocks) {
        // the norms of G come from the launch that wrote G; those of X are left to the weight half
        float *outs[1] = {pl.gsq};
        VCAS_TRY(rows_from_blocks(chain.g_sq_blocks, R, s.K_out, s.T, chain.kept_above, outs, 1, st));
    } else if (together_for(s, xnorms))
        VCAS_TRY(row_sumsq_pair(G, s.K_out, pl.gsq, X, s.K_in, pl.xsq, s.dtype, R, rng, 1u, uw, pl.score, pl.q, s.T,
                                chain.kept_above, st));
    else
        VCAS_TRY(row_sumsq(G, s.dtype, R, s.K_out, s.T, chain.kept_above, pl.gsq, st));
    // SampleA keeps about N*rho samples (Sec. 4.1): the row count the dgrad tile choice plans for
    const int64_t rows_expected = (int64_t)((double)R * rho + 0.5);
    if (norms_for_dgrad || (sample_a_in_dgrad && dX && s.dtype == VCAS_BF16 && s.N <= 64 && R <= 4096)) {
        // one launch and its gap less on the chain row norms -> SampleA -> dX: the dgrad workgroups
        // decide SampleA themselves.  Worth it only while the vector of row norms is short: every
        // workgroup reads all of it (BERT-base, R = 4096: step 2.78 -> 2.70 ms; ViT, N = 64,
        // R = 12608: 3.93 -> 4.44 ms)
        InlineSampleA sa = {};
        if (norms_for_dgrad) sa.norms = pl.gnorm;
        else sa.gsq = pl.gsq;
        sa.budget = (double)s.N * rho;
        sa.seed = rng.seed;
        sa.layer = rng.layer;
        sa.draw = rng.draw;
        sa.draw_offset = rng.draw_offset;
        sa.gnorm = pl.gnorm;
        sa.p = pl.p;
        sa.maskA = pl.maskA;
        sa.idxA = pl.idxA;
        sa.cntA = pl.cntA;
        return dgrad_bf16(s, G, W, pl.p, pl.idxA, pl.cntA, dX, chain.J, chain.fill, rows_expected, &sa, chain.dx_sq_blocks, st);
    }
    VCAS_TRY(sampler_a(pl.gsq, s.N, s.T, (double)s.N * rho, rng, pl.gnorm, pl.p, pl.maskA, pl.idxA, pl.cntA, st));
    if (dX)
        VCAS_TRY(dispatch_dgrad(s, G, W, pl.p, pl.idxA, pl.cntA, dX, chain.J, chain.fill, rows_expected, st,
                                chain.dx_sq_blocks));
    return VCAS_OK;
}

// Weight half, after the data half of the same layer and draw: row norms of X on kept samples
// (large layers), SampleW, dW.
static vcas_status weight_half(const vcas_shape &s, const void *G, const void *X, double rho, double nu,
                               const vcas_rng &rng, int token_sampling, const vcas_plan &pl, float *dW,
                               void *workspace, hipStream_t st, XNorms xnorms = kXNormsByShape,
                               const float *xsq_forward = nullptr)
{
    const int64_t R = (int64_t)s.N * s.T;
    float *u = uniforms_of(s, workspace);
    // cached norms of X: whatever the data half may have left in score and q is not used
    const bool together = !xsq_forward && together_for(s, xnorms);
    if (xsq_forward)
        VCAS_TRY(cached_xsq_scores_uniforms(xsq_forward, R, s.T, pl.maskA, pl.xsq, pl.gsq, pl.p, pl.score, rng, 1u,
                                            token_sampling ? u : nullptr, st));
    else if (!together)
        VCAS_TRY(row_sumsq_scores_uniforms(X, s.dtype, R, s.K_in, s.T, pl.maskA, pl.xsq, pl.gsq, pl.p, pl.score, rng, 1u,
                                           token_sampling ? u : nullptr, st));
    // what the norm passes have left in score and q: roots (together) or the scores themselves
    VCAS_TRY(sampler_w(pl.gsq, pl.xsq, together ? 1 : 0, pl.p, pl.maskA, u, s.N, s.T, (double)R * rho * nu,
                       token_sampling, together ? 1 : 2, pl.score, pl.q, pl.maskW, pl.scaleW, pl.idxW, pl.cntW, st));
    if (dW)
        VCAS_TRY(dispatch_wgrad(s, G, X, pl.scaleW, pl.idxW, pl.cntW, dW, workspace, st));
    return VCAS_OK;
}

static bool same_shape(const vcas_shape &s, const vcas_shape &t)
{
    return s.N == t.N && s.T == t.T && s.K_in == t.K_in && s.K_out == t.K_out && s.dtype == t.dtype;
}

// Can layer b of a stack share the launches of its data half with layer a in front of it?  Only
// where the caller says that b's G does not depend on a's dX and the two have one shape (bf16, a
// dX wanted, at most 1024 samples: the one-workgroup SampleA).
static bool shares_data_half(const vcas_layer_args &a, const vcas_layer_args &b)
{
    const vcas_shape &s = a.shape;
    return b.sibling != 0 && same_shape(s, b.shape) && s.dtype == VCAS_BF16 && s.N <= 1024 && a.dX && b.dX &&
           (a.leave_dropped_rows != 0) == (b.leave_dropped_rows != 0) && (a.g_sq_blocks != nullptr) == (b.g_sq_blocks != nullptr);
}

// Data halves of n sibling layers (shares_data_half): the row norms of every G in one launch,
// every dX in one launch.  SampleA in between: on short vectors each dgrad workgroup decides its
// own layer's (as in data_half), else one launch with a workgroup per layer.  Bit for bit what
// n calls of data_half compute.
static vcas_status data_half_siblings(const vcas_layer_args *layers, int n, hipStream_t st)
{
    const vcas_shape &s = layers[0].shape;
    const int64_t R = (int64_t)s.N * s.T;
    const bool in_dgrad = s.N <= 64 && R <= 4096;
    // with the block sums of G at hand the sample norms come with the row sums and dgrad decides from those (see data_half)
    const bool norms_for_dgrad = layers[0].g_sq_blocks && s.N <= 64 && sample_norms_from_blocks_fits(s.N, s.T);
    RowNormGroup norms = {};
    SampleAGroup samplers = {};
    DgradProblem probs[kMaxSiblings];
    double rho_max = 0.0;
    for (int i = 0; i < n; ++i) {
        const vcas_layer_args &a = layers[i];
        norms.A[i] = static_cast<const uint4 *>(a.G);
        norms.out[i] = a.plan.gsq;
        norms.keep[i] = a.kept_above;
        InlineSampleA sa = {};
        sa.gsq = a.plan.gsq;
        sa.budget = (double)s.N * a.rho;
        sa.seed = a.rng.seed;
        sa.layer = a.rng.layer;
        sa.draw = a.rng.draw;
        sa.draw_offset = a.rng.draw_offset;
        sa.gnorm = a.plan.gnorm;
        sa.p = a.plan.p;
        sa.maskA = a.plan.maskA;
        sa.idxA = a.plan.idxA;
        sa.cntA = a.plan.cntA;
        samplers.prob[i] = sa;
        DgradProblem &q = probs[i];
        q.G = static_cast<const uint16_t *>(a.G);
        q.W = static_cast<const uint16_t *>(a.W);
        q.p = a.plan.p;
        q.idxA = a.plan.idxA;
        q.cntA = a.plan.cntA;
        q.dX = static_cast<uint16_t *>(a.dX);
        q.J = static_cast<const uint16_t *>(a.J);
        q.sa = sa;
        if (!in_dgrad || norms_for_dgrad) q.sa.gsq = nullptr;
        if (norms_for_dgrad) q.sa.norms = a.plan.gnorm;
        q.sq_blocks = a.dx_sq_blocks;
        if (a.rho > rho_max) rho_max = a.rho;
    }
    if (layers[0].g_sq_blocks) {
        // norms of G from the launch that wrote it: one pass over the block sums serves every
        // sibling that was handed the same G; the others take a pass of their own
        for (int i = 0; i < n;) {
            float *outs[kMaxSiblings], *gnorms[kMaxSiblings];
            int m = 0;
            for (; i + m < n && layers[i + m].g_sq_blocks == layers[i].g_sq_blocks &&
                   layers[i + m].kept_above == layers[i].kept_above; ++m) {
                outs[m] = layers[i + m].plan.gsq;
                gnorms[m] = layers[i + m].plan.gnorm;
            }
            if (norms_for_dgrad)
                VCAS_TRY(sample_norms_from_blocks(layers[i].g_sq_blocks, s.N, s.T, s.K_out, layers[i].kept_above, outs,
                                                  gnorms, m, st));
            else
                VCAS_TRY(rows_from_blocks(layers[i].g_sq_blocks, R, s.K_out, s.T, layers[i].kept_above, outs, m, st));
            i += m;
        }
    } else
        VCAS_TRY(row_sumsq_group(norms, n, s.dtype, R, s.K_out, s.T, st));
    if (!in_dgrad && !norms_for_dgrad) VCAS_TRY(sampler_a_group(samplers, n, s.N, s.T, st));
    return dgrad_bf16_group(s, probs, n, layers[0].leave_dropped_rows == 0, (int64_t)((double)R * rho_max + 0.5), st);
}

// Can layer b share the SampleW launches of layer a in front of it?  Siblings of one shape and
// dtype with the same kind of token sampling, the rows of X still to be swept, and few enough
// rows for the one-workgroup sampler.
static bool shares_weight_half(const vcas_layer_args &a, const vcas_layer_args &b)
{
    const vcas_shape &s = a.shape;
    return b.sibling != 0 && same_shape(s, b.shape) && (int64_t)s.N * s.T <= 16384 && !a.xsq_forward &&
           !b.xsq_forward && (a.token_sampling != 0) == (b.token_sampling != 0);
}

// What weight_half does before dW, for n sibling layers (shares_weight_half) whose data halves
// left the norms of X to it: the row norms of X on kept samples with the SampleW scores and
// uniforms in one launch, SampleW in one launch (a workgroup per layer).  The same bits.
static vcas_status weight_half_siblings(const vcas_layer_args *layers, int n, hipStream_t st)
{
    const vcas_shape &s = layers[0].shape;
    const int64_t R = (int64_t)s.N * s.T;
    const int token_sampling = layers[0].token_sampling;
    RowJobGroup norms = {};
    SampleWGroup samplers = {};
    for (int i = 0; i < n; ++i) {
        const vcas_layer_args &a = layers[i];
        float *u = uniforms_of(a.shape, a.workspace);
        norms.A[i] = static_cast<const uint4 *>(a.X);
        norms.keep[i] = a.plan.maskA;
        norms.out[i] = a.plan.xsq;
        norms.job[i] = {token_sampling ? u : nullptr, a.rng.seed, a.rng.layer, 1u, a.rng.draw, a.rng.draw_offset};
        norms.sj[i] = {a.plan.gsq, a.plan.p, a.plan.score};
        SampleWProblem &w = samplers.prob[i];
        w.gsq = a.plan.gsq;
        w.xsq = a.plan.xsq;
        w.p = a.plan.p;
        w.maskA = a.plan.maskA;
        w.u = u;
        w.budget = (double)R * a.rho * a.nu;
        w.score = a.plan.score;
        w.q = a.plan.q;
        w.maskW = a.plan.maskW;
        w.scaleW = a.plan.scaleW;
        w.idxW = a.plan.idxW;
        w.cntW = a.plan.cntW;
    }
    VCAS_TRY(row_sumsq_scores_uniforms_group(norms, n, s.dtype, R, s.K_in, s.T, st));
    return sampler_w_group(samplers, n, 0, s.N, s.T, token_sampling, 2, st);
}

// Weight gradients of the layers [l0, l1) of a stack that want one (bf16 layers in batched
// launches, fp32 layers one by one).  A layer with wgrad_fill == 0 gets the tile and the slices a
// call on its own would pick, hence that call's bits; the others are planned per launch: the
// tiles of every layer of the batch count towards `fill`, so a block's weight gradients fill the
// chip together and are rarely sliced at all.
static vcas_status wgrad_of_layers(const vcas_layer_args *layers, int l0, int l1, hipStream_t st)
{
    for (int l = l0; l < l1;) {
        const vcas_layer_args &a = layers[l];
        if (!a.dW) {
            ++l;
            continue;
        }
        if (a.shape.dtype != VCAS_BF16) {
            VCAS_TRY(dispatch_wgrad(a.shape, a.G, a.X, a.plan.scaleW, a.plan.idxW, a.plan.cntW, a.dW, a.workspace, st,
                                    a.wgrad_fill));
            ++l;
            continue;
        }
        // a run of bf16 layers that plan their launch the same way
        const bool alone = a.wgrad_fill == 0 || a.wgrad_fill >= kWgradFill;
        int picked[kWgradBatch], n = 0, next = l;
        int tiles256 = 0, tiles128 = 0;
        for (; next < l1 && n < kWgradBatch; ++next) {
            const vcas_layer_args &b = layers[next];
            if (!b.dW) continue;
            if (b.shape.dtype != VCAS_BF16 || (b.wgrad_fill == 0 || b.wgrad_fill >= kWgradFill) != alone) break;
            const int t256 = wgrad_tiles_bf16(b.shape.K_out, b.shape.K_in, 256), t128 = wgrad_tiles_bf16(b.shape.K_out, b.shape.K_in, 128);
            if (alone && n > 0 &&
                wgrad_tile_choice(t256, t128, kWgradFill) !=
                    wgrad_tile_choice(wgrad_tiles_bf16(layers[picked[0]].shape.K_out, layers[picked[0]].shape.K_in, 256),
                                      wgrad_tiles_bf16(layers[picked[0]].shape.K_out, layers[picked[0]].shape.K_in, 128), kWgradFill))
                break;
            picked[n++] = next;
            tiles256 += t256;
            tiles128 += t128;
        }
        const int fill = fill_or_default(a.wgrad_fill);
        const vcas_shape &s0 = layers[picked[0]].shape;
        const int tile = alone ? wgrad_tile_choice(wgrad_tiles_bf16(s0.K_out, s0.K_in, 256), wgrad_tiles_bf16(s0.K_out, s0.K_in, 128), fill)
                               : wgrad_tile_choice(tiles256, tiles128, fill);
        int launch_tiles = 0;
        for (int i = 0; i < n; ++i) launch_tiles += wgrad_tiles_bf16(layers[picked[i]].shape.K_out, layers[picked[i]].shape.K_in, tile);
        WgradItem items[kWgradBatch];
        for (int i = 0; i < n; ++i) {
            const vcas_layer_args &b = layers[picked[i]];
            const WorkspaceLayout w = workspace_layout(&b.shape);
            unsigned char *base = static_cast<unsigned char *>(b.workspace);
            items[i] = wgrad_item(b.shape, b.G, b.X, b.plan.scaleW, b.plan.idxW, b.plan.cntW, b.dW,
                                  reinterpret_cast<float *>(base + w.partials), reinterpret_cast<uint16_t *>(base + w.packed));
            items[i].splits = wgrad_slices_bf16(b.shape, alone ? wgrad_tiles_bf16(b.shape.K_out, b.shape.K_in, tile) : launch_tiles, fill);
        }
        VCAS_TRY(wgrad_bf16_batch(items, n, tile, st));
        l = next;
    }
    return VCAS_OK;
}

static vcas_status linear_backward_impl(const vcas_shape &s, const void *G, const void *X, const void *W, double rho,
                                        double nu, const vcas_rng &rng, int token_sampling, const vcas_plan &pl,
                                        void *dX, float *dW, void *workspace, hipStream_t st, hipStream_t side)
{
    const int64_t R = (int64_t)s.N * s.T;
    const bool forked = side && side != st;
    // Small layers with short vectors, everything on one stream: norms, SampleA and SampleW in
    // ONE launch (the workgroup that finishes its rows last does the two samplers).  With a side
    // stream the samplers stay separate launches: SampleW then runs beside dX instead of before it.
    if (!forked && norms_together(s) && plan_fused_fits(s.N, s.T)) {
        uint32_t *tickets = reinterpret_cast<uint32_t *>(static_cast<unsigned char *>(workspace) +
                                                         workspace_layout(&s).control);
        VCAS_TRY(plan_fused(G, s.K_out, X, s.K_in, s.dtype, s.N, s.T, (double)s.N * rho, (double)R * rho * nu,
                            token_sampling, rng, uniforms_of(s, workspace), tickets, pl, st));
        if (dX) VCAS_TRY(dispatch_dgrad(s, G, W, pl.p, pl.idxA, pl.cntA, dX, nullptr, true, (int64_t)((double)R * rho + 0.5), st));
        if (dW) VCAS_TRY(dispatch_wgrad(s, G, X, pl.scaleW, pl.idxW, pl.cntW, dW, workspace, st));
        return VCAS_OK;
    }
    if (!forked) {
        VCAS_TRY(data_half(s, G, X, W, rho, rng, token_sampling, pl, dX, ChainArgs(), workspace, st));
        return weight_half(s, G, X, rho, nu, rng, token_sampling, pl, dW, workspace, st);
    }
    // The weight half needs SampleA's outcome but not dX: order it after SampleA, beside dX.
    VCAS_TRY(data_half(s, G, X, W, rho, rng, token_sampling, pl, nullptr, ChainArgs(), workspace, st));
    hipEvent_t ev = fork_event();
    if (!ev || hipEventRecord(ev, st) != hipSuccess || hipStreamWaitEvent(side, ev, 0) != hipSuccess) return VCAS_EHIP;
    if (dX) VCAS_TRY(dispatch_dgrad(s, G, W, pl.p, pl.idxA, pl.cntA, dX, nullptr, true, (int64_t)((double)R * rho + 0.5), st));
    return weight_half(s, G, X, rho, nu, rng, token_sampling, pl, dW, workspace, side);
}

}  // namespace vcas

using namespace vcas;

extern "C" {

const char *vcas_status_string(vcas_status s)
{
    switch (s) {
    case VCAS_OK: return "ok";
    case VCAS_EINVAL: return "invalid size, ratio or alignment";
    case VCAS_ENULL: return "required pointer is null";
    case VCAS_EDTYPE: return "unknown dtype";
    case VCAS_EWORKSPACE: return "workspace missing";
    case VCAS_EHIP: return "HIP launch failed";
    case VCAS_ETOOBIG: return "problem needs more scratch than the library's static buffer holds";
    }
    return "unknown status";
}

size_t vcas_workspace_bytes(const vcas_shape *shape)
{
    if (check_shape(shape) != VCAS_OK) return 0;
    return workspace_layout(shape).total;
}

vcas_status vcas_workspace_init(const vcas_shape *shape, void *workspace, void *stream)
{
    VCAS_TRY(check_shape(shape));
    if (!workspace) return VCAS_EWORKSPACE;
    if (!aligned16(workspace)) return VCAS_EINVAL;
    const WorkspaceLayout w = workspace_layout(shape);
    uint32_t *control = reinterpret_cast<uint32_t *>(static_cast<unsigned char *>(workspace) + w.control);
    const int words = (int)((w.partials - w.control) / 4);
    // a fill kernel rather than hipMemsetAsync, so that the call may be captured in a graph
    hipLaunchKernelGGL(fill_zero_kernel, dim3((words + 255) / 256), dim3(256), 0, as_stream(stream), control,
                       (size_t)words);
    return launch_status();
}

vcas_status vcas_row_norms(const vcas_shape *shape, const void *G, const void *X, const uint8_t *sample_mask,
                           float *gsq, float *xsq, float *gnorm, void *stream)
{
    VCAS_TRY(check_shape(shape));
    if (!G && !X) return VCAS_ENULL;
    if (G && !gsq) return VCAS_ENULL;
    if (X && !xsq) return VCAS_ENULL;
    if (gnorm && !G) return VCAS_ENULL;
    if ((G && !aligned16(G)) || (X && !aligned16(X))) return VCAS_EINVAL;
    const int64_t R = (int64_t)shape->N * shape->T;
    hipStream_t st = as_stream(stream);
    if (G) {
        VCAS_TRY(row_sumsq(G, shape->dtype, R, shape->K_out, shape->T, nullptr, gsq, st));
        if (gnorm) VCAS_TRY(sample_norms(gsq, shape->N, shape->T, gnorm, st));
    }
    if (X) VCAS_TRY(row_sumsq(X, shape->dtype, R, shape->K_in, shape->T, sample_mask, xsq, st));
    return VCAS_OK;
}

vcas_status vcas_keep_probs(const float *score, int32_t n, double budget, float *prob, void *stream)
{
    if (n < 0 || !(budget >= 0.0)) return VCAS_EINVAL;
    if (n == 0) return VCAS_OK;
    if (!score || !prob) return VCAS_ENULL;
    return keep_probs(score, n, budget, prob, as_stream(stream));
}

vcas_status vcas_sample_compact(const float *prob, int32_t n, const vcas_rng *rng, uint32_t stream_id, uint8_t *mask,
                                int32_t *idx, int32_t *count, void *stream)
{
    if (n < 0) return VCAS_EINVAL;
    if (!rng || !count) return VCAS_ENULL;
    if (n > 0 && (!prob || !mask || !idx)) return VCAS_ENULL;
    return sample_compact(prob, n, *rng, stream_id, mask, idx, count, as_stream(stream));
}

vcas_status vcas_leverage_scores(const vcas_shape *shape, const float *gsq, const float *xsq, const float *p,
                                 const uint8_t *maskA, float *score, void *stream)
{
    VCAS_TRY(check_shape(shape));
    if (!gsq || !xsq || !p || !maskA || !score) return VCAS_ENULL;
    return leverage_scores(gsq, xsq, p, maskA, (int64_t)shape->N * shape->T, shape->T, score, as_stream(stream));
}

vcas_status vcas_row_scale(const vcas_shape *shape, const float *p, const float *q, const uint8_t *maskW,
                           float *scaleW, void *stream)
{
    VCAS_TRY(check_shape(shape));
    if (!p || !q || !maskW || !scaleW) return VCAS_ENULL;
    return row_scale(p, q, maskW, (int64_t)shape->N * shape->T, shape->T, scaleW, as_stream(stream));
}

vcas_status vcas_sampled_dgrad(const vcas_shape *shape, const void *G, const void *W, const float *p,
                               const int32_t *idxA, const int32_t *cntA, void *dX, void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !W || !p || !idxA || !cntA || !dX) return VCAS_ENULL;
    if (!aligned16(G) || !aligned16(W) || !aligned16(dX)) return VCAS_EINVAL;
    return dispatch_dgrad(*shape, G, W, p, idxA, cntA, dX, nullptr, true, 0, as_stream(stream));
}

vcas_status vcas_sampled_dgrad_jac(const vcas_shape *shape, const void *G, const void *W, const float *p,
                                   const int32_t *idxA, const int32_t *cntA, const void *J, void *dX, void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !W || !p || !idxA || !cntA || !J || !dX) return VCAS_ENULL;
    if (!aligned16(G) || !aligned16(W) || !aligned16(J) || !aligned16(dX)) return VCAS_EINVAL;
    return dispatch_dgrad(*shape, G, W, p, idxA, cntA, dX, J, true, 0, as_stream(stream));
}

vcas_status vcas_sampled_dgrad_norms(const vcas_shape *shape, const void *G, const void *W, const float *p,
                                     const int32_t *idxA, const int32_t *cntA, const void *J, void *dX,
                                     float *sq_blocks, void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (shape->dtype != VCAS_BF16) return VCAS_EDTYPE;
    if (!G || !W || !p || !idxA || !cntA || !dX || !sq_blocks) return VCAS_ENULL;
    if (!aligned16(G) || !aligned16(W) || (J && !aligned16(J)) || !aligned16(dX) || !aligned16(sq_blocks)) return VCAS_EINVAL;
    return dispatch_dgrad(*shape, G, W, p, idxA, cntA, dX, J, true, 0, as_stream(stream), sq_blocks);
}

size_t vcas_sq_blocks_bytes(int64_t R, int32_t K)
{
    if (R <= 0 || K <= 0) return 0;
    return (size_t)16 * (size_t)R * (size_t)(((K + 63) / 64 + 3) / 4);
}

vcas_status vcas_row_norms_from_blocks(int32_t N, int32_t T, int32_t K, const float *sq_blocks,
                                       const uint8_t *sample_mask, float *sq, float *norm, void *stream)
{
    if (N <= 0 || T <= 0 || K <= 0 || (int64_t)N * T > (int64_t)1 << 30) return VCAS_EINVAL;
    if (!sq_blocks || !sq) return VCAS_ENULL;
    if (!aligned16(sq_blocks)) return VCAS_EINVAL;
    float *outs[1] = {sq};
    VCAS_TRY(rows_from_blocks(sq_blocks, (int64_t)N * T, K, T, sample_mask, outs, 1, as_stream(stream)));
    if (norm) VCAS_TRY(sample_norms(sq, N, T, norm, as_stream(stream)));
    return VCAS_OK;
}

vcas_status vcas_sampled_wgrad(const vcas_shape *shape, const void *G, const void *X, const float *row_scale_,
                               const int32_t *idxW, const int32_t *cntW, float *dW, void *workspace, void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !X || !row_scale_ || !idxW || !cntW || !dW) return VCAS_ENULL;
    if (!workspace) return VCAS_EWORKSPACE;
    if (!aligned16(G) || !aligned16(X) || !aligned16(dW) || !aligned16(workspace)) return VCAS_EINVAL;
    return dispatch_wgrad(*shape, G, X, row_scale_, idxW, cntW, dW, workspace, as_stream(stream));
}

size_t vcas_static_scratch_bytes(void) { return kStaticScratchBytes; }

vcas_status vcas_sampled_wgrad_static(const vcas_shape *shape, const void *G, const void *X, const float *row_scale_,
                                      const int32_t *idxW, const int32_t *cntW, float *dW, void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !X || !row_scale_ || !idxW || !cntW || !dW) return VCAS_ENULL;
    if (!aligned16(G) || !aligned16(X) || !aligned16(dW)) return VCAS_EINVAL;
    if (wgrad_scratch_bytes(*shape) > kStaticScratchBytes) return VCAS_ETOOBIG;
    void *buf = nullptr;
    VCAS_TRY(static_scratch(&buf));
    // the partial tiles and the packed rows are written in full before anything reads them, so
    // whatever the last call left in the buffer does not matter and nothing is cleared
    unsigned char *base = static_cast<unsigned char *>(buf);
    return dispatch_wgrad_into(*shape, G, X, row_scale_, idxW, cntW, dW, reinterpret_cast<float *>(base),
                               reinterpret_cast<uint16_t *>(base + wgrad_partial_bytes(*shape)), as_stream(stream));
}

vcas_status vcas_linear_backward(const vcas_shape *shape, const void *G, const void *X, const void *W, double rho,
                                 double nu, const vcas_rng *rng, int32_t token_sampling, const vcas_plan *plan,
                                 void *dX, float *dW, void *workspace, void *stream, void *side_stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !X || !rng || !plan_complete(plan)) return VCAS_ENULL;
    if (dX && !W) return VCAS_ENULL;
    if (!workspace) return VCAS_EWORKSPACE;
    if (!ratio_ok(rho) || !ratio_ok(nu)) return VCAS_EINVAL;
    if (!aligned16(G) || !aligned16(X) || (W && !aligned16(W)) || (dX && !aligned16(dX)) || (dW && !aligned16(dW)) ||
        (workspace && !aligned16(workspace)))
        return VCAS_EINVAL;
    return linear_backward_impl(*shape, G, X, W, rho, nu, *rng, token_sampling, *plan, dX, dW, workspace,
                                as_stream(stream), as_stream(side_stream));
}

vcas_status vcas_backward_stack(const vcas_layer_args *layers, int32_t L, int32_t group, void *stream,
                                void *sampler_stream, void *gemm_stream)
{
    if (!layers) return VCAS_ENULL;
    if (L <= 0 || group <= 0) return VCAS_EINVAL;
    hipStream_t st = as_stream(stream);
    hipStream_t s2 = sampler_stream ? as_stream(sampler_stream) : st;
    hipStream_t s3 = gemm_stream ? as_stream(gemm_stream) : s2;
    for (int l = 0; l < L; ++l) {
        const vcas_layer_args &a = layers[l];
        VCAS_TRY(check_shape(&a.shape));
        VCAS_TRY(check_gemm_limits(&a.shape));
        if (!a.G || !a.X || !plan_complete(&a.plan)) return VCAS_ENULL;
        if (a.dX && !a.W) return VCAS_ENULL;
        if (!a.workspace) return VCAS_EWORKSPACE;
        if (!ratio_ok(a.rho) || !ratio_ok(a.nu) || (a.xsq_forward && a.xsq_forward == a.plan.xsq)) return VCAS_EINVAL;
        if (a.wgrad_fill < 0) return VCAS_EINVAL;
        if (a.J && !a.dX) return VCAS_ENULL;
        if (a.J && !aligned16(a.J)) return VCAS_EINVAL;
        if ((a.g_sq_blocks || a.dx_sq_blocks) && a.shape.dtype != VCAS_BF16) return VCAS_EDTYPE;
        if (a.dx_sq_blocks && !a.dX) return VCAS_ENULL;
        if (a.g_sq_blocks && !a.kept_above) return VCAS_ENULL;
        if (!aligned16(a.g_sq_blocks) || !aligned16(a.dx_sq_blocks)) return VCAS_EINVAL;
        if (!aligned16(a.G) || !aligned16(a.X) || (a.W && !aligned16(a.W)) || (a.dX && !aligned16(a.dX)) ||
            (a.dW && !aligned16(a.dW)) || !aligned16(a.workspace))
            return VCAS_EINVAL;
    }
    // Groups of `group` layers; the last ones shrink (half of what is left), so that the side
    // streams are not a whole group behind when the main stream reaches the end of the stack.
    std::vector<int> first;
    for (int l = 0; l < L;) {
        first.push_back(l);
        const int left = L - l;
        int n = left > 2 * group ? group : (left + 1) / 2;
        if (n < 1) n = 1;
        while (l + n < L && layers[l + n].sibling) ++n;   // a run of siblings is not cut: it shares launches
        l += n;
    }
    first.push_back(L);
    const int groups = (int)first.size() - 1;
    // two events per group, created on first use and kept
    static std::vector<hipEvent_t> events;
    while ((int)events.size() < 2 * groups) {
        hipEvent_t ev;
        if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return VCAS_EHIP;
        events.push_back(ev);
    }
    // with a stream of its own for the weight halves, the norms of X go there too
    const XNorms xnorms_default = s2 != st ? kXNormsAfterSampleA : kXNormsByShape;
    // The host issues the data halves of group g + 1 before the side-stream work of group g: the
    // main stream, which carries the chain every other launch waits for, is then always a group
    // ahead of the host, whatever the side streams' launches cost it.
    auto issue_data = [&](int g) -> vcas_status {
        const int l0 = first[g], l1 = first[g + 1];
        for (int l = l0; l < l1;) {
            const vcas_layer_args &a = layers[l];
            // siblings share launches only where the norms of X are not taken beside those of G
            int n = 1;
            if (s2 != st)
                while (l + n < l1 && n < kMaxSiblings && shares_data_half(a, layers[l + n])) ++n;
            if (n > 1)
                VCAS_TRY(data_half_siblings(layers + l, n, st));
            else {
                ChainArgs chain;
                chain.J = a.J;
                chain.kept_above = a.kept_above;
                chain.fill = a.leave_dropped_rows == 0;
                chain.g_sq_blocks = a.g_sq_blocks;
                chain.dx_sq_blocks = a.dx_sq_blocks;
                VCAS_TRY(data_half(a.shape, a.G, a.X, a.W, a.rho, a.rng, a.token_sampling, a.plan, a.dX, chain,
                                   a.workspace, st,
                                   a.xsq_forward || a.g_sq_blocks ? kXNormsAfterSampleA : xnorms_default, true));
            }
            l += n;
        }
        if (s2 != st && hipEventRecord(events[2 * g], st) != hipSuccess) return VCAS_EHIP;
        return VCAS_OK;
    };
    auto issue_side = [&](int g) -> vcas_status {
        const int l0 = first[g], l1 = first[g + 1];
        if (s2 != st && hipStreamWaitEvent(s2, events[2 * g], 0) != hipSuccess) return VCAS_EHIP;
        for (int l = l0; l < l1;) {
            const vcas_layer_args &a = layers[l];
            int n = 1;
            if (s2 != st)
                while (l + n < l1 && n < kMaxSiblings && shares_weight_half(a, layers[l + n])) ++n;
            if (n > 1)
                VCAS_TRY(weight_half_siblings(layers + l, n, s2));
            else
                VCAS_TRY(weight_half(a.shape, a.G, a.X, a.rho, a.nu, a.rng, a.token_sampling, a.plan, nullptr,
                                     a.workspace, s2,
                                     a.xsq_forward || a.g_sq_blocks ? kXNormsAfterSampleA : xnorms_default,
                                     a.xsq_forward));
            l += n;
        }
        if (s3 != s2 && (hipEventRecord(events[2 * g + 1], s2) != hipSuccess ||
                         hipStreamWaitEvent(s3, events[2 * g + 1], 0) != hipSuccess))
            return VCAS_EHIP;
        VCAS_TRY(wgrad_of_layers(layers, l0, l1, s3));
            return VCAS_OK;
    };
    VCAS_TRY(issue_data(0));
    for (int g = 0; g < groups; ++g) {
        if (g + 1 < groups) VCAS_TRY(issue_data(g + 1));
        VCAS_TRY(issue_side(g));
    }
    return VCAS_OK;
}

vcas_status vcas_backward_data(const vcas_shape *shape, const void *G, const void *X, const void *W, double rho,
                               const vcas_rng *rng, int32_t token_sampling, const vcas_plan *plan, void *dX,
                               void *workspace, void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !X || !rng || !plan_complete(plan)) return VCAS_ENULL;
    if (dX && !W) return VCAS_ENULL;
    if (!workspace) return VCAS_EWORKSPACE;
    if (!ratio_ok(rho)) return VCAS_EINVAL;
    if (!aligned16(G) || !aligned16(X) || (W && !aligned16(W)) || (dX && !aligned16(dX)) || !aligned16(workspace))
        return VCAS_EINVAL;
    return data_half(*shape, G, X, W, rho, *rng, token_sampling, *plan, dX, ChainArgs(), workspace, as_stream(stream));
}

vcas_status vcas_backward_data_chained(const vcas_shape *shape, const void *G, const void *X, const void *W,
                                       const void *J, const uint8_t *kept_above, int32_t fill_dropped_rows,
                                       double rho, const vcas_rng *rng, int32_t token_sampling,
                                       const vcas_plan *plan, void *dX, void *workspace, void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !X || !rng || !plan_complete(plan)) return VCAS_ENULL;
    if (dX && !W) return VCAS_ENULL;
    if (J && !dX) return VCAS_ENULL;
    if (!workspace) return VCAS_EWORKSPACE;
    if (!ratio_ok(rho)) return VCAS_EINVAL;
    if (!aligned16(G) || !aligned16(X) || (W && !aligned16(W)) || (J && !aligned16(J)) || (dX && !aligned16(dX)) ||
        !aligned16(workspace))
        return VCAS_EINVAL;
    ChainArgs chain;
    chain.J = J;
    chain.kept_above = kept_above;
    chain.fill = fill_dropped_rows != 0;
    return data_half(*shape, G, X, W, rho, *rng, token_sampling, *plan, dX, chain, workspace, as_stream(stream));
}

vcas_status vcas_backward_weight(const vcas_shape *shape, const void *G, const void *X, double rho, double nu,
                                 const vcas_rng *rng, int32_t token_sampling, const vcas_plan *plan, float *dW,
                                 void *workspace, void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !X || !rng || !plan_complete(plan)) return VCAS_ENULL;
    if (!workspace) return VCAS_EWORKSPACE;
    if (!ratio_ok(rho) || !ratio_ok(nu)) return VCAS_EINVAL;
    if (!aligned16(G) || !aligned16(X) || (dW && !aligned16(dW)) || !aligned16(workspace)) return VCAS_EINVAL;
    return weight_half(*shape, G, X, rho, nu, *rng, token_sampling, *plan, dW, workspace, as_stream(stream));
}

vcas_status vcas_backward_weight_cached(const vcas_shape *shape, const void *G, const void *X, const float *xsq_forward,
                                        double rho, double nu, const vcas_rng *rng, int32_t token_sampling,
                                        const vcas_plan *plan, float *dW, void *workspace, void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !X || !xsq_forward || !rng || !plan_complete(plan)) return VCAS_ENULL;
    if (!workspace) return VCAS_EWORKSPACE;
    if (!ratio_ok(rho) || !ratio_ok(nu) || xsq_forward == plan->xsq) return VCAS_EINVAL;
    if (!aligned16(G) || !aligned16(X) || (dW && !aligned16(dW)) || !aligned16(workspace)) return VCAS_EINVAL;
    return weight_half(*shape, G, X, rho, nu, *rng, token_sampling, *plan, dW, workspace, as_stream(stream),
                       kXNormsAfterSampleA, xsq_forward);
}

vcas_status vcas_variance_probe(const vcas_shape *shape, const void *G, const void *X, double rho, double nu,
                                const vcas_rng *base, int32_t M, const vcas_plan *plan, double *out, void *workspace,
                                void *stream)
{
    VCAS_TRY(check_shape(shape));
    VCAS_TRY(check_gemm_limits(shape));
    if (!G || !X || !base || !out || !plan_complete(plan)) return VCAS_ENULL;
    if (!workspace) return VCAS_EWORKSPACE;
    if (!ratio_ok(rho) || !ratio_ok(nu) || M <= 0) return VCAS_EINVAL;
    if (!aligned16(G) || !aligned16(X) || !aligned16(workspace)) return VCAS_EINVAL;
    const vcas_shape &s = *shape;
    hipStream_t st = as_stream(stream);
    const WorkspaceLayout w = workspace_layout(&s);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    float *exact = reinterpret_cast<float *>(ws + w.probe_exact);
    float *draw = reinterpret_cast<float *>(ws + w.probe_draw);
    double *partial = reinterpret_cast<double *>(ws + w.probe_acc);  // 32 doubles
    const int64_t R = (int64_t)s.N * s.T, nW = (int64_t)s.K_out * s.K_in;
    const int blocks = 32;
    const double wgt = 1.0 / (double)M;

    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(64), 0, st, reinterpret_cast<uint32_t *>(out), (size_t)8);
    if (hipGetLastError() != hipSuccess) return VCAS_EHIP;
    vcas_rng rng = *base;
    VCAS_TRY(linear_backward_impl(s, G, X, nullptr, 1.0, 1.0, rng, 1, *plan, nullptr, exact, workspace, st, nullptr));
    for (int j = 0; j < M; ++j) {
        rng.draw = base->draw + (uint32_t)j;
        // SampleA only
        VCAS_TRY(linear_backward_impl(s, G, X, nullptr, rho, nu, rng, 0, *plan, nullptr, draw, workspace, st, nullptr));
        hipLaunchKernelGGL(sq_diff_partial_kernel, dim3(blocks), dim3(256), 0, st, draw, exact, nW, partial);
        hipLaunchKernelGGL(sq_diff_final_kernel, dim3(1), dim3(64), 0, st, partial, blocks, wgt, out + 2);
        // SampleA and SampleW
        VCAS_TRY(linear_backward_impl(s, G, X, nullptr, rho, nu, rng, 1, *plan, nullptr, draw, workspace, st, nullptr));
        hipLaunchKernelGGL(sq_diff_partial_kernel, dim3(blocks), dim3(256), 0, st, draw, exact, nW, partial);
        hipLaunchKernelGGL(sq_diff_final_kernel, dim3(1), dim3(64), 0, st, partial, blocks, wgt, out + 3);
        if (j == 0)
            hipLaunchKernelGGL(var_closed_kernel, dim3(1), dim3(256), 0, st, plan->p, plan->gnorm, (int64_t)s.N, 1,
                               1.0, 0, out + 0);
        hipLaunchKernelGGL(var_closed_kernel, dim3(1), dim3(256), 0, st, plan->q, plan->score, R, 1, wgt, 1, out + 1);
        if (hipGetLastError() != hipSuccess) return VCAS_EHIP;
    }
    return VCAS_OK;
}

vcas_status vcas_profile_begin(void)
{
    KernelTimer &t = kernel_timer();
    for (auto &v : t.pairs) {
        for (auto &pr : v) {
            (void)hipEventDestroy(pr.first);
            (void)hipEventDestroy(pr.second);
        }
        v.clear();
    }
    t.on = true;
    return VCAS_OK;
}

vcas_status vcas_profile_end(double *total_ms, int64_t *launches)
{
    if (!total_ms || !launches) return VCAS_ENULL;
    KernelTimer &t = kernel_timer();
    t.on = false;
    vcas_status status = VCAS_OK;
    for (int w = 0; w < 2; ++w) {
        total_ms[w] = 0.0;
        launches[w] = 0;
        for (auto &pr : t.pairs[w]) {
            float ms = 0.0f;
            if (hipEventSynchronize(pr.second) == hipSuccess && hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) {
                total_ms[w] += ms;
                ++launches[w];
            } else {
                status = VCAS_EHIP;
            }
            (void)hipEventDestroy(pr.first);
            (void)hipEventDestroy(pr.second);
        }
        t.pairs[w].clear();
    }
    return status;
}

}  // extern "C"
