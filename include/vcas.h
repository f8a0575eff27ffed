/*
 * vcas.h -- C ABI of the MI355X (gfx950) library for the sampled backward pass
 * of a transformer linear layer Z = X W^T under VCAS, "variance-controlled
 * adaptive sampling" (Wang, Chen, Zhu, ICLR 2024).
 *
 * Notation follows the paper (Sec. 4): batch N, tokens per sample T, rows
 * R = N*T, G = grad of Z [R, K_out], X = layer input [R, K_in],
 * W [K_out, K_in], data keep ratio rho, token keep ratio nu, data keep
 * probabilities p[N], token keep probabilities q[R].
 *
 * Conventions that hold for every call:
 *  - Every pointer is a DEVICE pointer unless its comment says "host".
 *    Structs (vcas_shape, vcas_rng, vcas_plan, vcas_layer_args) are read on the host.
 *  - Tensors are dense row-major.  dtype VCAS_F32: float; VCAS_BF16: 16-bit
 *    bfloat16 bit patterns.  K_in and K_out must be multiples of 8 (one 16-byte
 *    vector of bf16; fp32 needs only a multiple of 4 but the same rule is kept),
 *    and tensor base addresses 16-byte aligned.
 *  - The caller owns every buffer.  The library allocates no device memory;
 *    calls that need scratch take a `workspace` of at least
 *    vcas_workspace_bytes(shape) bytes, 16-byte aligned, on which
 *    vcas_workspace_init has run once; the rest of its contents don't matter.
 *    bf16 tensors must be smaller than 2 GiB each and K_in, K_out <= 8184
 *    (buffer-addressing limits of the GEMM kernels).
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *    default stream); calls return without synchronising.  Kept counts stay on
 *    the device.  Two calls that share a workspace must be ordered (same stream).
 *  - Errors are reported by the return value and detected on the host before
 *    anything is launched (null pointer, non-positive size, bad dtype, keep
 *    ratio outside (0,1], K not a multiple of 8).  Nothing throws or exits.
 *  - Results are a pure function of the arguments: the same inputs, seed,
 *    layer and draw give the same bits on every call and launch geometry.
 */
#ifndef VCAS_H
#define VCAS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VCAS_OK = 0,
    VCAS_EINVAL = 1,     /* size / ratio / alignment out of range */
    VCAS_ENULL = 2,      /* required pointer is null */
    VCAS_EDTYPE = 3,     /* dtype is neither VCAS_F32 nor VCAS_BF16 */
    VCAS_EWORKSPACE = 4, /* workspace missing */
    VCAS_EHIP = 5,       /* a HIP launch failed; hipGetLastError has the cause */
    VCAS_ETOOBIG = 6     /* the problem needs more scratch than the library's static buffer holds */
} vcas_status;

typedef enum { VCAS_F32 = 0, VCAS_BF16 = 1 } vcas_dtype;

typedef struct {
    int32_t N, T, K_in, K_out;
    int32_t dtype; /* vcas_dtype of G, X, W and dX */
} vcas_shape;

/* Randomness of one layer and one draw.  Row r of sampler s (0 = SampleA over
 * samples, 1 = SampleW over tokens) is decided by the Philox4x32-10 block with
 * counter (r, layer, s, draw) and key (seed low word, seed high word): the top
 * 24 bits of output word 0, scaled to [0,1), are compared with the keep
 * probability.  (The paper writes Bern(p; eps) without naming a generator.)
 * draw_offset, if not null, is a DEVICE pointer to one uint32 that the kernels
 * add to `draw` when they run: a caller that replays a captured HIP graph
 * bumps that word between replays to get fresh masks without new launches. */
typedef struct {
    uint64_t seed;
    uint32_t layer;
    uint32_t draw;
    const uint32_t *draw_offset;
} vcas_rng;

/* Everything the sampling steps decide for one layer; all device pointers,
 * all required, caller-allocated. */
typedef struct {
    float *gsq;     /* [R]  ||g_t||^2                                   */
    float *gnorm;   /* [N]  ||G_i||_F                                   */
    float *p;       /* [N]  data keep probabilities, sum = min(N rho, #nonzero) */
    uint8_t *maskA; /* [N]  1 = sample kept                             */
    int32_t *idxA;  /* [N]  kept samples, ascending; first *cntA valid  */
    int32_t *cntA;  /* [1]                                              */
    float *xsq;     /* [R]  ||x_t||^2 for rows of kept samples, else 0  */
    float *score;   /* [R]  leverage score ||ghat_t|| ||x_t||           */
    float *q;       /* [R]  token keep probabilities                    */
    uint8_t *maskW; /* [R]  1 = token kept                              */
    int32_t *idxW;  /* [R]  kept tokens, ascending; first *cntW valid   */
    int32_t *cntW;  /* [1]                                              */
    float *scaleW;  /* [R]  1/(p_i q_t) for kept tokens, else 0         */
} vcas_plan;

const char *vcas_status_string(vcas_status s);

/* Bytes of scratch the calls below need for this shape (host query; 0 on a
 * bad shape). */
size_t vcas_workspace_bytes(const vcas_shape *shape);

/*
 * Zeroes the workspace's control words, its first 8 KiB (a small fill kernel on
 * `stream`, so the call may be captured in a graph).  Must run once after the
 * buffer is allocated and before vcas_linear_backward or vcas_variance_probe
 * first use it: the launch that fuses the row norms with SampleA and SampleW
 * (Sec. 4.1, 4.2) counts finished workgroups there to find the last one.  Every
 * call leaves the words zero again, so one initialisation lasts as long as the
 * buffer; it is needed again only after a call was aborted mid-flight.
 */
vcas_status vcas_workspace_init(const vcas_shape *shape, void *workspace, void *stream);

/*
 * Squared row norms, the ||.||_2^2 factors of Eq. 3 and the ||G_i||_F of
 * Sec. 4.1.  G [R,K_out] and/or X [R,K_in] (either may be null, not both).
 *   gsq[t]   = sum_k G[t,k]^2            (required if G is given)
 *   gnorm[i] = sqrt(sum_{t in i} gsq[t]) (optional, needs G)
 *   xsq[t]   = sum_k X[t,k]^2, or 0 if sample_mask is given and the row's
 *              sample has mask 0        (required if X is given)
 * fp32, each row summed in a fixed order that does not depend on the launch:
 * pairwise, neighbours first.  The squares v*v (fp32 product of the element's
 * fp32 image, one rounding), padded with +0 to the next power of two, are added
 * as a balanced binary tree in index order: s[2m] + s[2m+1] first, then those
 * results pairwise, and so on.  gnorm: value t of a sample on accumulator
 * t mod 64, accumulators add their values in ascending t and are combined by
 * the same kind of tree (2m with 2m+1, distances 1, 2, 4, 8, 16, 32), then a
 * correctly rounded square root.
 */
vcas_status vcas_row_norms(const vcas_shape *shape, const void *G, const void *X,
                           const uint8_t *sample_mask, float *gsq, float *xsq, float *gnorm,
                           void *stream);

/*
 * Keep probabilities proportional to score[n] (Sec. 4.1: p_i ~ ||G_i||_F with
 * sum N rho; Sec. 4.2: q_t ~ leverage score with sum N T rho nu), capped at
 * one: prob_i = min(1, c score_i) with c such that sum prob = min(budget,
 * number of positive scores); zero (or negative) scores get 0.  Scores must be
 * finite.  Sums are taken in fp64 in a fixed order; prob is fp32.
 */
vcas_status vcas_keep_probs(const float *score, int32_t n, double budget, float *prob, void *stream);

/*
 * Bernoulli masks and the kept-row list (Sec. 4.1 / 4.2: m = Bern(p)/p; the
 * division is applied later as a scale).  mask[r] = [u_r < prob[r]] with u_r
 * from vcas_rng and stream_id (0 = SampleA, 1 = SampleW); idx = kept r in
 * ascending order (idx has room for n entries; entries past *count are left
 * untouched); *count = number kept.
 */
vcas_status vcas_sample_compact(const float *prob, int32_t n, const vcas_rng *rng, uint32_t stream_id,
                                uint8_t *mask, int32_t *idx, int32_t *count, void *stream);

/* Leverage scores of Sec. 4.2 on the already data-sampled gradient:
 * score[t] = maskA[i] * ((1/p[i]) * sqrt(gsq[t])) * sqrt(xsq[t]), fp32. */
vcas_status vcas_leverage_scores(const vcas_shape *shape, const float *gsq, const float *xsq,
                                 const float *p, const uint8_t *maskA, float *score, void *stream);

/* scaleW[t] = maskW[t] ? 1 / (p[i] * q[t]) : 0, the product of the two masks'
 * 1/probability factors that a kept token carries into the weight gradient. */
vcas_status vcas_row_scale(const vcas_shape *shape, const float *p, const float *q,
                           const uint8_t *maskW, float *scaleW, void *stream);

/*
 * Sampled activation gradient (Eq. 2, upper line; SampleA only):
 *   dX[r,:] = (1/p[i]) * G[r,:] W   for the T rows r of every kept sample i,
 *   dX[r,:] = 0                     for rows of dropped samples.
 * idxA/cntA: kept samples ascending and their count (device).  dX [R,K_in] in
 * the layer dtype is written completely.  bf16: MFMA with fp32 accumulation;
 * fp32: fp32 MFMA.
 */
vcas_status vcas_sampled_dgrad(const vcas_shape *shape, const void *G, const void *W, const float *p,
                               const int32_t *idxA, const int32_t *cntA, void *dX, void *stream);

/*
 * The same through an elementwise layer below the linear one (App. E, proof of unbiasedness: for a
 * non-linear layer such as ReLU the activation gradient is multiplied, entry by
 * entry, by the Jacobian saved in the forward pass):
 *   dX[r,:] = ((1/p[i]) * G[r,:] W) * J[r,:]   on rows of kept samples, 0 elsewhere.
 * J [R,K_in], device, layer dtype, 16-byte aligned, read on kept rows only; the
 * product is formed in fp32 before the one rounding to the layer dtype.  What
 * comes out is the output gradient of the layer below the elementwise one.
 */
vcas_status vcas_sampled_dgrad_jac(const vcas_shape *shape, const void *G, const void *W, const float *p,
                                   const int32_t *idxA, const int32_t *cntA, const void *J, void *dX,
                                   void *stream);

/*
 * The norms of a layer's incoming gradient from the launch that produced it.  In a
 * stack of layers the G of a layer is the dX the layer above has just written
 * (Sec. 4: samplers at every layer), and Sec. 4.1 needs ||G_i||_F of it; a second
 * pass over HBM for those norms is avoided by letting the dgrad epilogue add up the
 * squares of what it stores.
 * vcas_sampled_dgrad_norms: vcas_sampled_dgrad_jac (J may be null: no Jacobian)
 * that also writes, for every row r of a kept sample and every block b of 64
 * columns, the sum of squares of dX[r, 64 b .. 64 b + 63] as stored (after the
 * rounding to bf16), b < nb = ceil(K_in / 64); pairwise, neighbours first, i.e.
 * the 64-column subtrees of the order vcas_row_norms uses.  Layout: four
 * neighbouring blocks of a row side by side,
 *   sq_blocks[((b / 4) * R + r) * 4 + b % 4],
 * so that both sides move 16 bytes per row and neighbouring rows touch
 * neighbouring addresses; vcas_sq_blocks_bytes gives the size.  Slots with
 * b >= nb and rows of dropped samples are not written.  bf16 only (VCAS_EDTYPE
 * otherwise).  sq_blocks 16-byte aligned.
 * vcas_row_norms_from_blocks: sq[r] = the nb block sums of row r added pairwise,
 * neighbours first (zero-padded to a power of two): bit for bit what
 * vcas_row_norms computes from the stored matrix itself.  K = row length of that
 * matrix; sample_mask (N bytes, null: all): rows of samples with mask 0 are not
 * read and get 0 (pass the producing layer's maskA).  norm (null: skip): the
 * per-sample Frobenius norms, as vcas_row_norms' gnorm.
 * vcas_sq_blocks_bytes (host query): bytes of the block sums of a matrix of R
 * rows and K columns, 16 R ceil(ceil(K / 64) / 4); 0 on bad sizes.
 */
size_t vcas_sq_blocks_bytes(int64_t R, int32_t K);
vcas_status vcas_sampled_dgrad_norms(const vcas_shape *shape, const void *G, const void *W, const float *p,
                                     const int32_t *idxA, const int32_t *cntA, const void *J, void *dX,
                                     float *sq_blocks, void *stream);
vcas_status vcas_row_norms_from_blocks(int32_t N, int32_t T, int32_t K, const float *sq_blocks,
                                       const uint8_t *sample_mask, float *sq, float *norm, void *stream);

/*
 * Sampled weight gradient (Sec. 4.2, grad_W = Gtilde^T X):
 *   dW[o,k] = sum over the *cntW rows t = idxW[.] of row_scale[t] G[t,o] X[t,k].
 * dW [K_out,K_in] fp32 is overwritten.  Needs the workspace (split-K partial
 * tiles, added up in a fixed order by a second small launch, so the result is
 * deterministic).
 */
vcas_status vcas_sampled_wgrad(const vcas_shape *shape, const void *G, const void *X,
                               const float *row_scale, const int32_t *idxW, const int32_t *cntW,
                               float *dW, void *workspace, void *stream);

/*
 * vcas_sampled_wgrad for callers that cannot allocate or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without `workspace`, same kernels, the same bits in
 * dW.  The split-K partial tiles go to a buffer of vcas_static_scratch_bytes()
 * (64 MiB) that is part of the library's device image: each GPU the library runs
 * on holds its own copy until the process ends, and its address is looked up once
 * per device, on the first call there (with that device current).  The call
 * allocates and frees nothing.  A shape whose partial tiles do not fit
 * (K_out * K_in * 4 bytes times the number of split-K slices, at most 8) is
 * refused with VCAS_ETOOBIG before anything is launched; every shape of the
 * benchmark configurations fits.  All calls on one GPU share that buffer: calls
 * that may overlap there (different streams without an ordering between them,
 * different host threads) race on it and must be ordered by the caller.  Nothing
 * needs clearing between calls: the kernels overwrite what they later read.
 */
size_t vcas_static_scratch_bytes(void);
vcas_status vcas_sampled_wgrad_static(const vcas_shape *shape, const void *G, const void *X,
                                      const float *row_scale, const int32_t *idxW, const int32_t *cntW,
                                      float *dW, void *stream);

/*
 * The whole path for one layer and one draw, in the paper's order: row norms
 * of G, p, SampleA mask, dX; row norms of X on kept samples, leverage scores,
 * q, SampleW mask, scale, dW.  Fills every field of *plan.  With
 * token_sampling = 0 SampleW is skipped (Alg. 1's "SampleA only" backward):
 * q = maskW = the data mask repeated over tokens.  dX may be null (skip the
 * activation gradient), dW may be null.
 *
 * side_stream (a second hipStream_t, or null): the weight-gradient half of the
 * path (row norms of X, SampleW, dW) depends only on SampleA's outcome, not on
 * dX, so with a side stream it is enqueued there, ordered after SampleA by an
 * event, while dX proceeds on `stream`.  The call does NOT join the two: xsq,
 * score, q, maskW, idxW, cntW, scaleW and dW are complete once side_stream has
 * drained (the caller waits on it, or makes `stream` wait for it with an
 * event).  Consecutive calls may share one side stream; their weight-gradient
 * halves then run in call order behind each other.  Both streams must have the
 * default priority.  With side_stream null everything is on `stream`.
 * The event that orders the two streams belongs to the library and is shared
 * by all calls: with a side stream, call this (and every other entry point that
 * takes more than one stream) from one host thread at a time.
 */
vcas_status vcas_linear_backward(const vcas_shape *shape, const void *G, const void *X, const void *W,
                                 double rho, double nu, const vcas_rng *rng, int32_t token_sampling,
                                 const vcas_plan *plan, void *dX, float *dW, void *workspace,
                                 void *stream, void *side_stream);

/* One layer of a stack: the arguments of vcas_linear_backward (host struct), then optional
 * fields, every one of which is off when zero: a zero-initialised tail gives the plain layer. */
typedef struct {
    vcas_shape shape;
    const void *G, *X, *W;
    double rho, nu;
    vcas_rng rng;
    int32_t token_sampling;
    vcas_plan plan;
    void *dX;        /* may be null */
    float *dW;       /* may be null */
    void *workspace; /* of this layer's shape; layers must not share one */
    const float *xsq_forward; /* null, or the cached row norms of X: see vcas_backward_weight_cached */
    int32_t sibling; /* nonzero: this layer's G does not depend on the dX of the entry before it (the
                        Q, K and V projections of one attention block all get their gradients from
                        the attention backward), so vcas_backward_stack may launch the two data
                        halves together instead of one behind the other; results are the same bits */
    /* The three additions of vcas_backward_data_chained, for a stack whose entries feed each other
       (an entry's dX buffer is the next entry's G): all optional, zero = off. */
    const void *J;             /* elementwise Jacobian [R,K_in] multiplied into dX; needs dX */
    const uint8_t *kept_above; /* N bytes, device: 0 = sample dropped by a layer above (its rows of G are
                                  never read); usually the maskA array of the previous entry's plan */
    int32_t leave_dropped_rows; /* nonzero: rows of dX of samples this layer does not keep are not written */
    int32_t wgrad_fill; /* 0, or how many workgroups the weight-gradient launch should have before it stops
                           cutting the contraction into split-K slices (1..384; larger values count as 384).
                           0 = 384, what every other entry point uses: right for a launch that has the chip
                           to itself.  Beside the data chain of a stack fewer, longer slices (64) make the
                           step shorter.  The number of slices fixes the order of a weight gradient's sums:
                           dW is the same bits for the same value of this field, and within rounding
                           (fp32 sums in another order) across values. */
    /* The norms of G from the launch that wrote G (see vcas_sampled_dgrad_norms), for entries that feed
       each other; bf16 only, both optional. */
    float *dx_sq_blocks;       /* vcas_sq_blocks_bytes(R, K_in) bytes, device: this entry's dgrad also leaves the block sums of
                                  squares of its dX here (rows of kept samples only); needs dX */
    const float *g_sq_blocks;  /* vcas_sq_blocks_bytes(R, K_out) bytes, device: block sums of squares of this entry's G, as
                                  the entry that wrote G left them; the pass over G is replaced by a pass over
                                  them (the same bits), which for N <= 64 and T <= 1024 also leaves the sample
                                  norms, so that dgrad decides SampleA itself and no launch of its own does.
                                  Needs kept_above: rows of samples dropped above have no block sums */
} vcas_layer_args;

/*
 * A stack of L layers in one call: computes, bit for bit, what calling
 * vcas_linear_backward on layers[0], layers[1], ... computes (dW: where wgrad_fill
 * is left at zero; see there), with the launches
 * laid out over up to three streams so that a dependency between streams is
 * paid once per group of layers instead of once per layer (on this hardware a
 * cross-stream wait costs about as much as two small kernels):
 *   stream          data halves (row norms of G, SampleA, dX) in layer order, as
 *                   a backward pass imposes;
 *   sampler_stream  for each group of `group` consecutive layers, after the
 *                   group's last SampleA: row norms of X where still due, SampleW;
 *   gemm_stream     after the group's SampleW: dW (and its split-K reduction).
 * Consecutive entries marked `sibling` that have one shape may share the launches
 * of their data halves and of their weight gradients (up to four layers per
 * launch); a group is extended rather than cut inside such a run.
 * Towards the end of the stack the groups shrink (each takes half of the layers
 * that are left), so that the side streams finish shortly after `stream`.
 * sampler_stream and gemm_stream may be the same stream, or null (= `stream`).
 * layers: HOST array, read during the call only.  group >= 1.  The call joins
 * nothing: results of the weight halves are complete when the streams they ran
 * on have drained, and work that reuses any of the layers' buffers (the next
 * call on the same stack included) must be ordered after all three streams.
 * All streams at default priority.  Meant for eager launching; under graph
 * capture it is correct but gains nothing over per-layer calls.
 * Every layer's arguments are checked before anything is launched.  The events
 * that order the streams belong to the library and are shared by all calls:
 * call it from one host thread at a time.
 */
vcas_status vcas_backward_stack(const vcas_layer_args *layers, int32_t L, int32_t group, void *stream,
                                void *sampler_stream, void *gemm_stream);

/*
 * The two halves of vcas_linear_backward as calls of their own, for callers
 * that schedule them apart (e.g. the weight gradients of a block of layers on a
 * second stream while the chain of activation gradients goes on).
 * vcas_backward_data: row norms of G, p, SampleA mask and kept list (Sec. 4.1),
 * dX (Eq. 2, upper line; dX may be null); on small layers also the row norms of
 * X and the SampleW uniforms, which do not depend on SampleA.  Fills gsq, gnorm,
 * p, maskA, idxA, cntA of *plan; the score and q arrays of *plan carry
 * intermediate values (square roots of the row norms) to the weight call and
 * must be left alone until it has run: one weight call per data call.
 * vcas_backward_weight: must be ordered after vcas_backward_data with the same
 * shape, G, X, rho, rng, token_sampling, plan and workspace (same stream, or an
 * event).  Row norms of X on kept samples if not taken yet, leverage scores, q,
 * SampleW mask, scale (Sec. 4.2), dW (may be null).  Fills the remaining fields
 * of *plan.  Together the two calls compute bit for bit what
 * vcas_linear_backward computes.
 */
vcas_status vcas_backward_data(const vcas_shape *shape, const void *G, const void *X, const void *W,
                               double rho, const vcas_rng *rng, int32_t token_sampling,
                               const vcas_plan *plan, void *dX, void *workspace, void *stream);
/*
 * vcas_backward_data for a layer inside a stack of layers (Sec. 4: the
 * activation gradient grows sparser layer by layer; App. E: elementwise layers
 * in between multiply by their Jacobian).  Three additions, each optional:
 *   J (null: none): elementwise Jacobian [R,K_in] of the layer below, multiplied
 *     into dX as in vcas_sampled_dgrad_jac; needs dX.
 *   kept_above (null: all): N bytes, device; 0 marks a sample that a layer above
 *     has dropped.  Its rows of G are never read and count as zero, so it gets
 *     p_i = 0 and stays dropped.  The maskA array of the upper layer's plan can
 *     be passed as it is.
 *   fill_dropped_rows: 0 leaves the rows of dX that belong to samples this layer
 *     does not keep as they are (for a consumer that gets this layer's maskA as
 *     its kept_above); otherwise they are written as zeros.
 * The weight call that follows is vcas_backward_weight, unchanged: it reads rows
 * of kept tokens only.
 */
vcas_status vcas_backward_data_chained(const vcas_shape *shape, const void *G, const void *X, const void *W,
                                       const void *J, const uint8_t *kept_above, int32_t fill_dropped_rows,
                                       double rho, const vcas_rng *rng, int32_t token_sampling,
                                       const vcas_plan *plan, void *dX, void *workspace, void *stream);
vcas_status vcas_backward_weight(const vcas_shape *shape, const void *G, const void *X, double rho,
                                 double nu, const vcas_rng *rng, int32_t token_sampling,
                                 const vcas_plan *plan, float *dW, void *workspace, void *stream);

/*
 * vcas_backward_weight for a caller that already has the squared row norms of X
 * (the ||x_t||^2 of Eq. 3): X is an input of the forward pass, so its norms can
 * be taken there, once, by vcas_row_norms (xsq of EVERY row, no sample_mask) and
 * kept with the activations.  xsq_forward [R] is read instead of sweeping the
 * kept rows of X again; everything else, and every bit of the results, is as in
 * vcas_backward_weight (plan->xsq receives the norms with zeros on dropped
 * samples, as there).  xsq_forward must not be plan->xsq.  Whatever the data
 * call may have prepared for the weight call (on small layers it takes the norms
 * of X beside those of G) is ignored; vcas_backward_stack skips that work for
 * layers whose xsq_forward is set.
 */
vcas_status vcas_backward_weight_cached(const vcas_shape *shape, const void *G, const void *X,
                                        const float *xsq_forward, double rho, double nu,
                                        const vcas_rng *rng, int32_t token_sampling,
                                        const vcas_plan *plan, float *dW, void *workspace, void *stream);

/*
 * Variance probe for the adaptive keep ratios (Sec. 4.1 variance, Eq. 3, and
 * the Monte-Carlo lines of Alg. 1) over M mask draws, draw j using
 * rng.draw = base->draw + j.  out[4] (device, fp64):
 *   out[0] = sum_i (1-p_i)/p_i ||G_i||_F^2
 *   out[1] = mean_j of Eq. 3, sum_t (1-q_t)/q_t score_t^2, under draw j's data mask
 *   out[2] = mean_j ||dW(SampleA only, draw j) - dW exact||_F^2
 *   out[3] = mean_j ||dW(SampleA and SampleW, draw j) - dW exact||_F^2
 * dW exact is this library's dW at keep ratio one.  `plan` is scratch for the
 * draws (left holding the last one).
 */
vcas_status vcas_variance_probe(const vcas_shape *shape, const void *G, const void *X, double rho,
                                double nu, const vcas_rng *base, int32_t M, const vcas_plan *plan,
                                double *out, void *workspace, void *stream);

/*
 * Adaptive keep ratios (Sec. 5).  One update of Alg. 1 needs, besides the probe
 * above: Eq. 4's gradient-norm sparsity of every layer at s - alpha and
 * s + alpha, the SGD variance V_s from the running mean and running mean of
 * squares that App. D keeps on a subset of the parameters, the squared
 * difference of V_act on the same subset, and the update rules themselves.
 *
 * vcas_sparsity_ratio: Eq. 4, p(s) = min{ n/N : the n largest of gnorm[N] sum to
 * at least s times the sum of all }, n >= 1 (the paper leaves "largest" unsaid;
 * fp64 sums over the norms in descending order).  s: HOST array of ns <= 8 levels
 * in [0,1]; p: device [ns].  N <= 1024.
 */
vcas_status vcas_sparsity_ratio(const float *gnorm, int32_t N, const double *s, int32_t ns, float *p,
                                void *stream);

/*
 * App. D's running statistics over entries 0, stride, 2*stride, ... of a
 * gradient (m entries): after the call with index i = 1, 2, ... `mean` and
 * `sqmean` (device [m], zero before i = 1) hold the mean and the mean of squares
 * of the first i gradients (fp32: mean += (x - mean)/i, sqmean += (x*x - sqmean)/i).
 * vcas_grad_stats_variance: Alg. 1's V_s = 1/(M-1) sum_i ||g_i - gbar||^2
 * = M/(M-1) sum_j (sqmean_j - mean_j^2), fp64, into out[0] (device).
 * vcas_sq_diff_strided: out[0] = (accumulate ? out[0] : 0) + weight * sum over
 * the same subset of (a - b)^2 (Alg. 1's V_act line on the kept parameters).
 */
vcas_status vcas_grad_stats_update(const float *grad, int64_t m, int64_t stride, int32_t i, float *mean,
                                   float *sqmean, void *stream);
vcas_status vcas_grad_stats_variance(const float *mean, const float *sqmean, int64_t m, int32_t M,
                                     double *out, void *stream);
vcas_status vcas_sq_diff_strided(const float *a, const float *b, int64_t m, int64_t stride, double weight,
                                 int32_t accumulate, double *out, void *stream);

/*
 * The update rules of Alg. 1, HOST arithmetic on HOST pointers (nothing is
 * launched).  Layers 0..L-1 run from the input to the output.
 *   Eq. 5: *s += alpha * sign(V_act - tau_act * V_s), sign(0) = +1, kept in [0,1];
 *   Eq. 4: rho[l] = max_{j <= l} p_j, with p_j = p_plus[j] if s went up, else
 *          p_minus[j] (App. D: both sides are measured inside the loops);
 *   Eq. 7: nu[l] *= beta^{-sign(V_w[l] - tau_w * V_s_layer[l])}, kept in [nu_min, 1].
 *          As printed (beta^{+sign}, beta < 1) the rule would lower the keep ratio
 *          when the variance is too high; the sign is read so that it raises it.
 * Requires 0 < beta < 1, alpha > 0, 0 < nu_min <= 1.
 */
typedef struct {
    double alpha;   /* step of s                         */
    double beta;    /* multiplier of nu, in (0,1)         */
    double tau_act; /* tolerated V_act / V_s              */
    double tau_w;   /* tolerated V_w,l / V_s,l            */
    double nu_min;  /* floor of the token keep ratio      */
} vcas_controller_params;

vcas_status vcas_controller_update(const vcas_controller_params *prm, int32_t L, double *s, double *rho,
                                   double *nu, double V_s, double V_act, const double *V_w,
                                   const double *V_s_layer, const double *p_minus, const double *p_plus);

/*
 * Profiling aid, not part of the method: between vcas_profile_begin and
 * vcas_profile_end every dgrad / wgrad GEMM launch (Eq. 2 upper line resp.
 * Sec. 4.2's grad_W) is bracketed by HIP events stamped by the kernel's own
 * dispatch.  vcas_profile_end waits for them and returns, in HOST arrays of two
 * entries ([0] dgrad, [1] wgrad), the summed kernel durations in milliseconds
 * and the number of launches.  Not for use under graph capture; creates and
 * destroys HIP events (the only calls of the library that do).
 */
vcas_status vcas_profile_begin(void);
vcas_status vcas_profile_end(double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* VCAS_H */
