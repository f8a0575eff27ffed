// Argument blocks of the grouped launches: several layers of one shape whose upstream gradients
// do not depend on each other (the Q, K and V projections of an attention block) run each step of
// the path in ONE launch, blockIdx.y (blockIdx.x for the one-workgroup samplers) picking the layer.
// Every layer is computed by the code of the single-layer kernel, so its bits do not change.
#pragma once

#include "rowsum.hpp"
#include "sample_a_small.hpp"

namespace vcas {

constexpr int kMaxSiblings = 4;

// One layer of a grouped dgrad launch (layers of one shape that do not depend on each other):
// the pointer arguments of the bf16 dgrad kernel.
struct DgradProblem {
    const uint16_t *G, *W;
    const float *p;
    const int32_t *idxA, *cntA;
    uint16_t *dX;
    const uint16_t *J;   // null: no Jacobian
    InlineSampleA sa;    // sa.gsq null: SampleA has been decided, p / idxA / cntA hold its outcome
    float *sq_blocks;    // null, or the sums of squares of the written dX by blocks of 64 columns (layout: rows_from_blocks)
};
struct DgradGroup {
    DgradProblem prob[kMaxSiblings];
};

// SampleA of several layers in one launch: one workgroup each, the fields of InlineSampleA.
struct SampleAGroup {
    InlineSampleA prob[kMaxSiblings];
};

// One layer of a batched bf16 weight-gradient launch (host view): the arguments of
// vcas_sampled_wgrad, where its split-K partial tiles and its packed (gathered and pre-scaled)
// narrower operand go, and how many slices its contraction is cut into.
constexpr int kWgradBatch = 8;
struct WgradItem {
    vcas_shape shape;
    const void *G, *X;
    const float *row_scale;
    const int32_t *idxW, *cntW;
    float *dW, *partials;
    uint16_t *packed;
    int splits;
};

// One layer of a grouped SampleW launch: the pointer arguments of the one-workgroup sampler.
struct SampleWProblem {
    const float *gsq;
    float *xsq;
    const float *p;
    const uint8_t *maskA;
    const float *u;
    double budget;
    float *score, *q;
    uint8_t *maskW;
    float *scaleW;
    int32_t *idxW, *cntW;
};
struct SampleWGroup {
    SampleWProblem prob[kMaxSiblings];
};

// The same for the row-norm launch: matrix, where its row sums go, and (null: all) the samples
// whose rows are read at all.
struct RowNormGroup {
    const uint4 *A[kMaxSiblings];
    float *out[kMaxSiblings];
    const uint8_t *keep[kMaxSiblings];
};

// Row norms with their side jobs for up to kMaxSiblings matrices of one shape in one launch.
struct RowJobGroup {
    const uint4 *A[kMaxSiblings];
    const uint8_t *keep[kMaxSiblings];
    float *out[kMaxSiblings];
    UniformJob job[kMaxSiblings];
    ScoreJob sj[kMaxSiblings];
};

}  // namespace vcas
