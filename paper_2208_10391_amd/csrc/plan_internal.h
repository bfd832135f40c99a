// Internal layout of a plan: shared by the planner (host only) and the evaluator.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "launch_params.h"

namespace mom {

// kDiagonal is the property set {lowerTri, upperTri}: zeros off the diagonal, the diagonal stored.
enum : int { kGeneral = 0, kLower = 1, kUpper = 2, kIdentity = 3, kDiagonal = 4 };

// Where an operand of a binary product lives.
enum class Where : int { Factor = 0, Temp = 1, Out = 2 };

struct Operand {
    Where where;
    int index;     // original factor index, or temporary id
};

// One binary product C(m x n) = A(m x k) * B(k x n), in evaluation (post-) order.
struct ProductStep {
    Operand a, b, c;
    int64_t m, k, n;
    int pa, pb, pc;            // properties of A, B (as the product reads them) and of the result
    int ta, tb;                // the buffer of A / B holds its transpose (factors only)
    uint64_t mults;            // scalar multiplications with no structurally-zero operand
    int level;                 // 1 + the highest level among the products it consumes (factors: 0);
                               // products of one level are independent of each other
    size_t scratch_offset;     // split-K partial sums: bytes from the start of the scratch region
};

struct Temp {
    size_t offset;             // bytes from the start of the workspace, 256-byte aligned
    size_t bytes;              // rows * cols * 4 (dense storage; a triangular temporary is
                               // stored dense and only its triangle is ever written or read)
};

// One kernel launch of the evaluation, laid out at plan time: the evaluator copies `batch`
// (and `reduce`), fills in the pointers, row strides and alignment flags of its operands and
// launches.  A launch carries up to kMaxFused independent products of one level; when some of
// them are cut along k, one slice-sum launch follows.
struct PlannedLaunch {
    int kind;                        // kLaunchProduct, or kLaunchScale: one product with a diagonal
                                     // operand, run as an element-wise scaling pass (batch.prob[0]
                                     // carries its shapes and properties)
    int shape;                       // TileShape of the product kernel
    int variant;                     // which operands are stored transposed (ProductVariant)
    int step[kMaxFused];             // index into mom_plan::steps of batch.prob[i]
    int64_t row0[kMaxFused];         // batch.prob[i] is the sub-product of the result's rows from row0 on (see choose_tail)
    ProductBatch batch;              // geometry complete; A, B, C, ld*, *_vec patched per call
    ReduceBatch reduce;              // count == 0: no product of this launch is split
    int reduce_of[kMaxFused];        // reduce.prob[i] sums the slices of batch.prob[reduce_of[i]]
    unsigned reduce_grid_x;
};

// kLaunchPair: two products (X * Y) * Z with a narrow intermediate in one launch of the
// skinny-pair kernel; step[0] is X * Y (whose temporary is never written), step[1] the consumer.
enum : int { kLaunchProduct = 0, kLaunchScale = 1, kLaunchPair = 2 };

constexpr int kBatchedSlots = 8;     // surviving factors the batched kernels hold at once

}  // namespace mom

struct mom_plan {
    int32_t n = 0;
    std::vector<int64_t> dims;       // n + 1
    std::vector<int32_t> props;      // n: properties of the STORED matrices
    std::vector<int32_t> trans;      // n: factor t enters the chain as the transpose of its buffer
    std::vector<int32_t> chain_props;   // n: properties inside the chain (a transposed triangle mirrored)
    int32_t objective = 0;           // what the tree minimises (MOM_PLAN_MIN_MULTS / MOM_PLAN_MIN_TIME)
    std::vector<int32_t> survivors;  // original indices of the non-Identity factors
    std::vector<int32_t> splits;     // preorder, original indices, survivors-1 entries
    uint64_t cost = 0;               // scalar multiplications of the tree
    uint64_t time_ps = 0;            // modelled time of the tree (sum over its products)
    int64_t rows = 0, cols = 0;
    int32_t result_prop = 0;
    std::vector<mom::ProductStep> steps;      // post-order
    std::vector<int32_t> order;              // indices into steps, by level: the evaluation order
    std::vector<mom::Temp> temps;
    size_t temp_bytes = 0;           // bytes of workspace used by temporaries
    size_t scratch_offset = 0;       // split-K partial sums start here
    size_t scratch_bytes = 0;
    size_t workspace_bytes = 0;
    std::string text;
    std::vector<int32_t> absorbed_by;         // per step: the step whose launch also runs this one (a
                                              // narrow left operand computed on the fly), or -1
    std::vector<mom::PlannedLaunch> launches;   // the evaluation, launch by launch
    // batched evaluation: largest dimension and operand-stack depth of the post-order walk;
    // product s multiplies LDS slot a_slot[s] by slot b_slot[s] and leaves the result in a_slot[s]
    // (filled only when the plan has at most kBatchedSlots surviving factors)
    int64_t max_dim = 0;
    int32_t stack_depth = 0;
    int32_t a_slot[mom::kBatchedSlots] = {}, b_slot[mom::kBatchedSlots] = {};
};

// A sum of chain products (the paper's Equation holding variadic Add and Mul): one plan per
// addend, all of one shape.
struct mom_equation {
    std::vector<mom_plan *> chains;          // owned
    std::vector<int32_t> first_factor;       // position of chain c's first factor in the caller's arrays
    int64_t rows = 0, cols = 0;
    int32_t result_prop = 0;
    int32_t direct_chain = -1;               // addend with products whose result has the sum's own
                                             // structure: evaluated straight into the output
    uint64_t cost = 0, time_ps = 0;
    size_t chain_bytes = 0;                  // largest workspace of any addend
    size_t temp_offset = 0;                  // one rows x cols temporary behind it (0 bytes if unused)
    size_t workspace_bytes = 0;
    ~mom_equation()
    {
        for (mom_plan *p : chains) delete p;
    }
};
