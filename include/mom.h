/*
 * mom.h - C ABI of the MI355X (gfx950) evaluator for property-annotated matrix chains.
 *
 * The library evaluates the paper's variadic Mul (MOM: Matrix Operations in MLIR, Sec. 2,
 * "Operations"): a product A_0 * A_1 * ... * A_{n-1} of f32 matrices, each a Linnea Matrix
 * type with static dimensions and one property (Sec. 2, "Matrix Attribute", "Types").  As the
 * paper's transformations prescribe (Sec. 2, "Transformations"), Identity factors are
 * simplified away (A*I -> A, I*I = I), the properties of intermediate results are inferred,
 * and the chain is rewritten into binary products whose parenthesisation minimises the number
 * of scalar multiplications, counted with the structural zeros of the operands left out.
 * Each binary product then runs as one HIP kernel that skips the tiles a property makes zero;
 * this realises the non-rectangular iteration space that Sec. 5 leaves as future work.
 *
 * Conventions
 *   - All matrices are dense, row-major f32 (the paper's memref materialisation, Sec. 2).
 *     Factor t has dims[t] rows and dims[t+1] columns.
 *   - lowerTri: entries above the diagonal are zero; upperTri: entries below it are zero; the
 *     diagonal is stored data.  Only the triangle of a triangular factor defines the value: the
 *     other half of its (dense, fully allocated) buffer may be loaded but is masked before any
 *     arithmetic, so whatever it holds, NaN included, never reaches a result.  Identity factors
 *     have no buffer.
 *   - lowerTri, upperTri, diagonal and Identity factors must be square.
 *   - Plans live in host memory, belong to the library until mom_plan_destroy, are immutable
 *     and may be evaluated concurrently on different streams with different workspaces.
 *   - The library never allocates, frees or synchronises device memory.  Inputs, output and
 *     workspace are the caller's; inputs are read-only and must not overlap the output or the
 *     workspace.  Evaluation calls only enqueue kernels on the given stream and return.
 *   - Every call reports failure through mom_status_t and no C++ exception leaves the library.
 *     Every check of an evaluation call comes before its first launch, so nothing is enqueued
 *     on failure; the one exception is MOM_ERR_HIP (the runtime rejected a launch), after which
 *     earlier launches of the same call may already be on the stream.
 *   - "host" / "device" below say where a pointer must point.
 */
#ifndef MOM_H
#define MOM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Matrix properties (Sec. 2, "Matrix Attribute"; Identity is the paper's Identity type).
 * The paper's attribute is a SET of non-conflicting properties; the one set with two members
 * that this library knows is {lowerTri, upperTri} = MOM_DIAGONAL: zeros off the diagonal, the
 * diagonal stored in a dense square buffer of which nothing else is ever read.  A product with
 * a diagonal operand scales the rows (D*X) or columns (X*D) of the other operand, keeps that
 * operand's structure, costs one multiplication per structural entry of it, and runs as an
 * element-wise pass. */
typedef enum {
    MOM_GENERAL   = 0,
    MOM_LOWER_TRI = 1,
    MOM_UPPER_TRI = 2,
    MOM_IDENTITY  = 3,
    MOM_DIAGONAL  = 4
} mom_prop_t;

typedef enum {
    MOM_OK = 0,
    MOM_ERR_NULL,              /* a required pointer is NULL */
    MOM_ERR_BAD_N,             /* n <= 0 or above MOM_MAX_FACTORS, batch < 0 */
    MOM_ERR_BAD_DIM,           /* a dimension is <= 0 or above MOM_MAX_DIM */
    MOM_ERR_BAD_PROP,          /* a property is not one of mom_prop_t */
    MOM_ERR_NOT_SQUARE,        /* a lowerTri / upperTri / Identity factor is not square */
    MOM_ERR_OVERFLOW,          /* a multiplication count does not fit in 64 bits */
    MOM_ERR_BAD_SPLITS,        /* forced parenthesisation is not a tree over the chain */
    MOM_ERR_WORKSPACE,         /* workspace NULL or smaller than mom_plan_workspace_bytes */
    MOM_ERR_BUFFER_TOO_SMALL,  /* caller's host buffer cannot hold the answer */
    MOM_ERR_BAD_STRIDE,        /* a row or batch stride is smaller than the matrix needs */
    MOM_ERR_UNSUPPORTED,       /* the batched kernel does not cover this plan's shapes, or a product
                                  would need more workgroups than one launch can have */
    MOM_ERR_HIP,               /* the HIP runtime rejected a call */
    MOM_ERR_NOMEM,             /* host memory for a plan could not be allocated */
    MOM_ERR_BAD_FLAGS,         /* flag bits that this version does not define */
    MOM_ERR_NOT_READY,         /* first evaluation on this device was attempted while its stream
                                  is being captured: call mom_init (or evaluate once) before */
    MOM_ERR_BAD_TRANS          /* a transposition flag is neither 0 nor 1 */
} mom_status_t;

#define MOM_MAX_FACTORS 1024
#define MOM_MAX_DIM 2147483392          /* 2^31 - 256: tile arithmetic in the kernels stays in 32 bits */

/* mom_chain_eval flag: also write zeros into the other half of a triangular RESULT, which
 * restores the fully materialised buffer of the paper's bufferization (Sec. 2).  Without it
 * only the triangle of a triangular result is written and the rest of d_out is untouched. */
#define MOM_OUT_ZERO_FILL_TRIANGLE 1u

typedef struct mom_plan mom_plan_t;   /* opaque */

/*
 * Plan a chain (Sec. 2, "Transformations": identity simplification, property propagation,
 * matrix-chain reordering generalised to properties).
 *   dims  [host] n+1 dimensions, props [host] n values of mom_prop_t.
 *   *out receives a new plan (NULL on error); release it with mom_plan_destroy.
 * Cost of X(m x k)*Y(k x n) = number of scalar products with no structurally-zero operand:
 *   general*general m*k*n; tri*general n*m(m+1)/2; general*tri m*n(n+1)/2;
 *   L*L, U*U n(n+1)(n+2)/6 (result keeps the triangle); L*U, U*L n(n+1)(2n+1)/6 (general);
 *   with a diagonal operand: the structural entries of the other one.
 * Among equal-cost trees the one with the smallest root split wins, recursively.
 */
mom_status_t mom_chain_plan(const int64_t *dims, const int32_t *props, int32_t n, mom_plan_t **out);

/*
 * Plan with a forced parenthesisation, e.g. the left-to-right tree Sec. 4 starts from.
 *   preorder_splits [host]: one entry per binary product (survivors-1 entries; survivors =
 *   factors that are not Identity), in preorder: a node's split, then its left subtree's
 *   entries, then its right subtree's.  A split is the ORIGINAL index of the last factor of
 *   the node's left operand and must be a surviving factor inside the node's range.
 */
mom_status_t mom_plan_from_splits(const int64_t *dims, const int32_t *props, int32_t n,
                                  const int32_t *preorder_splits, mom_plan_t **out);

/* What the parenthesisation minimises. */
#define MOM_PLAN_MIN_MULTS 0            /* scalar multiplications (Sec. 2, "Transformations") */
#define MOM_PLAN_MIN_TIME  1            /* modelled run time on the GPU, see below */

/*
 * MOM_PLAN_MIN_TIME: the paper minimises the multiplication count, and its own experiment
 * (Sec. 4, "Results": 5.94 times fewer multiplications, 1.24 times the speed) shows that the
 * count is not the run time.  This opt-in objective minimises, by the same dynamic program, the
 * sum over the tree's products of an integer estimate in picoseconds of the tiled kernel's
 * time for X (m x k) * Y (k x n):
 *   T = 64 if m <= 64 or n <= 64 or ceil(m/128) * ceil(n/128) <= limit, else 128 (square output
 *   tiles), with limit = 192 when neither operand is triangular, 448 for one triangular operand,
 *   900 for lowerTri * upperTri and upperTri * lowerTri, 1400 for two equal triangles; k-chunks of 32;
 *   a tile (I, J) exists unless it lies wholly in the zero half of a triangular result;
 *   its k-range is [0, k) clipped by the operands' structures (X lowerTri: k < min((I+1)T, m);
 *   X upperTri: k >= I*T; Y lowerTri: k >= J*T; Y upperTri: k < min((J+1)T, n)), start rounded
 *   down to a chunk; a product with fewer than 256 tiles and at least 64
 *   chunks in the full k is cut into s = min(ceil(768/tiles), chunks/8) > 1 k-slices (every tile's
 *   chunks dealt out to s workgroups, ceil(tile's chunks / s) each), plus a summing launch;
 *   matrix = max(longest workgroup's chunks, ceil(all chunks / 256)) * (1706667 for T = 128,
 *   426667 for T = 64: one chunk of one tile at 256 FLOP per clock and 2.4 GHz);
 *   memory = 4 * (structural entries of X, Y and the result) / 8 (8 bytes per picosecond);
 *   time = 6000000 + max(matrix, memory)  [+ 6000000 + 4 * (s+1) * (structural entries of the
 *   result) / 8 when sliced];
 *   a product with a diagonal operand is an element-wise pass: time = 6000000 + memory.
 * Ties go to the smallest root split, recursively, as for the multiplication count.
 */

/*
 * The general planning call: mom_chain_plan / mom_plan_from_splits plus transposed factors
 * (Table 1, "Transpose").
 *   trans [host] n flags or NULL (= none).  trans[t] = 1: factor t of the chain is the
 *         TRANSPOSE of the matrix in its buffer.  dims still describe the chain (factor t is
 *         dims[t] x dims[t+1]), so the buffer holds a dims[t+1] x dims[t] matrix, row-major;
 *         props[t] is the property of that STORED matrix, and inside the chain the factor
 *         carries the mirrored one: lowerTri(A) -> upperTri(A^T) (Sec. 2, "Transformations",
 *         the inference rule printed there); general and Identity are their own mirror image.
 *         Nothing is transposed in memory: the product kernels read the buffer as it is.
 *   objective        MOM_PLAN_MIN_MULTS or MOM_PLAN_MIN_TIME (anything else: MOM_ERR_BAD_FLAGS).
 *   preorder_splits  [host] NULL: the optimal tree; else a forced tree as in mom_plan_from_splits.
 * Costs, the tree and the result's property follow from the properties inside the chain.
 */
mom_status_t mom_chain_plan_ex(const int64_t *dims, const int32_t *props, const int32_t *trans, int32_t n,
                               int32_t objective, const int32_t *preorder_splits, mom_plan_t **out);

void mom_plan_destroy(mom_plan_t *plan);                       /* NULL is allowed */

/* The accessors below read what the transformations of Sec. 2 produced for the chain: the
 * multiplication count that the chain reordering minimised, the binary products the variadic
 * Mul was rewritten into, and the inferred type of the result. */

/* Scalar multiplications of the plan's tree (0 for a NULL plan). */
uint64_t mom_plan_cost_mults(const mom_plan_t *plan);

/* Modelled time of the plan's tree in picoseconds (the MOM_PLAN_MIN_TIME objective, whatever
 * objective the plan was made with; 0 for a NULL plan). */
uint64_t mom_plan_cost_time_ps(const mom_plan_t *plan);

/* Number of binary products the evaluation launches: survivors-1, or 0. */
int32_t mom_plan_num_products(const mom_plan_t *plan);

/* Shape and inferred property of the result (the concrete type that replaces the paper's
 * Term type).  All-Identity chains report MOM_IDENTITY.  Any out pointer may be NULL. */
mom_status_t mom_plan_result(const mom_plan_t *plan, int64_t *rows, int64_t *cols, int32_t *prop);

/* Parenthesised form with original factor indices, e.g. "(0 (2 (3 4)))"; a single survivor
 * prints as its index, an all-Identity chain as "I".  buf [host], cap bytes incl. the NUL. */
mom_status_t mom_plan_string(const mom_plan_t *plan, char *buf, size_t cap);

/* Preorder splits (original indices) of the plan; cap entries available in out [host]. */
mom_status_t mom_plan_splits(const mom_plan_t *plan, int32_t *out, int32_t cap);

/* The i-th binary product (0 <= i < mom_plan_num_products) in evaluation order, i.e. level by
 * level of the tree: shape[3] = rows, inner dimension, columns; props[3] = properties of the
 * left operand, the right operand and the result; *mults = its scalar multiplications;
 * *level = its height in the tree (products of one level are independent).  Any out pointer
 * may be NULL.  MOM_ERR_BAD_N for an index out of range. */
mom_status_t mom_plan_product(const mom_plan_t *plan, int32_t i, int64_t *shape, int32_t *props,
                              uint64_t *mults, int32_t *level);

/* Kernel launches one mom_chain_eval of this plan enqueues (products that share a launch count
 * once, slice sums count, the optional zero-fill pass does not). */
int32_t mom_plan_num_launches(const mom_plan_t *plan);

/* Bytes of device workspace mom_chain_eval needs for temporaries and k-slices (may be 0). */
size_t mom_plan_workspace_bytes(const mom_plan_t *plan);

/*
 * One-time set-up of the CURRENT device (kernel attributes), for callers that record
 * evaluations into a HIP graph: the set-up is not allowed while a stream is being captured.
 * Without this call the first evaluation on a device does the same, unless its stream is being
 * captured, in which case it returns MOM_ERR_NOT_READY and enqueues nothing.  Idempotent and
 * cheap after the first time; allocates no device memory.
 */
mom_status_t mom_init(void);

/*
 * Enqueue the evaluation of the plan on `stream` (a hipStream_t passed as void*; NULL = the
 * default stream).  Asynchronous.  The products run level by level of the tree; small
 * independent products of one level share a kernel launch, a product cut along k is followed
 * by a launch that adds its slices, and a zero-fill pass runs last when asked for.  The
 * library allocates nothing and never synchronises; calls on one stream run in order, calls
 * that share a workspace or an output on different streams race.
 *   d_factors [host] array of n DEVICE pointers, entry t -> dims[t] x dims[t+1] f32 (for a
 *             factor planned as transposed: the dims[t+1] x dims[t] matrix whose transpose it
 *             is); entries of Identity factors are ignored and may be NULL.
 *   lds       [host] n row strides in elements (>= the columns of the stored matrix), or NULL
 *             for packed rows.
 *   d_out     [device] rows x cols result, row stride ld_out elements (0 = packed).
 *   d_workspace [device] at least mom_plan_workspace_bytes bytes, 256-byte aligned; may be
 *             NULL when that is 0.  Contents are scratch.
 *   flags     0 or MOM_OUT_ZERO_FILL_TRIANGLE; any other bit is MOM_ERR_BAD_FLAGS.
 * A chain whose factors are all Identity writes the identity matrix; a chain with a single
 * surviving factor copies it (its triangle only, for a triangular factor).
 */
mom_status_t mom_chain_eval(const mom_plan_t *plan, const float *const *d_factors, const int64_t *lds,
                            float *d_out, int64_t ld_out, void *d_workspace, size_t workspace_bytes,
                            uint32_t flags, void *stream);

/*
 * mom_chain_eval for callers that cannot hand over (or allocate) a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments and
 * behaviour as mom_chain_eval, except that temporaries and k-slices live in an array that is
 * part of the library's device code: MOM_STATIC_WORKSPACE_BYTES per GPU, held from the moment
 * the library is loaded on a GPU until the process ends.  The call allocates and frees nothing.
 *   - A plan with mom_plan_workspace_bytes above MOM_STATIC_WORKSPACE_BYTES is refused with
 *     MOM_ERR_WORKSPACE and nothing is enqueued.
 *   - Every call on a GPU shares that GPU's array: calls on ONE stream run in order and are
 *     safe; calls that may overlap on one GPU (different streams, different threads) race.
 *   - The array keeps the last call's contents; nothing in it needs to start at zero.
 *   - The array's address is looked up at the device's one-time set-up (mom_init or the first
 *     evaluation outside capture), so the capture rule of mom_init applies here as well.
 */
#define MOM_STATIC_WORKSPACE_BYTES (64u << 20)
mom_status_t mom_chain_eval_static(const mom_plan_t *plan, const float *const *d_factors, const int64_t *lds,
                                   float *d_out, int64_t ld_out, uint32_t flags, void *stream);

/*
 * The same variadic Mul (Sec. 2, "Operations") for many small chains at once: evaluate
 * `batch` independent chains that share one plan (one shape, one property list, hence one
 * parenthesisation by Sec. 2, "Transformations") in ONE kernel launch; each chain is
 * handled by one 64-lane wavefront and intermediates never leave the compute unit.
 *   d_factor_bases [host] n DEVICE pointers; chain b's factor t starts at
 *             d_factor_bases[t] + b * batch_strides[t] and is packed row-major (the stored
 *             matrix, for a factor planned as transposed).
 *   batch_strides [host] n strides in elements, or NULL for dims[t]*dims[t+1].
 *   d_out [device], chain b's result at d_out + b * out_batch_stride (0 = rows*cols), packed.
 * Covers plans whose dimensions are all <= 32 and that have at most 8 surviving factors
 * (MOM_ERR_UNSUPPORTED otherwise).  Triangular results are written in full (zeros included).
 */
mom_status_t mom_chain_eval_batched(const mom_plan_t *plan, const float *const *d_factor_bases,
                                    const int64_t *batch_strides, float *d_out,
                                    int64_t out_batch_stride, int32_t batch, void *stream);

/*
 * Sums of chain products: the paper's Equation with its variadic Add and Mul (Table 1, "Add",
 * "Mul", "Equation"; Sec. 2, "Operations").  out = C_0 + C_1 + ... where every addend C_c is a
 * chain of chain_len[c] factors (a chain of one factor is a plain matrix term, so a pure
 * variadic Add is an equation whose chains all have length 1; an all-Identity chain adds I).
 *   chain_len [host] n_chains lengths, each 1..MOM_MAX_FACTORS.
 *   dims      [host] the chains' dimension lists one after the other (chain_len[c] + 1 each);
 *   props, trans (may be NULL) [host] one entry per factor, chain after chain, with the
 *             meaning they have in mom_chain_plan_ex; every chain must have the same rows x cols
 *             (MOM_ERR_BAD_DIM otherwise).
 *   objective as in mom_chain_plan_ex; every addend gets its own optimal tree.
 * The sum's property is the smallest structure that holds every addend's: one addend keeps its
 * property; Identity / diagonal addends give MOM_DIAGONAL (I + I is not an Identity); adding
 * lowerTri addends gives lowerTri, upperTri likewise; anything else is general.
 * No algebraic rewriting across addends (common factors are not pulled out).
 */
typedef struct mom_equation mom_equation_t;   /* opaque, host memory, immutable */
mom_status_t mom_equation_plan(const int64_t *dims, const int32_t *props, const int32_t *trans,
                               const int32_t *chain_len, int32_t n_chains, int32_t objective, mom_equation_t **out);
void mom_equation_destroy(mom_equation_t *eq);                 /* NULL is allowed */
mom_status_t mom_equation_result(const mom_equation_t *eq, int64_t *rows, int64_t *cols, int32_t *prop);
uint64_t mom_equation_cost_mults(const mom_equation_t *eq);    /* multiplications of all addends */
size_t mom_equation_workspace_bytes(const mom_equation_t *eq);
int32_t mom_equation_num_chains(const mom_equation_t *eq);
/* The plan of addend c (borrowed: it lives as long as the equation), NULL when out of range. */
const mom_plan_t *mom_equation_chain(const mom_equation_t *eq, int32_t c);

/*
 * Enqueue the evaluation of the equation on `stream`; same rules as mom_chain_eval (caller's
 * memory, no allocation, no synchronisation, only the sum's structure is written unless
 * MOM_OUT_ZERO_FILL_TRIANGLE is set).  d_factors / lds [host]: one entry per factor, chain
 * after chain.  Addends that are plain matrices are summed by one element-wise launch per eight
 * of them; an addend with products is evaluated by the chain evaluator, straight into d_out
 * when its result has the sum's structure, otherwise (and for every further one) into a
 * temporary in the workspace that an element-wise launch then adds to d_out.
 */
mom_status_t mom_equation_eval(const mom_equation_t *eq, const float *const *d_factors, const int64_t *lds,
                               float *d_out, int64_t ld_out, void *d_workspace, size_t workspace_bytes,
                               uint32_t flags, void *stream);

/*
 * Calibration aid for measurements (not a step of the method): enqueue one launch of a
 * register-only v_mfma_f32_32x32x2_f32 loop, the rate the matrix pipes of this GPU sustain
 * with no memory traffic at all, which is what the product kernels' f32 throughput (the f32
 * operands of Sec. 4) is to be read against.  The caller times the launch with events.
 *   iters   loop trips per wavefront (32 MFMAs each), > 0.
 *   d_sink  [device] at least 1024 bytes; kept only so that the loop has a visible result, it
 *           is written if the accumulators reach a value they cannot reach.
 *   flop    [host] receives the floating-point operations of one launch.
 */
mom_status_t mom_probe_mfma_peak(int32_t iters, float *d_sink, double *flop, void *stream);

/* Static, NUL-terminated description of a status code. */
const char *mom_status_string(mom_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* MOM_H */
