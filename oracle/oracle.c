/*
 * CPU oracle for property-annotated matrix-chain products (MOM / Linnea dialect).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain statement of what the
 * chain evaluator must compute, used only by the test-suite, the smoke check and
 * the CPU-baseline leg of the benchmark.  It shares no code, header, table or
 * helper with the GPU library and nothing in the product path may call it.
 *
 * What it states (paper sections in brackets):
 *   - a chain  A_0 * A_1 * ... * A_{n-1}  of f32 matrices, each carrying one
 *     property: general, lowerTri, upperTri or Identity, or the set
 *     {lowerTri, upperTri} = diagonal                          [Sec. 2, "Matrix
 *     Attribute" and "Types: Matrix, Term and Identity"]
 *   - memory of a triangular matrix is a plain dense row-major buffer whose
 *     other half holds zeros; the diagonal is stored             [Sec. 2, bufferization]
 *   - Identity is square with ones on the diagonal, A*I = A, I*I = I  [Sec. 2, Types]
 *   - a factor may enter the chain transposed; the transpose of a lowerTri
 *     matrix is upperTri and vice versa     [Table 1 "Transpose"; Sec. 2,
 *     "Transformations", the inference rule printed there]
 *   - the variadic product is rewritten into binary products whose
 *     parenthesisation minimises the number of scalar multiplications, taking
 *     the properties of operands and intermediates into account
 *                                      [Sec. 2, "Operations" and "Transformations"]
 *
 *   - Add is variadic as well: the sum of any number of equally shaped terms,
 *     whose structure is the union of the terms' structures
 *                                      [Table 1 "Add"; Sec. 2, "Operations"]
 *   - an opt-in second objective: a stated integer time model of one tiled
 *     product on the GPU, summed over the tree  [motivated by Sec. 4, Results]
 *
 * All floating point work is done in double precision.
 *
 * Pins (tests/test_oracle_*.py): the paper's 5x5 lowerTri*lowerTri example with
 * fill value 1 (closed form i-j+1), the Sec. 4 chain 800x1100x900x1200x100 and its
 * two parenthesisations, numpy.matmul in f64 on general chains, counted
 * multiplications against the closed-form costs, identity rules bit-exactly,
 * structure invariants, agreement of every parenthesisation on tiny inputs;
 * transposed factors: (A*B)^T = B^T * A^T and explicit .T chains against numpy,
 * lowerTri^T is upperTri, costs and plans equal those of the mirrored chain.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* P_DIAGONAL is the property SET {lowerTri, upperTri}: a matrix that is both
 * has zeros above and below the diagonal and an arbitrary stored diagonal
 * [Sec. 2, Matrix Attribute: a set of non-conflicting properties].          */
enum { P_GENERAL = 0, P_LOWER = 1, P_UPPER = 2, P_IDENTITY = 3, P_DIAGONAL = 4 };

/* ------------------------------------------------------------------------ */
/* Structure of a property: is position (i,j) allowed to be non-zero?       */
/* lowerTri: zeros above the diagonal; upperTri: zeros below it; the        */
/* diagonal itself is stored data.  [Sec. 2, bufferization remark]          */
static int structurally_nonzero(int prop, int64_t i, int64_t j)
{
    switch (prop) {
    case P_LOWER:    return j <= i;
    case P_UPPER:    return j >= i;
    case P_IDENTITY: return j == i;
    case P_DIAGONAL: return j == i;
    default:         return 1;
    }
}

/* Number of scalar products X[i][t]*Y[t][j] in which neither operand is a
 * structural zero, counted one by one.  This is the planner's cost unit
 * (the multiplication count of Sec. 2, Transformations) written as
 * its definition; the closed forms below are checked against it.           */
uint64_t oracle_count_mults(int64_t m, int64_t k, int64_t n, int32_t pX, int32_t pY)
{
    uint64_t c = 0;
    for (int64_t i = 0; i < m; ++i)
        for (int64_t t = 0; t < k; ++t)
            for (int64_t j = 0; j < n; ++j)
                if (structurally_nonzero(pX, i, t) && structurally_nonzero(pY, t, j))
                    ++c;
    return c;
}

/* ------------------------------------------------------------------------ */
/* Property of a product of two operands.  Identity is neutral; a diagonal   */
/* operand only scales rows or columns, so the other operand's structure    */
/* stays; equal triangles keep their triangle; everything else is general.  */
static int product_property(int pX, int pY)
{
    if (pX == P_IDENTITY) return pY;
    if (pY == P_IDENTITY) return pX;
    if (pX == P_DIAGONAL) return pY;          /* scaling rows keeps the structure of Y */
    if (pY == P_DIAGONAL) return pX;          /* scaling columns keeps that of X       */
    if (pX == pY && (pX == P_LOWER || pX == P_UPPER)) return pX;
    return P_GENERAL;
}

/* Property of the transpose of a matrix with property p: the mirror image of
 * its structure, lowerTri(A) -> upperTri(A^T) and back; general, Identity
 * stay what they are.  [Sec. 2, Transformations: the inference rule printed
 * there; Table 1, Transpose]                                               */
int32_t oracle_transposed_property(int32_t p)
{
    if (p == P_LOWER) return P_UPPER;
    if (p == P_UPPER) return P_LOWER;
    return p;
}

typedef unsigned __int128 u128;

/* Closed-form count of the non-structurally-zero scalar products of
 * X (m x k, pX) times Y (k x n, pY).  A product with an Identity operand is
 * no computation at all (A*I -> A).                                        */
static u128 product_cost(int64_t m, int64_t k, int64_t n, int pX, int pY)
{
    u128 M = (u128)m, K = (u128)k, N = (u128)n;
    int triX = (pX == P_LOWER || pX == P_UPPER);
    int triY = (pY == P_LOWER || pY == P_UPPER);
    if (pX == P_IDENTITY || pY == P_IDENTITY) return 0;
    /* a diagonal operand meets every structural entry of the other exactly once */
    if (pX == P_DIAGONAL) return pY == P_DIAGONAL ? N : (triY ? N * (N + 1) / 2 : K * N);
    if (pY == P_DIAGONAL) return triX ? M * (M + 1) / 2 : M * K;
    if (!triX && !triY) return M * K * N;
    if (triX && !triY)  return N * (M * (M + 1) / 2);          /* m == k */
    if (!triX && triY)  return M * (N * (N + 1) / 2);          /* k == n */
    if (pX == pY)       return N * (N + 1) * (N + 2) / 6;      /* tri*tri, same side */
    return N * (N + 1) * (2 * N + 1) / 6;                      /* L*U or U*L */
}

/* ------------------------------------------------------------------------ */
/* Brute-force search over every parenthesisation.                          */
/*                                                                          */
/* A binary tree over factors lo..hi is written as its preorder list of     */
/* splits: the root's split s (left = lo..s, right = s+1..hi), then the     */
/* left subtree's list, then the right subtree's.  Positions index the      */
/* chain handed to the enumerator.                                          */

typedef struct { int64_t rows, cols; int prop; u128 cost; } subresult_t;

/* Cost a complete tree bottom-up; *pos walks the preorder split list. */
static subresult_t cost_tree(const int64_t *dims, const int32_t *props,
                             int lo, int hi, const int32_t *splits, int *pos)
{
    subresult_t r;
    if (lo == hi) {
        r.rows = dims[lo]; r.cols = dims[lo + 1]; r.prop = props[lo]; r.cost = 0;
        return r;
    }
    int s = splits[(*pos)++];
    subresult_t a = cost_tree(dims, props, lo, s, splits, pos);
    subresult_t b = cost_tree(dims, props, s + 1, hi, splits, pos);
    r.rows = a.rows; r.cols = b.cols;
    r.prop = product_property(a.prop, b.prop);
    r.cost = a.cost + b.cost + product_cost(a.rows, a.cols, b.cols, a.prop, b.prop);
    return r;
}

/* All trees over lo..hi, each as (hi-lo) ints, concatenated; returns count. */
static int64_t all_trees(int lo, int hi, int32_t **out)
{
    int len = hi - lo;                       /* number of splits in one tree */
    if (len == 0) { *out = NULL; return 1; } /* one (empty) tree */
    int64_t cap = 16, cnt = 0;
    int32_t *buf = (int32_t *)malloc(sizeof(int32_t) * cap * len);
    for (int s = lo; s < hi; ++s) {
        int32_t *L, *R;
        int64_t nl = all_trees(lo, s, &L), nr = all_trees(s + 1, hi, &R);
        int ll = s - lo, rl = hi - s - 1;
        for (int64_t a = 0; a < nl; ++a)
            for (int64_t b = 0; b < nr; ++b) {
                if (cnt == cap) { cap *= 2; buf = (int32_t *)realloc(buf, sizeof(int32_t) * cap * len); }
                int32_t *t = buf + cnt * len;
                t[0] = s;
                if (ll) memcpy(t + 1, L + a * ll, sizeof(int32_t) * ll);
                if (rl) memcpy(t + 1 + ll, R + b * rl, sizeof(int32_t) * rl);
                ++cnt;
            }
        free(L); free(R);
    }
    *out = buf;
    return cnt;
}

static int lex_less(const int32_t *a, const int32_t *b, int len)
{
    for (int i = 0; i < len; ++i) { if (a[i] != b[i]) return a[i] < b[i]; }
    return 0;
}

/*
 * Minimum-multiplication parenthesisation by exhaustive enumeration.
 *
 * elide != 0: Identity factors are dropped first (A*I -> A, I*I = I) and the
 *             trees range over the survivors.
 * elide == 0: every factor stays in the chain and a product with an Identity
 *             operand costs nothing (used to cross-check the elision rule).
 *
 * Outputs: *cost (minimum), *n_eff (factors the trees range over),
 * out_splits[n_eff-1] = preorder splits of the minimiser, expressed as ORIGINAL
 * factor indices (the index of the last factor of each left subtree); among
 * equal-cost trees the lexicographically smallest preorder list wins.
 * *result_prop = property of the whole product, *num_trees = trees enumerated.
 * Returns 0, or 1 when a cost does not fit in 64 bits.
 */
int oracle_plan_bruteforce(int32_t n, const int64_t *dims, const int32_t *props, int32_t elide,
                           uint64_t *cost, int32_t *n_eff, int32_t *out_splits,
                           int32_t *result_prop, int64_t *num_trees)
{
    int64_t *d = (int64_t *)malloc(sizeof(int64_t) * (n + 1));
    int32_t *p = (int32_t *)malloc(sizeof(int32_t) * n);
    int32_t *orig = (int32_t *)malloc(sizeof(int32_t) * n);
    int m = 0;
    for (int i = 0; i < n; ++i) {
        if (elide && props[i] == P_IDENTITY) continue;
        d[m] = dims[i]; p[m] = props[i]; orig[m] = i; ++m;
    }
    d[m] = dims[n];
    *n_eff = m;
    *num_trees = 0;
    if (m == 0) {                     /* every factor was an Identity: I*I = I */
        *cost = 0; *result_prop = P_IDENTITY;
        free(d); free(p); free(orig); return 0;
    }
    int len = m - 1;
    int32_t *trees;
    int64_t cnt = all_trees(0, m - 1, &trees);
    u128 best = 0; int64_t best_idx = -1; int prop = p[0];
    for (int64_t t = 0; t < cnt; ++t) {
        int pos = 0;
        subresult_t r = cost_tree(d, p, 0, m - 1, trees ? trees + t * len : NULL, &pos);
        prop = r.prop;
        if (best_idx < 0 || r.cost < best ||
            (r.cost == best && lex_less(trees + t * len, trees + best_idx * len, len))) {
            best = r.cost; best_idx = t;
        }
    }
    for (int i = 0; i < len; ++i) out_splits[i] = orig[trees[best_idx * len + i]];
    *result_prop = prop;
    *num_trees = cnt;
    int overflow = (best >> 64) != 0;
    *cost = (uint64_t)best;
    free(trees); free(d); free(p); free(orig);
    return overflow;
}

/*
 * Cost of one given tree.  `splits` is a preorder list over the chain with
 * Identity factors removed, in ORIGINAL factor indices.  Returns 0, 1 on
 * 64-bit overflow, 2 when a split is not a surviving factor inside its range.
 */
int oracle_tree_cost(int32_t n, const int64_t *dims, const int32_t *props,
                     const int32_t *splits, uint64_t *cost, int32_t *result_prop)
{
    int64_t *d = (int64_t *)malloc(sizeof(int64_t) * (n + 1));
    int32_t *p = (int32_t *)malloc(sizeof(int32_t) * n);
    int32_t *where = (int32_t *)malloc(sizeof(int32_t) * n);   /* original -> elided position */
    int m = 0, rc = 0;
    for (int i = 0; i < n; ++i) {
        where[i] = -1;
        if (props[i] == P_IDENTITY) continue;
        d[m] = dims[i]; p[m] = props[i]; where[i] = m; ++m;
    }
    d[m] = dims[n];
    if (m == 0) { *cost = 0; *result_prop = P_IDENTITY; goto done; }
    {
        int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (m > 1 ? m - 1 : 1));
        for (int i = 0; i + 1 < m; ++i) {
            if (splits[i] < 0 || splits[i] >= n || where[splits[i]] < 0) { rc = 2; }
            else s[i] = where[splits[i]];
        }
        if (rc == 0) {
            /* validate ranges while walking */
            int stack_lo[64], stack_hi[64], sp = 0, pos = 0;
            stack_lo[0] = 0; stack_hi[0] = m - 1; sp = 1;
            while (sp > 0 && rc == 0) {
                int lo = stack_lo[sp - 1], hi = stack_hi[sp - 1]; --sp;
                if (lo == hi) continue;
                int k = s[pos++];
                if (k < lo || k >= hi) { rc = 2; break; }
                /* preorder: left first, so push right then left */
                stack_lo[sp] = k + 1; stack_hi[sp] = hi; ++sp;
                stack_lo[sp] = lo;    stack_hi[sp] = k;  ++sp;
            }
        }
        if (rc == 0) {
            int pos = 0;
            subresult_t r = cost_tree(d, p, 0, m - 1, s, &pos);
            *result_prop = r.prop;
            if (r.cost >> 64) rc = 1;
            *cost = (uint64_t)r.cost;
        }
        free(s);
    }
done:
    free(d); free(p); free(where);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Time model of one binary product on the GPU, and the tree that minimises  */
/* its sum.  The paper's objective is the multiplication count [Sec. 2,      */
/* Transformations]; its own experiment shows that count and run time are    */
/* different things (5.94 times fewer multiplications bought 1.24 times the  */
/* speed) [Sec. 4, Results].  This is the opt-in alternative objective: an    */
/* estimate, in integer picoseconds, of what the tiled product kernel        */
/* spends on X (m x k, pX) * Y (k x n, pY).  Stated so that both sides can   */
/* compute it exactly:                                                       */
/*   T  = 64 if m <= 64 or n <= 64 or ceil(m/128) * ceil(n/128) <= limit,    */
/*        else 128 (square output tiles); limit = 192 when neither operand   */
/*        is triangular, 448 for one triangular operand, 900 for lowerTri *  */
/*        upperTri and upperTri * lowerTri, 1400 for two equal triangles     */
/*   a tile (I, J) of the result exists unless the result is triangular and  */
/*   the tile lies wholly in its zero half                                   */
/*   k-range of a tile: [0, k) clipped by the operands' structures           */
/*     X lowerTri: k < min((I+1)T, m)      X upperTri: k >= I*T              */
/*     Y lowerTri: k >= J*T                Y upperTri: k < min((J+1)T, n)    */
/*   start rounded down to a multiple of 32; chunks = ceil(length / 32)      */
/*   a product with fewer than 256 tiles and at least 64                     */
/*   chunks in the full k is cut into s = min(ceil(768 / tiles), chunks / 8) */
/*   slices (s > 1): every tile's own chunks are dealt out to s workgroups,  */
/*   ceil(chunks of the tile / s) each, followed by a launch that adds the   */
/*   slices                                                                  */
/*   matrix time = max(longest workgroup, ceil(all chunks / 256)) * chunk_ps */
/*     (256 compute units; chunk_ps = one T x T x 32 chunk at 256 FLOP per   */
/*     clock and 2.4 GHz: 1706667 ps for T = 128, 426667 ps for T = 64)      */
/*   memory time = 4 bytes * (structural entries of X, Y and the result) at  */
/*     8 bytes per picosecond                                                */
/*   time = 6000000 (launch) + max(matrix, memory)                           */
/*          + [split] 6000000 + 4 * (s + 1) * (entries of the result) / 8    */
/*   a product with a diagonal operand is an element-wise scaling pass:      */
/*   time = 6000000 + memory                                                 */

enum { TIME_LAUNCH_PS = 6000000, TIME_CHUNK128_PS = 1706667, TIME_CHUNK64_PS = 426667 };

static u128 structural_entries(int64_t rows, int64_t cols, int prop)
{
    if (prop == P_LOWER || prop == P_UPPER) return (u128)rows * (u128)(rows + 1) / 2;
    if (prop == P_DIAGONAL) return (u128)rows;
    return (u128)rows * (u128)cols;
}

static u128 product_time(int64_t m, int64_t k, int64_t n, int pX, int pY)
{
    if (pX == P_IDENTITY || pY == P_IDENTITY) return 0;           /* no computation at all */
    if (pX == P_DIAGONAL || pY == P_DIAGONAL) {
        /* rows or columns of the other operand scaled: an element-wise pass, memory only */
        int pD = product_property(pX, pY);
        return TIME_LAUNCH_PS + 4 * (structural_entries(m, k, pX) + structural_entries(k, n, pY) +
                                     structural_entries(m, n, pD)) / 8;
    }
    int triX = pX == P_LOWER || pX == P_UPPER, triY = pY == P_LOWER || pY == P_UPPER;
    int64_t limit = (triX && triY) ? (pX == pY ? 1400 : 900) : ((triX || triY) ? 448 : 192);
    int64_t T = (m <= 64 || n <= 64 || ((m + 127) / 128) * ((n + 127) / 128) <= limit) ? 64 : 128;
    u128 chunk_ps = T == 128 ? TIME_CHUNK128_PS : TIME_CHUNK64_PS;
    int pR = product_property(pX, pY);
    int64_t tm = (m + T - 1) / T, tn = (n + T - 1) / T;
    u128 tiles = 0, all_chunks = 0, longest = 0;
    for (int64_t I = 0; I < tm; ++I)
        for (int64_t J = 0; J < tn; ++J) {
            if (pR == P_LOWER && J > I) continue;
            if (pR == P_UPPER && J < I) continue;
            int64_t r0 = I * T, r1 = r0 + T < m ? r0 + T : m;
            int64_t c0 = J * T, c1 = c0 + T < n ? c0 + T : n;
            int64_t lo = 0, hi = k;
            if (pX == P_LOWER && r1 < hi) hi = r1;
            if (pX == P_UPPER && r0 > lo) lo = r0;
            if (pY == P_LOWER && c0 > lo) lo = c0;
            if (pY == P_UPPER && c1 < hi) hi = c1;
            lo = (lo / 32) * 32;
            u128 chunks = hi > lo ? (u128)((hi - lo + 31) / 32) : 0;
            ++tiles;
            all_chunks += chunks;
            if (chunks > longest) longest = chunks;
        }
    u128 extra = 0;
    int64_t chunks_full = (k + 31) / 32;
    if (tiles < 256 && chunks_full >= 64) {
        u128 want = (768 + tiles - 1) / tiles, most = (u128)(chunks_full / 8);
        u128 s = want < most ? want : most;
        if (s > 1) {
            longest = (longest + s - 1) / s;                     /* the longest tile's slice */
            extra = TIME_LAUNCH_PS + 4 * (s + 1) * structural_entries(m, n, pR) / 8;
        }
    }
    u128 spread = (all_chunks + 255) / 256;
    u128 matrix = (longest > spread ? longest : spread) * chunk_ps;
    u128 memory = 4 * (structural_entries(m, k, pX) + structural_entries(k, n, pY) +
                       structural_entries(m, n, pR)) / 8;
    return TIME_LAUNCH_PS + (matrix > memory ? matrix : memory) + extra;
}

uint64_t oracle_product_time_ps(int64_t m, int64_t k, int64_t n, int32_t pX, int32_t pY)
{
    u128 t = product_time(m, k, n, pX, pY);
    return (t >> 64) ? UINT64_MAX : (uint64_t)t;
}

/* Modelled time of a complete tree: the sum over its products. */
static subresult_t time_tree(const int64_t *dims, const int32_t *props,
                             int lo, int hi, const int32_t *splits, int *pos)
{
    subresult_t r;
    if (lo == hi) {
        r.rows = dims[lo]; r.cols = dims[lo + 1]; r.prop = props[lo]; r.cost = 0;
        return r;
    }
    int s = splits[(*pos)++];
    subresult_t a = time_tree(dims, props, lo, s, splits, pos);
    subresult_t b = time_tree(dims, props, s + 1, hi, splits, pos);
    r.rows = a.rows; r.cols = b.cols;
    r.prop = product_property(a.prop, b.prop);
    r.cost = a.cost + b.cost + product_time(a.rows, a.cols, b.cols, a.prop, b.prop);
    return r;
}

/*
 * The tree with the smallest modelled time, by exhaustive enumeration, ties to
 * the lexicographically smallest preorder split list.  Identity factors are
 * dropped first.  Outputs as oracle_plan_bruteforce, with *time_ps the
 * minimum and *mults the multiplication count of that same tree.
 * Returns 0, or 1 when a sum does not fit in 64 bits.
 */
int oracle_plan_bruteforce_time(int32_t n, const int64_t *dims, const int32_t *props,
                                uint64_t *time_ps, uint64_t *mults, int32_t *n_eff, int32_t *out_splits)
{
    int64_t *d = (int64_t *)malloc(sizeof(int64_t) * (n + 1));
    int32_t *p = (int32_t *)malloc(sizeof(int32_t) * (n > 0 ? n : 1));
    int32_t *orig = (int32_t *)malloc(sizeof(int32_t) * (n > 0 ? n : 1));
    int m = 0;
    for (int i = 0; i < n; ++i) {
        if (props[i] == P_IDENTITY) continue;
        d[m] = dims[i]; p[m] = props[i]; orig[m] = i; ++m;
    }
    d[m] = dims[n];
    *n_eff = m; *time_ps = 0; *mults = 0;
    if (m == 0) { free(d); free(p); free(orig); return 0; }
    int len = m - 1;
    int32_t *trees;
    int64_t cnt = all_trees(0, m - 1, &trees);
    u128 best = 0; int64_t best_idx = -1;
    for (int64_t t = 0; t < cnt; ++t) {
        int pos = 0;
        subresult_t r = time_tree(d, p, 0, m - 1, trees ? trees + t * len : NULL, &pos);
        if (best_idx < 0 || r.cost < best ||
            (r.cost == best && lex_less(trees + t * len, trees + best_idx * len, len))) {
            best = r.cost; best_idx = t;
        }
    }
    int pos = 0;
    subresult_t c = cost_tree(d, p, 0, m - 1, trees ? trees + best_idx * len : NULL, &pos);
    for (int i = 0; i < len; ++i) out_splits[i] = orig[trees[best_idx * len + i]];
    int overflow = (best >> 64) != 0 || (c.cost >> 64) != 0;
    *time_ps = (uint64_t)best; *mults = (uint64_t)c.cost;
    free(trees); free(d); free(p); free(orig);
    return overflow;
}

/* Modelled time of one given tree (splits as in oracle_tree_cost). */
int oracle_tree_time(int32_t n, const int64_t *dims, const int32_t *props,
                     const int32_t *splits, uint64_t *time_ps)
{
    uint64_t cost; int32_t rp;
    int rc = oracle_tree_cost(n, dims, props, splits, &cost, &rp);     /* validates the split list */
    if (rc == 2) return 2;
    int64_t *d = (int64_t *)malloc(sizeof(int64_t) * (n + 1));
    int32_t *p = (int32_t *)malloc(sizeof(int32_t) * (n > 0 ? n : 1));
    int32_t *where = (int32_t *)malloc(sizeof(int32_t) * (n > 0 ? n : 1));
    int m = 0;
    for (int i = 0; i < n; ++i) {
        where[i] = -1;
        if (props[i] == P_IDENTITY) continue;
        d[m] = dims[i]; p[m] = props[i]; where[i] = m; ++m;
    }
    d[m] = dims[n];
    *time_ps = 0;
    if (m > 0) {
        int32_t *s = (int32_t *)malloc(sizeof(int32_t) * m);
        for (int i = 0; i + 1 < m; ++i) s[i] = where[splits[i]];
        int pos = 0;
        subresult_t r = time_tree(d, p, 0, m - 1, s, &pos);
        free(s);
        if (r.cost >> 64) { free(d); free(p); free(where); return 1; }
        *time_ps = (uint64_t)r.cost;
    }
    free(d); free(p); free(where);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Values.                                                                   */

/* Entry (i,j) of factor t, promoted to double.  An Identity factor has no   */
/* buffer: it is the matrix with ones on the diagonal [Sec. 2, Types].       */
/* With trans[t] != 0 the chain holds the TRANSPOSE of the stored matrix      */
/* [Table 1, Transpose]: the buffer is the dims[t+1] x dims[t] matrix S,     */
/* row-major, and entry (i,j) of the factor is S[j][i].                      */
static double factor_entry(const float *const *factors, const int64_t *dims, const int32_t *props,
                           const int32_t *trans, int t, int64_t i, int64_t j)
{
    if (props[t] == P_IDENTITY) return i == j ? 1.0 : 0.0;
    if (trans && trans[t]) return (double)factors[t][j * dims[t] + i];
    return (double)factors[t][i * dims[t + 1] + j];
}

/*
 * The plain definition: every factor materialised as the dense matrix it is
 * (zeros of triangular factors are whatever the buffers hold - the input
 * generator enforces them), Identity as eye, and the chain multiplied left to
 * right with the textbook triple loop  C[i][j] = sum_k A[i][k] * B[k][j].
 * No property logic.  out: dims[0] x dims[n] doubles, row-major.
 */
int oracle_eval_dense_t(int32_t n, const int64_t *dims, const int32_t *props, const int32_t *trans,
                        const float *const *factors, double *out)
{
    if (n <= 0) return 1;
    int64_t rows = dims[0], cols = dims[1];
    double *acc = (double *)malloc(sizeof(double) * rows * cols);
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j)
            acc[i * cols + j] = factor_entry(factors, dims, props, trans, 0, i, j);
    for (int t = 1; t < n; ++t) {
        int64_t k = dims[t], nc = dims[t + 1];
        double *b = (double *)malloc(sizeof(double) * k * nc);
        for (int64_t i = 0; i < k; ++i)
            for (int64_t j = 0; j < nc; ++j)
                b[i * nc + j] = factor_entry(factors, dims, props, trans, t, i, j);
        double *c = (double *)calloc((size_t)(rows * nc), sizeof(double));
        #pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < rows; ++i)
            for (int64_t kk = 0; kk < k; ++kk) {
                double a = acc[i * k + kk];
                for (int64_t j = 0; j < nc; ++j)
                    c[i * nc + j] += a * b[kk * nc + j];
            }
        free(acc); free(b);
        acc = c; cols = nc;
    }
    memcpy(out, acc, sizeof(double) * rows * cols);
    free(acc);
    return 0;
}

int oracle_eval_dense(int32_t n, const int64_t *dims, const int32_t *props,
                      const float *const *factors, double *out)
{
    return oracle_eval_dense_t(n, dims, props, NULL, factors, out);
}

/*
 * Selected rows of the chain product, for sizes where the whole product is
 * out of reach on a CPU: row r of A_0*A_1*...*A_{n-1} is the row vector
 * A_0[r,:] pushed through the remaining factors one after the other,
 * w[j] = sum_k v[k] * A_t[k][j].  Same plain definition, no property logic.
 * out: nrows x dims[n] doubles.
 */
int oracle_eval_rows_t(int32_t n, const int64_t *dims, const int32_t *props, const int32_t *trans,
                       const float *const *factors, int32_t nrows, const int64_t *row_idx, double *out)
{
    if (n <= 0) return 1;
    int64_t widest = 0;
    for (int t = 0; t <= n; ++t) if (dims[t] > widest) widest = dims[t];
    #pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < nrows; ++r) {
        double *v = (double *)malloc(sizeof(double) * widest);
        double *w = (double *)malloc(sizeof(double) * widest);
        for (int64_t j = 0; j < dims[1]; ++j)
            v[j] = factor_entry(factors, dims, props, trans, 0, row_idx[r], j);
        for (int t = 1; t < n; ++t) {
            int64_t k = dims[t], nc = dims[t + 1];
            for (int64_t j = 0; j < nc; ++j) w[j] = 0.0;
            for (int64_t kk = 0; kk < k; ++kk) {
                double a = v[kk];
                for (int64_t j = 0; j < nc; ++j)
                    w[j] += a * factor_entry(factors, dims, props, trans, t, kk, j);
            }
            double *tmp = v; v = w; w = tmp;
        }
        memcpy(out + (int64_t)r * dims[n], v, sizeof(double) * dims[n]);
        free(v); free(w);
    }
    return 0;
}

int oracle_eval_rows(int32_t n, const int64_t *dims, const int32_t *props,
                     const float *const *factors, int32_t nrows, const int64_t *row_idx, double *out)
{
    return oracle_eval_rows_t(n, dims, props, NULL, factors, nrows, row_idx, out);
}

/* ------------------------------------------------------------------------ */
/* Evaluation along a given tree with loops restricted by the properties:   */
/* exactly the scalar products the cost model counts are executed.          */

typedef struct { double *a; int64_t rows, cols; int prop; } dmat_t;

static void k_range(int prop, int64_t i, int64_t k, int64_t *lo, int64_t *hi)   /* t with X[i][t] != 0 */
{
    *lo = 0; *hi = k;
    if (prop == P_LOWER) *hi = i + 1;
    if (prop == P_UPPER) *lo = i;
    if (prop == P_DIAGONAL) { *lo = i; *hi = i + 1; }
}

static void j_range(int prop, int64_t t, int64_t n, int64_t *lo, int64_t *hi)   /* j with Y[t][j] != 0 */
{
    *lo = 0; *hi = n;
    if (prop == P_LOWER) *hi = t + 1;
    if (prop == P_UPPER) *lo = t;
    if (prop == P_DIAGONAL) { *lo = t; *hi = t + 1; }
}

/* p holds the properties the factors have INSIDE the chain (a transposed     */
/* factor's property already mirrored); tr says which buffers hold the       */
/* transpose of their factor.                                                */
static dmat_t eval_tree(const int64_t *d, const int32_t *p, const int32_t *tr, const float *const *f,
                        int lo, int hi, const int32_t *splits, int *pos)
{
    dmat_t r;
    if (lo == hi) {                                /* leaf: promote, reading only the structure */
        r.rows = d[lo]; r.cols = d[lo + 1]; r.prop = p[lo];
        r.a = (double *)calloc((size_t)(r.rows * r.cols), sizeof(double));
        for (int64_t i = 0; i < r.rows; ++i)
            for (int64_t j = 0; j < r.cols; ++j)
                if (structurally_nonzero(r.prop, i, j))
                    r.a[i * r.cols + j] = tr[lo] ? (double)f[lo][j * r.rows + i]
                                                 : (double)f[lo][i * r.cols + j];
        return r;
    }
    int s = splits[(*pos)++];
    dmat_t X = eval_tree(d, p, tr, f, lo, s, splits, pos);
    dmat_t Y = eval_tree(d, p, tr, f, s + 1, hi, splits, pos);
    r.rows = X.rows; r.cols = Y.cols; r.prop = product_property(X.prop, Y.prop);
    r.a = (double *)calloc((size_t)(r.rows * r.cols), sizeof(double));
    int64_t K = X.cols, N = Y.cols;
    #pragma omp parallel for schedule(dynamic, 8)
    for (int64_t i = 0; i < X.rows; ++i) {
        int64_t t0, t1;
        k_range(X.prop, i, K, &t0, &t1);
        for (int64_t t = t0; t < t1; ++t) {
            double a = X.a[i * K + t];
            int64_t j0, j1;
            j_range(Y.prop, t, N, &j0, &j1);
            for (int64_t j = j0; j < j1; ++j)
                r.a[i * N + j] += a * Y.a[t * N + j];
        }
    }
    free(X.a); free(Y.a);
    return r;
}

/*
 * Evaluate the chain along the tree `splits` (preorder, ORIGINAL factor
 * indices, over the chain with Identity factors removed).  trans (may be
 * NULL): which factors enter the chain transposed [Table 1, Transpose].  out receives the
 * dense dims[0] x dims[n] result (zeros outside the triangle of a triangular
 * result; the identity matrix when every factor is an Identity).
 * Returns 0, or 2 for a malformed split list.
 */
int oracle_eval_plan_t(int32_t n, const int64_t *dims, const int32_t *props, const int32_t *trans,
                       const float *const *factors, const int32_t *splits,
                       double *out, int32_t *result_prop)
{
    /* props describe the STORED matrices; inside the chain a transposed factor
     * carries the mirrored property [Sec. 2, Transformations]                */
    int32_t *eff = (int32_t *)malloc(sizeof(int32_t) * (n > 0 ? n : 1));
    for (int i = 0; i < n; ++i)
        eff[i] = (trans && trans[i]) ? oracle_transposed_property(props[i]) : props[i];
    uint64_t cost; int32_t rp;
    int rc = oracle_tree_cost(n, dims, eff, splits, &cost, &rp);
    if (rc == 2) { free(eff); return 2; }
    *result_prop = rp;
    int64_t *d = (int64_t *)malloc(sizeof(int64_t) * (n + 1));
    int32_t *p = (int32_t *)malloc(sizeof(int32_t) * n);
    int32_t *tr = (int32_t *)malloc(sizeof(int32_t) * n);
    const float **f = (const float **)malloc(sizeof(float *) * n);
    int32_t *where = (int32_t *)malloc(sizeof(int32_t) * n);
    int m = 0;
    for (int i = 0; i < n; ++i) {
        where[i] = -1;
        if (props[i] == P_IDENTITY) continue;
        d[m] = dims[i]; p[m] = eff[i]; tr[m] = (trans && trans[i]) ? 1 : 0; f[m] = factors[i]; where[i] = m; ++m;
    }
    d[m] = dims[n];
    if (m == 0) {
        int64_t r = dims[0];
        for (int64_t i = 0; i < r; ++i)
            for (int64_t j = 0; j < r; ++j) out[i * r + j] = (i == j) ? 1.0 : 0.0;
    } else {
        int32_t *s = (int32_t *)malloc(sizeof(int32_t) * m);
        for (int i = 0; i + 1 < m; ++i) s[i] = where[splits[i]];
        int pos = 0;
        dmat_t r = eval_tree(d, p, tr, f, 0, m - 1, s, &pos);
        memcpy(out, r.a, sizeof(double) * r.rows * r.cols);
        free(r.a); free(s);
    }
    free(d); free(p); free(tr); free((void *)f); free(where); free(eff);
    return 0;
}

int oracle_eval_plan(int32_t n, const int64_t *dims, const int32_t *props,
                     const float *const *factors, const int32_t *splits,
                     double *out, int32_t *result_prop)
{
    return oracle_eval_plan_t(n, dims, props, NULL, factors, splits, out, result_prop);
}

/* ------------------------------------------------------------------------ */
/* Variadic Add [Table 1, "Add"; Sec. 2, Operations: Mul and Add take an     */
/* arbitrary number of values].                                              */

/*
 * Property of a sum of terms with the given properties (as they stand in the
 * sum, transposed terms already mirrored): the smallest structure that holds
 * every term's structure.  One term keeps its property; several terms that
 * are all Identity or diagonal give a diagonal (I + I has 2 on its diagonal:
 * no Identity); diagonal / Identity / lowerTri terms give lowerTri; the same
 * for upperTri; anything else is general.
 */
int32_t oracle_sum_property(int32_t n, const int32_t *props)
{
    if (n == 1) return props[0];
    int any_lower = 0, any_upper = 0, any_general = 0;
    for (int t = 0; t < n; ++t) {
        if (props[t] == P_LOWER) any_lower = 1;
        else if (props[t] == P_UPPER) any_upper = 1;
        else if (props[t] == P_GENERAL) any_general = 1;
    }
    if (any_general || (any_lower && any_upper)) return P_GENERAL;
    if (any_lower) return P_LOWER;
    if (any_upper) return P_UPPER;
    return P_DIAGONAL;
}

/*
 * out[i][j] = sum over the terms, in their order, of term t's entry (i, j),
 * in double precision; every term is rows x cols (a transposed term is
 * stored cols x rows), Identity terms are eye.  No property logic.
 */
int oracle_add_dense(int64_t rows, int64_t cols, int32_t n, const int32_t *props, const int32_t *trans,
                     const float *const *terms, double *out)
{
    if (n <= 0) return 1;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            double s = 0.0;
            for (int t = 0; t < n; ++t) {
                if (props[t] == P_IDENTITY) s += (i == j) ? 1.0 : 0.0;
                else if (trans && trans[t]) s += (double)terms[t][j * rows + i];
                else s += (double)terms[t][i * cols + j];
            }
            out[i * cols + j] = s;
        }
    return 0;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
