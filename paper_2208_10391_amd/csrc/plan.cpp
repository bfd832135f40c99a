// Host-side planner: identity simplification, property propagation and the
// property-aware matrix-chain dynamic program (MOM paper, Sec. 2 "Transformations"),
// followed by the schedule: the binary products in evaluation order and the placement
// of temporaries in the caller's workspace.  Integer work only; no HIP calls.
#include "../../include/mom.h"
#include "plan_internal.h"
#include "schedule.h"

#include <algorithm>
#include <limits>
#include <memory>
#include <new>

namespace {

using mom::kDiagonal;
using mom::kGeneral;
using mom::kIdentity;
using mom::kLower;
using mom::kUpper;
typedef unsigned __int128 u128;

constexpr u128 kU64Max = (u128)std::numeric_limits<uint64_t>::max();

inline bool is_tri(int p) { return p == kLower || p == kUpper; }

// Property of X*Y (Sec. 2: properties of intermediate results are inferred).  With Identity
// below diagonal (= {lowerTri, upperTri}) below the triangles below general, this is the join of
// the two operand properties: equal triangles keep their triangle, anything else fills the matrix.
inline int join(int px, int py)
{
    if (px == kIdentity) return py;
    if (py == kIdentity) return px;
    if (px == kDiagonal) return py;      // rows scaled: the structure of the other operand stays
    if (py == kDiagonal) return px;      // columns scaled
    if (px == py) return px;
    return kGeneral;
}

// Scalar multiplications of X(m x k)*Y(k x n) in which neither operand is a structural zero.
u128 product_mults(int64_t m, int64_t k, int64_t n, int px, int py)
{
    const u128 M = (u128)m, K = (u128)k, N = (u128)n;
    // a diagonal operand meets every structural entry of the other operand exactly once
    if (px == kDiagonal) return py == kDiagonal ? N : (is_tri(py) ? N * (N + 1) / 2 : K * N);
    if (py == kDiagonal) return is_tri(px) ? M * (M + 1) / 2 : M * K;
    if (!is_tri(px) && !is_tri(py)) return M * K * N;
    if (is_tri(px) && !is_tri(py)) return N * (M * (M + 1) / 2);       // row i of X has i+1 (or m-i) entries
    if (!is_tri(px) && is_tri(py)) return M * (N * (N + 1) / 2);
    if (px == py) return N * (N + 1) * (N + 2) / 6;                     // sum over i>=j of (i-j+1)
    return N * (N + 1) * (2 * N + 1) / 6;                               // sum over i,j of min(i,j)+1
}

// Property of the transpose: the structure mirrored at the diagonal (Sec. 2, Transformations:
// lowerTri(A) -> upperTri(A^T)).
inline int mirrored(int p) { return p == kLower ? kUpper : (p == kUpper ? kLower : p); }

// Modelled time of X(m x k)*Y(k x n) on the GPU in picoseconds: the objective of
// MOM_PLAN_MIN_TIME (include/mom.h states the model).  The tile shape and the slice cut are the
// ones the evaluator will use (choose_launch); the k-chunks of all tiles are summed in closed
// form per tile row, tile column, diagonal or shell, never tile by tile.
constexpr uint64_t kLaunchPs = 6000000, kChunk128Ps = 1706667, kChunk64Ps = 426667;

u128 structural_entries(int64_t rows, int64_t cols, int p)
{
    if (p == kDiagonal) return (u128)rows;
    return is_tri(p) ? (u128)rows * (u128)(rows + 1) / 2 : (u128)rows * (u128)cols;
}

u128 product_time_ps(int64_t m, int64_t k, int64_t n, int px, int py)
{
    mom::ProductStep st{};
    st.m = m; st.k = k; st.n = n; st.pa = px; st.pb = py; st.pc = join(px, py);
    if (mom::is_scaling(st))           // element-wise pass: launch + bytes
        return kLaunchPs + 4 * (structural_entries(m, k, px) + structural_entries(k, n, py) +
                                structural_entries(m, n, st.pc)) / 8;
    const mom::Launch L = mom::choose_launch(st);
    const int64_t T = L.bm, q = T / 32, tm = L.tiles_m, tn = L.tiles_n;
    const u128 chunk_ps = L.shape == mom::kTile128 ? kChunk128Ps : kChunk64Ps;
    auto chunks_up_to = [](int64_t x) { return (u128)((x + 31) / 32); };          // chunks covering [0, x)
    auto row_end = [&](int64_t I, int64_t extent) { return std::min((I + 1) * T, extent); };
    u128 all = 0, longest = 0;
    const bool xt = is_tri(px), yt = is_tri(py);
    if (!xt && !yt) {
        longest = chunks_up_to(k);
        all = (u128)tm * (u128)tn * longest;
    } else if (xt && !yt) {            // the k-range depends on the tile row only
        u128 rows = 0;
        for (int64_t I = 0; I < tm; ++I) {
            const u128 c = px == kLower ? chunks_up_to(row_end(I, m)) : chunks_up_to(k - I * T);
            rows += c;
            longest = std::max(longest, c);
        }
        all = rows * (u128)tn;
    } else if (!xt && yt) {            // ... on the tile column only
        u128 cols = 0;
        for (int64_t J = 0; J < tn; ++J) {
            const u128 c = py == kLower ? chunks_up_to(k - J * T) : chunks_up_to(row_end(J, n));
            cols += c;
            longest = std::max(longest, c);
        }
        all = cols * (u128)tm;
    } else if (px == py) {             // L*L -> L (tiles I >= J: [J*T, end(I))), U*U -> U mirrored
        for (int64_t I = 0; I < tm; ++I) {
            const u128 c = chunks_up_to(row_end(I, n));
            all += (u128)(I + 1) * c - (u128)q * (u128)I * (u128)(I + 1) / 2;
            longest = std::max(longest, c);
        }
    } else if (px == kLower) {         // L*U: [0, end(min(I, J))): shell s has 2*(tm-s)-1 tiles
        for (int64_t s = 0; s < tm; ++s) {
            const u128 c = chunks_up_to(row_end(s, n));
            all += c * (u128)(2 * (tm - s) - 1);
            longest = std::max(longest, c);
        }
    } else {                           // U*L: [max(I, J)*T, n): shell s has 2*s+1 tiles
        for (int64_t s = 0; s < tm; ++s) {
            const u128 c = chunks_up_to(n - s * T);
            all += c * (u128)(2 * s + 1);
            longest = std::max(longest, c);
        }
    }
    if (L.split_k > 1) longest = (longest + L.split_k - 1) / L.split_k;            // the longest tile's slice
    const u128 spread = (all + mom::kComputeUnits - 1) / mom::kComputeUnits;
    const u128 matrix = std::max(longest, spread) * chunk_ps;
    const u128 memory = 4 * (structural_entries(m, k, px) + structural_entries(k, n, py) +
                             structural_entries(m, n, st.pc)) / 8;
    u128 t = kLaunchPs + std::max(matrix, memory);
    if (L.split_k > 1) t += kLaunchPs + 4 * (u128)(L.split_k + 1) * structural_entries(m, n, st.pc) / 8;
    return t;
}

mom_status_t validate(const int64_t *dims, const int32_t *props, const int32_t *trans, int32_t n)
{
    if (!dims || !props) return MOM_ERR_NULL;
    if (n <= 0 || n > MOM_MAX_FACTORS) return MOM_ERR_BAD_N;
    for (int i = 0; i <= n; ++i)
        if (dims[i] <= 0 || dims[i] > (int64_t)MOM_MAX_DIM) return MOM_ERR_BAD_DIM;
    for (int i = 0; i < n; ++i) {
        if (props[i] < kGeneral || props[i] > kDiagonal) return MOM_ERR_BAD_PROP;
        if (props[i] != kGeneral && dims[i] != dims[i + 1]) return MOM_ERR_NOT_SQUARE;
        if (trans && trans[i] != 0 && trans[i] != 1) return MOM_ERR_BAD_TRANS;
    }
    return MOM_OK;
}

// First-fit allocator over the workspace, 256-byte granules; temporaries are released as
// soon as the product that consumes them has been scheduled, so their space is reused.
class Arena {
public:
    size_t alloc(size_t bytes)
    {
        bytes = (bytes + 255) & ~(size_t)255;
        for (size_t i = 0; i < free_.size(); ++i) {
            if (free_[i].second >= bytes) {
                size_t off = free_[i].first;
                free_[i].first += bytes;
                free_[i].second -= bytes;
                if (free_[i].second == 0) free_.erase(free_.begin() + i);
                return off;
            }
        }
        const size_t off = top_;      // release() never leaves a free block touching top_
        top_ = off + bytes;
        peak_ = std::max(peak_, top_);
        return off;
    }
    void release(size_t off, size_t bytes)
    {
        bytes = (bytes + 255) & ~(size_t)255;
        free_.emplace_back(off, bytes);
        std::sort(free_.begin(), free_.end());
        for (size_t i = 0; i + 1 < free_.size();) {       // merge neighbours
            if (free_[i].first + free_[i].second == free_[i + 1].first) {
                free_[i].second += free_[i + 1].second;
                free_.erase(free_.begin() + i + 1);
            } else {
                ++i;
            }
        }
        if (!free_.empty() && free_.back().first + free_.back().second == top_) {
            top_ = free_.back().first;
            free_.pop_back();
        }
    }
    size_t peak() const { return peak_; }

private:
    std::vector<std::pair<size_t, size_t>> free_;
    size_t top_ = 0, peak_ = 0;
};

struct Builder {
    mom_plan *plan;
    const std::vector<int64_t> &d;     // dims of the survivors chain
    const std::vector<int32_t> &p;     // props of the survivors chain
    const std::vector<int32_t> &split_pos;   // preorder, positions in the survivors chain
    std::vector<int> producer;         // temporary id -> index of the step that writes it
    size_t cursor = 0;
    int depth = 0, max_depth = 0;
    u128 total = 0, total_time = 0;
    bool ok = true;

    struct Value { mom::Operand op; int64_t rows, cols; int prop; };

    Value walk(int lo, int hi, bool is_root)
    {
        if (lo == hi) {
            ++depth; max_depth = std::max(max_depth, depth);
            return Value{{mom::Where::Factor, plan->survivors[lo]}, d[lo], d[lo + 1], p[lo]};
        }
        if (cursor >= split_pos.size()) { ok = false; return Value{}; }
        const int s = split_pos[cursor++];
        if (s < lo || s >= hi) { ok = false; return Value{}; }
        Value a = walk(lo, s, false);
        if (!ok) return Value{};
        Value b = walk(s + 1, hi, false);
        if (!ok) return Value{};
        mom::ProductStep st;
        st.a = a.op; st.b = b.op;
        st.m = a.rows; st.k = a.cols; st.n = b.cols;
        st.pa = a.prop; st.pb = b.prop; st.pc = join(a.prop, b.prop);
        st.ta = a.op.where == mom::Where::Factor && plan->trans[a.op.index];
        st.tb = b.op.where == mom::Where::Factor && plan->trans[b.op.index];
        const u128 c = product_mults(st.m, st.k, st.n, st.pa, st.pb);
        total += c;
        total_time += product_time_ps(st.m, st.k, st.n, st.pa, st.pb);
        st.mults = c > kU64Max ? std::numeric_limits<uint64_t>::max() : (uint64_t)c;
        auto level_of = [&](const mom::Operand &o) {
            return o.where == mom::Where::Temp ? plan->steps[producer[o.index]].level : 0;
        };
        st.level = 1 + std::max(level_of(a.op), level_of(b.op));
        st.scratch_offset = 0;
        if (is_root) {
            st.c = {mom::Where::Out, 0};
        } else {
            plan->temps.push_back({0, (size_t)st.m * (size_t)st.n * sizeof(float)});
            producer.push_back((int)plan->steps.size());
            st.c = {mom::Where::Temp, (int)plan->temps.size() - 1};
        }
        plan->steps.push_back(st);
        --depth;    // two operands popped, one result pushed
        return Value{st.c, st.m, st.n, st.pc};
    }
};

void render(const mom_plan *plan, const std::vector<int32_t> &split_pos, size_t &cursor, int lo, int hi,
            std::string &out)
{
    if (lo == hi) { out += std::to_string(plan->survivors[lo]); return; }
    const int s = split_pos[cursor++];
    out += '(';
    render(plan, split_pos, cursor, lo, s, out);
    out += ' ';
    render(plan, split_pos, cursor, s + 1, hi, out);
    out += ')';
}

// (X * Y) * Z with a narrow X * Y runs as ONE launch that reads X, Y and Z and never writes
// X * Y.  That launch happens where the outer product stands in the evaluation order, so the
// inner product is moved to the outer one's level: its operands then stay alive (and its
// never-written temporary stays reserved) until that launch has run, and nothing placed at
// that level can overlap them.
void find_shared_launches(mom_plan *plan)
{
    using namespace mom;
    plan->absorbed_by.assign(plan->steps.size(), -1);
    for (size_t j = 0; j < plan->steps.size(); ++j) {
        const ProductStep &outer = plan->steps[j];
        if (outer.a.where != Where::Temp) continue;
        for (size_t i = 0; i < plan->steps.size(); ++i) {
            ProductStep &inner = plan->steps[i];
            if (inner.c.where == Where::Temp && inner.c.index == outer.a.index && fits_skinny_pair(inner, outer)) {
                plan->absorbed_by[i] = (int32_t)j;
                inner.level = outer.level;
            }
        }
    }
}

// The evaluation as a list of launches.  Level by level; the products of a level that share a
// tile shape go out in one launch (at most kMaxFused at a time), followed by one launch that
// sums their split-K slices.  Only small products share a launch: a big one fills the chip by
// itself and keeps its longest-first tile order only when it is alone.  Everything but the
// operands' addresses is fixed here, so an evaluation call allocates and decides nothing.
mom_status_t lay_out_launches(mom_plan *plan)
{
    using namespace mom;
    const std::vector<int32_t> &order = plan->order;
    // products whose narrow result is consumed as the left operand of a product they share a
    // launch with (found before the workspace was laid out, see find_shared_launches)
    const std::vector<int32_t> &absorbed_by = plan->absorbed_by;
    std::vector<int> absorbs(plan->steps.size(), -1);
    for (size_t i = 0; i < plan->steps.size(); ++i)
        if (absorbed_by[i] >= 0) absorbs[absorbed_by[i]] = (int)i;
    size_t next = 0;
    while (next < order.size()) {
        const int level = plan->steps[order[next]].level;
        size_t level_end = next;
        while (level_end < order.size() && plan->steps[order[level_end]].level == level) ++level_end;
        std::vector<char> done(level_end - next, 0);
        for (size_t first = next; first < level_end; ++first) {
            if (done[first - next]) continue;
            PlannedLaunch pl{};
            if (absorbed_by[order[first]] >= 0) {               // runs inside its consumer's launch
                done[first - next] = 1;
                continue;
            }
            if (absorbs[order[first]] >= 0) {                   // (X * Y) * Z in one launch
                done[first - next] = 1;
                pl.kind = kLaunchPair;
                pl.step[0] = absorbs[order[first]];
                pl.step[1] = order[first];
                plan->launches.push_back(pl);
                continue;
            }
            if (is_scaling(plan->steps[order[first]])) {        // an element-wise pass of its own
                const ProductStep &st = plan->steps[order[first]];
                done[first - next] = 1;
                pl.kind = kLaunchScale;
                pl.step[0] = order[first];
                pl.batch.count = 1;
                ProductParams &p = pl.batch.prob[0];
                p.M = (int)st.m; p.N = (int)st.n; p.K = (int)st.k;
                p.pa = st.pa; p.pb = st.pb; p.pc = st.pc;
                plan->launches.push_back(pl);
                continue;
            }
            pl.kind = kLaunchProduct;
            pl.shape = choose_launch(plan->steps[order[first]]).shape;
            pl.variant = (plan->steps[order[first]].ta ? 1 : 0) + (plan->steps[order[first]].tb ? 2 : 0);
            {   // a product whose last round of tiles is cut along k: two sub-products, one launch
                const ProductStep &st = plan->steps[order[first]];
                const Launch L = choose_launch(st);
                const Tail tail = choose_tail(st, L);
                if (tail.tile_rows_main > 0) {
                    done[first - next] = 1;
                    const int64_t rows_main = (int64_t)tail.tile_rows_main * L.bm;
                    for (int slot = 0; slot < 2; ++slot) {
                        pl.step[slot] = order[first];
                        pl.row0[slot] = slot ? rows_main : 0;
                        ProductParams &p = pl.batch.prob[slot];
                        p.M = (int)(slot ? st.m - rows_main : rows_main); p.N = (int)st.n; p.K = (int)st.k;
                        p.pa = st.pa; p.pb = st.pb; p.pc = st.pc;
                        p.tiles_m = slot ? L.tiles_m - tail.tile_rows_main : tail.tile_rows_main;
                        p.tiles_n = L.tiles_n; p.num_tiles = p.tiles_m * p.tiles_n;
                        p.order = L.order; p.paired = 0; p.mirrored = 0; p.k_walk = 0; p.folded = 0;
                        p.grid = slot ? p.num_tiles : std::min(p.num_tiles, 2 * kComputeUnits);
                        p.split_k = slot ? tail.split : 1;
                        p.slice_stride = slot ? (int64_t)p.M * p.N : 0;
                        const int64_t blocks = (int64_t)(slot ? pl.batch.block_end[0] : 0) + (int64_t)p.grid * p.split_k;
                        pl.batch.block_end[pl.batch.count++] = (int)blocks;
                    }
                    ReduceParams &r = pl.reduce.prob[0];
                    pl.reduce_of[0] = 1;
                    pl.reduce.count = 1;
                    r.slice_stride = pl.batch.prob[1].slice_stride;
                    r.slices = tail.split; r.M = pl.batch.prob[1].M; r.N = pl.batch.prob[1].N; r.pc = st.pc;
                    pl.reduce_grid_x = (unsigned)std::min<int64_t>((((int64_t)r.M * r.N + 3) / 4 + 31) / 32, 8192);
                    plan->launches.push_back(pl);
                    continue;
                }
            }
            int64_t reduce_quads = 0;
            bool batch_small = true;
            for (size_t i = first; i < level_end && pl.batch.count < kMaxFused; ++i) {
                const ProductStep &st = plan->steps[order[i]];
                const Launch L = choose_launch(st);
                if (done[i - next] || is_scaling(st) || absorbed_by[order[i]] >= 0 || absorbs[order[i]] >= 0 ||
                    L.shape != pl.shape || (st.ta ? 1 : 0) + (st.tb ? 2 : 0) != pl.variant) continue;
                const bool small_launch = (int64_t)L.grid * L.split_k <= 4 * kComputeUnits;
                if (pl.batch.count > 0 && (!small_launch || !batch_small)) continue;
                batch_small = small_launch;
                done[i - next] = 1;
                const int slot = pl.batch.count;
                pl.step[slot] = order[i];
                ProductParams &p = pl.batch.prob[slot];
                p.M = (int)st.m; p.N = (int)st.n; p.K = (int)st.k;
                p.pa = st.pa; p.pb = st.pb; p.pc = st.pc;
                p.tiles_m = L.tiles_m; p.tiles_n = L.tiles_n; p.num_tiles = L.num_tiles;
                p.order = L.order; p.paired = L.paired; p.mirrored = L.mirrored; p.k_walk = L.k_walk; p.folded = L.folded; p.grid = L.grid;
                p.split_k = L.split_k;
                p.slice_stride = L.split_k > 1 ? st.m * st.n : 0;
                if (L.split_k > 1) {
                    ReduceParams &r = pl.reduce.prob[pl.reduce.count];
                    pl.reduce_of[pl.reduce.count++] = slot;
                    r.slice_stride = p.slice_stride;
                    r.slices = L.split_k; r.M = p.M; r.N = p.N; r.pc = st.pc;
                    reduce_quads = std::max<int64_t>(reduce_quads, (st.m * st.n + 3) / 4);
                }
                const int64_t blocks = (int64_t)(slot ? pl.batch.block_end[slot - 1] : 0) + (int64_t)L.grid * L.split_k;
                if (blocks > 0x7fffffff) return MOM_ERR_UNSUPPORTED;
                pl.batch.block_end[pl.batch.count++] = (int)blocks;
            }
            pl.reduce_grid_x = (unsigned)std::min<int64_t>((reduce_quads + 31) / 32, 8192);
            plan->launches.push_back(pl);
        }
        next = level_end;
    }
    return MOM_OK;
}

// Batched evaluation keeps every value of a chain in an LDS slot: a factor sits in the slot of
// its position among the survivors, a product's result takes over the slot of its left operand.
void assign_batched_slots(mom_plan *plan)
{
    using namespace mom;
    const int nl = (int)plan->survivors.size();
    if (nl > kBatchedSlots) return;
    std::vector<int> temp_slot(plan->temps.size(), -1);
    auto slot_of = [&](const Operand &o) {
        if (o.where == Where::Temp) return temp_slot[o.index];
        for (int i = 0; i < nl; ++i)
            if (plan->survivors[i] == o.index) return i;
        return -1;
    };
    for (size_t s = 0; s < plan->steps.size(); ++s) {
        const ProductStep &st = plan->steps[s];
        plan->a_slot[s] = slot_of(st.a);
        plan->b_slot[s] = slot_of(st.b);
        if (st.c.where == Where::Temp) temp_slot[st.c.index] = plan->a_slot[s];
    }
}

// Build everything that follows from a chosen tree (given as positions in the survivors chain).
mom_status_t finish(mom_plan *plan, const std::vector<int64_t> &d, const std::vector<int32_t> &p,
                    const std::vector<int32_t> &split_pos)
{
    const int m = (int)plan->survivors.size();
    plan->rows = plan->dims.front();
    plan->cols = plan->dims.back();
    plan->max_dim = *std::max_element(plan->dims.begin(), plan->dims.end());
    if (m == 0) {                       // I*I = I
        plan->result_prop = kIdentity;
        plan->cost = 0;
        plan->text = "I";
        return MOM_OK;
    }
    if ((int)split_pos.size() != m - 1) return MOM_ERR_BAD_SPLITS;
    Builder b{plan, d, p, split_pos, {}};
    Builder::Value root = b.walk(0, m - 1, true);
    if (!b.ok || b.cursor != split_pos.size()) return MOM_ERR_BAD_SPLITS;
    if (b.total > kU64Max) return MOM_ERR_OVERFLOW;
    plan->cost = (uint64_t)b.total;
    plan->time_ps = b.total_time > kU64Max ? std::numeric_limits<uint64_t>::max() : (uint64_t)b.total_time;
    plan->result_prop = root.prop;
    plan->stack_depth = b.max_depth;
    plan->splits.clear();
    for (int s : split_pos) plan->splits.push_back(plan->survivors[s]);
    size_t cursor = 0;
    render(plan, split_pos, cursor, 0, m - 1, plan->text);

    find_shared_launches(plan);

    // Evaluation order: level by level.  The products of one level do not depend on each
    // other, so the evaluator may put them into one launch; a temporary lives from the level
    // that writes it to the level that reads it.  Split-K partial sums of a level's products
    // sit side by side in a scratch region behind the temporaries.
    int top = 0;
    for (const mom::ProductStep &st : plan->steps) top = std::max(top, st.level);
    Arena arena;
    size_t scratch = 0;
    for (int level = 1; level <= top; ++level) {
        size_t level_scratch = 0;
        for (size_t i = 0; i < plan->steps.size(); ++i) {
            mom::ProductStep &st = plan->steps[i];
            if (st.level != level) continue;
            plan->order.push_back((int32_t)i);
            if (st.c.where == mom::Where::Temp) plan->temps[st.c.index].offset = arena.alloc(plan->temps[st.c.index].bytes);
            st.scratch_offset = level_scratch;
            const mom::Launch L = mom::choose_launch(st);
            level_scratch += (L.scratch_bytes + mom::choose_tail(st, L).scratch_bytes + 255) & ~(size_t)255;
        }
        scratch = std::max(scratch, level_scratch);
        for (const mom::ProductStep &st : plan->steps) {
            if (st.level != level) continue;
            for (const mom::Operand &o : {st.a, st.b})
                if (o.where == mom::Where::Temp) arena.release(plan->temps[o.index].offset, plan->temps[o.index].bytes);
        }
    }
    plan->temp_bytes = arena.peak();
    plan->scratch_offset = (plan->temp_bytes + 255) & ~(size_t)255;
    plan->scratch_bytes = scratch;
    plan->workspace_bytes = scratch ? plan->scratch_offset + scratch : plan->temp_bytes;
    mom_status_t st = lay_out_launches(plan);
    if (st != MOM_OK) return st;
    assign_batched_slots(plan);
    return MOM_OK;
}

// identity simplification: A*I -> A, I*A -> A, I*I = I.  d / p receive the survivors' chain.
void start(mom_plan *plan, const int64_t *dims, const int32_t *props, const int32_t *trans, int32_t n,
           std::vector<int64_t> &d, std::vector<int32_t> &p)
{
    plan->n = n;
    plan->dims.assign(dims, dims + n + 1);
    plan->props.assign(props, props + n);
    plan->trans.assign(n, 0);
    plan->chain_props.assign(props, props + n);
    for (int i = 0; i < n; ++i) {
        if (trans && trans[i] && props[i] != kIdentity) {       // the transpose of I is I
            plan->trans[i] = 1;
            plan->chain_props[i] = mirrored(props[i]);
        }
        if (props[i] == kIdentity) continue;
        plan->survivors.push_back(i);
        d.push_back(dims[i]);
        p.push_back(plan->chain_props[i]);
    }
    d.push_back(dims[n]);
}

// The chain DP: the smallest sum of product costs (multiplications, or modelled picoseconds)
// for every sub-chain of the survivors, smallest split on ties; returns the chosen tree as
// preorder positions.  Both costs are sums over the products of a tree, and the shape and
// property of a sub-chain's product do not depend on its tree, so the recurrence is exact.
mom_status_t optimal_splits(const std::vector<int64_t> &d, const std::vector<int32_t> &p, int objective,
                            std::vector<int32_t> &split_pos)
{
    const int m = (int)p.size();
    if (m <= 1) return MOM_OK;
    // best[i][j]: fewest multiplications for survivors i..j; prop[i][j]: their product's
    // property (independent of the parenthesisation); cut[i][j]: chosen split.
    std::vector<u128> best((size_t)m * m, 0);
    std::vector<int32_t> cut((size_t)m * m, -1);
    std::vector<int8_t> prop((size_t)m * m, 0);
    auto at = [m](int i, int j) { return (size_t)i * m + j; };
    for (int i = 0; i < m; ++i) {
        prop[at(i, i)] = (int8_t)p[i];
        for (int j = i + 1; j < m; ++j) prop[at(i, j)] = (int8_t)join(prop[at(i, j - 1)], p[j]);
    }
    for (int len = 2; len <= m; ++len) {
        for (int i = 0; i + len <= m; ++i) {
            const int j = i + len - 1;
            u128 lowest = 0;
            int where = -1;
            for (int k = i; k < j; ++k) {       // ascending; only a strictly smaller cost
                const u128 c = best[at(i, k)] + best[at(k + 1, j)] +
                               (objective == MOM_PLAN_MIN_TIME
                                    ? product_time_ps(d[i], d[k + 1], d[j + 1], prop[at(i, k)], prop[at(k + 1, j)])
                                    : product_mults(d[i], d[k + 1], d[j + 1], prop[at(i, k)], prop[at(k + 1, j)]));
                if (where < 0 || c < lowest) { lowest = c; where = k; }   // replaces: smallest split wins ties
            }
            best[at(i, j)] = lowest;
            cut[at(i, j)] = where;
        }
    }
    if (best[at(0, m - 1)] > kU64Max) return MOM_ERR_OVERFLOW;
    // preorder read-out of the chosen tree
    std::vector<std::pair<int, int>> todo{{0, m - 1}};
    while (!todo.empty()) {
        auto [lo, hi] = todo.back();
        todo.pop_back();
        if (lo == hi) continue;
        const int s = cut[at(lo, hi)];
        split_pos.push_back(s);
        todo.emplace_back(s + 1, hi);
        todo.emplace_back(lo, s);
    }
    return MOM_OK;
}

// Plan with the DP's tree (forced == nullptr) or with a given one.  Exceptions (allocation
// failures of the containers) are turned into a status by the callers.
mom_status_t make_plan(const int64_t *dims, const int32_t *props, const int32_t *trans, int32_t n,
                       int32_t objective, bool forced_tree, const int32_t *forced, mom_plan_t **out)
{
    mom_status_t st = validate(dims, props, trans, n);
    if (st != MOM_OK) return st;
    if (objective != MOM_PLAN_MIN_MULTS && objective != MOM_PLAN_MIN_TIME) return MOM_ERR_BAD_FLAGS;
    std::unique_ptr<mom_plan> plan(new mom_plan());
    plan->objective = objective;
    std::vector<int64_t> d;
    std::vector<int32_t> p;
    start(plan.get(), dims, props, trans, n, d, p);
    const int m = (int)p.size();
    std::vector<int32_t> split_pos;
    if (!forced_tree) {
        st = optimal_splits(d, p, objective, split_pos);
        if (st != MOM_OK) return st;
    } else if (m > 1) {
        if (!forced) return MOM_ERR_NULL;
        std::vector<int32_t> position(n, -1);
        for (int i = 0; i < m; ++i) position[plan->survivors[i]] = i;
        for (int i = 0; i < m - 1; ++i) {
            const int32_t s = forced[i];
            if (s < 0 || s >= n || position[s] < 0) return MOM_ERR_BAD_SPLITS;
            split_pos.push_back(position[s]);
        }
    }
    st = finish(plan.get(), d, p, split_pos);
    if (st != MOM_OK) return st;
    *out = plan.release();
    return MOM_OK;
}

// No exception leaves the library: allocation failures become MOM_ERR_NOMEM.
template <class F>
mom_status_t guarded(F &&body)
{
    try {
        return body();
    } catch (const std::bad_alloc &) {
        return MOM_ERR_NOMEM;
    } catch (...) {
        return MOM_ERR_NOMEM;
    }
}

}  // namespace

extern "C" {

mom_status_t mom_chain_plan(const int64_t *dims, const int32_t *props, int32_t n, mom_plan_t **out)
{
    if (!out) return MOM_ERR_NULL;
    *out = nullptr;
    return guarded([&] { return make_plan(dims, props, nullptr, n, MOM_PLAN_MIN_MULTS, false, nullptr, out); });
}

mom_status_t mom_plan_from_splits(const int64_t *dims, const int32_t *props, int32_t n,
                                  const int32_t *preorder_splits, mom_plan_t **out)
{
    if (!out) return MOM_ERR_NULL;
    *out = nullptr;
    return guarded([&] { return make_plan(dims, props, nullptr, n, MOM_PLAN_MIN_MULTS, true, preorder_splits, out); });
}

mom_status_t mom_chain_plan_ex(const int64_t *dims, const int32_t *props, const int32_t *trans, int32_t n,
                               int32_t objective, const int32_t *preorder_splits, mom_plan_t **out)
{
    if (!out) return MOM_ERR_NULL;
    *out = nullptr;
    return guarded([&] {
        return make_plan(dims, props, trans, n, objective, preorder_splits != nullptr, preorder_splits, out);
    });
}

// Property of a sum: the smallest structure that holds every addend's structure.  One addend
// keeps its property; several Identity / diagonal addends give a diagonal (never an Identity).
static int sum_property(const std::vector<int> &props)
{
    if (props.size() == 1) return props[0];
    bool lower = false, upper = false, general = false;
    for (int p : props) {
        lower |= p == kLower;
        upper |= p == kUpper;
        general |= p == kGeneral;
    }
    if (general || (lower && upper)) return kGeneral;
    return lower ? kLower : (upper ? kUpper : kDiagonal);
}

mom_status_t mom_equation_plan(const int64_t *dims, const int32_t *props, const int32_t *trans,
                               const int32_t *chain_len, int32_t n_chains, int32_t objective, mom_equation_t **out)
{
    if (!out) return MOM_ERR_NULL;
    *out = nullptr;
    if (!dims || !props || !chain_len) return MOM_ERR_NULL;
    if (n_chains <= 0 || n_chains > MOM_MAX_FACTORS) return MOM_ERR_BAD_N;
    return guarded([&]() -> mom_status_t {
        std::unique_ptr<mom_equation> eq(new mom_equation());
        std::vector<int> result_props;
        int64_t factor_at = 0, dim_at = 0;
        size_t largest_products_ws = 0;
        bool any_products = false;
        u128 cost = 0, time = 0;
        for (int c = 0; c < n_chains; ++c) {
            const int32_t len = chain_len[c];
            if (len <= 0 || len > MOM_MAX_FACTORS) return MOM_ERR_BAD_N;
            mom_plan_t *plan = nullptr;
            const mom_status_t st = make_plan(dims + dim_at, props + factor_at, trans ? trans + factor_at : nullptr, len,
                                              objective, false, nullptr, &plan);
            if (st != MOM_OK) return st;
            eq->chains.push_back(plan);
            eq->first_factor.push_back((int32_t)factor_at);
            if (c == 0) { eq->rows = plan->rows; eq->cols = plan->cols; }
            if (plan->rows != eq->rows || plan->cols != eq->cols) return MOM_ERR_BAD_DIM;
            result_props.push_back(plan->result_prop);
            cost += plan->cost;
            time += plan->time_ps;
            if (!plan->steps.empty()) {
                any_products = true;
                largest_products_ws = std::max(largest_products_ws, plan->workspace_bytes);
            }
            factor_at += len;
            dim_at += len + 1;
        }
        if (cost > kU64Max) return MOM_ERR_OVERFLOW;
        eq->cost = (uint64_t)cost;
        eq->time_ps = time > kU64Max ? std::numeric_limits<uint64_t>::max() : (uint64_t)time;
        eq->result_prop = sum_property(result_props);
        // the first addend with products whose result fills the sum's structure goes straight to
        // the output; every other addend with products passes through one temporary
        int through_temp = 0;
        for (int c = 0; c < n_chains; ++c) {
            if (eq->chains[c]->steps.empty()) continue;
            if (eq->direct_chain < 0 && eq->chains[c]->result_prop == eq->result_prop) eq->direct_chain = c;
            else ++through_temp;
        }
        eq->chain_bytes = any_products ? (largest_products_ws + 255) & ~(size_t)255 : 0;
        eq->temp_offset = eq->chain_bytes;
        const size_t temp = through_temp ? (size_t)eq->rows * (size_t)eq->cols * sizeof(float) : 0;
        eq->workspace_bytes = eq->chain_bytes + temp;
        *out = eq.release();
        return MOM_OK;
    });
}

void mom_equation_destroy(mom_equation_t *eq) { delete eq; }

mom_status_t mom_equation_result(const mom_equation_t *eq, int64_t *rows, int64_t *cols, int32_t *prop)
{
    if (!eq) return MOM_ERR_NULL;
    if (rows) *rows = eq->rows;
    if (cols) *cols = eq->cols;
    if (prop) *prop = eq->result_prop;
    return MOM_OK;
}

uint64_t mom_equation_cost_mults(const mom_equation_t *eq) { return eq ? eq->cost : 0; }

size_t mom_equation_workspace_bytes(const mom_equation_t *eq) { return eq ? eq->workspace_bytes : 0; }

int32_t mom_equation_num_chains(const mom_equation_t *eq) { return eq ? (int32_t)eq->chains.size() : 0; }

const mom_plan_t *mom_equation_chain(const mom_equation_t *eq, int32_t c)
{
    return (eq && c >= 0 && c < (int32_t)eq->chains.size()) ? eq->chains[c] : nullptr;
}

void mom_plan_destroy(mom_plan_t *plan) { delete plan; }

uint64_t mom_plan_cost_mults(const mom_plan_t *plan) { return plan ? plan->cost : 0; }

uint64_t mom_plan_cost_time_ps(const mom_plan_t *plan) { return plan ? plan->time_ps : 0; }

int32_t mom_plan_num_products(const mom_plan_t *plan) { return plan ? (int32_t)plan->steps.size() : 0; }

mom_status_t mom_plan_result(const mom_plan_t *plan, int64_t *rows, int64_t *cols, int32_t *prop)
{
    if (!plan) return MOM_ERR_NULL;
    if (rows) *rows = plan->rows;
    if (cols) *cols = plan->cols;
    if (prop) *prop = plan->result_prop;
    return MOM_OK;
}

mom_status_t mom_plan_string(const mom_plan_t *plan, char *buf, size_t cap)
{
    if (!plan || !buf) return MOM_ERR_NULL;
    if (cap < plan->text.size() + 1) return MOM_ERR_BUFFER_TOO_SMALL;
    std::copy(plan->text.begin(), plan->text.end(), buf);
    buf[plan->text.size()] = '\0';
    return MOM_OK;
}

mom_status_t mom_plan_splits(const mom_plan_t *plan, int32_t *out, int32_t cap)
{
    if (!plan || (!out && !plan->splits.empty())) return MOM_ERR_NULL;
    if (cap < (int32_t)plan->splits.size()) return MOM_ERR_BUFFER_TOO_SMALL;
    std::copy(plan->splits.begin(), plan->splits.end(), out);
    return MOM_OK;
}

mom_status_t mom_plan_product(const mom_plan_t *plan, int32_t i, int64_t *shape, int32_t *props,
                              uint64_t *mults, int32_t *level)
{
    if (!plan) return MOM_ERR_NULL;
    if (i < 0 || i >= (int32_t)plan->order.size()) return MOM_ERR_BAD_N;
    const mom::ProductStep &st = plan->steps[plan->order[i]];
    if (shape) { shape[0] = st.m; shape[1] = st.k; shape[2] = st.n; }
    if (props) { props[0] = st.pa; props[1] = st.pb; props[2] = st.pc; }
    if (mults) *mults = st.mults;
    if (level) *level = st.level;
    return MOM_OK;
}

int32_t mom_plan_num_launches(const mom_plan_t *plan)
{
    if (!plan) return 0;
    if (plan->steps.empty()) return 1;                    // identity write or copy
    int32_t n = 0;
    for (const mom::PlannedLaunch &pl : plan->launches) n += 1 + (pl.reduce.count > 0 ? 1 : 0);
    return n;
}

size_t mom_plan_workspace_bytes(const mom_plan_t *plan) { return plan ? plan->workspace_bytes : 0; }

const char *mom_status_string(mom_status_t status)
{
    switch (status) {
    case MOM_OK: return "ok";
    case MOM_ERR_NULL: return "a required pointer is NULL";
    case MOM_ERR_BAD_N: return "number of factors (or batch) out of range";
    case MOM_ERR_BAD_DIM: return "a dimension is not in 1..2^31-256";
    case MOM_ERR_BAD_PROP: return "unknown matrix property";
    case MOM_ERR_NOT_SQUARE: return "a triangular or Identity factor is not square";
    case MOM_ERR_OVERFLOW: return "multiplication count does not fit in 64 bits";
    case MOM_ERR_BAD_SPLITS: return "forced parenthesisation is not a tree over the chain";
    case MOM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case MOM_ERR_BUFFER_TOO_SMALL: return "host buffer too small";
    case MOM_ERR_BAD_STRIDE: return "stride smaller than the matrix needs";
    case MOM_ERR_UNSUPPORTED: return "plan not covered by the kernel (batched: a dimension above 32 or more than 8 factors)";
    case MOM_ERR_HIP: return "HIP runtime error";
    case MOM_ERR_BAD_TRANS: return "a transposition flag is neither 0 nor 1";
    case MOM_ERR_NOMEM: return "out of host memory";
    case MOM_ERR_BAD_FLAGS: return "unknown flag bits";
    case MOM_ERR_NOT_READY: return "first use on this device happened under stream capture: call mom_init before capturing";
    }
    return "unknown status";
}

}  // extern "C"
