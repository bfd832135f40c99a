// Launch geometry of one binary product: tile shape, tile order, pairing and split-K.
// Plain integer logic shared by the planner (which sizes the workspace) and the evaluator
// (which launches); written for the MI355X: 256 compute units in 8 XCDs.
#pragma once
#include <algorithm>

#include "launch_params.h"
#include "plan_internal.h"

namespace mom {

constexpr int kComputeUnits = 256;
constexpr int kXcds = 8;                   // accelerator dies, each with an L2 of its own; workgroup b is
                                           // dispatched to die b % 8
constexpr int kMinChunksPerSlice = 8;
constexpr int kSplitTargetWorkgroups = 768;
constexpr int kMinChunksToSplit = 64;      // below this the second launch costs more than it saves
constexpr int kChunk128 = 32, kChunk64 = 32;   // k-chunk (BK) of the 128x128 and of the 64x64 tile shape

// Tile shapes the product kernel is instantiated for.
enum TileShape : int { kTile128 = 0, kTile64 = 1, kNumTileShapes };

// Order in which workgroups take tiles.  A property clips the k-range of a tile, so tiles
// differ in length; the longest are handed out first.
enum TileOrder : int {
    kRowMajor = 0,     // general*general: all tiles equally long
    kRowsDesc,         // L*G : tile row I needs k <  (I+1)*BM      -> bottom rows first
    kRowsAsc,          // U*G : tile row I needs k >= I*BM          -> top rows first
    kColsAsc,          // G*L : tile col J needs k >= J*BN          -> left columns first
    kColsDesc,         // G*U : tile col J needs k <  (J+1)*BN      -> right columns first
    kDiagLower,        // L*L -> L: only I >= J, length I-J+1       -> far diagonals first
    kDiagUpper,        // U*U -> U: only J >= I, length J-I+1
    kShellMin,         // L*U : length min(I,J)+1                   -> bottom-right shells first
    kShellMax          // U*L : length nt - max(I,J)                -> top-left shells first
};

struct Launch {
    int shape;             // TileShape
    int bm, bn;
    int tiles_m, tiles_n;
    int num_tiles;         // tiles that exist (a triangular result has no tiles in its zero half)
    int order;             // TileOrder
    int paired;            // 1: workgroup b also takes tile num_tiles-1-b (longest with shortest);
                           // 2: pairs are dealt so that every die works on tile rows of its own
    int mirrored;          // pairs few enough to leave compute units with one workgroup: the two tiles of
                           // a pair go to two workgroups, b (long tile) and b + pairs (short tile), which
                           // the dispatcher places on the same compute unit; they then overlap each other
    int folded;            // single tiles, the second 256 workgroups in reverse order (see choose_launch)
    int k_walk;            // direction in which tiles walk their k-range (bit 0: a workgroup's first tile
                           // downwards, bit 1: its later tiles downwards)
    int grid;              // workgroups
    int split_k;           // >1: the k-range is cut into this many slices, summed by a second kernel
    size_t scratch_bytes;  // split_k * m * n floats of partial sums
};

inline int tile_order(const ProductStep &st)
{
    const bool la = st.pa == kLower, ua = st.pa == kUpper, lb = st.pb == kLower, ub = st.pb == kUpper;
    if (la && lb) return kDiagLower;
    if (ua && ub) return kDiagUpper;
    if (la && ub) return kShellMin;
    if (ua && lb) return kShellMax;
    if (la) return kRowsDesc;
    if (ua) return kRowsAsc;
    if (lb) return kColsAsc;
    if (ub) return kColsDesc;
    return kRowMajor;
}

// A product with a diagonal operand scales the rows or columns of the other operand: it runs
// as an element-wise pass, not through the tiled kernel.
inline bool is_scaling(const ProductStep &st) { return st.pa == kDiagonal || st.pb == kDiagonal; }

// (X * Y) * Z runs as one launch of the skinny-pair kernel when the intermediate has at most
// 64 columns, everything is general and stored as read, there are enough 32-row blocks to fill
// the chip, and the second product is wide enough to be worth keeping the rows in registers.
constexpr int kPairMinRowBlocks = 192, kPairMinCols = 256;
inline bool fits_skinny_pair(const ProductStep &inner, const ProductStep &outer)
{
    const bool general = inner.pa == kGeneral && inner.pb == kGeneral && outer.pb == kGeneral;
    const bool as_read = !inner.ta && !inner.tb && !outer.tb;
    return general && as_read && inner.n <= 64 && inner.n >= 8 && (inner.m + 31) / 32 >= kPairMinRowBlocks &&
           outer.n >= kPairMinCols;
}

// Up to how many 128x128 tiles of the result a product runs on 64x64 tiles instead.
inline int small_tile_limit(int pa, int pb)
{
    const bool ta = pa == kLower || pa == kUpper, tb = pb == kLower || pb == kUpper;
    if (ta && tb) return pa == pb ? 1400 : 900;
    return ta || tb ? 448 : 192;
}

inline Launch choose_launch(const ProductStep &st)
{
    Launch L{};
    if (is_scaling(st)) {
        L.shape = kTile128; L.bm = L.bn = 128; L.split_k = 1;
        return L;
    }
    // 64x64 tiles when a side is at most 64, and when 128x128 tiles would be too few to keep the
    // 256 compute units busy.  Triangular operands make a tile count worth less (the tiles' k-ranges
    // run from one chunk to all of k) and a triangular result leaves only half of the tiles.
    // Limits measured on square products (64x64 tiles run at about 80 % of the peak when they
    // fill the chip): general n <= 1664, one triangular operand n <= 2688, L*U and U*L
    // n <= 3840, L*L and U*U n <= 4736.
    const int64_t t128 = ((st.m + 127) / 128) * ((st.n + 127) / 128);
    const bool small = st.m <= 64 || st.n <= 64 || t128 <= small_tile_limit(st.pa, st.pb);
    L.shape = small ? kTile64 : kTile128;
    L.bm = L.bn = small ? 64 : 128;
    L.tiles_m = (int)((st.m + L.bm - 1) / L.bm);
    L.tiles_n = (int)((st.n + L.bn - 1) / L.bn);
    L.order = tile_order(st);
    if (L.order == kDiagLower || L.order == kDiagUpper)
        L.num_tiles = (int)((int64_t)L.tiles_m * (L.tiles_m + 1) / 2);      // square, bm == bn
    else
        L.num_tiles = L.tiles_m * L.tiles_n;
    // Pair the longest tile with the shortest, the second longest with the second shortest,
    // ...: for the linear length profile of one triangular operand every workgroup then does
    // the same amount of work, and a pair's second tile rides the pipeline of the first instead of
    // starting a workgroup of its own.  Equal workgroups only pay when they fill the chip evenly:
    // with 265 pairs on 256 compute units nine units do twice the work of the others (45 % of the
    // peak measured, 69 % with single tiles), so tiles are paired only when the pairs are a
    // multiple of the compute units (up to the 4096 tiles of an 8192^3 product, the largest
    // tried: +1.3 to +1.6 % against single tiles).  Two triangular operands have many short
    // tiles that do not pair up to equal sums: never paired.
    const bool linear = L.order == kRowsDesc || L.order == kRowsAsc || L.order == kColsAsc || L.order == kColsDesc;
    L.paired = (linear && L.num_tiles >= 2 * kComputeUnits && L.num_tiles < 17 * kComputeUnits &&
                ((L.num_tiles + 1) / 2) % kComputeUnits == 0) ? 1 : 0;
    // Otherwise single tiles, longest first, which the dispatcher hands to whichever compute unit
    // has a free slot; only the start is fixed: workgroups b and b + 256 share a compute unit, so
    // the second 256 take their tiles in reverse (compute unit c starts with the c-th longest and
    // the c-th shortest of the first 512 tiles: equal sums for a linear profile).
    L.folded = (!L.paired && L.order != kRowMajor && L.num_tiles > kComputeUnits) ? 1 : 0;
    // A tall triangular operand against a narrow right-hand side (more than twice as many tile
    // rows as tile columns): the triangle is the bulk of the traffic, and with the plain order
    // every die streams all of it, once per tile column it holds.  Give each die 1/8 of the tile
    // rows instead (rows x and 15-x of every group of 16, which pair up to equal work): the
    // triangle is then fetched once, the narrow operand once per die.
    if (L.paired && (L.order == kRowsDesc || L.order == kRowsAsc) && L.tiles_m % (2 * kXcds) == 0 &&
        L.tiles_m > 2 * L.tiles_n && L.num_tiles % (2 * kXcds) == 0)
        L.paired = 2;
    // Tiles that share an operand panel hit in a die's L2 only while they are at the same k at about
    // the same time (the L2 merges misses in flight, but holds only some ten chunks of what a die's
    // workgroups stream).  The clipped k-ranges of a triangular operand all share one end (k = 0 for
    // L*G and G*U, k = K for U*G and G*L): tiles that start together walk away from that end; the
    // second, short tile of a pair starts when its long partner ends, that is the later the shorter
    // it is, and walks towards the shared end, which puts all second tiles at the same k again.  The
    // same holds when the pair is two workgroups on one compute unit: the older one takes most of
    // the matrix pipe, so the short tile runs mostly after the long one.
    const bool high_end = L.order == kRowsAsc || L.order == kColsAsc;
    L.k_walk = (high_end ? 1 : 0) | (((L.paired || L.folded) ? !high_end : high_end) ? 2 : 0);
    if (L.order != kRowsDesc && L.order != kRowsAsc && L.order != kColsAsc && L.order != kColsDesc) L.k_walk = 0;
    L.grid = L.paired ? (L.num_tiles + 1) / 2 : L.num_tiles;
    L.mirrored = (L.paired && L.grid <= kComputeUnits) ? 1 : 0;
    if (L.mirrored) L.grid *= 2;
    // Equal tiles (general * general) beyond what the chip holds at once, with a k long enough
    // to matter: launch only as many workgroups as are resident together and let each walk
    // every grid-th tile, so that the loads of its next tile overlap the MFMAs of this one.
    const int resident = kComputeUnits * (small ? 4 : 2);
    if (L.order == kRowMajor && L.num_tiles > resident && st.k >= 8 * (small ? kChunk64 : kChunk128)) L.grid = resident;
    // Split-K: a product with few output tiles and a long k leaves most compute units idle; cut
    // every tile's k-range into slices (one workgroup per tile and slice, partial sums to scratch,
    // summed by a second small kernel) until about three workgroups per compute unit
    // exist, keeping at least kMinChunksPerSlice chunks per slice of a full k-range.  Operands and
    // result may be triangular: a tile's clipped k-range is what is dealt out, the slices are
    // dense m x n buffers of which only the result's structure is written and summed.
    L.split_k = 1;
    L.scratch_bytes = 0;
    const int bk = small ? kChunk64 : kChunk128;
    const int chunks = (int)((st.k + bk - 1) / bk);
    if (L.num_tiles < kComputeUnits && chunks >= kMinChunksToSplit) {
        const int want = (kSplitTargetWorkgroups + L.num_tiles - 1) / L.num_tiles;
        const int split = std::min(want, chunks / kMinChunksPerSlice);
        if (split > 1) {
            L.split_k = split;
            L.scratch_bytes = (size_t)split * (size_t)st.m * (size_t)st.n * sizeof(float);
        }
    }
    return L;
}

// The last round of a general * general product on 128x128 tiles.  Its tiles are all equally long,
// and a compute unit multiplies as fast with one workgroup as with two, so the product takes
// ceil(tiles / 256) tile times: when the tile count is a little above a multiple of 256, the last few
// tiles run on a few compute units while the rest of the chip waits (576 tiles: 2.25 per unit,
// 72 % of the peak; 2304 tiles: 9 per unit, 96 %).  Such a product is cut into two sub-products
// along the rows of the result: the first tile rows, a whole number of tiles per unit, and the
// remaining tile rows, whose tiles are cut along k into as many slices as fill the chip once
// (their partial sums are added by the slice-sum kernel).  Both run in one launch.  Only when the
// idle part of the last round is worth at least 24 chunk times per compute unit (some 40 us) and
// the tail is small: the slices cost a second launch and traffic.
struct Tail {
    int tile_rows_main;    // 0: the product is not cut
    int split;             // k-slices of the tail's tiles
    size_t scratch_bytes;  // split * (rows of the tail) * n floats
};

inline Tail choose_tail(const ProductStep &st, const Launch &L)
{
    Tail t{0, 1, 0};
    const int resident = 2 * kComputeUnits;
    const int chunks = (int)((st.k + kChunk128 - 1) / kChunk128);
    if (L.shape != kTile128 || L.order != kRowMajor || L.split_k != 1 || L.num_tiles <= kComputeUnits || chunks < 32)
        return t;
    const int per_unit = L.num_tiles / kComputeUnits, rounds_up = (L.num_tiles + kComputeUnits - 1) / kComputeUnits;
    const int64_t idle_tiles = (int64_t)rounds_up * kComputeUnits - L.num_tiles;
    if (idle_tiles * chunks < (int64_t)24 * kComputeUnits) return t;      // the last round is full enough, or k short
    const int main_rows = (int)(((int64_t)per_unit * kComputeUnits) / L.tiles_n);
    if (main_rows < 1 || main_rows >= L.tiles_m) return t;
    const int tail_tiles = (L.tiles_m - main_rows) * L.tiles_n;
    if (tail_tiles > kComputeUnits * 5 / 8) return t;      // (measured: a tail of 182 tiles loses, one of 160 gains)
    const int split = std::min((resident + tail_tiles - 1) / tail_tiles, chunks / kMinChunksPerSlice);
    if (split < 2) return t;
    t.tile_rows_main = main_rows;
    t.split = split;
    t.scratch_bytes = (size_t)split * (size_t)(st.m - (int64_t)main_rows * 128) * (size_t)st.n * sizeof(float);
    return t;
}

}  // namespace mom
