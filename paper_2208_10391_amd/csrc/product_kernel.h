// Tiled f32 MFMA product kernel for gfx950 (MI355X): C = A * B where A, B and C each carry
// one of the properties general / lowerTri / upperTri (MOM paper, Sec. 2).  One kernel covers
// GEMM, TRMM from either side and triangular*triangular products: a property only
//   - clips the k-range of an output tile (tiles of zeros are never loaded or multiplied),
//   - masks the operand elements of the chunks that straddle a diagonal (the zero half of a
//     triangular operand is never trusted to hold zeros),
//   - removes the output tiles of the zero half of a triangular result and masks the stores
//     of its diagonal tiles (only the triangle is written).
// This is the non-rectangular iteration space that Sec. 5 of the paper names as future work.
//
// Data path: global -> registers (16-byte loads through buffer descriptors that end with the
// matrix, two chunks ahead) -> LDS (two stages, one barrier per chunk) -> MFMA operands (read one
// group of 8 k-values ahead).
// v_mfma_f32_32x32x2_f32 computes D = X * Y + D with lane l supplying X[i = l%32][k = l/32] and
// Y[k = l/32][j = l%32]; register v of lane l holds D[8*(v/4) + 4*(l/32) + v%4][l%32].  The kernel
// feeds it the transposed problem, X = B^T and Y = A^T, so that D = C^T: a lane then owns one row
// of the 32x32 block of C and four consecutive registers are four consecutive columns of it, which
// go out as one 16-byte store.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch_params.h"
#include "schedule.h"

namespace mom {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// Fourth word of an untyped buffer descriptor (32-bit data format).  A load through such a
// descriptor takes its address as descriptor base + scalar byte offset + one 32-bit vector byte
// offset: everything that is the same for the whole workgroup stays in scalar registers.
constexpr int kRawBufferFlags = 0x00020000;

// Is (i, j) inside the structure of property p?  (p is never Identity here; diagonal, the last
// case, reaches the batched and the element-wise kernels only.)
__device__ __forceinline__ bool in_structure(int p, int i, int j)
{
    return p == kGeneral ? true : (p == kLower ? j <= i : (p == kUpper ? j >= i : j == i));
}

__device__ __forceinline__ int isqrt_floor(int64_t x)
{
    int64_t r = (int64_t)sqrt((double)x);
    while (r * r > x) --r;
    while ((r + 1) * (r + 1) <= x) ++r;
    return (int)r;
}

// Position t in the longest-first tile order -> tile coordinates.
__device__ __forceinline__ void tile_coords(int order, int t, int tm, int tn, int &I, int &J)
{
    switch (order) {
    case kRowsDesc: I = tm - 1 - t / tn; J = t % tn; break;
    case kColsAsc:  J = t / tm; I = t % tm; break;
    case kColsDesc: J = tn - 1 - t / tm; I = t % tm; break;
    case kDiagLower:
    case kDiagUpper: {
        // diagonals d = tm-1, tm-2, ..., 0; diagonal d has tm-d tiles of length d+1
        const int s = (isqrt_floor(8 * (int64_t)t + 1) - 1) / 2;      // complete diagonals before t
        const int d = tm - 1 - s, pos = t - s * (s + 1) / 2;
        const int hi = d + pos, lo = pos;
        if (order == kDiagLower) { I = hi; J = lo; } else { I = lo; J = hi; }
        break;
    }
    case kShellMin:
    case kShellMax: {
        // shells of constant min(I,J) = s, largest s first; the shell has 2*(tm-s)-1 tiles
        const int q = isqrt_floor(t), side = q + 1, s = tm - side, pos = t - q * q;
        int i, j;
        if (pos < side) { i = s; j = s + pos; } else { i = s + (pos - side) + 1; j = s; }
        if (order == kShellMin) { I = i; J = j; } else { I = tm - 1 - i; J = tn - 1 - j; }
        break;
    }
    default: I = t / tn; J = t % tn; break;     // kRowMajor, kRowsAsc
    }
}

// TA / TB: the operand's buffer holds the TRANSPOSE of what the product needs (paper Table 1,
// Transpose): A is stored as the K x M matrix S with A[i][k] = S[k][i], B as the N x K matrix
// with B[k][j] = S[j][k].  Nothing is transposed in memory: a transposed A tile is simply
// fetched and staged the way a plain B tile is ([k][i], contiguous along i, read from LDS
// with one 4-byte read per k), a transposed B tile the way a plain A tile is ([j][k + pad],
// read with one 16-byte read per lane).
// WORDS: the instance also knows how to load an operand 4 bytes at a time (rows that are not
// 16-byte aligned, edges that a 16-byte group could straddle); the instance without it keeps
// that code out of the way of the products whose operands never need it.
template <int BM_, int BN_, int BK_, int WM_, int WN_, int MIN_BLOCKS_, bool TA_ = false, bool TB_ = false, bool WORDS_ = false>
struct TileConfig {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr int MIN_BLOCKS = MIN_BLOCKS_;
    static constexpr bool TA = TA_, TB = TB_, WORDS = WORDS_;
    static constexpr int NT = WM * WN * 64;           // threads per workgroup
    static constexpr int WTM = BM / WM, WTN = BN / WN;   // tile of one wavefront
    static constexpr int FM = WTM / 32, FN = WTN / 32;   // 32x32 MFMA blocks per wavefront
    // A wavefront's blocks are spread over the tile, not adjacent: wavefront (wr, wc) owns the
    // row blocks wr, wr + WM, ... and the column blocks wc, wc + WN, ... (measured 1 % faster
    // than adjacent blocks on every large workload; the LDS access pattern is the same).
    static constexpr int RSTEP = WM * 32, CSTEP = WN * 32;   // rows / columns between a wavefront's blocks
    static constexpr int LDA = TA ? BM : BK + 4;      // LDS row stride of the A tile: [BM][BK + 4]
                                                      // (16-byte row reads hit distinct banks), or
                                                      // [BK][BM] when A is stored transposed
    static constexpr int LDB = TB ? BK + 4 : BN;      // LDS row stride of the B tile: [BK][BN], or
                                                      // [BN][BK + 4] when B is stored transposed
    static constexpr int A_STAGE = (TA ? BK : BM) * LDA, B_STAGE = (TB ? BN : BK) * LDB;
    static constexpr int LDS_BYTES = 2 * (A_STAGE + B_STAGE) * 4;
    static constexpr int A_F4 = BM * BK / 4 / NT;     // 16-byte loads per thread and chunk
    static constexpr int B_F4 = BK * BN / 4 / NT;
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % 8 == 0, "tile shape");
    static_assert(BM % BK == 0 && BN % BK == 0, "diagonals must fall on chunk boundaries");
    static_assert((BM * BK / 4) % NT == 0 && (BK * BN / 4) % NT == 0, "load decomposition");

    // Where the idx-th group of four consecutive stored elements of a chunk sits: row / column
    // of the product (i or j), k inside the chunk, and which of the two runs along the four.
    // A plain: idx -> (i = idx / (BK/4), k = 4 * (idx % (BK/4)) .. +3)
    // A transposed: idx -> (k = idx / (BM/4), i = 4 * (idx % (BM/4)) .. +3)
    static __device__ __forceinline__ int a_row(int idx) { return TA ? (idx % (BM / 4)) * 4 : idx / (BK / 4); }
    static __device__ __forceinline__ int a_k(int idx) { return TA ? idx / (BM / 4) : (idx % (BK / 4)) * 4; }
    static __device__ __forceinline__ int b_col(int idx) { return TB ? idx / (BK / 4) : (idx % (BN / 4)) * 4; }
    static __device__ __forceinline__ int b_k(int idx) { return TB ? (idx % (BK / 4)) * 4 : idx / (BN / 4); }
};

// Element-wise loads of one k-chunk for row strides too long for 32-bit offsets (and, in the
// instance without the 4-byte descriptor loads, for whatever else cannot be loaded 16 bytes at a
// time): bounds-checked and predicated on the structure, so nothing outside the matrix or the
// triangle is touched; 64-bit addresses.
template <class T>
__device__ __forceinline__ void load_a_checked(const ProductParams &p, int r0, int kc, int tid, f32x4 (&ra)[T::A_F4])
{
#pragma unroll
    for (int q = 0; q < T::A_F4; ++q) {
        const int idx = tid + q * T::NT;
        const int gi = r0 + T::a_row(idx), gk = kc + T::a_k(idx);
        const float *src = T::TA ? p.A + (int64_t)gk * p.lda + gi : p.A + (int64_t)gi * p.lda + gk;
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = T::TA ? gi + e : gi, k = T::TA ? gk : gk + e;
            const bool ok = i < p.M && k < p.K && in_structure(p.pa, i, k);
            v[e] = ok ? src[e] : 0.0f;
        }
        ra[q] = v;
    }
}

template <class T>
__device__ __forceinline__ void load_b_checked(const ProductParams &p, int c0, int kc, int tid, f32x4 (&rb)[T::B_F4])
{
#pragma unroll
    for (int q = 0; q < T::B_F4; ++q) {
        const int idx = tid + q * T::NT;
        const int gk = kc + T::b_k(idx), gj = c0 + T::b_col(idx);
        const float *src = T::TB ? p.B + (int64_t)gj * p.ldb + gk : p.B + (int64_t)gk * p.ldb + gj;
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = T::TB ? gk + e : gk, j = T::TB ? gj : gj + e;
            const bool ok = k < p.K && j < p.N && in_structure(p.pb, k, j);
            v[e] = ok ? src[e] : 0.0f;
        }
        rb[q] = v;
    }
}

template <class T>
__device__ __forceinline__ void stage_to_lds(float *As, float *Bs, int tid,
                                             const f32x4 (&ra)[T::A_F4], const f32x4 (&rb)[T::B_F4])
{
#pragma unroll
    for (int q = 0; q < T::A_F4; ++q) {
        const int idx = tid + q * T::NT;
        *reinterpret_cast<f32x4 *>(As + (T::TA ? T::a_k(idx) * T::LDA + T::a_row(idx)
                                                 : T::a_row(idx) * T::LDA + T::a_k(idx))) = ra[q];
    }
#pragma unroll
    for (int q = 0; q < T::B_F4; ++q) {
        const int idx = tid + q * T::NT;
        *reinterpret_cast<f32x4 *>(Bs + (T::TB ? T::b_col(idx) * T::LDB + T::b_k(idx)
                                                 : T::b_k(idx) * T::LDB + T::b_col(idx))) = rb[q];
    }
}

// MFMA operands of one group of 8 k-values: lane (l32, half) takes A[row l32][k = 4*half + e]
// for e = 0..3 with one 16-byte LDS read per 32-row block, and B[k = 4*half + e][col l32].
// a_lane / b_lane are the lane's own offsets inside a stage: (wr0 + l32) * LDA + 4 * half and
// 4 * half * LDB + wc0 + l32; an operand stored transposed swaps the two patterns.
template <class T>
struct Fragments {
    f32x4 a[T::FM];
    float b[T::FN][4];
};

template <class T>
__device__ __forceinline__ void read_fragments(const float *As, const float *Bs, int a_lane, int b_lane, int kg,
                                               Fragments<T> &f)
{
#pragma unroll
    for (int bi = 0; bi < T::FM; ++bi) {
        if (T::TA) {
#pragma unroll
            for (int e = 0; e < 4; ++e) f.a[bi][e] = As[a_lane + (kg * 8 + e) * T::LDA + bi * T::RSTEP];
        } else {
            f.a[bi] = *reinterpret_cast<const f32x4 *>(As + a_lane + bi * T::RSTEP * T::LDA + kg * 8);
        }
    }
#pragma unroll
    for (int bj = 0; bj < T::FN; ++bj) {
        if (T::TB) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(Bs + b_lane + bj * T::CSTEP * T::LDB + kg * 8);
#pragma unroll
            for (int e = 0; e < 4; ++e) f.b[bj][e] = v[e];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) f.b[bj][e] = Bs[b_lane + (kg * 8 + e) * T::LDB + bj * T::CSTEP];
        }
    }
}

// The 4 * FM * FN MFMAs of one group of 8 k-values: step e multiplies k = 4*half + e (the
// order of summation over k is free).  The B operand goes first: the accumulators hold the
// transposed block (see the head of this file).
template <class T>
__device__ __forceinline__ void mfma_group(const Fragments<T> &f, f32x16 (&acc)[T::FM][T::FN])
{
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int bi = 0; bi < T::FM; ++bi)
#pragma unroll
            for (int bj = 0; bj < T::FN; ++bj)
                acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.b[bj][e], f.a[bi][e], acc[bi][bj], 0, 0, 0);
}

// What one output tile needs: where it sits, its k-range in chunks, and which chunks are
// interior for both operands.
struct TileWork {
    int r0, c0;            // first row / column of the tile
    int k0, kstep;         // chunk j starts at k = k0 + j * kstep (kstep = BK, or -BK for a range walked downwards)
    int nchunks;           // chunks of BK to multiply (0: the tile is all zeros)
    int f_lo, f_hi;        // chunks [f_lo, f_hi) need neither masking nor bounds checks
    int a_load, b_load;    // how the operand's part of the tile is loaded: 16 bytes at a time; 4 bytes at a time
                           // (rows not 16-byte aligned, or the tile pokes over the matrix edge and a 16-byte
                           // group could straddle the end of a row); or 0: element-wise with 64-bit
                           // addresses (a row stride out of reach of 32-bit offsets)
};

template <class T>
__device__ __forceinline__ TileWork tile_work(const ProductParams &p, int t, int slice, bool down)
{
    int I, J;
    tile_coords(p.order, t, p.tiles_m, p.tiles_n, I, J);
    TileWork w;
    w.r0 = I * T::BM;
    w.c0 = J * T::BN;
    const int r1 = min(w.r0 + T::BM, p.M), c1 = min(w.c0 + T::BN, p.N);
    // k-range: the k for which some A[i][k] and some B[k][j] are both inside their
    // structures, widened to whole chunks
    int klo = 0, khi = p.K;
    if (p.pa == kLower) khi = min(khi, r1);          // A[i][k] = 0 for k > i
    if (p.pa == kUpper) klo = max(klo, w.r0);        // A[i][k] = 0 for k < i
    if (p.pb == kLower) klo = max(klo, w.c0);        // B[k][j] = 0 for k < j
    if (p.pb == kUpper) khi = min(khi, c1);          // B[k][j] = 0 for k > j
    klo = (klo / T::BK) * T::BK;
    int nchunks = khi > klo ? (khi - klo + T::BK - 1) / T::BK : 0;
    if (p.split_k > 1) {                             // this slice's share of the chunks
        const int per = (nchunks + p.split_k - 1) / p.split_k;
        const int first = min(slice * per, nchunks);
        nchunks = min(per, nchunks - first);
        klo += first * T::BK;
    }
    w.nchunks = nchunks;
    w.a_load = p.a_vec && (w.r0 + T::BM <= p.M || p.a_tail) ? 16 : (T::WORDS && p.a_word ? 4 : 0);
    w.b_load = p.b_vec && (w.c0 + T::BN <= p.N || p.b_tail) ? 16 : (T::WORDS && p.b_word ? 4 : 0);
    // What a property or an edge makes special is always a run of chunks at the head and a
    // run at the tail of the k-range; the chunks in between are interior.
    w.f_lo = w.f_hi = 0;
    if (w.a_load != 0 && w.b_load != 0) {
        int k_from = klo, k_to = (p.K / T::BK) * T::BK;
        if (p.pa == kUpper) k_from = max(k_from, w.r0 + T::BM);
        if (p.pb == kLower) k_from = max(k_from, w.c0 + T::BN);
        if (p.pa == kLower) k_to = min(k_to, w.r0);
        if (p.pb == kUpper) k_to = min(k_to, w.c0);
        w.f_lo = min((k_from - klo) / T::BK, nchunks);
        w.f_hi = max(min((k_to - klo) / T::BK, nchunks), w.f_lo);
    }
    w.k0 = klo;
    w.kstep = T::BK;
    if (down) {                                      // the same chunks, last one first
        const int lo = nchunks - w.f_hi, hi = nchunks - w.f_lo;
        w.f_lo = lo; w.f_hi = hi;
        w.k0 = klo + (nchunks - 1) * T::BK;
        w.kstep = -T::BK;
    }
    return w;
}

// How the operands of chunk j of a tile get from HBM to LDS (uniform over the workgroup):
//   kPlain  16-byte loads, staged as they are
//   kDiag   loads through descriptors, 16 bytes at a time or, where rows are not 16-byte aligned or
//           a group could straddle a matrix edge, 4 bytes at a time; the elements outside the
//           structure or beyond a ragged end of k are zeroed when the registers are staged (one
//           chunk after the load, when the data has long arrived)
//   kEdge   a row stride beyond the reach of 32-bit offsets: element-wise loads with 64-bit
//           addresses, bounds-checked and predicated on the structure; staged as they are
// Descriptor loads go through buffer descriptors that end with the matrix: what lies past its last
// element (rows below the last one, the tail of the last row) reads as zero and is never
// touched.  What a tile reads beyond an edge INSIDE the buffer (the next row's head in place of
// columns past the edge) only reaches rows or columns of the tile that are not stored, except
// along k, which the mask covers.
enum ChunkKind : int { kPlain = 0, kDiag = 1, kEdge = 2 };

template <class T>
__device__ __forceinline__ int chunk_kind(const ProductParams &p, const TileWork &w, int j)
{
    if (j >= w.f_lo && j < w.f_hi) return kPlain;
    // through descriptors (16 or 4 bytes at a time), masked at staging where a mask is due: next to a
    // diagonal and at a ragged end of k
    return (w.a_load == 0 || w.b_load == 0) ? kEdge : kDiag;
}

// How the rectangle rows [r_lo, r_hi] x columns [c_lo, c_hi] of a triangular matrix lies to its
// structure: 1 wholly inside, 0 wholly outside, 2 across the diagonal.
__device__ __forceinline__ int structure_class(int prop, int r_lo, int r_hi, int c_lo, int c_hi)
{
    if (prop == kLower) return c_hi <= r_lo ? 1 : (c_lo > r_hi ? 0 : 2);       // kept: column <= row
    if (prop == kUpper) return c_lo >= r_hi ? 1 : (c_hi < r_lo ? 0 : 2);       // kept: column >= row
    return 1;
}

// Zero what lies outside the structures in the registers of the chunk that starts at k = kc.
// The q-th 16-byte group of all threads together covers a rectangle of the operand (32 rows of
// an A tile by the chunk's k-range when A is stored as it is read, a few k-values by all rows
// when it is stored transposed; B likewise): where that rectangle lies wholly inside or outside
// the structure, which the whole workgroup knows at once, no element is compared.
template <class T>
__device__ __forceinline__ void mask_registers(const ProductParams &p, int r0, int c0, int kc, int tid,
                                               f32x4 (&ra)[T::A_F4], f32x4 (&rb)[T::B_F4])
{
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    if (kc + T::BK > p.K) {      // ragged end of k, where k runs along the rows of the buffer
        if (!T::TA) {
#pragma unroll
            for (int q = 0; q < T::A_F4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (kc + T::a_k(tid + q * T::NT) + e >= p.K) ra[q][e] = 0.0f;
        }
        if (T::TB) {
#pragma unroll
            for (int q = 0; q < T::B_F4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (kc + T::b_k(tid + q * T::NT) + e >= p.K) rb[q][e] = 0.0f;
        }
    }
    if (p.pa != kGeneral) {
        constexpr int ROWS = T::TA ? T::BM : T::NT / (T::BK / 4);      // rows and k-values one group index spans
        constexpr int KS = T::TA ? T::NT / (T::BM / 4) : T::BK;
#pragma unroll
        for (int q = 0; q < T::A_F4; ++q) {
            const int i_lo = r0 + (T::TA ? 0 : q * ROWS), k_lo = kc + (T::TA ? q * KS : 0);
            // (stored transposed, a group spans all rows of the tile: next to a diagonal always across)
            const int cls = T::TA ? 2 : structure_class(p.pa, i_lo, i_lo + ROWS - 1, k_lo, k_lo + KS - 1);
            if (cls == 0) ra[q] = zero;
            if (cls != 2) continue;
            const int idx = tid + q * T::NT;
            const int gi = r0 + T::a_row(idx), gk = kc + T::a_k(idx);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                ra[q][e] = in_structure(p.pa, T::TA ? gi + e : gi, T::TA ? gk : gk + e) ? ra[q][e] : 0.0f;
        }
    }
    if (p.pb != kGeneral) {
        constexpr int COLS = T::TB ? T::NT / (T::BK / 4) : T::BN;
        constexpr int KS = T::TB ? T::BK : T::NT / (T::BN / 4);
#pragma unroll
        for (int q = 0; q < T::B_F4; ++q) {
            const int j_lo = c0 + (T::TB ? q * COLS : 0), k_lo = kc + (T::TB ? 0 : q * KS);
            const int cls = T::TB ? structure_class(p.pb, k_lo, k_lo + KS - 1, j_lo, j_lo + COLS - 1) : 2;
            if (cls == 0) rb[q] = zero;
            if (cls != 2) continue;
            const int idx = tid + q * T::NT;
            const int gk = kc + T::b_k(idx), gj = c0 + T::b_col(idx);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                rb[q][e] = in_structure(p.pb, T::TB ? gk + e : gk, T::TB ? gj : gj + e) ? rb[q][e] : 0.0f;
        }
    }
}

// The MFMAs of one group of 8 k-values for a chunk next to a diagonal: 32x32 blocks of a triangular operand that lie wholly
// outside its structure are not multiplied at all.  Bit bi of `skip` drops row block bi of the
// wavefront, bit 8 + bj column block bj (the same for the whole wavefront: scalar branches).
template <class T>
__device__ __forceinline__ void mfma_group_some(const Fragments<T> &f, f32x16 (&acc)[T::FM][T::FN], int skip)
{
    // (one plain condition per block, none nested and none with an else: each block's accumulator is
    // updated in place; with anything richer the compiler copies accumulators at the joins)
#pragma unroll
    for (int bi = 0; bi < T::FM; ++bi)
#pragma unroll
        for (int bj = 0; bj < T::FN; ++bj) {
            if (skip & ((1 << bi) | (256 << bj))) continue;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.b[bj][e], f.a[bi][e], acc[bi][bj], 0, 0, 0);
        }
}

// Which of a wavefront's blocks chunk [kc, kc + BK) of a tile cannot touch: the skip mask of
// mfma_group_some.  wr0 / wc0: first row / column of the wavefront inside the tile.
template <class T>
__device__ __forceinline__ int blocks_outside(const ProductParams &p, int r0, int c0, int kc, int wr0, int wc0)
{
    int skip = 0;
#pragma unroll
    for (int bi = 0; bi < T::FM; ++bi) {
        const int r_lo = r0 + wr0 + bi * T::RSTEP;
        if (structure_class(p.pa, r_lo, r_lo + 31, kc, kc + T::BK - 1) == 0) skip |= 1 << bi;
    }
#pragma unroll
    for (int bj = 0; bj < T::FN; ++bj) {
        const int c_lo = c0 + wc0 + bj * T::CSTEP;
        if (structure_class(p.pb, kc, kc + T::BK - 1, c_lo, c_lo + 31) == 0) skip |= 256 << bj;
    }
    return skip;
}

// Scheduling groups (masks of __builtin_amdgcn_sched_group_barrier).
constexpr int kSchedMfma = 0x008, kSchedVmemRead = 0x020, kSchedLdsRead = 0x100, kSchedLdsWrite = 0x200;

// Per-thread state of the software pipeline of one workgroup.  The pipeline is flat over the
// (tile, chunk) pairs of the workgroup: the fetch side runs two chunks ahead of the MFMAs and
// simply carries on into the next tile, so a tile's first chunks arrive while the previous
// tile is still being multiplied and stored.
template <class T>
struct Pipeline {
    f32x4 ra[T::A_F4], rb[T::B_F4];     // the chunk on its way from HBM to LDS
    // Where the next chunk to load starts (its first element: the same for the whole workgroup,
    // scalar registers) and this thread's byte offsets from there (the same for every chunk).
    const float *a_chunk, *b_chunk;
    const float *a_end, *b_end;         // one past the last element of A / B: where their descriptors end
    int a_step, b_step;                 // elements from one chunk of the fetch tile to the next
    int a_off[T::A_F4], b_off[T::B_F4];
    Fragments<T> f0, f1;                // MFMA operands: current group, next group
    // fetch cursor: the next chunk to load is chunk fj of tile fw (the f_seq-th of the workgroup)
    TileWork fw;
    int f_seq, fj;
    bool f_live;                        // false once every chunk of the workgroup has been loaded
    // the chunk that sits in ra / rb
    bool in_regs;
    int reg_kind, reg_r0, reg_c0, reg_kc;
};

// Whether the i-th tile of a workgroup walks its k-range downwards.
__device__ __forceinline__ bool walks_down(const ProductParams &p, int block, int i)
{
    const bool second = p.mirrored ? block >= (p.num_tiles + 1) / 2
                                   : (p.folded ? block >= kComputeUnits && block < 2 * kComputeUnits : i > 0);
    return (p.k_walk >> (second ? 1 : 0)) & 1;
}

// The i-th tile of a workgroup (-1: none): tile `block` and its partner from the other end of
// the longest-first order when tiles are paired, else every grid-th tile.
__device__ __forceinline__ int tile_at(const ProductParams &p, int block, int i)
{
    if (p.mirrored) {            // the pair's two tiles belong to workgroups block and block + pairs
        if (i > 0) return -1;
        const int pairs = (p.num_tiles + 1) / 2;
        i = block / pairs;
        block %= pairs;
    }
    if (p.paired == 2) {
        // die x = block % 8 owns tile rows 16j + x and 16j + 15 - x (counted from the short end);
        // in descending length these are D[2i] = 16(nb-1-i) + 15 - x, D[2i+1] = 16(nb-1-i) + x, and
        // pair q = (D[q], D[2nb-1-q]) always adds up to 16(nb-1) + 15: equal work everywhere
        if (i > 1) return -1;
        const int x = block % kXcds, s = block / kXcds, J = s % p.tiles_n, q = s / p.tiles_n;
        const int nb = p.tiles_m / (2 * kXcds), pos = i == 0 ? q : 2 * nb - 1 - q;
        const int len = 16 * (nb - 1 - pos / 2) + ((pos & 1) ? x : 15 - x);      // 0 = shortest row
        // position of that row in the longest-first order of tile_coords
        return (p.tiles_m - 1 - len) * p.tiles_n + J;
    }
    if (p.paired) {
        const int partner = p.num_tiles - 1 - block;
        return i == 0 ? block : (i == 1 && partner > block ? partner : -1);
    }
    if (p.folded) {              // one tile each; the second 256 workgroups in reverse
        if (i > 0) return -1;
        const int hi = min(p.num_tiles, 2 * kComputeUnits);
        return block >= kComputeUnits && block < hi ? hi - 1 - (block - kComputeUnits) : block;
    }
    const int64_t t = block + (int64_t)i * p.grid;
    return t < p.num_tiles ? (int)t : -1;
}

template <class T>
__device__ __forceinline__ void next_fetch_tile(const ProductParams &p, int block, int slice, int tid, Pipeline<T> &pl)
{
    for (;;) {
        const int t = tile_at(p, block, ++pl.f_seq);
        if (t < 0) { pl.f_live = false; return; }
        pl.fw = tile_work<T>(p, t, slice, walks_down(p, block, pl.f_seq));
        if (pl.fw.nchunks > 0) break;
    }
    pl.fj = 0;
    pl.a_chunk = T::TA ? p.A + (int64_t)pl.fw.k0 * p.lda + pl.fw.r0 : p.A + (int64_t)pl.fw.r0 * p.lda + pl.fw.k0;
    pl.b_chunk = T::TB ? p.B + (int64_t)pl.fw.c0 * p.ldb + pl.fw.k0 : p.B + (int64_t)pl.fw.k0 * p.ldb + pl.fw.c0;
    pl.a_step = T::TA ? pl.fw.kstep * (int)p.lda : pl.fw.kstep;      // (row strides of 16-byte-loadable operands are below 2^22)
    pl.b_step = T::TB ? pl.fw.kstep : pl.fw.kstep * (int)p.ldb;
}

// The 16-byte loads of one plain (or diagonal) chunk: through descriptors whose base is the
// chunk's first element, then on to the next chunk with scalar arithmetic only.
template <class T>
__device__ __forceinline__ void load_chunk_vectors(const ProductParams &p, Pipeline<T> &pl)
{
    // (bytes from the chunk's first element to the end of the matrix; a thread's offsets stay below 2^31)
    const uint64_t a_left = (uint64_t)(pl.a_end - pl.a_chunk) * 4, b_left = (uint64_t)(pl.b_end - pl.b_chunk) * 4;
    // (clamped to 2^31 - 1 in 32-bit pieces: there is no scalar 64-bit ordering compare)
    const uint32_t a_lo = (uint32_t)a_left, b_lo = (uint32_t)b_left;
    const uint32_t a_over = (uint32_t)(a_left >> 32) | (a_lo >> 31), b_over = (uint32_t)(b_left >> 32) | (b_lo >> 31);
    const int a_bytes = a_over != 0 ? 0x7fffffff : (int)a_lo, b_bytes = b_over != 0 ? 0x7fffffff : (int)b_lo;
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(pl.a_chunk), 0, a_bytes, kRawBufferFlags);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(pl.b_chunk), 0, b_bytes, kRawBufferFlags);
#pragma unroll
    for (int q = 0; q < T::A_F4; ++q) pl.ra[q] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(ra, pl.a_off[q], 0, 0));
#pragma unroll
    for (int q = 0; q < T::B_F4; ++q) pl.rb[q] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, pl.b_off[q], 0, 0));
}

// The same through descriptors for a chunk of which an operand has to be loaded 4 bytes at a time.
template <class T>
__device__ __forceinline__ void load_chunk_words(const ProductParams &p, Pipeline<T> &pl, bool a_wide, bool b_wide)
{
    const uint64_t a_left = (uint64_t)(pl.a_end - pl.a_chunk) * 4, b_left = (uint64_t)(pl.b_end - pl.b_chunk) * 4;
    const uint32_t a_lo = (uint32_t)a_left, b_lo = (uint32_t)b_left;
    const uint32_t a_over = (uint32_t)(a_left >> 32) | (a_lo >> 31), b_over = (uint32_t)(b_left >> 32) | (b_lo >> 31);
    const int a_bytes = a_over != 0 ? 0x7fffffff : (int)a_lo, b_bytes = b_over != 0 ? 0x7fffffff : (int)b_lo;
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(pl.a_chunk), 0, a_bytes, kRawBufferFlags);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(pl.b_chunk), 0, b_bytes, kRawBufferFlags);
#pragma unroll
    for (int q = 0; q < T::A_F4; ++q) {
        if (a_wide) {
            pl.ra[q] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(ra, pl.a_off[q], 0, 0));
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)      // (the next element along the rows of the buffer, or the next row of it)
                pl.ra[q][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ra, pl.a_off[q] + 4 * e, 0, 0));
        }
    }
#pragma unroll
    for (int q = 0; q < T::B_F4; ++q) {
        if (b_wide) {
            pl.rb[q] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, pl.b_off[q], 0, 0));
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                pl.rb[q][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, pl.b_off[q] + 4 * e, 0, 0));
        }
    }
}

// Loads of a chunk that needs no element-wise path: 16 bytes at a time, or, in the instance that
// knows how, 4 bytes at a time for the operands that need it.
template <class T>
__device__ __forceinline__ void load_chunk(const ProductParams &p, Pipeline<T> &pl)
{
    if (!T::WORDS || (pl.fw.a_load == 16 && pl.fw.b_load == 16))
        load_chunk_vectors<T>(p, pl);
    else
        load_chunk_words<T>(p, pl, pl.fw.a_load == 16, pl.fw.b_load == 16);
}

template <class T>
__device__ __forceinline__ void advance_chunk(const ProductParams &p, Pipeline<T> &pl)
{
    pl.a_chunk += pl.a_step;      // one chunk further along k
    pl.b_chunk += pl.b_step;
}

// Next chunk of the flat sequence: HBM -> registers.
template <class T>
__device__ __forceinline__ void fetch_chunk(const ProductParams &p, int block, int slice, int tid, Pipeline<T> &pl)
{
    pl.in_regs = pl.f_live;
    if (!pl.f_live) return;
    const int kind = chunk_kind<T>(p, pl.fw, pl.fj), kc = pl.fw.k0 + pl.fj * pl.fw.kstep;
    if (kind == kEdge) {
        load_a_checked<T>(p, pl.fw.r0, kc, tid, pl.ra);
        load_b_checked<T>(p, pl.fw.c0, kc, tid, pl.rb);
    } else {
        load_chunk<T>(p, pl);
    }
    advance_chunk<T>(p, pl);
    pl.reg_kind = kind; pl.reg_r0 = pl.fw.r0; pl.reg_c0 = pl.fw.c0; pl.reg_kc = kc;
    if (++pl.fj == pl.fw.nchunks) next_fetch_tile<T>(p, block, slice, tid, pl);
}

// One k-chunk: the MFMAs of flat chunk g out of LDS stage s while chunk g+1 moves from the
// registers to the other stage and the loads of chunk g+2 are issued.  On entry pl.f0 holds
// the operands of the chunk's first group; on exit those of chunk g+1's first group.  The
// workgroup barrier sits before the last group's MFMAs: by then every read of stage s has
// returned and the other stage is complete, so the first operands of chunk g+1 are read under
// the last MFMAs.
// With HOT the chunk in the registers and the one to load are both plain and s is the
// compile-time S: the body is a single basic block whose instruction mix is laid out by
// scheduling groups, LDS writes and global loads one per MFMA in the first group, LDS reads
// spread over the MFMAs of every group.  Without HOT the body decides as it goes: mask
// (kDiag), element-wise loads (kEdge), a new fetch tile, the end of the workgroup's chunks.
template <class T, bool HOT, int S>
__device__ __forceinline__ void chunk_step(float *smem, const ProductParams &p, int block, int slice, int s_, int tid,
                                           int a_lane, int b_lane, Pipeline<T> &pl, f32x16 (&acc)[T::FM][T::FN], int skip = 0)
{
    constexpr int NKG = T::BK / 8;
    static_assert(NKG % 2 == 0, "the operand double buffer returns to f0 after an even number of groups");
    constexpr int NMFMA = 4 * T::FM * T::FN, NMOVE = T::A_F4 + T::B_F4;
    // LDS read instructions per k-group: one 16-byte read per block of an operand laid out
    // [row][k], two paired 4-byte reads per block of one laid out [k][row]
    constexpr int NREAD = (T::TA ? 2 : 1) * T::FM + (T::TB ? 1 : 2) * T::FN;
    const int s = HOT ? S : s_;
    const float *As = smem + s * T::A_STAGE, *Bs = smem + 2 * T::A_STAGE + s * T::B_STAGE;
    float *An = smem + (s ^ 1) * T::A_STAGE, *Bn = smem + 2 * T::A_STAGE + (s ^ 1) * T::B_STAGE;

    // The chunk on its way to LDS is staged, and the next loads are issued, in the group before
    // the barrier rather than in the first one: the stores of a tile that has just ended (and
    // that an in-order memory counter makes the staging wait for) then have the first groups'
    // MFMAs to drain under.
    constexpr int MOVE = NKG >= 2 ? NKG - 2 : 0;
    bool staged = HOT;
#pragma unroll
    for (int kg = 0; kg < NKG; ++kg) {
        Fragments<T> &now = (kg & 1) ? pl.f1 : pl.f0;
        Fragments<T> &next = (kg & 1) ? pl.f0 : pl.f1;
        if (kg + 1 < NKG) {
            read_fragments<T>(As, Bs, a_lane, b_lane, kg + 1, next);
        } else {
            __syncthreads();
            if (staged) read_fragments<T>(An, Bn, a_lane, b_lane, 0, next);
        }
        if (kg == MOVE) {
            if (HOT) {
                stage_to_lds<T>(An, Bn, tid, pl.ra, pl.rb);
                load_chunk<T>(p, pl);
                advance_chunk<T>(p, pl);
            } else {
                staged = pl.in_regs;
                if (pl.in_regs) {
                    if (pl.reg_kind == kDiag) mask_registers<T>(p, pl.reg_r0, pl.reg_c0, pl.reg_kc, tid, pl.ra, pl.rb);
                    stage_to_lds<T>(An, Bn, tid, pl.ra, pl.rb);
                }
                fetch_chunk<T>(p, block, slice, tid, pl);
            }
        }
        if (HOT) mfma_group<T>(now, acc); else mfma_group_some<T>(now, acc, skip);
        if (!HOT || T::WORDS) {
            // the general body, and the steady state of the instance with 4-byte loads (whose load count
            // is only known at run time), are left to the compiler's own scheduling
        } else if (kg == MOVE) {
            __builtin_amdgcn_sched_group_barrier(kSchedLdsRead, NREAD, 0);
#pragma unroll
            for (int i = 0; i < NMOVE; ++i) {
                __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
                __builtin_amdgcn_sched_group_barrier(kSchedLdsWrite, 1, 0);
            }
#pragma unroll
            for (int i = 0; i < NMOVE; ++i) {
                __builtin_amdgcn_sched_group_barrier(kSchedMfma, 1, 0);
                __builtin_amdgcn_sched_group_barrier(kSchedVmemRead, 1, 0);
            }
        } else {
            constexpr int PER = NMFMA / NREAD > 0 ? NMFMA / NREAD : 1;
#pragma unroll
            for (int i = 0; i < NREAD; ++i) {
                __builtin_amdgcn_sched_group_barrier(kSchedLdsRead, 1, 0);
                __builtin_amdgcn_sched_group_barrier(kSchedMfma, PER, 0);
            }
            if (NMFMA > PER * NREAD) __builtin_amdgcn_sched_group_barrier(kSchedMfma, NMFMA - PER * NREAD, 0);
        }
    }
}

template <class T>
__global__ __launch_bounds__(T::NT, T::MIN_BLOCKS) void product_kernel(const ProductBatch batch)
{
    int which = 0;
    while (which + 1 < batch.count && (int)blockIdx.x >= batch.block_end[which]) ++which;
    const ProductParams &p = batch.prob[which];
    const int local = (int)blockIdx.x - (which ? batch.block_end[which - 1] : 0);
    const int slice = local / p.grid, block = local % p.grid;

    extern __shared__ __align__(16) float smem[];     // A stages 0 and 1, then B stages 0 and 1

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wr0 = (wave / T::WN) * 32, wc0 = (wave % T::WN) * 32;     // first row / column block of this wavefront
    const int a_lane = T::TA ? 4 * half * T::LDA + wr0 + l32 : (wr0 + l32) * T::LDA + 4 * half;
    const int b_lane = T::TB ? (wc0 + l32) * T::LDB + 4 * half : 4 * half * T::LDB + wc0 + l32;

    // prologue of the whole workgroup: flat chunk 0 into stage 0, flat chunk 1 into the registers
    Pipeline<T> pl;
#pragma unroll
    for (int q = 0; q < T::A_F4; ++q) {
        const int idx = tid + q * T::NT;
        pl.a_off[q] = (T::TA ? T::a_k(idx) * (int)p.lda + T::a_row(idx) : T::a_row(idx) * (int)p.lda + T::a_k(idx)) * 4;
    }
#pragma unroll
    for (int q = 0; q < T::B_F4; ++q) {
        const int idx = tid + q * T::NT;
        pl.b_off[q] = (T::TB ? T::b_col(idx) * (int)p.ldb + T::b_k(idx) : T::b_k(idx) * (int)p.ldb + T::b_col(idx)) * 4;
    }
    pl.a_end = T::TA ? p.A + (int64_t)(p.K - 1) * p.lda + p.M : p.A + (int64_t)(p.M - 1) * p.lda + p.K;
    pl.b_end = T::TB ? p.B + (int64_t)(p.N - 1) * p.ldb + p.K : p.B + (int64_t)(p.K - 1) * p.ldb + p.N;
    pl.f_seq = -1;
    pl.f_live = true;
    next_fetch_tile<T>(p, block, slice, tid, pl);
    fetch_chunk<T>(p, block, slice, tid, pl);
    if (pl.in_regs) {
        if (pl.reg_kind == kDiag) mask_registers<T>(p, pl.reg_r0, pl.reg_c0, pl.reg_kc, tid, pl.ra, pl.rb);
        stage_to_lds<T>(smem, smem + 2 * T::A_STAGE, tid, pl.ra, pl.rb);
        fetch_chunk<T>(p, block, slice, tid, pl);
    }
    __syncthreads();
    read_fragments<T>(smem, smem + 2 * T::A_STAGE, a_lane, b_lane, 0, pl.f0);

    int g = 0;                                         // flat chunk counter: chunk g sits in stage g & 1
    for (int seq = 0;; ++seq) {
        const int t = tile_at(p, block, seq);
        if (t < 0) break;
        const TileWork w = tile_work<T>(p, t, slice, walks_down(p, block, seq));
        const int n = w.nchunks;

        f32x16 acc[T::FM][T::FN];
#pragma unroll
        for (int bi = 0; bi < T::FM; ++bi)
#pragma unroll
            for (int bj = 0; bj < T::FN; ++bj)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[bi][bj][v] = 0.0f;

        int c = 0;
        while (c < n) {
            // Pairs of chunks (stage 0, stage 1) run the decision-free body for as long as the
            // chunk in the registers and the ones to load are plain chunks of the fetch tile.
            if (!(g & 1) && pl.in_regs && pl.reg_kind == kPlain && pl.f_live && pl.fj >= pl.fw.f_lo) {
                const int pairs = __builtin_amdgcn_readfirstlane(min(n - c, pl.fw.f_hi - pl.fj) / 2);     // (uniform: a scalar loop counter)
                if (pairs > 0) {
                    for (int i = 0; i < pairs; ++i) {
                        chunk_step<T, true, 0>(smem, p, block, slice, 0, tid, a_lane, b_lane, pl, acc);
                        chunk_step<T, true, 1>(smem, p, block, slice, 1, tid, a_lane, b_lane, pl, acc);
                    }
                    c += 2 * pairs;
                    g += 2 * pairs;
                    pl.fj += 2 * pairs;                          // the registers hold chunk fj-1 of the fetch tile
                    pl.reg_r0 = pl.fw.r0; pl.reg_c0 = pl.fw.c0; pl.reg_kc = pl.fw.k0 + (pl.fj - 1) * pl.fw.kstep;
                    if (pl.fj == pl.fw.nchunks) next_fetch_tile<T>(p, block, slice, tid, pl);
                    continue;
                }
            }
            const int swave = __builtin_amdgcn_readfirstlane(wave);       // (the wavefront's place in the tile, in scalar registers)
            const int skip = blocks_outside<T>(p, w.r0, w.c0, w.k0 + c * w.kstep, (swave / T::WN) * 32, (swave % T::WN) * 32);
            chunk_step<T, false, 0>(smem, p, block, slice, g & 1, tid, a_lane, b_lane, pl, acc, skip);
            ++c;
            ++g;
        }

        // store: register v of lane (l32, half) is C[row l32][column 8*(v/4) + 4*half + v%4] of its
        // 32x32 block.  Full tiles of a general result (or tiles strictly inside the triangle) go out
        // unchecked, 16 bytes at a time when the result allows; so do the groups of four of an edge
        // tile that lie inside the matrix; the rest and diagonal tiles element by element, the
        // triangle only
        float *const C = p.C + (int64_t)slice * p.slice_stride;
        bool inside = true;                                // no element of the tile lies outside the result's structure
        if (p.pc == kLower) inside = w.c0 + T::BN - 1 <= w.r0;
        if (p.pc == kUpper) inside = w.r0 + T::BM - 1 <= w.c0;
        const bool plain = inside && w.r0 + T::BM <= p.M && w.c0 + T::BN <= p.N;
#pragma unroll
        for (int bi = 0; bi < T::FM; ++bi)
#pragma unroll
            for (int bj = 0; bj < T::FN; ++bj)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int gi = w.r0 + wr0 + bi * T::RSTEP + l32;
                    const int gj = w.c0 + wc0 + bj * T::CSTEP + 8 * q + 4 * half;
                    float *dst = C + (int64_t)gi * p.ldc + gj;
                    if (p.c_vec && (plain || (inside && gi < p.M && gj + 4 <= p.N))) {
                        const f32x4 v = {acc[bi][bj][4 * q], acc[bi][bj][4 * q + 1], acc[bi][bj][4 * q + 2], acc[bi][bj][4 * q + 3]};
                        *reinterpret_cast<f32x4 *>(dst) = v;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (plain || (gi < p.M && gj + e < p.N && in_structure(p.pc, gi, gj + e))) dst[e] = acc[bi][bj][4 * q + e];
                    }
                }
    }
}

}  // namespace mom
