// Kernel argument blocks of the product and slice-sum kernels: plain data, filled by the
// planner at plan time (shapes, tile geometry) and completed by the evaluator at launch time
// (pointers, row strides, alignment flags).  No HIP types: the host-only planner includes this.
#pragma once
#include <stdint.h>

namespace mom {

constexpr int kMaxFused = 4;          // independent products one launch can carry

struct ProductParams {
    const float *A;
    const float *B;
    float *C;              // result, or split-K partial sums (slice s at C + s * slice_stride)
    int64_t lda, ldb, ldc;
    int64_t slice_stride;  // elements between split-K slices (0 when split_k == 1)
    int M, N, K;
    int pa, pb, pc;
    int tiles_m, tiles_n, num_tiles, order, paired, mirrored;
    int folded;            // single tiles; workgroups 256..511 take tiles min(T, 512) - 1 - (b - 256)
    int k_walk;            // bit 0: the first tile of a workgroup walks its k-range downwards, bit 1: its later tiles (the short tiles of mirrored and folded launches) do
    int grid;              // workgroups per k-slice
    int a_vec, b_vec;      // 16-byte loads at 32-bit offsets are legal for A / B (base and row stride aligned,
                           // row stride below 2^22 elements)
    int a_word, b_word;    // the row stride is below 2^22 elements: 32-bit byte offsets reach every element of a tile
    int a_tail, b_tail;    // ... and the extent along which the buffer is contiguous is a multiple of four, so no
                           // 16-byte group straddles the end of a row: tiles that poke over the matrix edge can
                           // then be loaded 16 bytes at a time through a descriptor that ends with the matrix
    int c_vec;             // 16-byte stores are legal for C
    int split_k;
};

// Several independent products in one launch: workgroups [block_end[i-1], block_end[i]) belong
// to product i, slice-major (split_k slices of `grid` workgroups each).
struct ProductBatch {
    int count;
    int block_end[kMaxFused];
    ProductParams prob[kMaxFused];
};

// Sum of split-K slices: C[i][j] = sum_s P[s][i][j], for up to kMaxFused products at once.
struct ReduceParams {
    const float *P;
    float *C;
    int64_t slice_stride, ldc;
    int slices, M, N;
    int pc;                               // structure of the result: only that part of the slices exists
};
struct ReduceBatch {
    int count;
    ReduceParams prob[kMaxFused];
};

}  // namespace mom
