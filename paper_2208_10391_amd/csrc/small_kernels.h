// The small kernels around the product kernel: sum of split-K slices, copy of a single
// surviving factor, identity write, zero fill of the other half of a triangular result.
// Included by the evaluator only (these are ordinary, non-template kernels).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "product_kernel.h"

namespace mom {

// Sum of split-K slices (ReduceBatch; blockIdx.y selects the product).  The order of summation
// is fixed, so results repeat bit for bit from run to run.  Only the structure of the result
// is summed and written: outside it the slices were never written.
// 256 threads = 32 groups of 4 consecutive floats x 8 lanes over the slices: lane g of a group
// sums slices g, g+8, ... with all its loads in flight, the 8 partial sums meet in LDS.
__global__ __launch_bounds__(256) void reduce_slices_kernel(const ReduceBatch batch)
{
    __shared__ f32x4 part[8][32];
    const ReduceParams &r = batch.prob[blockIdx.y];
    const int64_t total = (int64_t)r.M * r.N;              // scratch slices are packed: M*N floats each
    const int64_t quads = (total + 3) / 4;
    const bool vec = (total % 4) == 0 && (r.N % 4) == 0 && (r.ldc % 4) == 0 && (reinterpret_cast<uintptr_t>(r.C) & 15) == 0;
    const int q_in_block = threadIdx.x % 32, g = threadIdx.x / 32;
    for (int64_t q0 = (int64_t)blockIdx.x * 32; q0 < quads; q0 += (int64_t)gridDim.x * 32) {
        const int64_t q = q0 + q_in_block, e = q * 4;
        // where the quad sits in the result's structure: 2 wholly inside, 1 partly, 0 outside
        // (with N % 4 == 0 a quad lies in one row; otherwise every element is checked)
        int inside = 0;
        if (q < quads) {
            if (r.pc == kGeneral) {
                inside = 2;
            } else if (vec) {
                const int i = (int)(e / r.N), j = (int)(e % r.N);
                const bool first = in_structure(r.pc, i, j), last = in_structure(r.pc, i, j + 3);
                inside = (first && last) ? 2 : (first || last) ? 1 : 0;
            } else {
                inside = 1;
            }
        }
        f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f};
        if (inside == 2 && vec) {
#pragma unroll 8
            for (int k = g; k < r.slices; k += 8) s += *reinterpret_cast<const f32x4 *>(r.P + k * r.slice_stride + e);
        } else if (inside) {
            for (int k = g; k < r.slices; k += 8)
                for (int c = 0; c < 4; ++c)
                    if (e + c < total && in_structure(r.pc, (int)((e + c) / r.N), (int)((e + c) % r.N)))
                        s[c] += r.P[k * r.slice_stride + e + c];
        }
        part[g][q_in_block] = s;
        __syncthreads();
        if (g == 0 && inside) {
#pragma unroll
            for (int k = 1; k < 8; ++k) s += part[k][q_in_block];
            if (inside == 2 && vec) {
                *reinterpret_cast<f32x4 *>(r.C + (e / r.N) * r.ldc + (e % r.N)) = s;
            } else {
                for (int c = 0; c < 4; ++c)
                    if (e + c < total && in_structure(r.pc, (int)((e + c) / r.N), (int)((e + c) % r.N)))
                        r.C[((e + c) / r.N) * r.ldc + ((e + c) % r.N)] = s[c];
            }
        }
        __syncthreads();
    }
}

// The three element-wise kernels below walk a matrix row by row: blockIdx.y strides over the
// rows, the threads of a workgroup over groups of four consecutive columns (one 16-byte access
// when base and row stride allow, element-wise otherwise); no division per element.
constexpr int kRowUnroll = 4;          // rows a thread has in flight at once

// Columns [lo, hi) of row i that lie inside the structure of property p (N columns in all).
__device__ __forceinline__ void structure_span(int p, int i, int N, int &lo, int &hi)
{
    lo = (p == kUpper || p == kDiagonal) ? min(i, N) : 0;
    hi = (p == kLower || p == kDiagonal) ? min(i + 1, N) : N;
}

// out = A restricted to its structure (single surviving factor: A*I -> A).  Whole 16-byte
// groups move with non-temporal loads and stores: every line is touched once, and keeping it
// out of the caches' way is worth a sixth of the time (100 -> 87 us for 8192 x 8192).
__global__ __launch_bounds__(256) void copy_structure_kernel(const float *A, int64_t lda, float *C, int64_t ldc, int M, int N,
                                                             int prop, int vec)
{
    const int quads = (N + 3) / 4;
    for (int i0 = blockIdx.y * kRowUnroll; i0 < M; i0 += gridDim.y * kRowUnroll) {
        for (int q = blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += gridDim.x * blockDim.x) {
            const int j = 4 * q;
            f32x4 v[kRowUnroll];
            bool whole[kRowUnroll], some[kRowUnroll];
#pragma unroll
            for (int r = 0; r < kRowUnroll; ++r) {          // all loads first
                const int i = i0 + r;
                int lo, hi;
                structure_span(prop, i, N, lo, hi);
                some[r] = i < M && j < hi && j + 4 > lo;
                whole[r] = some[r] && vec && j >= lo && j + 4 <= hi;
                if (whole[r]) {
                    v[r] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(A + (int64_t)i * lda + j));
                } else if (some[r]) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[r][e] = (j + e >= lo && j + e < hi) ? A[(int64_t)i * lda + j + e] : 0.0f;
                }
            }
#pragma unroll
            for (int r = 0; r < kRowUnroll; ++r) {
                const int i = i0 + r;
                if (whole[r]) {
                    __builtin_nontemporal_store(v[r], reinterpret_cast<f32x4 *>(C + (int64_t)i * ldc + j));
                } else if (some[r]) {
                    int lo, hi;
                    structure_span(prop, i, N, lo, hi);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (j + e >= lo && j + e < hi) C[(int64_t)i * ldc + j + e] = v[r][e];
                }
            }
        }
    }
}

// out = S^T restricted to the structure `prop` of the result (single surviving factor that
// enters the chain transposed): 64 x 64 blocks through LDS, reads and writes both along rows.
// A block that lies wholly inside the matrix and the structure moves with 16-byte non-temporal
// accesses on both sides (`vec`: bases and row strides allow them); edge and diagonal blocks go
// element by element.
constexpr int kTransposeTile = 64;
__global__ __launch_bounds__(256) void copy_transposed_kernel(const float *S, int64_t lds_, float *C, int64_t ldc, int M, int N,
                                                              int prop, int vec)
{
    constexpr int T = kTransposeTile;
    __shared__ float tile[T][T + 1];                             // tile[j][i] = S[j0 + j][i0 + i]
    const int tid = threadIdx.x, c4 = 4 * (tid % 16), r4 = tid / 16;
    const int bj = (N + T - 1) / T, blocks = ((M + T - 1) / T) * bj;
    for (int b = blockIdx.x; b < blocks; b += gridDim.x) {
        const int i0 = (b / bj) * T, j0 = (b % bj) * T;          // block of the result
        bool whole = vec && i0 + T <= M && j0 + T <= N;
        if (prop == kLower) whole = whole && j0 + T - 1 <= i0;
        if (prop == kUpper) whole = whole && i0 + T - 1 <= j0;
        if (prop == kDiagonal) whole = false;
        if (whole) {
            f32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)                          // S is N x M: rows j0.., columns i0..
                v[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(S + (int64_t)(j0 + r4 + 16 * u) * lds_ + i0 + c4));
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) tile[r4 + 16 * u][c4 + e] = v[u][e];
            __syncthreads();
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = r4 + 16 * u;
                const f32x4 w = {tile[c4][i], tile[c4 + 1][i], tile[c4 + 2][i], tile[c4 + 3][i]};
                __builtin_nontemporal_store(w, reinterpret_cast<f32x4 *>(C + (int64_t)(i0 + i) * ldc + j0 + c4));
            }
        } else {
            for (int idx = tid; idx < T * T; idx += 256) {
                const int r = idx / T, x = idx % T, j = j0 + r, i = i0 + x;
                tile[r][x] = (j < N && i < M && in_structure(prop, i, j)) ? S[(int64_t)j * lds_ + i] : 0.0f;
            }
            __syncthreads();
            for (int idx = tid; idx < T * T; idx += 256) {
                const int r = idx / T, x = idx % T, i = i0 + r, j = j0 + x;
                if (i < M && j < N && in_structure(prop, i, j)) C[(int64_t)i * ldc + j] = tile[x][r];
            }
        }
        __syncthreads();
    }
}

// A product with a diagonal operand: C = D * X (side 0: row i of X scaled by D[i][i]) or
// C = X * D (side 1: column j scaled by D[j][j]), written inside the structure px of X, which
// is also the result's.  X is addressed through a row and a column stride, so a factor stored
// transposed is read in place; D's own transposition does not matter.
struct ScaleParams {
    const float *D;
    int64_t ldd;
    const float *X;
    int64_t x_rs, x_cs;
    float *C;
    int64_t ldc;
    int M, N, side, px, vec;
};

__global__ __launch_bounds__(256) void diag_scale_kernel(const ScaleParams p)
{
    const int quads = (p.N + 3) / 4;
    for (int i = blockIdx.y; i < p.M; i += gridDim.y) {
        int lo, hi;
        structure_span(p.px, i, p.N, lo, hi);
        const float di = p.side == 0 ? p.D[(int64_t)i * (p.ldd + 1)] : 0.0f;
        for (int q = blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += gridDim.x * blockDim.x) {
            const int j = 4 * q;
            if (j >= hi || j + 4 <= lo) continue;
            if (p.vec && j >= lo && j + 4 <= hi) {
                f32x4 v = *reinterpret_cast<const f32x4 *>(p.X + (int64_t)i * p.x_rs + j);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] *= p.side == 0 ? di : p.D[(int64_t)(j + e) * (p.ldd + 1)];
                *reinterpret_cast<f32x4 *>(p.C + (int64_t)i * p.ldc + j) = v;
            } else {
                for (int e = 0; e < 4; ++e) {
                    const int c = j + e;
                    if (c < lo || c >= hi) continue;
                    const float d = p.side == 0 ? di : p.D[(int64_t)c * (p.ldd + 1)];
                    p.C[(int64_t)i * p.ldc + c] = d * p.X[(int64_t)i * p.x_rs + (int64_t)c * p.x_cs];
                }
            }
        }
    }
}

// Variadic Add (paper Table 1): C = [C +] sum of up to kMaxAddTerms terms, each with its own
// structure (an Identity term has no buffer and adds 1 on the diagonal), written inside the
// structure `pc` of the sum.  Terms are addressed through a row and a column stride, so a term
// stored transposed is read in place.
constexpr int kMaxAddTerms = 8;
struct AddParams {
    const float *X[kMaxAddTerms];
    int64_t rs[kMaxAddTerms], cs[kMaxAddTerms];
    int prop[kMaxAddTerms], vec[kMaxAddTerms];
    int count;
    float *C;
    int64_t ldc;
    int M, N, pc, accumulate, c_vec;
};

__global__ __launch_bounds__(256) void add_terms_kernel(const AddParams p)
{
    const int quads = (p.N + 3) / 4;
    for (int i = blockIdx.y; i < p.M; i += gridDim.y) {
        int lo, hi;
        structure_span(p.pc, i, p.N, lo, hi);
        for (int q = blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += gridDim.x * blockDim.x) {
            const int j = 4 * q;
            if (j >= hi || j + 4 <= lo) continue;
            const bool whole = p.c_vec && j >= lo && j + 4 <= hi;
            float *dst = p.C + (int64_t)i * p.ldc + j;
            f32x4 s = {0.0f, 0.0f, 0.0f, 0.0f};
            if (p.accumulate) {
                if (whole) {
                    s = *reinterpret_cast<const f32x4 *>(dst);
                } else {
                    for (int e = 0; e < 4; ++e)
                        if (j + e >= lo && j + e < hi) s[e] = dst[e];
                }
            }
            for (int t = 0; t < p.count; ++t) {
                if (p.prop[t] == kIdentity) {
                    for (int e = 0; e < 4; ++e) s[e] += (j + e == i) ? 1.0f : 0.0f;
                    continue;
                }
                int tlo, thi;
                structure_span(p.prop[t], i, p.N, tlo, thi);
                if (j >= thi || j + 4 <= tlo) continue;
                if (p.vec[t] && j >= tlo && j + 4 <= thi) {
                    s += *reinterpret_cast<const f32x4 *>(p.X[t] + (int64_t)i * p.rs[t] + j);
                } else {
                    for (int e = 0; e < 4; ++e)
                        if (j + e >= tlo && j + e < thi) s[e] += p.X[t][(int64_t)i * p.rs[t] + (int64_t)(j + e) * p.cs[t]];
                }
            }
            if (whole) {
                *reinterpret_cast<f32x4 *>(dst) = s;
            } else {
                for (int e = 0; e < 4; ++e)
                    if (j + e >= lo && j + e < hi) dst[e] = s[e];
            }
        }
    }
}

// out = I (every factor was an Identity: I*I = I)
__global__ __launch_bounds__(256) void write_identity_kernel(float *C, int64_t ldc, int M, int vec)
{
    const int quads = (M + 3) / 4;
    for (int i = blockIdx.y; i < M; i += gridDim.y)
        for (int q = blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += gridDim.x * blockDim.x) {
            const int j = 4 * q;
            if (vec && j + 4 <= M) {
                const f32x4 v = {j == i ? 1.0f : 0.0f, j + 1 == i ? 1.0f : 0.0f, j + 2 == i ? 1.0f : 0.0f, j + 3 == i ? 1.0f : 0.0f};
                *reinterpret_cast<f32x4 *>(C + (int64_t)i * ldc + j) = v;
            } else {
                for (int e = 0; e < 4 && j + e < M; ++e) C[(int64_t)i * ldc + j + e] = (j + e == i) ? 1.0f : 0.0f;
            }
        }
}

// zeros into the half of a triangular result that the product kernel leaves untouched
__global__ __launch_bounds__(256) void zero_other_half_kernel(float *C, int64_t ldc, int M, int prop, int vec)
{
    const int quads = (M + 3) / 4;
    for (int i = blockIdx.y; i < M; i += gridDim.y) {
        // the other half of row i: columns (i, M) of a lowerTri result, [0, i) of an upperTri
        // one, both for a diagonal one; [s0, s1) is the structure, which is left alone
        int s0, s1;
        structure_span(prop, i, M, s0, s1);
        for (int q = blockIdx.x * blockDim.x + threadIdx.x; q < quads; q += gridDim.x * blockDim.x) {
            const int j = 4 * q;
            if (j >= s0 && j + 4 <= s1) continue;
            if (vec && j + 4 <= M && (j + 4 <= s0 || j >= s1)) {
                const f32x4 z = {0.0f, 0.0f, 0.0f, 0.0f};
                *reinterpret_cast<f32x4 *>(C + (int64_t)i * ldc + j) = z;
            } else {
                for (int e = 0; e < 4; ++e)
                    if (j + e < M && (j + e < s0 || j + e >= s1)) C[(int64_t)i * ldc + j + e] = 0.0f;
            }
        }
    }
}

}  // namespace mom
