// Batched small chains: many independent chains that share one plan, all in one launch.
// One 64-lane wavefront (= one workgroup) evaluates one chain: its factors (each at most
// 32x32) are fetched with all loads in flight at once, parked in LDS, and the plan's binary
// products run as 32x32x32 MFMA sequences whose results replace their left operand in LDS.
// Only the factors are read from and only the final result is written to HBM.
// (Variadic Mul rewritten into binary products, MOM paper Sec. 2 "Operations".)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan_internal.h"
#include "product_kernel.h"

namespace mom {

constexpr int kBatchedMaxDim = 32;
constexpr int kBatchedMaxFactors = kBatchedSlots;
constexpr int kSlotLd = 36;                       // LDS row stride of a 32x32 slot, floats
constexpr int kSlotFloats = 32 * kSlotLd;

struct BatchedParams {
    const float *base[kBatchedMaxFactors];
    int64_t stride[kBatchedMaxFactors];           // elements between consecutive chains
    int rows[kBatchedMaxFactors], cols[kBatchedMaxFactors], prop[kBatchedMaxFactors];
    int vec[kBatchedMaxFactors];                  // factor is a full 32x32, 16-byte aligned
    int trans[kBatchedMaxFactors];                // the buffer holds the factor's transpose (rows, cols:
                                                  // of the STORED matrix; prop: of the factor in the chain)
    int num_products;
    int a_slot[kBatchedMaxFactors], b_slot[kBatchedMaxFactors];   // product s: slot[a] = slot[a] * slot[b]
    float *out;
    int64_t out_stride;
    int out_rows, out_cols;
    int result_slot;
    int batch;
};

// NL = number of surviving factors (0: every factor is an Identity, the result is I).
template <int NL>
__global__ __launch_bounds__(64) void batched_chain_kernel(const BatchedParams p)
{
    __shared__ __align__(16) float slots[(NL > 0 ? NL : 1) * kSlotFloats];
    const int chain = blockIdx.x;
    const int lane = threadIdx.x, l32 = lane & 31, half = lane >> 5;
    float *const out = p.out + (int64_t)chain * p.out_stride;

    if (NL == 0) {
        for (int e = lane; e < p.out_rows * p.out_cols; e += 64)
            out[e] = (e / p.out_cols == e % p.out_cols) ? 1.0f : 0.0f;
        return;
    }

    // 1. every factor of this chain: global -> registers, all loads issued before any is used
    f32x4 reg[NL > 0 ? NL : 1][4];
#pragma unroll
    for (int f = 0; f < NL; ++f) {
        const float *src = p.base[f] + (int64_t)chain * p.stride[f];
        if (p.vec[f]) {
#pragma unroll
            for (int q = 0; q < 4; ++q) reg[f][q] = *reinterpret_cast<const f32x4 *>(src + (lane + 64 * q) * 4);
        } else {                                   // any shape up to 32x32: element-wise, zero padded
            const int rows = p.rows[f], cols = p.cols[f];
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = (lane + 64 * q) / 8, j = ((lane + 64 * q) % 8) * 4 + e;
                    reg[f][q][e] = (i < rows && j < cols) ? src[i * cols + j] : 0.0f;
                }
        }
    }
    // 2. registers -> LDS slot f, keeping only the factor's structure; a factor whose buffer
    //    holds its transpose is mirrored on the way (stored entry (i, j) is entry (j, i) of the chain)
#pragma unroll
    for (int f = 0; f < NL; ++f)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = (lane + 64 * q) / 8, j0 = ((lane + 64 * q) % 8) * 4;
            f32x4 v = reg[f][q];
            if (p.trans[f]) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    slots[f * kSlotFloats + (j0 + e) * kSlotLd + i] = in_structure(p.prop[f], j0 + e, i) ? v[e] : 0.0f;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = in_structure(p.prop[f], i, j0 + e) ? v[e] : 0.0f;
                *reinterpret_cast<f32x4 *>(&slots[f * kSlotFloats + i * kSlotLd + j0]) = v;
            }
        }
    __syncthreads();

    // 3. the products, in the plan's order
    for (int s = 0; s < p.num_products; ++s) {
        const float *A = &slots[p.a_slot[s] * kSlotFloats];
        const float *B = &slots[p.b_slot[s] * kSlotFloats];
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) {
            const f32x4 a = *reinterpret_cast<const f32x4 *>(A + l32 * kSlotLd + kg * 8 + 4 * half);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], B[(kg * 8 + 4 * half + e) * kSlotLd + l32], acc, 0, 0, 0);
        }
        __syncthreads();                           // every lane has read A before it is replaced
        if (s + 1 < p.num_products) {
            float *D = &slots[p.a_slot[s] * kSlotFloats];
#pragma unroll
            for (int v = 0; v < 16; ++v) D[(8 * (v / 4) + 4 * half + v % 4) * kSlotLd + l32] = acc[v];
            __syncthreads();
        } else {                                   // last product: accumulators -> HBM
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = 8 * (v / 4) + 4 * half + v % 4;
                if (i < p.out_rows && l32 < p.out_cols) out[i * p.out_cols + l32] = acc[v];
            }
        }
    }
    if (p.num_products == 0) {                     // a single surviving factor: A * I -> A
        const float *S = &slots[p.result_slot * kSlotFloats];
        for (int e = lane; e < p.out_rows * p.out_cols; e += 64)
            out[e] = S[(e / p.out_cols) * kSlotLd + e % p.out_cols];
    }
}

// Register-only fast path for the chain X0 * (X1 * X2) of three full 32x32 factors (the
// canonical plan of lowerTri * general * upperTri): nothing touches LDS.
//   P = X1 * X2: X1 is the A operand (lane (l32, half) loads X1[l32][8kg + 4half .. +3] as one
//   16-byte load per group kg), X2 the B operand (X2[8kg + 4half + e][l32], a coalesced 4-byte
//   load per step).  Accumulator register v = 4kg + e of P then holds P[8kg + 4half + e][l32],
//   which is exactly the B operand of step (kg, e) of the second product: X0 * P runs
//   straight out of the accumulators of the first.
// The three properties are template parameters: a general factor then costs no masking at
// all and a triangular one a compare against a constant and a select per element.
template <int P>
__device__ __forceinline__ float keep(float x, int i, int j)
{
    if (P == kLower) return j <= i ? x : 0.0f;
    if (P == kUpper) return j >= i ? x : 0.0f;
    return x;
}

template <int P0, int P1, int P2>
__global__ __launch_bounds__(256) void batched_chain3_right_kernel(const BatchedParams p)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const int64_t chain = (int64_t)blockIdx.x * 4 + wave;
    if (chain >= p.batch) return;
    const float *X0 = p.base[0] + chain * p.stride[0];
    const float *X1 = p.base[1] + chain * p.stride[1];
    const float *X2 = p.base[2] + chain * p.stride[2];
    f32x4 x0[4], x1[4];
    float x2[16];
#pragma unroll
    for (int kg = 0; kg < 4; ++kg) x1[kg] = *reinterpret_cast<const f32x4 *>(X1 + l32 * 32 + kg * 8 + 4 * half);
#pragma unroll
    for (int v = 0; v < 16; ++v) x2[v] = X2[((v / 4) * 8 + 4 * half + v % 4) * 32 + l32];
#pragma unroll
    for (int kg = 0; kg < 4; ++kg) x0[kg] = *reinterpret_cast<const f32x4 *>(X0 + l32 * 32 + kg * 8 + 4 * half);

    __builtin_amdgcn_sched_barrier(0);     // all 24 loads are in flight before the first use
    const int row = l32 - 4 * half;        // (k <= l32) with k = c + 4*half  <=>  c <= row, c a constant
    f32x16 prod, res;
#pragma unroll
    for (int v = 0; v < 16; ++v) prod[v] = res[v] = 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int c = (v / 4) * 8 + v % 4;
        prod = __builtin_amdgcn_mfma_f32_32x32x2f32(keep<P1>(x1[v / 4][v % 4], row, c), keep<P2>(x2[v], c, row), prod, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int c = (v / 4) * 8 + v % 4;
        res = __builtin_amdgcn_mfma_f32_32x32x2f32(keep<P0>(x0[v / 4][v % 4], row, c), prod[v], res, 0, 0, 0);
    }
    float *out = p.out + chain * p.out_stride;
#pragma unroll
    for (int v = 0; v < 16; ++v) out[(8 * (v / 4) + 4 * half + v % 4) * 32 + l32] = res[v];
}

typedef void (*Chain3Kernel)(const BatchedParams);
template <int P0, int P1>
inline Chain3Kernel chain3_kernel_for(int p2)
{
    return p2 == kLower ? batched_chain3_right_kernel<P0, P1, kLower>
         : p2 == kUpper ? batched_chain3_right_kernel<P0, P1, kUpper> : batched_chain3_right_kernel<P0, P1, kGeneral>;
}
template <int P0>
inline Chain3Kernel chain3_kernel_for(int p1, int p2)
{
    return p1 == kLower ? chain3_kernel_for<P0, kLower>(p2)
         : p1 == kUpper ? chain3_kernel_for<P0, kUpper>(p2) : chain3_kernel_for<P0, kGeneral>(p2);
}
inline Chain3Kernel chain3_kernel_for(int p0, int p1, int p2)
{
    return p0 == kLower ? chain3_kernel_for<kLower>(p1, p2)
         : p0 == kUpper ? chain3_kernel_for<kUpper>(p1, p2) : chain3_kernel_for<kGeneral>(p1, p2);
}

inline hipError_t launch_batched(const mom_plan *plan, const float *const *bases, const int64_t *strides,
                                 float *d_out, int64_t out_stride, int32_t batch, hipStream_t stream)
{
    BatchedParams p{};
    const int nl = (int)plan->survivors.size();
    for (int i = 0; i < nl; ++i) {
        const int f = plan->survivors[i];
        p.base[i] = bases[f];
        p.trans[i] = plan->trans[f];
        p.rows[i] = (int)plan->dims[p.trans[i] ? f + 1 : f];
        p.cols[i] = (int)plan->dims[p.trans[i] ? f : f + 1];
        p.prop[i] = plan->chain_props[f];
        p.stride[i] = strides ? strides[f] : plan->dims[f] * plan->dims[f + 1];
        p.vec[i] = p.rows[i] == 32 && p.cols[i] == 32 && (reinterpret_cast<uintptr_t>(bases[f]) & 15) == 0 &&
                   (p.stride[i] & 3) == 0;
    }
    // slots were assigned with the plan
    p.num_products = (int)plan->steps.size();
    for (int s = 0; s < p.num_products; ++s) {
        p.a_slot[s] = plan->a_slot[s];
        p.b_slot[s] = plan->b_slot[s];
    }
    p.result_slot = 0;
    p.out = d_out;
    p.out_stride = out_stride;
    p.out_rows = (int)plan->rows;
    p.out_cols = (int)plan->cols;
    p.batch = batch;
    // three full, aligned 32x32 factors multiplied as X0 * (X1 * X2): the register-only kernel
    const bool no_diagonal = p.prop[0] != kDiagonal && p.prop[1] != kDiagonal && p.prop[2] != kDiagonal;
    if (nl == 3 && no_diagonal && p.vec[0] && p.vec[1] && p.vec[2] && !p.trans[0] && !p.trans[1] && !p.trans[2] && p.num_products == 2 && p.a_slot[0] == 1 && p.b_slot[0] == 2 &&
        p.a_slot[1] == 0 && p.b_slot[1] == 1) {
        hipLaunchKernelGGL(chain3_kernel_for(p.prop[0], p.prop[1], p.prop[2]), dim3((batch + 3) / 4), dim3(256), 0, stream, p);
        return hipGetLastError();
    }
    const dim3 grid(batch), block(64);
    switch (nl) {
    case 0: hipLaunchKernelGGL(batched_chain_kernel<0>, grid, block, 0, stream, p); break;
    case 1: hipLaunchKernelGGL(batched_chain_kernel<1>, grid, block, 0, stream, p); break;
    case 2: hipLaunchKernelGGL(batched_chain_kernel<2>, grid, block, 0, stream, p); break;
    case 3: hipLaunchKernelGGL(batched_chain_kernel<3>, grid, block, 0, stream, p); break;
    case 4: hipLaunchKernelGGL(batched_chain_kernel<4>, grid, block, 0, stream, p); break;
    case 5: hipLaunchKernelGGL(batched_chain_kernel<5>, grid, block, 0, stream, p); break;
    case 6: hipLaunchKernelGGL(batched_chain_kernel<6>, grid, block, 0, stream, p); break;
    case 7: hipLaunchKernelGGL(batched_chain_kernel<7>, grid, block, 0, stream, p); break;
    case 8: hipLaunchKernelGGL(batched_chain_kernel<8>, grid, block, 0, stream, p); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace mom
