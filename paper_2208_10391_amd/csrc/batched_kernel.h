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
constexpr int kBatchedMaxFactors = 8;
constexpr int kSlotLd = 36;                       // LDS row stride of a 32x32 slot, floats
constexpr int kSlotFloats = 32 * kSlotLd;

struct BatchedParams {
    const float *base[kBatchedMaxFactors];
    int64_t stride[kBatchedMaxFactors];           // elements between consecutive chains
    int rows[kBatchedMaxFactors], cols[kBatchedMaxFactors], prop[kBatchedMaxFactors];
    int vec[kBatchedMaxFactors];                  // factor is a full 32x32, 16-byte aligned
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
    // 2. registers -> LDS slot f, keeping only the factor's structure
#pragma unroll
    for (int f = 0; f < NL; ++f)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = (lane + 64 * q) / 8, j0 = ((lane + 64 * q) % 8) * 4;
            f32x4 v = reg[f][q];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = in_structure(p.prop[f], i, j0 + e) ? v[e] : 0.0f;
            *reinterpret_cast<f32x4 *>(&slots[f * kSlotFloats + i * kSlotLd + j0]) = v;
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

inline hipError_t launch_batched(const mom_plan *plan, const float *const *bases, const int64_t *strides,
                                 float *d_out, int64_t out_stride, int32_t batch, hipStream_t stream)
{
    BatchedParams p{};
    const int nl = (int)plan->survivors.size();
    for (int i = 0; i < nl; ++i) {
        const int f = plan->survivors[i];
        p.base[i] = bases[f];
        p.rows[i] = (int)plan->dims[f];
        p.cols[i] = (int)plan->dims[f + 1];
        p.prop[i] = plan->props[f];
        p.stride[i] = strides ? strides[f] : plan->dims[f] * plan->dims[f + 1];
        p.vec[i] = p.rows[i] == 32 && p.cols[i] == 32 && (reinterpret_cast<uintptr_t>(bases[f]) & 15) == 0 &&
                   (p.stride[i] & 3) == 0;
    }
    // slot of every value: factor -> its position among the survivors; a product's result
    // takes over the slot of its left operand
    std::vector<int> temp_slot(plan->temps.size(), -1);
    auto slot_of = [&](const Operand &o) {
        if (o.where == Where::Temp) return temp_slot[o.index];
        for (int i = 0; i < nl; ++i)
            if (plan->survivors[i] == o.index) return i;
        return -1;
    };
    p.num_products = (int)plan->steps.size();
    for (int s = 0; s < p.num_products; ++s) {
        const ProductStep &st = plan->steps[s];
        p.a_slot[s] = slot_of(st.a);
        p.b_slot[s] = slot_of(st.b);
        if (st.c.where == Where::Temp) temp_slot[st.c.index] = p.a_slot[s];
    }
    p.result_slot = 0;
    p.out = d_out;
    p.out_stride = out_stride;
    p.out_rows = (int)plan->rows;
    p.out_cols = (int)plan->cols;
    p.batch = batch;
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
