// Evaluator: walks a plan's binary products level by level and enqueues their kernels on the
// caller's stream (MOM paper, Sec. 2 "Operations": a variadic Mul rewritten into binary
// multiplications).  No allocation, no synchronisation, no device memory owned here.
#include "../../include/mom.h"
#include "plan_internal.h"
#include "product_kernel.h"
#include "schedule.h"
#include "batched_kernel.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <vector>

namespace {

using namespace mom;

// 128x128 tiles, 4 wavefronts of 64x64, two workgroups per compute unit: the workhorse.
// 64x64 tiles, 4 wavefronts of 32x32, four or more per compute unit: products with a short side.
typedef TileConfig<128, 128, kChunk128, 2, 2, 2> Tile128;
typedef TileConfig<64, 64, kChunk64, 2, 2, 4> Tile64;

constexpr int kMaxDevices = 64;       // devices whose kernel attributes are remembered

template <class T>
hipError_t launch_product(const ProductBatch &batch, hipStream_t stream)
{
    // the tile's LDS footprint exceeds the default dynamic limit: raise it once per device (a
    // second thread doing the same at the same moment is harmless)
    static std::atomic<bool> configured[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices || !configured[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&product_kernel<T>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < kMaxDevices) configured[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(product_kernel<T>, dim3(batch.block_end[batch.count - 1]), dim3(T::NT), T::LDS_BYTES, stream,
                       batch);
    return hipGetLastError();
}

// Register-only MFMA loop: 4 independent accumulator blocks per wavefront keep the pipe full.
constexpr int kProbeWorkgroups = 2 * kComputeUnits, kProbeBlocks = 4, kProbeUnroll = 8;

__global__ __launch_bounds__(256) void probe_mfma_kernel(float *sink, int iters, float a0, float b0)
{
    f32x16 acc[kProbeBlocks];
#pragma unroll
    for (int i = 0; i < kProbeBlocks; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    const float a = a0 + threadIdx.x, b = b0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < kProbeUnroll; ++r)
#pragma unroll
            for (int i = 0; i < kProbeBlocks; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < kProbeBlocks; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    if (s == 12345.0f) sink[threadIdx.x] = s;       // sums of products of 1.x and 2 never land here
}

inline bool aligned16(const void *ptr, int64_t ld) { return (reinterpret_cast<uintptr_t>(ptr) & 15) == 0 && (ld & 3) == 0; }

inline int elementwise_grid(int64_t total) { return (int)std::min<int64_t>((total + 255) / 256, 4096); }

struct Resolved { const float *ptr; int64_t ld; };

}  // namespace

extern "C" mom_status_t mom_chain_eval(const mom_plan_t *plan, const float *const *d_factors, const int64_t *lds,
                                       float *d_out, int64_t ld_out, void *d_workspace, size_t workspace_bytes,
                                       uint32_t flags, void *stream_)
{
    if (!plan || !d_out) return MOM_ERR_NULL;
    if (!d_factors && !plan->survivors.empty()) return MOM_ERR_NULL;
    for (int32_t f : plan->survivors)
        if (!d_factors[f]) return MOM_ERR_NULL;
    if (lds)
        for (int32_t f : plan->survivors)
            if (lds[f] < plan->dims[f + 1]) return MOM_ERR_BAD_STRIDE;
    if (ld_out == 0) ld_out = plan->cols;
    if (ld_out < plan->cols) return MOM_ERR_BAD_STRIDE;
    if (plan->workspace_bytes > 0 &&
        (!d_workspace || workspace_bytes < plan->workspace_bytes || (reinterpret_cast<uintptr_t>(d_workspace) & 255)))
        return MOM_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    char *const ws = static_cast<char *>(d_workspace);
    const bool zero_fill = (flags & MOM_OUT_ZERO_FILL_TRIANGLE) != 0;
    const int M = (int)plan->rows, N = (int)plan->cols;

    if (plan->survivors.empty()) {                         // I * I * ... = I
        hipLaunchKernelGGL(write_identity_kernel, dim3(elementwise_grid((int64_t)M * M)), dim3(256), 0, stream,
                           d_out, ld_out, M);
        return hipGetLastError() == hipSuccess ? MOM_OK : MOM_ERR_HIP;
    }
    auto factor = [&](int32_t f) { return Resolved{d_factors[f], lds ? lds[f] : plan->dims[f + 1]}; };

    if (plan->steps.empty()) {                             // one survivor: A * I -> A
        const int32_t f = plan->survivors[0];
        const Resolved a = factor(f);
        hipLaunchKernelGGL(copy_structure_kernel, dim3(elementwise_grid((int64_t)M * N)), dim3(256), 0, stream,
                           a.ptr, a.ld, d_out, ld_out, M, N, plan->props[f]);
        if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
    }

    // Level by level; the products of a level that share a tile shape go out in one launch
    // (at most kMaxFused at a time), followed by one launch that sums their split-K slices.
    auto resolve = [&](const Operand &o, int64_t cols) {
        if (o.where == Where::Factor) return factor(o.index);
        if (o.where == Where::Temp)
            return Resolved{reinterpret_cast<const float *>(ws + plan->temps[o.index].offset), cols};
        return Resolved{d_out, ld_out};
    };
    size_t next = 0;
    while (next < plan->order.size()) {
        const int level = plan->steps[plan->order[next]].level;
        size_t level_end = next;
        while (level_end < plan->order.size() && plan->steps[plan->order[level_end]].level == level) ++level_end;
        std::vector<bool> done(level_end - next, false);
        for (size_t first = next; first < level_end; ++first) {
            if (done[first - next]) continue;
            const int shape = choose_launch(plan->steps[plan->order[first]]).shape;
            ProductBatch batch{};
            ReduceBatch reduce{};
            int64_t reduce_quads = 0;
            bool batch_small = true;
            for (size_t i = first; i < level_end && batch.count < kMaxFused; ++i) {
                const ProductStep &st = plan->steps[plan->order[i]];
                const Launch L = choose_launch(st);
                if (done[i - next] || L.shape != shape) continue;
                // only small products share a launch: a big one fills the chip by itself and
                // keeps its longest-first tile order only when it is alone
                const bool small_launch = (int64_t)L.grid * L.split_k <= 4 * kComputeUnits;
                if (batch.count > 0 && (!small_launch || !batch_small)) continue;
                batch_small = small_launch;
                done[i - next] = true;
                const Resolved a = resolve(st.a, st.k), b = resolve(st.b, st.n), c = resolve(st.c, st.n);
                ProductParams &p = batch.prob[batch.count];
                p.A = a.ptr; p.B = b.ptr; p.C = const_cast<float *>(c.ptr);
                p.lda = a.ld; p.ldb = b.ld; p.ldc = c.ld;
                p.M = (int)st.m; p.N = (int)st.n; p.K = (int)st.k;
                p.pa = st.pa; p.pb = st.pb; p.pc = st.pc;
                p.tiles_m = L.tiles_m; p.tiles_n = L.tiles_n; p.num_tiles = L.num_tiles;
                p.order = L.order; p.paired = L.paired; p.grid = L.grid;
                p.a_vec = aligned16(a.ptr, a.ld); p.b_vec = aligned16(b.ptr, b.ld);
                p.split_k = L.split_k;
                p.slice_stride = 0;
                if (L.split_k > 1) {                       // partial sums go to the scratch region
                    p.C = reinterpret_cast<float *>(ws + plan->scratch_offset + st.scratch_offset);
                    p.ldc = st.n;
                    p.slice_stride = st.m * st.n;
                    ReduceParams &r = reduce.prob[reduce.count++];
                    r.P = p.C; r.C = const_cast<float *>(c.ptr);
                    r.slice_stride = p.slice_stride; r.ldc = c.ld;
                    r.slices = L.split_k; r.M = p.M; r.N = p.N;
                    reduce_quads = std::max<int64_t>(reduce_quads, (st.m * st.n + 3) / 4);
                }
                p.c_vec = aligned16(p.C, p.ldc);
                const int64_t blocks = (int64_t)(batch.count ? batch.block_end[batch.count - 1] : 0) + (int64_t)L.grid * L.split_k;
                if (blocks > 0x7fffffff) return MOM_ERR_UNSUPPORTED;
                batch.block_end[batch.count++] = (int)blocks;
            }
            const hipError_t e = shape == kTile128 ? launch_product<Tile128>(batch, stream)
                                                   : launch_product<Tile64>(batch, stream);
            if (e != hipSuccess) return MOM_ERR_HIP;
            if (reduce.count > 0) {
                hipLaunchKernelGGL(reduce_slices_kernel, dim3((unsigned)std::min<int64_t>((reduce_quads + 31) / 32, 8192), reduce.count),
                                   dim3(256), 0, stream, reduce);
                if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
            }
        }
        next = level_end;
    }

    if (zero_fill && (plan->result_prop == kLower || plan->result_prop == kUpper)) {
        hipLaunchKernelGGL(zero_other_half_kernel, dim3(elementwise_grid((int64_t)M * M)), dim3(256), 0, stream,
                           d_out, ld_out, M, plan->result_prop);
        if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
    }
    return MOM_OK;
}

extern "C" mom_status_t mom_chain_eval_batched(const mom_plan_t *plan, const float *const *d_factor_bases,
                                               const int64_t *batch_strides, float *d_out,
                                               int64_t out_batch_stride, int32_t batch, void *stream_)
{
    if (!plan || !d_out) return MOM_ERR_NULL;
    if (batch < 0) return MOM_ERR_BAD_N;
    if (!d_factor_bases && !plan->survivors.empty()) return MOM_ERR_NULL;
    for (int32_t f : plan->survivors)
        if (!d_factor_bases[f]) return MOM_ERR_NULL;
    if (plan->max_dim > kBatchedMaxDim || (int)plan->survivors.size() > kBatchedMaxFactors) return MOM_ERR_UNSUPPORTED;
    if (batch_strides)
        for (int32_t f : plan->survivors)
            if (batch_strides[f] < plan->dims[f] * plan->dims[f + 1]) return MOM_ERR_BAD_STRIDE;
    if (out_batch_stride == 0) out_batch_stride = plan->rows * plan->cols;
    if (out_batch_stride < plan->rows * plan->cols) return MOM_ERR_BAD_STRIDE;
    if (batch == 0) return MOM_OK;
    return launch_batched(plan, d_factor_bases, batch_strides, d_out, out_batch_stride, batch,
                          static_cast<hipStream_t>(stream_)) == hipSuccess ? MOM_OK : MOM_ERR_HIP;
}

extern "C" mom_status_t mom_probe_mfma_peak(int32_t iters, float *d_sink, double *flop, void *stream_)
{
    if (!d_sink || !flop) return MOM_ERR_NULL;
    if (iters <= 0) return MOM_ERR_BAD_N;
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(kProbeWorkgroups), dim3(256), 0, static_cast<hipStream_t>(stream_), d_sink,
                       iters, 1.0f, 2.0f);
    if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
    // 32x32x2: 2 * 32 * 32 * 2 = 4096 floating-point operations per MFMA
    *flop = (double)kProbeWorkgroups * 4 /* wavefronts */ * (double)iters * kProbeUnroll * kProbeBlocks * 4096.0;
    return MOM_OK;
}
