// Evaluator: walks a plan's binary products level by level and enqueues their kernels on the
// caller's stream (MOM paper, Sec. 2 "Operations": a variadic Mul rewritten into binary
// multiplications).  No allocation, no synchronisation, no device memory owned here.
#include "../../include/mom.h"
#include "plan_internal.h"
#include "product_kernel.h"
#include "product_variant.h"
#include "schedule.h"
#include "small_kernels.h"
#include "skinny_pair_kernel.h"
#include "batched_kernel.h"

#include <hip/hip_runtime.h>

#include <atomic>

namespace {

using namespace mom;

constexpr int kMaxDevices = 64;       // devices whose one-time set-up is remembered

// One-time set-up per device: the tiles' LDS footprint exceeds the default dynamic limit, so
// the limit of each product kernel is raised once (hipFuncSetAttribute is not allowed while a
// stream is being captured, which is why this is not left to the launch itself).
std::atomic<bool> g_device_ready[kMaxDevices];

// Workspace of mom_chain_eval_static: one array per GPU, part of the loaded code object, held
// until the process ends.  `scratch` is a host-side stand-in here; its device address on the
// current GPU comes from hipGetSymbolAddress and is kept per device in g_scratch.
static __device__ __align__(256) unsigned char scratch[MOM_STATIC_WORKSPACE_BYTES];
char *g_scratch[kMaxDevices];

hipError_t scratch_address(char **ptr)
{
    return hipGetSymbolAddress(reinterpret_cast<void **>(ptr), HIP_SYMBOL(scratch));
}

const ProductLauncher kLaunchers[kNumVariants] = {launch_product_nn, launch_product_tn, launch_product_nt, launch_product_tt};
const ProductConfigurer kConfigurers[kNumVariants] = {configure_product_nn, configure_product_tn, configure_product_nt,
                                                      configure_product_tt};

hipError_t configure_kernels()
{
    for (int v = 0; v < kNumVariants; ++v) {
        const hipError_t e = kConfigurers[v]();
        if (e != hipSuccess) return e;
    }
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&skinny_pair_kernel<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kPairLdsBytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&skinny_pair_kernel<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kPairLdsBytes);
}

// Make the current device ready for launches.  `stream` is the stream an evaluation is about
// to use (nullptr from mom_init): a first use under capture is refused instead of breaking the
// capture.  A second thread doing the same set-up at the same moment is harmless.
mom_status_t ensure_device_ready(bool have_stream, hipStream_t stream)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOM_ERR_HIP;
    const bool remembered = dev >= 0 && dev < kMaxDevices;
    if (remembered && g_device_ready[dev].load(std::memory_order_acquire)) return MOM_OK;
    if (have_stream) {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream, &cs) != hipSuccess) return MOM_ERR_HIP;
        if (cs != hipStreamCaptureStatusNone) return MOM_ERR_NOT_READY;
    }
    if (configure_kernels() != hipSuccess) return MOM_ERR_HIP;
    if (remembered) {
        char *ptr = nullptr;
        if (scratch_address(&ptr) != hipSuccess || !ptr) return MOM_ERR_HIP;
        g_scratch[dev] = ptr;                        // published by the release store below
        g_device_ready[dev].store(true, std::memory_order_release);
    }
    return MOM_OK;
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

// Grid of the row-wise element-wise kernels: x over groups of four columns, y over rows.
inline dim3 rowwise_grid(int rows, int cols, int rows_per_block)
{
    const int quads = (cols + 3) / 4;
    const int gx = std::max(1, std::min((quads + 255) / 256, 16));
    const int gy = std::max(1, std::min((rows + rows_per_block - 1) / rows_per_block, 16384));
    return dim3(gx, gy);
}

struct Resolved { const float *ptr; int64_t ld; };

// The evaluation proper: every check that can fail comes before the first launch.
mom_status_t eval_chain(const mom_plan_t *plan, const float *const *d_factors, const int64_t *lds, float *d_out,
                        int64_t ld_out, char *ws, uint32_t flags, hipStream_t stream)
{
    const bool zero_fill = (flags & MOM_OUT_ZERO_FILL_TRIANGLE) != 0;
    const int M = (int)plan->rows, N = (int)plan->cols;

    if (plan->survivors.empty()) {                         // I * I * ... = I
        hipLaunchKernelGGL(write_identity_kernel, rowwise_grid(M, M, 1), dim3(256), 0, stream, d_out, ld_out, M,
                           (int)aligned16(d_out, ld_out));
        return hipGetLastError() == hipSuccess ? MOM_OK : MOM_ERR_HIP;
    }
    auto factor = [&](int32_t f) {                         // packed rows of the STORED matrix by default
        return Resolved{d_factors[f], lds ? lds[f] : (plan->trans[f] ? plan->dims[f] : plan->dims[f + 1])};
    };

    if (plan->steps.empty()) {                             // one survivor: A * I -> A
        const int32_t f = plan->survivors[0];
        const Resolved a = factor(f);
        if (plan->trans[f]) {
            const int64_t blocks = (int64_t)((M + kTransposeTile - 1) / kTransposeTile) * ((N + kTransposeTile - 1) / kTransposeTile);
            hipLaunchKernelGGL(copy_transposed_kernel, dim3((unsigned)std::min<int64_t>(blocks, 1 << 20)), dim3(256), 0, stream,
                               a.ptr, a.ld, d_out, ld_out, M, N, plan->chain_props[f],
                               (int)(aligned16(a.ptr, a.ld) && aligned16(d_out, ld_out)));
        } else {
            hipLaunchKernelGGL(copy_structure_kernel, rowwise_grid(M, N, kRowUnroll), dim3(256), 0, stream, a.ptr, a.ld,
                               d_out, ld_out, M, N, plan->props[f], (int)(aligned16(a.ptr, a.ld) && aligned16(d_out, ld_out)));
        }
        if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
    }

    auto resolve = [&](const Operand &o, int64_t cols) {
        if (o.where == Where::Factor) return factor(o.index);
        if (o.where == Where::Temp)
            return Resolved{reinterpret_cast<const float *>(ws + plan->temps[o.index].offset), cols};
        return Resolved{d_out, ld_out};
    };
    // The launches were laid out with the plan; only addresses are filled in here.
    for (const PlannedLaunch &pl : plan->launches) {
        if (pl.kind == kLaunchScale) {                     // a diagonal operand: element-wise pass
            const ProductStep &st = plan->steps[pl.step[0]];
            const bool left = st.pa == kDiagonal;          // D * X, else X * D
            const Resolved d = left ? resolve(st.a, st.k) : resolve(st.b, st.n);
            const Resolved x = left ? resolve(st.b, st.n) : resolve(st.a, st.k);
            const Resolved c = resolve(st.c, st.n);
            const bool x_trans = left ? st.tb : st.ta;
            ScaleParams sp;
            sp.D = d.ptr; sp.ldd = d.ld;
            sp.X = x.ptr; sp.x_rs = x_trans ? 1 : x.ld; sp.x_cs = x_trans ? x.ld : 1;
            sp.C = const_cast<float *>(c.ptr); sp.ldc = c.ld;
            sp.M = (int)st.m; sp.N = (int)st.n; sp.side = left ? 0 : 1;
            sp.px = left ? st.pb : st.pa;
            sp.vec = !x_trans && aligned16(x.ptr, x.ld) && aligned16(c.ptr, c.ld);
            hipLaunchKernelGGL(diag_scale_kernel, rowwise_grid(sp.M, sp.N, 1), dim3(256), 0, stream, sp);
            if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
            continue;
        }
        if (pl.kind == kLaunchPair) {                      // (X * Y) * Z, narrow intermediate kept on chip
            const ProductStep &inner = plan->steps[pl.step[0]], &outer = plan->steps[pl.step[1]];
            const Resolved x = resolve(inner.a, inner.k), y = resolve(inner.b, inner.n);
            const Resolved z = resolve(outer.b, outer.n), c = resolve(outer.c, outer.n);
            SkinnyPairParams sp;
            sp.X = x.ptr; sp.Y = y.ptr; sp.Z = z.ptr; sp.C = const_cast<float *>(c.ptr);
            sp.ldx = x.ld; sp.ldy = y.ld; sp.ldz = z.ld; sp.ldc = c.ld;
            sp.M = (int)inner.m; sp.K1 = (int)inner.k; sp.W = (int)inner.n; sp.N = (int)outer.n;
            sp.x_vec = aligned16(x.ptr, x.ld); sp.c_vec = aligned16(c.ptr, c.ld);
            sp.yz_vec = ((reinterpret_cast<uintptr_t>(y.ptr) | reinterpret_cast<uintptr_t>(z.ptr)) & 7) == 0 &&
                        ((y.ld | z.ld) & 1) == 0;
            const dim3 grid((sp.M + kPairRows - 1) / kPairRows);
            if (skinny_pair_is_fast(sp))
                hipLaunchKernelGGL(skinny_pair_kernel<true>, grid, dim3(kPairThreads), kPairLdsBytes, stream, sp);
            else
                hipLaunchKernelGGL(skinny_pair_kernel<false>, grid, dim3(kPairThreads), kPairLdsBytes, stream, sp);
            if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
            continue;
        }
        ProductBatch batch = pl.batch;
        for (int i = 0; i < batch.count; ++i) {
            const ProductStep &st = plan->steps[pl.step[i]];
            ProductParams &p = batch.prob[i];
            // (the column count only matters for temporaries, which are never stored transposed)
            const Resolved a = resolve(st.a, st.k), b = resolve(st.b, st.n), c = resolve(st.c, st.n);
            // (a sub-product of the result's rows from row0 on: the same rows of A, which are columns of
            // its buffer when that holds the transpose)
            const int64_t row0 = pl.row0[i];
            p.A = a.ptr + ((pl.variant & 1) ? row0 : row0 * a.ld); p.B = b.ptr;
            p.C = const_cast<float *>(c.ptr) + row0 * c.ld;
            p.lda = a.ld; p.ldb = b.ld; p.ldc = c.ld;
            // (a row stride of 2^22 elements or more leaves the reach of the kernel's 32-bit offsets)
            p.a_vec = aligned16(a.ptr, a.ld) && a.ld < (1 << 22);
            p.b_vec = aligned16(b.ptr, b.ld) && b.ld < (1 << 22);
            p.a_word = a.ld < (1 << 22); p.b_word = b.ld < (1 << 22);
            p.a_tail = p.a_vec && ((pl.variant & 1) ? p.M : p.K) % 4 == 0;      // (bit 0 of the variant: A is stored transposed)
            p.b_tail = p.b_vec && ((pl.variant & 2) ? p.K : p.N) % 4 == 0;
            if (p.split_k > 1) {                           // partial sums go to the scratch region
                p.C = reinterpret_cast<float *>(ws + plan->scratch_offset + st.scratch_offset);
                p.ldc = st.n;
            }
            p.c_vec = aligned16(p.C, p.ldc);
        }
        bool words = false;
        for (int i = 0; i < batch.count; ++i) words = words || needs_words(batch.prob[i]);
        if (kLaunchers[pl.variant](pl.shape, words, batch, stream) != hipSuccess) return MOM_ERR_HIP;
        if (pl.reduce.count > 0) {
            ReduceBatch reduce = pl.reduce;
            for (int i = 0; i < reduce.count; ++i) {
                const int slot = pl.reduce_of[i];
                const Resolved c = resolve(plan->steps[pl.step[slot]].c, plan->steps[pl.step[slot]].n);
                reduce.prob[i].P = batch.prob[slot].C;
                reduce.prob[i].C = const_cast<float *>(c.ptr) + pl.row0[slot] * c.ld;
                reduce.prob[i].ldc = c.ld;
            }
            hipLaunchKernelGGL(reduce_slices_kernel, dim3(pl.reduce_grid_x, reduce.count), dim3(256), 0, stream, reduce);
            if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
        }
    }

    if (zero_fill && (plan->result_prop == kLower || plan->result_prop == kUpper || plan->result_prop == kDiagonal)) {
        hipLaunchKernelGGL(zero_other_half_kernel, rowwise_grid(M, M, 1), dim3(256), 0, stream, d_out, ld_out, M,
                           plan->result_prop, (int)aligned16(d_out, ld_out));
        if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
    }
    return MOM_OK;
}

// Argument checks shared by the evaluation entry points; ld_out is resolved (0 = packed).
mom_status_t check_eval_arguments(const mom_plan_t *plan, const float *const *d_factors, const int64_t *lds,
                                  const float *d_out, int64_t &ld_out, uint32_t flags)
{
    if (!plan || !d_out) return MOM_ERR_NULL;
    if (!d_factors && !plan->survivors.empty()) return MOM_ERR_NULL;
    for (int32_t f : plan->survivors)
        if (!d_factors[f]) return MOM_ERR_NULL;
    if (lds)
        for (int32_t f : plan->survivors)
            if (lds[f] < (plan->trans[f] ? plan->dims[f] : plan->dims[f + 1])) return MOM_ERR_BAD_STRIDE;
    if (ld_out == 0) ld_out = plan->cols;
    if (ld_out < plan->cols) return MOM_ERR_BAD_STRIDE;
    if (flags & ~(uint32_t)MOM_OUT_ZERO_FILL_TRIANGLE) return MOM_ERR_BAD_FLAGS;
    return MOM_OK;
}

}  // namespace

extern "C" mom_status_t mom_init(void)
{
    return ensure_device_ready(false, nullptr);
}

extern "C" mom_status_t mom_chain_eval(const mom_plan_t *plan, const float *const *d_factors, const int64_t *lds,
                                       float *d_out, int64_t ld_out, void *d_workspace, size_t workspace_bytes,
                                       uint32_t flags, void *stream_)
{
    mom_status_t st = check_eval_arguments(plan, d_factors, lds, d_out, ld_out, flags);
    if (st != MOM_OK) return st;
    if (plan->workspace_bytes > 0 &&
        (!d_workspace || workspace_bytes < plan->workspace_bytes || (reinterpret_cast<uintptr_t>(d_workspace) & 255)))
        return MOM_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    st = ensure_device_ready(true, stream);
    if (st != MOM_OK) return st;
    return eval_chain(plan, d_factors, lds, d_out, ld_out, static_cast<char *>(d_workspace), flags, stream);
}

extern "C" mom_status_t mom_chain_eval_static(const mom_plan_t *plan, const float *const *d_factors, const int64_t *lds,
                                              float *d_out, int64_t ld_out, uint32_t flags, void *stream_)
{
    mom_status_t st = check_eval_arguments(plan, d_factors, lds, d_out, ld_out, flags);
    if (st != MOM_OK) return st;
    if (plan->workspace_bytes > (size_t)MOM_STATIC_WORKSPACE_BYTES) return MOM_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    st = ensure_device_ready(true, stream);
    if (st != MOM_OK) return st;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOM_ERR_HIP;
    char *ws = nullptr;
    if (dev >= 0 && dev < kMaxDevices) {
        ws = g_scratch[dev];
    } else if (scratch_address(&ws) != hipSuccess) {   // a device beyond the remembered ones: ask every time
        return MOM_ERR_HIP;
    }
    if (!ws) return MOM_ERR_HIP;
    // nothing in the workspace has to start at zero: temporaries are written before they are
    // read and every k-slice of a split product writes its whole partial tile
    return eval_chain(plan, d_factors, lds, d_out, ld_out, ws, flags, stream);
}

// Sum of chain products: addends without products (single matrices, Identity) are summed by the
// add kernel, up to kMaxAddTerms per launch; an addend with products is evaluated by the chain
// evaluator, straight into the output when it may go first, else into a temporary that the add
// kernel then accumulates.
extern "C" mom_status_t mom_equation_eval(const mom_equation_t *eq, const float *const *d_factors, const int64_t *lds,
                                          float *d_out, int64_t ld_out, void *d_workspace, size_t workspace_bytes,
                                          uint32_t flags, void *stream_)
{
    if (!eq || !d_out) return MOM_ERR_NULL;
    if (flags & ~(uint32_t)MOM_OUT_ZERO_FILL_TRIANGLE) return MOM_ERR_BAD_FLAGS;
    if (ld_out == 0) ld_out = eq->cols;
    if (ld_out < eq->cols) return MOM_ERR_BAD_STRIDE;
    const int n_chains = (int)eq->chains.size();
    for (int c = 0; c < n_chains; ++c) {                   // every addend's own argument checks first
        const mom_plan_t *plan = eq->chains[c];
        int64_t ld = ld_out;
        const int32_t at = eq->first_factor[c];
        if (!d_factors && !plan->survivors.empty()) return MOM_ERR_NULL;
        const mom_status_t st = check_eval_arguments(plan, d_factors ? d_factors + at : nullptr, lds ? lds + at : nullptr,
                                                     d_out, ld, 0);
        if (st != MOM_OK) return st;
    }
    if (eq->workspace_bytes > 0 &&
        (!d_workspace || workspace_bytes < eq->workspace_bytes || (reinterpret_cast<uintptr_t>(d_workspace) & 255)))
        return MOM_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    mom_status_t st = ensure_device_ready(true, stream);
    if (st != MOM_OK) return st;
    char *const ws = static_cast<char *>(d_workspace);
    float *const temp = reinterpret_cast<float *>(ws + eq->temp_offset);
    const int M = (int)eq->rows, N = (int)eq->cols;

    bool written = false;                                  // does the output hold a partial sum yet?
    if (eq->direct_chain >= 0) {
        const int c = eq->direct_chain, at = eq->first_factor[c];
        st = eval_chain(eq->chains[c], d_factors + at, lds ? lds + at : nullptr, d_out, ld_out, ws, 0, stream);
        if (st != MOM_OK) return st;
        written = true;
    }
    AddParams ap{};
    auto flush = [&]() -> mom_status_t {                   // launch what has been gathered
        if (ap.count == 0 && written) return MOM_OK;
        ap.C = d_out; ap.ldc = ld_out; ap.M = M; ap.N = N; ap.pc = eq->result_prop;
        ap.accumulate = written ? 1 : 0;
        ap.c_vec = aligned16(d_out, ld_out);
        hipLaunchKernelGGL(add_terms_kernel, rowwise_grid(M, N, 1), dim3(256), 0, stream, ap);
        if (hipGetLastError() != hipSuccess) return MOM_ERR_HIP;
        written = true;
        ap.count = 0;
        return MOM_OK;
    };
    auto gather = [&](const float *ptr, int64_t ld, bool transposed, int prop) -> mom_status_t {
        const int t = ap.count++;
        ap.X[t] = ptr;
        ap.rs[t] = transposed ? 1 : ld;
        ap.cs[t] = transposed ? ld : 1;
        ap.prop[t] = prop;
        ap.vec[t] = ptr && !transposed && aligned16(ptr, ld);
        return ap.count == kMaxAddTerms ? flush() : MOM_OK;
    };
    for (int c = 0; c < n_chains; ++c) {                   // addends that are plain matrices
        const mom_plan_t *plan = eq->chains[c];
        if (!plan->steps.empty()) continue;
        if (plan->survivors.empty()) {
            st = gather(nullptr, 0, false, kIdentity);
        } else {
            const int32_t f = plan->survivors[0], at = eq->first_factor[c];
            const int64_t ld = lds ? lds[at + f] : (plan->trans[f] ? plan->dims[f] : plan->dims[f + 1]);
            st = gather(d_factors[at + f], ld, plan->trans[f] != 0, plan->chain_props[f]);
        }
        if (st != MOM_OK) return st;
    }
    for (int c = 0; c < n_chains; ++c) {                   // addends with products, through the temporary
        const mom_plan_t *plan = eq->chains[c];
        if (plan->steps.empty() || c == eq->direct_chain) continue;
        st = flush();                                      // the temporary is about to be overwritten
        if (st != MOM_OK) return st;
        const int at = eq->first_factor[c];
        st = eval_chain(plan, d_factors + at, lds ? lds + at : nullptr, temp, N, ws, 0, stream);
        if (st != MOM_OK) return st;
        st = gather(temp, N, false, plan->result_prop);
        if (st != MOM_OK) return st;
        st = flush();
        if (st != MOM_OK) return st;
    }
    st = flush();
    if (st != MOM_OK) return st;
    const int rp = eq->result_prop;
    if ((flags & MOM_OUT_ZERO_FILL_TRIANGLE) && (rp == kLower || rp == kUpper || rp == kDiagonal)) {
        hipLaunchKernelGGL(zero_other_half_kernel, rowwise_grid(M, M, 1), dim3(256), 0, stream, d_out, ld_out, M, rp,
                           (int)aligned16(d_out, ld_out));
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
