// Two products in one launch when the intermediate is narrow: C = (X * Y) * Z with X (M x K1),
// Y (K1 x W), W <= 64, and Z (W x N), all general and stored as they are read.  The tiled
// kernel would run X * Y on few workgroups (M/64 tiles of 64 x 64) and then (X Y) * Z as a
// k = W product that spends its time loading, storing and starting up; here a workgroup
// keeps its 32 rows of T = X * Y in registers and multiplies them into every column strip of
// the result, so T never reaches memory and one launch replaces two.
//
// Layout trick (the one the batched kernel uses): v_mfma_f32_32x32x2_f32 is fed B-operand
// first, so register v of lane (l32, half) of an accumulator holds row l32 and the block's
// column i(v) = 8*(v/4) + 4*half + v%4.  A 64-column strip is handled as two 32-column blocks
// that INTERLEAVE: block b holds the strip's columns 2*i + b, so a lane fetches both blocks'
// operand values for one k with a single 8-byte load (columns 2*l32, 2*l32 + 1) and holds
// eight consecutive columns of its row in registers 4q .. 4q+3 of the two accumulators.
//   phase 1: T = X * Y.  The workgroup's 32 rows of X go to LDS, 512 columns at a time, with
//            coalesced 16-byte loads that are all in flight at once (read lane-per-row straight
//            from memory, a wavefront would touch 32 cache lines per load).  The four
//            wavefronts split k (groups of 8 k-values, interleaved), each accumulates a partial
//            T in two accumulators (even / odd columns of T) with Y straight from memory; the
//            partials are summed through LDS so that every wavefront holds T.  A lane then
//            owns T[l32][2*i(v) + b] for v = 0..15, b = 0, 1.
//   phase 2: since the order of summation over k is free, those 32 values ARE the A-operand
//            values of the second product when MFMA step (b, v) sums k = 2*i(v) + b; Z is
//            fetched in that same k order.  Wavefront w takes column strips w, w+4, ... (from
//            a starting point that differs between workgroups); per strip 64 MFMAs from
//            registers, Z straight from memory, the next strip requested a whole strip ahead; a
//            finished strip leaves through LDS as whole 256-byte row segments.
// Both phases are one even stream of MFMA pairs with at most one load, one LDS access and one
// store between two pairs: a wavefront is alone on its SIMD, so whatever it issues in a burst
// (sixteen loads, a strip's stores, the read-out of the accumulators) is time the matrix pipe
// idles.  Loads go two batches (a whole strip) ahead into the registers that have just been
// consumed, never behind a branch (past the end the last valid batch is fetched again and
// dropped), with fewer than 63 memory operations outstanding (the hardware counter has six
// bits).  Y, Z and the result are addressed through buffer descriptors: descriptor and uniform
// offset in scalar registers, the lane's own offset in one vector register, so that no vector
// arithmetic is spent on addresses (64-bit vector adds per access cost this kernel a tenth of
// its time).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "product_kernel.h"

namespace mom {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kPairRows = 32;            // rows of the result per workgroup
constexpr int kPairMaxWidth = 64;        // widest intermediate (two interleaved 32-column blocks)
constexpr int kPairWaves = 4;            // wavefronts per workgroup, one per SIMD
constexpr int kPairThreads = 64 * kPairWaves;
constexpr int kPairBatch = 4;            // k-groups of 8 a wavefront fetches per register set (16 loads of Y)
constexpr int kPartLd = 36;              // LDS floats per lane and wavefront (32 + pad, 16-byte aligned)
constexpr int kPairChunk = 512;          // columns of X staged in LDS at a time
constexpr int kPairXLd = kPairChunk + 4; // LDS row stride of the staged X block: 16-byte reads of 32 rows
                                         // at one k fall into distinct banks
constexpr int kPatchLd = 68;             // LDS row stride of a wavefront's 32 x 64 patch of the result
constexpr int kPairLdsFloats = kPairRows * kPairXLd > kPairWaves * 64 * kPartLd ? kPairRows * kPairXLd
                                                                                : kPairWaves * 64 * kPartLd;
constexpr int kPairLdsBytes = kPairLdsFloats * 4;      // X stage and partial sums share the space

struct SkinnyPairParams {
    const float *X, *Y, *Z;
    float *C;
    int64_t ldx, ldy, ldz, ldc;
    int M, K1, W, N;
    int x_vec, c_vec;                    // 16-byte loads of X rows / stores of C rows are legal
    int yz_vec;                          // 8-byte loads of Y and Z rows are legal
};

// FAST (chosen by the host, see skinny_pair_is_fast): whole row blocks, K1 a multiple of 8,
// W = 64, N a multiple of 64, aligned rows: no bounds checks anywhere.  The checked version
// predicates every access.
template <bool FAST>
__device__ __forceinline__ void skinny_pair_body(const SkinnyPairParams &p, float *lds)
{
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // (tells the compiler that it is uniform)
    const int row0 = blockIdx.x * kPairRows;
    // Y and Z are read at (uniform row and column) + (this lane's rows below and 2*l32 columns):
    // the lane's part sits in one pointer, everything else is scalar arithmetic
    const float *yl = p.Y + (int64_t)(4 * half) * p.ldy + 2 * l32;      // phase 1: k = 8g + 4*half + e
    const float *zl = p.Z + (int64_t)(8 * half) * p.ldz + 2 * l32;      // phase 2: k = 16q + 2r + b + 8*half
    // (FAST: all of Y, of Z and of this workgroup's rows of C lie within 2 GiB of their first byte)
    const int y_lane_bytes = (int)((4 * half) * p.ldy + 2 * l32) * 4;
    const __amdgpu_buffer_rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.Y), 0, FAST ? (int)(((int64_t)(p.K1 - 1) * p.ldy + p.W) * 4) : 0, kRawBufferFlags);
    const __amdgpu_buffer_rsrc_t c_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        p.C + (int64_t)row0 * p.ldc, 0, FAST ? (int)(((int64_t)(kPairRows - 1) * p.ldc + p.N) * 4) : 0, kRawBufferFlags);
    const int z_lane_bytes = (int)((8 * half) * p.ldz + 2 * l32) * 4;
    const __amdgpu_buffer_rsrc_t z_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.Z), 0, FAST ? (int)(((int64_t)(p.W - 1) * p.ldz + p.N) * 4) : 0, kRawBufferFlags);

    // ---- Z as phase 2 reads it: this wavefront's 64-column strips, half of the k-values (one of the two
    // interleaved blocks of T) at a time: z[v] = Z[k][strip's columns 2*l32, 2*l32 + 1] for
    // k = 2*i(v) + b = (16*(v/4) + 2*(v%4) + b) + 8*half
    const int strips = (p.N + 63) / 64;
    auto load_one = [&](int strip, int b, int v, f32x2 (&z)[16]) {
        {
            const int kc = 16 * (v / 4) + 2 * (v % 4) + b, k = kc + 8 * half;
            const float *src = zl + (int64_t)kc * p.ldz + strip * 64;         // (uniform part is scalar)
            if (FAST) {
                // buffer load: descriptor and the uniform byte offset in scalar registers, this lane's
                // offset in one vector register: no vector arithmetic per load
                const u32x2 raw = __builtin_amdgcn_raw_buffer_load_b64(z_rsrc, z_lane_bytes, (kc * (int)p.ldz + strip * 64) * 4, 0);
                z[v] = __builtin_bit_cast(f32x2, raw);
            } else if (p.yz_vec && k < p.W && strip * 64 + 2 * l32 + 2 <= p.N) {
                z[v] = *reinterpret_cast<const f32x2 *>(src);
            } else {
                z[v][0] = (k < p.W && strip * 64 + 2 * l32 < p.N) ? src[0] : 0.0f;
                z[v][1] = (k < p.W && strip * 64 + 2 * l32 + 1 < p.N) ? src[1] : 0.0f;
            }
        }
    };
    auto load_half = [&](int strip, int b, f32x2 (&z)[16]) {
#pragma unroll
        for (int v = 0; v < 16; ++v) load_one(strip, b, v, z);
    };
    const int my_strips = strips > wave ? (strips - wave + kPairWaves - 1) / kPairWaves : 0;
    const int last_strip = wave + kPairWaves * (my_strips - 1);
    // Every workgroup walks the strips from a different starting point: rows of Z are a power
    // of two apart more often than not, so the 64 rows of one strip sit in the same few L2
    // channels, and workgroups that all asked for the same strip at the same moment would queue
    // up there.
    const int rotate = blockIdx.x % strips;
    auto rotated = [&](int s) { const int r = s + rotate; return r >= strips ? r - strips : r; };
    // The first strip's part of Z is requested before anything else: it does not depend on
    // phase 1, and its way from memory is as long as that of X and Y.
    f32x2 a0[16], b0[16];
    if (my_strips > 0) {
        load_half(rotated(wave), 0, a0);
        load_half(rotated(wave), 1, b0);
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- phase 1: partial T over this wavefront's share of k
    f32x16 acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc0[v] = acc1[v] = 0.0f;
    struct Batch {
        f32x2 y[kPairBatch][4];
    };
    for (int kb = 0; kb < p.K1; kb += kPairChunk) {
        // the workgroup's rows of X, columns [kb, kb + 512), into LDS (zeros past the matrix)
        if (kb > 0) __syncthreads();                       // the previous block has been read
        // (only the columns that exist, rounded up to whole groups of 8 k-values, are staged)
        const int kc = min(kPairChunk, p.K1 - kb), quads_per_row = ((kc + 7) / 8) * 2, quads = kPairRows * quads_per_row;
#pragma unroll 4
        for (int idx = tid; idx < quads; idx += kPairThreads) {
            const int r = idx / quads_per_row, c = (idx % quads_per_row) * 4;
            const float *src = p.X + (int64_t)(row0 + r) * p.ldx + kb + c;
            f32x4 v;
            if (FAST || (p.x_vec && row0 + r < p.M && kb + c + 4 <= p.K1)) {
                v = *reinterpret_cast<const f32x4 *>(src);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (row0 + r < p.M && kb + c + e < p.K1) ? src[e] : 0.0f;
            }
            *reinterpret_cast<f32x4 *>(lds + r * kPairXLd + c) = v;
        }
        // this wavefront's k-groups of the block are wave, wave + 4, ...
        const int kgroups = (kc + 7) / 8;
        const int mine_count = kgroups > wave ? (kgroups - wave + kPairWaves - 1) / kPairWaves : 0;
        auto group_of = [&](int i) { return wave + kPairWaves * min(i, mine_count - 1); };
        auto load_y = [&](int i, int e, f32x2 &y) {        // Y: 8-byte loads, row kb + 8g + 4*half + e
            const int g = group_of(i);                     // (past the end: the last valid group again)
            if (FAST) {
                const u32x2 raw = __builtin_amdgcn_raw_buffer_load_b64(y_rsrc, y_lane_bytes, (kb + 8 * g + e) * (int)p.ldy * 4, 0);
                y = __builtin_bit_cast(f32x2, raw);
            } else {
                const float *src = yl + (int64_t)(kb + 8 * g + e) * p.ldy;
                const bool k_ok = kb + 8 * g + 4 * half + e < p.K1;
                y[0] = (k_ok && 2 * l32 < p.W) ? src[0] : 0.0f;
                y[1] = (k_ok && 2 * l32 + 1 < p.W) ? src[1] : 0.0f;
            }
        };
        auto load_batch = [&](int i0, Batch &bt) {
#pragma unroll
            for (int u = 0; u < kPairBatch; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) load_y(i0 + u, e, bt.y[u][e]);
        };
        auto read_x = [&](int i) {
            return *reinterpret_cast<const f32x4 *>(lds + l32 * kPairXLd + 8 * group_of(i) + 4 * half);
        };
        // One batch (four k-groups): the MFMAs of `cur`, every MFMA pair followed by one load of the
        // batch after next into the registers it has just consumed; the X values of the following
        // group are read one group ahead.
        // A k-group past the end is skipped (its loads fetched the last valid group again).
        auto multiply_batch = [&](int i0, Batch &cur, int n0) {
            f32x4 x = read_x(i0);
#pragma unroll
            for (int u = 0; u < kPairBatch; ++u) {
                const f32x4 x_next = read_x(u + 1 < kPairBatch ? i0 + u + 1 : n0 - kPairBatch);
                if (i0 + u < mine_count) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(cur.y[u][e][0], x[e], acc0, 0, 0, 0);
                        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(cur.y[u][e][1], x[e], acc1, 0, 0, 0);
                        load_y(n0 + u, e, cur.y[u][e]);    // (the registers just consumed take the next values)
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) load_y(n0 + u, e, cur.y[u][e]);
                }
                x = x_next;
            }
        };
        Batch b0, b1;
        if (mine_count > 0) {                              // in flight while the X block lands
            load_batch(0, b0);
            load_batch(kPairBatch, b1);
        }
        __syncthreads();
        if (mine_count > 0) {
            for (int i = 0; i < mine_count; i += 2 * kPairBatch) {
                multiply_batch(i, b0, i + 2 * kPairBatch);
                multiply_batch(i + kPairBatch, b1, i + 3 * kPairBatch);
            }
        }
    }
    __syncthreads();                                       // the X block is dead: its space takes the partial sums
    // partial sums meet in LDS: part[wave][lane][0..15] from acc0, [16..31] from acc1
    float *part = lds;
    float *mine = part + (wave * 64 + lane) * kPartLd;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const f32x4 v0 = {acc0[4 * q], acc0[4 * q + 1], acc0[4 * q + 2], acc0[4 * q + 3]};
        const f32x4 v1 = {acc1[4 * q], acc1[4 * q + 1], acc1[4 * q + 2], acc1[4 * q + 3]};
        *reinterpret_cast<f32x4 *>(mine + 4 * q) = v0;
        *reinterpret_cast<f32x4 *>(mine + 16 + 4 * q) = v1;
    }
    __syncthreads();
    // t[16b + v] = T[row l32][2*i(v) + b], summed over the wavefronts in a fixed order
    float t[32];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        f32x4 s = *reinterpret_cast<const f32x4 *>(part + (0 * 64 + lane) * kPartLd + 4 * q);
#pragma unroll
        for (int w = 1; w < kPairWaves; ++w) s += *reinterpret_cast<const f32x4 *>(part + (w * 64 + lane) * kPartLd + 4 * q);
#pragma unroll
        for (int r = 0; r < 4; ++r) t[4 * q + r] = s[r];
    }

    // ---- phase 2
    // acc[v] of block 0 / block 1: row l32, strip columns 2*i(v) / 2*i(v) + 1; registers 4q .. 4q+3
    // of both together are the eight consecutive columns 16q + 8*half .. + 7.  Stored from there,
    // one instruction would write 16-byte pieces of 32 different rows; a finished strip goes
    // through this wavefront's 32 x 64 patch of LDS instead and leaves it as whole 256-byte row
    // segments, four rows per store instruction.  That trip rides on the NEXT strip's MFMAs: two
    // accumulator sets take turns, and between two MFMA pairs there is at most one load of Z, one
    // LDS access and one store of the finished strip, so that the matrix pipe never waits for a
    // burst of other instructions, for LDS, or for the accumulators to be read out.
    __syncthreads();                                       // every wavefront has read the partial sums
    float *patch = lds + wave * (kPairRows * kPatchLd);
    // (a piece is one accumulator's four consecutive registers: every other column of eight, written
    // as two two-address LDS writes straight from the accumulator registers)
    auto stash_piece = [&](int piece, const f32x16 &d0, const f32x16 &d1) {
        const int blk = piece / 4, q = piece % 4;
        const f32x16 &d = blk ? d1 : d0;
        float *dst = patch + l32 * kPatchLd + 16 * q + 8 * half + blk;
        dst[0] = d[4 * q];
        dst[2] = d[4 * q + 1];
        dst[4] = d[4 * q + 2];
        dst[6] = d[4 * q + 3];
    };
    auto read_piece = [&](int piece) {
        return *reinterpret_cast<const f32x4 *>(patch + (4 * piece + (lane >> 4)) * kPatchLd + 4 * (lane & 15));
    };
    auto store_piece = [&](int piece, int strip, const f32x4 &v) {
        const int r = 4 * piece + (lane >> 4), c = 4 * (lane & 15), col = strip * 64 + c;
        float *dst = p.C + (int64_t)(row0 + r) * p.ldc + col;
        if (FAST) {
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), c_rsrc, (r * (int)p.ldc + c) * 4, strip * 256, 0);
        } else if (row0 + r < p.M && p.c_vec && col + 4 <= p.N) {
            *reinterpret_cast<f32x4 *>(dst) = v;
        } else if (row0 + r < p.M) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < p.N) dst[e] = v[e];
        }
    };
    if (my_strips > 0) {
        // Two pairs of register sets take turns, a strip each: the next strip's two halves are
        // requested while this strip is multiplied, a whole strip (4096 MFMA cycles) ahead of their
        // use; after the last strip it is fetched once more and dropped.
        f32x2 a1[16], b1[16];
        f32x16 set0, set1, alt0, alt1;                     // two accumulator sets of two blocks each
        const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        // Strip j into (c0, c1) while the finished strip j-1 leaves (d0, d1); have_done is false
        // for the first strip only.
        auto strip_step = [&](auto have_done, int j, const f32x2 (&ca)[16], const f32x2 (&cb)[16], f32x2 (&na)[16],
                              f32x2 (&nb)[16], f32x16 &c0, f32x16 &c1, const f32x16 &d0, const f32x16 &d1) {
            constexpr bool HAVE_DONE = decltype(have_done)::value;
            const int next = rotated(min(wave + kPairWaves * (j + 1), last_strip));
            const int done = rotated(wave + kPairWaves * (j - 1));
#pragma unroll
            for (int v = 0; v < 16; ++v) {                 // first half of k; the finished strip goes to LDS
                load_one(next, 0, v, na);
                c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(ca[v][0], t[v], v == 0 ? zero : c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(ca[v][1], t[v], v == 0 ? zero : c1, 0, 0, 0);
                if (HAVE_DONE && v >= 1 && v < 9) stash_piece(v - 1, d0, d1);
                __builtin_amdgcn_sched_barrier(0);
            }
            f32x4 piece[8];
#pragma unroll
            for (int v = 0; v < 16; ++v) {                 // second half; the finished strip goes LDS -> memory
                load_one(next, 1, v, nb);
                c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(cb[v][0], t[16 + v], c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(cb[v][1], t[16 + v], c1, 0, 0, 0);
                if (HAVE_DONE && v < 8) piece[v] = read_piece(v);
                if (HAVE_DONE && v >= 4 && v < 12) store_piece(v - 4, done, piece[v - 4]);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        using yes = std::integral_constant<bool, true>;
        using no = std::integral_constant<bool, false>;
        strip_step(no{}, 0, a0, b0, a1, b1, set0, set1, alt0, alt1);
        int j = 1;
        for (; j + 1 < my_strips; j += 2) {
            strip_step(yes{}, j, a1, b1, a0, b0, alt0, alt1, set0, set1);
            strip_step(yes{}, j + 1, a0, b0, a1, b1, set0, set1, alt0, alt1);
        }
        if (j < my_strips) {
            strip_step(yes{}, j, a1, b1, a0, b0, alt0, alt1, set0, set1);
            ++j;
        }
        // the last strip: strip j-1 sits in the first set when j is odd
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (j & 1) stash_piece(i, set0, set1);
            else stash_piece(i, alt0, alt1);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) store_piece(i, rotated(last_strip), read_piece(i));
    }
}

// Four wavefronts, one per SIMD: a workgroup overlaps its own loads, MFMAs and stores, and
// two workgroups share a compute unit when there are more than the chip has units.
template <bool FAST>
__global__ __launch_bounds__(kPairThreads, 1) void skinny_pair_kernel(const SkinnyPairParams p)
{
    extern __shared__ __align__(16) float pair_lds[];
    skinny_pair_body<FAST>(p, pair_lds);
}

// FAST needs: aligned rows of X, Y, Z and C, M a multiple of 32, K1 of 8, N of 64, W = 64; Y, Z and 32 rows of C within 2 GiB each.
inline bool skinny_pair_is_fast(const SkinnyPairParams &p)
{
    return p.x_vec && p.c_vec && p.yz_vec && p.M % kPairRows == 0 && p.K1 % 8 == 0 && p.W == kPairMaxWidth &&
           p.N % 64 == 0 && ((int64_t)(p.W - 1) * p.ldz + p.N) * 4 < (int64_t)1 << 31 &&
           ((int64_t)(p.K1 - 1) * p.ldy + p.W) * 4 < (int64_t)1 << 31 &&
           ((int64_t)(kPairRows - 1) * p.ldc + p.N) * 4 < (int64_t)1 << 31;
}

}  // namespace mom
