// One translation unit per combination of stored-transposed operands: each instantiates the
// product kernel for both tile shapes and exports a launcher and the one-time attribute set-up.
#pragma once
#include <hip/hip_runtime.h>

#include "launch_params.h"

namespace mom {

// (ta, tb) -> variant index
enum ProductVariant : int { kVariantNN = 0, kVariantTN = 1, kVariantNT = 2, kVariantTT = 3, kNumVariants };
inline int product_variant(bool ta, bool tb) { return (ta ? 1 : 0) + (tb ? 2 : 0); }

// words: some operand of the batch has to be loaded 4 bytes at a time somewhere (see needs_words)
typedef hipError_t (*ProductLauncher)(int shape, bool words, const ProductBatch &batch, hipStream_t stream);
typedef hipError_t (*ProductConfigurer)();

hipError_t launch_product_nn(int shape, bool words, const ProductBatch &batch, hipStream_t stream);
hipError_t launch_product_tn(int shape, bool words, const ProductBatch &batch, hipStream_t stream);
hipError_t launch_product_nt(int shape, bool words, const ProductBatch &batch, hipStream_t stream);
hipError_t launch_product_tt(int shape, bool words, const ProductBatch &batch, hipStream_t stream);
hipError_t configure_product_nn();
hipError_t configure_product_tn();
hipError_t configure_product_nt();
hipError_t configure_product_tt();

// Does the product need the kernel instance that can load 4 bytes at a time?  (An operand whose
// rows are not 16-byte aligned, or whose contiguous extent is not a multiple of four while some
// tile pokes over an edge; a row stride out of reach of 32-bit offsets takes the element-wise
// path, which every instance has.)
inline bool needs_words(const ProductParams &p)
{
    return (p.a_word && !(p.a_vec && p.a_tail)) || (p.b_word && !(p.b_vec && p.b_tail));
}

}  // namespace mom

// 128x128 tiles, 4 wavefronts of 64x64, two workgroups per compute unit: the workhorse.
// 64x64 tiles, 4 wavefronts of 32x32, four or more per compute unit: products with a short side.
#define MOM_DEFINE_PRODUCT_VARIANT(NAME, TA, TB)                                                                     \
    namespace mom {                                                                                                  \
    namespace {                                                                                                      \
    typedef TileConfig<128, 128, kChunk128, 2, 2, 2, TA, TB, false> Tile128;                                         \
    typedef TileConfig<64, 64, kChunk64, 2, 2, 4, TA, TB, false> Tile64;                                             \
    typedef TileConfig<128, 128, kChunk128, 2, 2, 2, TA, TB, true> Tile128W;                                         \
    typedef TileConfig<64, 64, kChunk64, 2, 2, 4, TA, TB, true> Tile64W;                                             \
    template <class T>                                                                                               \
    hipError_t launch_one(const ProductBatch &batch, hipStream_t stream)                                             \
    {                                                                                                                \
        hipLaunchKernelGGL(product_kernel<T>, dim3(batch.block_end[batch.count - 1]), dim3(T::NT), T::LDS_BYTES,     \
                           stream, batch);                                                                           \
        return hipGetLastError();                                                                                    \
    }                                                                                                                \
    template <class T>                                                                                               \
    hipError_t raise_lds_limit()                                                                                     \
    {                                                                                                                \
        return hipFuncSetAttribute(reinterpret_cast<const void *>(&product_kernel<T>),                               \
                                   hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);                        \
    }                                                                                                                \
    }                                                                                                                \
    hipError_t launch_product_##NAME(int shape, bool words, const ProductBatch &batch, hipStream_t stream)           \
    {                                                                                                                \
        if (words)                                                                                                   \
            return shape == kTile128 ? launch_one<Tile128W>(batch, stream) : launch_one<Tile64W>(batch, stream);     \
        return shape == kTile128 ? launch_one<Tile128>(batch, stream) : launch_one<Tile64>(batch, stream);           \
    }                                                                                                                \
    hipError_t configure_product_##NAME()                                                                            \
    {                                                                                                                \
        hipError_t e = raise_lds_limit<Tile128>();                                                                   \
        if (e == hipSuccess) e = raise_lds_limit<Tile64>();                                                          \
        if (e == hipSuccess) e = raise_lds_limit<Tile128W>();                                                        \
        return e != hipSuccess ? e : raise_lds_limit<Tile64W>();                                                     \
    }                                                                                                                \
    }
