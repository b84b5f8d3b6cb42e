// The kernels for streams with one tuple per data block (see enec_per_block.hpp), one instance per
// element format, group length and direction.
#include "enec_per_block.hpp"

namespace enec {

template <int DT>
static PbCompressFn compress_for(unsigned L)
{
    if (L == 8) return &compress_per_block_kernel<DT, 1>;
    if (L == 32) return &compress_per_block_kernel<DT, 4>;
    return L == 16 ? &compress_per_block_kernel<DT, 2> : nullptr;
}

template <int DT>
static PbDecompressFn decompress_for(unsigned L)
{
    if (L == 8) return &decompress_per_block_kernel<DT, 1>;
    if (L == 32) return &decompress_per_block_kernel<DT, 4>;
    return L == 16 ? &decompress_per_block_kernel<DT, 2> : nullptr;
}

PbCompressFn pick_compress_per_block(int dtype, unsigned L)
{
    if (dtype == DT_FP16) return compress_for<DT_FP16>(L);
    if (dtype == DT_FP32) return compress_for<DT_FP32>(L);
    return dtype == DT_BF16 ? compress_for<DT_BF16>(L) : nullptr;
}

PbDecompressFn pick_decompress_per_block(int dtype, unsigned L)
{
    if (dtype == DT_FP16) return decompress_for<DT_FP16>(L);
    if (dtype == DT_FP32) return decompress_for<DT_FP32>(L);
    return dtype == DT_BF16 ? decompress_for<DT_BF16>(L) : nullptr;
}

}  // namespace enec
