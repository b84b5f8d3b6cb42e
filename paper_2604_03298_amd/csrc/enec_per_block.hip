// The kernels for streams with one tuple per data block (see enec_per_block.hpp), one instance per
// element format and direction.
#include "enec_per_block.hpp"

namespace enec {

PbCompressFn pick_compress_per_block(int dtype)
{
    if (dtype == DT_FP16) return &compress_per_block_kernel<DT_FP16>;
    if (dtype == DT_FP32) return &compress_per_block_kernel<DT_FP32>;
    return dtype == DT_BF16 ? &compress_per_block_kernel<DT_BF16> : nullptr;
}

PbDecompressFn pick_decompress_per_block(int dtype)
{
    if (dtype == DT_FP16) return &decompress_per_block_kernel<DT_FP16>;
    if (dtype == DT_FP32) return &decompress_per_block_kernel<DT_FP32>;
    return dtype == DT_BF16 ? &decompress_per_block_kernel<DT_BF16> : nullptr;
}

}  // namespace enec
