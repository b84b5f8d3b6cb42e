// Kernel tables of libenec: one function per element format and direction that maps a tuple
// (m, a = n - m) to the kernel instance built for it (nullptr if there is none).  Each of the
// six tables is compiled as a translation unit of its own (enec_kernels.hip with
// -DENEC_DT=<format> -DENEC_DIR=<0 compress | 1 decompress>) so that the build runs in parallel.
#pragma once
#include "enec_device.hpp"

namespace enec {

using CompressFn = void (*)(const CompressArgs);
using DecompressFn = void (*)(const DecompressArgs);

CompressFn pick_compress_bf16(int m, int a);
CompressFn pick_compress_fp16(int m, int a);
CompressFn pick_compress_fp32(int m, int a);
DecompressFn pick_decompress_bf16(int m, int a);
DecompressFn pick_decompress_fp16(int m, int a);
DecompressFn pick_decompress_fp32(int m, int a);

}  // namespace enec
