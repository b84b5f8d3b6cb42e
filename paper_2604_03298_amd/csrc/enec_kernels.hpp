// Kernel tables of libenec: one function per element format, group length and direction that maps
// a tuple (m, a = n - m) to the kernel instance built for it (nullptr if there is none).  Each of
// the 18 tables is compiled as a translation unit of its own (enec_kernels.hip with
// -DENEC_DT=<format 0|1|2> -DENEC_LPG=<lanes per group 1|2|4> -DENEC_DIR=<0 compress | 1 decompress>)
// so that the build runs in parallel.
#pragma once
#include "enec_device.hpp"

namespace enec {

using CompressFn = void (*)(const CompressArgs);
using DecompressFn = void (*)(const DecompressArgs);

#define ENEC_TABLES(dt)                               \
    CompressFn pick_compress_##dt##_lpg1(int m, int a);   \
    CompressFn pick_compress_##dt##_lpg2(int m, int a);   \
    CompressFn pick_compress_##dt##_lpg4(int m, int a);   \
    DecompressFn pick_decompress_##dt##_lpg1(int m, int a); \
    DecompressFn pick_decompress_##dt##_lpg2(int m, int a); \
    DecompressFn pick_decompress_##dt##_lpg4(int m, int a);
ENEC_TABLES(dt0)
ENEC_TABLES(dt1)
ENEC_TABLES(dt2)
#undef ENEC_TABLES

}  // namespace enec
