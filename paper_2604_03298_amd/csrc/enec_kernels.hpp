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

// Streams with one tuple per data block (enec_per_block.hpp, compiled in enec_per_block.hip): the
// widths are run-time values there, one kernel per element format, group length and direction.
// LDS copies of the block histogram in the compress kernel, and their distance in words
constexpr uint32_t PB_HIST_COPIES = 16, PB_HIST_STRIDE = 257;   // words; 16 * 257 * 4 bytes of LDS

// Data blocks are handed out by tickets (see the compress kernel): PB_TICKET_CLASSES counters,
// PB_TICKET_STRIDE 32-bit words apart (a cache line each)
constexpr uint32_t PB_TICKET_CLASSES = 8, PB_TICKET_STRIDE = 16;

struct PbCompressItem {         // one tensor of a launch
    const void *in;
    uint8_t *out;
    unsigned long long *out_bytes;
    uint64_t *words;            // nb look-back words, zero at launch
    uint64_t n_elems;
    uint64_t tuples_at;         // byte offset of the tuple table in the stream
    uint64_t tail_base;         // fp32: where the lower halves go
    uint64_t payload_base;
    uint32_t nb;
    uint32_t first;             // number of its first data block; the blocks of a call are numbered through
};

struct PbCompressArgs {
    PbCompressItem item[MAX_BATCH];
    uint32_t *ticket;           // PB_TICKET_CLASSES counters, zero before the call's first launch
    uint32_t n_items;
    uint32_t first_block;       // this launch codes blocks first_block .. first_block + n_blocks - 1
    uint32_t n_blocks;
    uint32_t B, logB, spin_limit;
    uint32_t park_at;           // byte offset in the dynamic LDS where raw bytes wait (behind the image)
};
constexpr int PB_SM_REG_ROWS = 4;               // rows of a thread's raw bytes kept in registers; the other rows wait in LDS

struct PbDecompressItem {       // one stream of a launch
    const uint8_t *in;
    void *out;
    uint64_t n_elems;
    uint64_t tuples_at, tail_base, payload_base, payload_bytes;
    uint32_t nb;
    uint32_t first;             // number of its first data block among the blocks of the launch
    uint32_t *status;           // device-accessible or null: set to 7 (format error) when a block is left undecoded
    uint32_t hdr[11];           // the header the launch was configured from
};

struct PbDecompressArgs {
    PbDecompressItem item[MAX_BATCH];
    uint32_t n_items, n_blocks;
    uint32_t B, logB;
};

using PbCompressFn = void (*)(const PbCompressArgs);
using PbDecompressFn = void (*)(const PbDecompressArgs);
PbCompressFn pick_compress_per_block(int dtype, unsigned L);
PbDecompressFn pick_decompress_per_block(int dtype, unsigned L);

}  // namespace enec
