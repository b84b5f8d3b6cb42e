// Device code of libenec: the ENEC codec (bf16, fp16, fp32 tensors) on CDNA4 (gfx950), wave64.
//
// Thread mapping (both directions).  A data block of B elements is seen as 8 rows of
// C = B/8 columns: element c + t*C is row t, column c.  Alg. 2 (hierarchical halving
// bit-packing, Sec. V-B) over a whole block only ever combines elements of one column,
// and the a bytes it produces for a column do not depend on B: its "normalized bytes"
// are a planes of C bytes, plane-major.  So a thread that owns 8 adjacent columns
//   * reads / writes, for each row, one 128-bit vector of 8 bf16 (fully coalesced),
//   * packs its 8 columns in registers with byte-lane SIMD-within-a-register
//     arithmetic (4 columns per 32-bit register),
//   * owns half of a group of 16 consecutive elements per row; the two halves sit in
//     adjacent lanes and are combined with one DPP operation.  (Template parameter LPG =
//     lanes per group: 1, 2 or 4 for group lengths 8, 16, 32; Eq. 4 searches the length.)
// A workgroup has B/64 threads (256 for the default B = 16384) and handles one block.
//
// Element formats (template parameter DT).  Only the exponent field is coded (Sec. VI-B);
// every format is first split into an exponent byte X and the raw byte sign<<7 | first seven
// mantissa bits, after which the three formats share all code:
//   DT_BF16  1|8|7   nothing is left over
//   DT_FP16  1|5|10  the last three mantissa bits ride on top of the m low bits of y in the low
//                    plane, which is therefore m + 3 bits wide
//   DT_FP32  1|8|23  the upper half of an element is a bf16 word; the lower halves are copied
//                    to a region between the offset table and the payloads, at positions that
//                    do not depend on any compressed size
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

// Three waves per SIMD for the compression kernel: the register budget (168) that lets three
// workgroups of 256 threads share a CU.  The 16-bit formats fit it once the waiting block's
// sign/mantissa bytes are parked in LDS (all group lengths; the layer with L = 8: 0.177 -> 0.154 ms,
// with L = 32: 0.207 -> 0.181 ms against two waves with the bytes in registers).  The fp32 instances
// (twice the row registers) spill at that budget and run faster with two.
#ifndef ENEC_COMPRESS_OCCUPANCY
#define ENEC_COMPRESS_WAVES (compress_sm_in_lds(DT, LPG) ? 3 : 2)
#define ENEC_COMPRESS_OCCUPANCY __attribute__((amdgpu_waves_per_eu(ENEC_COMPRESS_WAVES, ENEC_COMPRESS_WAVES)))
#endif

namespace enec {

constexpr int DT_BF16 = 0, DT_FP16 = 1, DT_FP32 = 2;
constexpr int low_plane_bits(int m, int dt) { return m + (dt == DT_FP16 ? 3 : 0); }
constexpr uint32_t exponent_bits(int dt) { return dt == DT_FP16 ? 5u : 8u; }
// the compress instances that run three waves per SIMD (the 16-bit formats) and therefore park the
// waiting block's sign/mantissa bytes in LDS; the others get two waves
constexpr bool compress_sm_in_lds(int dt, int /*lpg*/) { return dt != DT_FP32; }

// ---------------------------------------------------------------------------------
// Compile-time bit map of Alg. 2 for one column (8 values of W bits -> W bytes).
// A "field" says: bits of row t land in byte `plane` at a constant bit offset.
// ---------------------------------------------------------------------------------
struct HHTable {
    int count;
    int plane[64];
    int row[64];
    int shift[64];        // destination bit - source bit (may be negative)
    unsigned dmask[64];   // destination bits inside the byte
    bool clean[64];       // whole W-bit value fits without spilling into the next byte
};

template <int W>
constexpr HHTable make_hh_table()
{
    HHTable T{};
    int lab[8][16] = {};
    for (int i = 0; i < 8; ++i)
        for (int k = 0; k < 16; ++k) lab[i][k] = (k < W) ? i * 8 + k : -1;
    int width = W, length = 8, planes = 0, n = 0;
    while (width > 0) {
        while (length > 1 && width < 8) {
            length /= 2;
            for (int i = 0; i < length; ++i)
                for (int k = 0; k < width; ++k) lab[i][width + k] = lab[i + length][k];
            width *= 2;
        }
        for (int j = 0; j < length; ++j) {
            for (int t = 0; t < 8; ++t) {
                int shift = 0;
                unsigned dmask = 0, smask = 0;
                for (int k = 0; k < 8; ++k)
                    if (lab[j][k] >= 0 && lab[j][k] / 8 == t) {
                        int sb = lab[j][k] % 8;
                        shift = k - sb;
                        dmask |= 1u << k;
                        smask |= 1u << sb;
                    }
                if (dmask) {
                    T.plane[n] = planes + j;
                    T.row[n] = t;
                    T.shift[n] = shift;
                    T.dmask[n] = dmask;
                    T.clean[n] = (smask == ((1u << W) - 1u)) && shift >= 0 && shift + W <= 8;
                    ++n;
                }
            }
            for (int k = 0; k < 8; ++k) lab[j][k] = lab[j][k + 8];
            for (int k = 8; k < 16; ++k) lab[j][k] = -1;
        }
        planes += length;
        width -= 8;
    }
    T.count = n;
    return T;
}

template <int W> struct HH { static constexpr HHTable table = make_hh_table<W>(); };

__device__ __forceinline__ uint32_t shl_or_shr(uint32_t v, int s)
{
    return s >= 0 ? (v << s) : (v >> (-s));
}

// ---------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t byte_perm(uint32_t hi, uint32_t lo, uint32_t sel)
{
    // selector byte i picks output byte i: 0-3 = bytes of lo, 4-7 = bytes of hi
    return __builtin_amdgcn_perm(hi, lo, sel);
}

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b)
{
    return (a & mask) | (b & ~mask);
}

// per-byte (a - b) mod 256 without borrows between bytes
__device__ __forceinline__ uint32_t bytesub_safe(uint32_t a, uint32_t b)
{
    const uint32_t H = 0x80808080u;
    return ((a | H) - (b & ~H)) ^ ((a ^ ~b) & H);
}

// value of the neighbouring lane (lane ^ 1), one DPP move
__device__ __forceinline__ uint32_t swap_pair(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, false);
}

// keep the even bits of x, packed into 32 bits (wave-uniform: runs on the scalar unit)
__device__ __forceinline__ uint32_t compact_even_bits(uint64_t x)
{
    x &= 0x5555555555555555ull;
    x = (x | (x >> 1)) & 0x3333333333333333ull;
    x = (x | (x >> 2)) & 0x0F0F0F0F0F0F0F0Full;
    x = (x | (x >> 4)) & 0x00FF00FF00FF00FFull;
    x = (x | (x >> 8)) & 0x0000FFFF0000FFFFull;
    x = (x | (x >> 16)) & 0x00000000FFFFFFFFull;
    return (uint32_t)x;
}

// keep every fourth bit of x, packed into 16 bits
__device__ __forceinline__ uint32_t compact_fourth_bits(uint64_t x)
{
    x &= 0x1111111111111111ull;
    x = (x | (x >> 3)) & 0x0303030303030303ull;
    x = (x | (x >> 6)) & 0x000F000F000F000Full;
    x = (x | (x >> 12)) & 0x000000FF000000FFull;
    x = (x | (x >> 24)) & 0x000000000000FFFFull;
    return (uint32_t)x;
}

// OR over the four lanes of a quad, two DPP moves
__device__ __forceinline__ uint32_t quad_or(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, false);
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E /* quad_perm [2,3,0,1] */, 0xF, 0xF, false);
    return v;
}

// inclusive prefix sum over the 64 lanes with data-parallel-primitive moves: four shifts inside
// each row of 16 lanes, then the last lane of a row is broadcast into the next row (rows 1 and 3)
// and the last lane of the lower half into the upper half.  Six dependent VALU operations; the
// same through ds_bpermute (__shfl_up) is six round trips to the LDS crossbar.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, uint32_t /*lane*/)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111 /* row_shr:1 */, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112 /* row_shr:2 */, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114 /* row_shr:4 */, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118 /* row_shr:8 */, 0xF, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142 /* row_bcast:15 */, 0xA, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143 /* row_bcast:31 */, 0xC, 0xF, false);
    return v;
}

// Value of `v` in lane `idx`.  A thread's group of row t lies in mask word (index of the group) / 32;
// for groups of 16 and 32 elements that word index is the same for all lanes of a wave (it depends
// on t and on the wave's number only), so one v_readlane with a scalar index fetches it; for groups
// of 8 the two halves of a wave look at different words and the LDS crossbar is asked.
template <int LPG>
__device__ __forceinline__ uint32_t mask_word_lane(uint32_t v, uint32_t idx)
{
    if constexpr (LPG == 1) return (uint32_t)__shfl((int)v, (int)idx, 64);
    else return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)__builtin_amdgcn_readfirstlane((int)idx));
}

// sum over the 64 lanes of values whose total fits 32 bits, in every lane
__device__ __forceinline__ uint32_t wave_sum32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan(v, 0), 63);
}

__device__ __forceinline__ uint64_t wave_sum(uint64_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)v, d, 64);
        const uint32_t hi = __shfl_xor((uint32_t)(v >> 32), d, 64);
        v += ((uint64_t)hi << 32) | lo;
    }
    return v;
}

// ---------------------------------------------------------------------------------
// Inter-block scan (Fig. 4: prefix sums of per-block compressed sizes) and work distribution.
//
// Scan state.  Block and group words are self-contained: [63:24] tag of the call that wrote it,
// [23] range error, [22:0] a size in units of 16 bytes.  Relaxed device-scope loads and stores
// are enough, no fence is needed, and they are never cleared: a word whose tag is not the
// current call's tag is simply "not published yet".
//   block word k   size of data block k, stored as soon as the block's mask is known
//   group word g   sum of the sizes of the GROUP blocks of group g
//   accumulator g  [63:48] blocks counted, [47:32] of them with a range error, [31:0] sum of
//                  their sizes; zero between calls.  Every block adds itself with one atomic; the
//                  workgroup whose addition completes the group stores the group word and zeroes
//                  the accumulator.  So a group word appears as soon as its last block is known
//                  and no workgroup ever waits for blocks of its own generation (a designated
//                  owner polling the other blocks of its group turned the loop latency-bound as
//                  soon as the blocks took equal time and the workgroups ran in lockstep).
// The start of block k is the sum of the group words below its group plus the block words of the
// earlier blocks of its own group: few words, read by one wave.
//
// Work distribution.  The grid is persistent (at most as many workgroups as the device holds at
// once).  Data blocks are dealt into `ncls` classes, block k belongs to class k mod ncls, and
// class c is served only by the workgroups with blockIdx mod ncls == c, which draw its blocks
// in increasing order from the class's ticket counter.  A workgroup therefore holds blocks in
// increasing order and publishes a block's size before it waits for anything, so the lowest
// unpublished block is always held by (or next in line for) a workgroup that is not waiting for
// it: the scan cannot deadlock.  Eight classes keep the rate of atomics on one address (about
// 12 ns each on MI355X) far below the block rate.
//
// Pipelining.  A workgroup stores block i-1 only while it is working on block i: by then the
// sizes of all earlier blocks were published an iteration ago, so the reads of the scan state
// succeed at the first attempt and nobody spins on hot cache lines in the steady state.
//
// Control record of class c (WS_STRIDE words apart): [0] ticket counter, never reset; [1] value
// of the counter when the current call started; [2..3] tag of the last finished call; class 0 also
// [4..5] tag of the last call in which a workgroup gave up waiting for the scan: whoever writes a
// header looks at it, so that a give-up anywhere in the launch turns every header of the launch
// into status ENEC_E_HIP (the block that gave up was stored at a start computed from a partial sum).  A class
// with L blocks and W workgroups sees exactly L + W draws per call (every workgroup draws until
// its first draw beyond L), so the workgroup that receives draw number L + W - 1 knows that
// nobody will touch the record again in this call and writes the next call's base and tag.
// ---------------------------------------------------------------------------------
constexpr uint64_t ST_ERR = 1ull << 23;
constexpr uint64_t ST_VALUE = (1ull << 23) - 1;
constexpr uint32_t SPIN_LIMIT = 1u << 20;      // default of CompressArgs::spin_limit: seconds, far beyond any real wait
constexpr uint32_t NO_BLOCK = 0xFFFFFFFFu;
constexpr uint32_t WS_STRIDE = 32;            // control records sit 128 bytes apart
constexpr uint32_t WS_CLASSES = 8;
// blocks per scan group: with G blocks a start costs G - 1 block words plus (blocks in flight) / G
// group words, and G additions meet on one accumulator at about 12 ns each
constexpr uint32_t GROUP_LOG = 3, GROUP = 1u << GROUP_LOG;

__device__ __forceinline__ uint64_t ld_state(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_state(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void spin_pause(uint32_t spins)
{
    if (spins < 4) __builtin_amdgcn_s_sleep(4);
    else if (spins < 16) __builtin_amdgcn_s_sleep(16);
    else __builtin_amdgcn_s_sleep(64);
}

// One launch handles up to MAX_BATCH tensors that share (m, n - m, block size): their data blocks
// form one global sequence (tensor after tensor), item[i].first is the global index of tensor i's
// first block.
constexpr int MAX_BATCH = 16;

struct CompressItem {
    const uint16_t *in;
    uint8_t *out;
    uint64_t *out_bytes;    // device-accessible or null
    uint64_t *ws_block;     // nb block words
    uint64_t *ws_group;     // ceil(nb / GROUP) group words
    uint64_t *ws_acc;       // ceil(nb / GROUP) group accumulators, zero between calls
    uint64_t n_elems;
    uint64_t payload_base;
    uint32_t nb, first;
    uint32_t b, mode;       // mode 0: window clear of 0 and 255; 1: n = exponent width; 2: window touches an end
    uint64_t tail_base;     // fp32: where the lower halves of the elements go
};

struct CompressArgs {
    uint32_t *ws_ctl;       // WS_CLASSES control records
    uint32_t B, logB;
    uint32_t total;         // data blocks of all items
    uint32_t ncls;          // number of block classes = min(8, gridDim.x)
    uint32_t lookahead;     // draw the next ticket while working on the current block
    uint32_t n_items;
    uint32_t spin_limit;    // polls of the scan state after which a workgroup gives up (status ENEC_E_HIP)
    CompressItem item[MAX_BATCH];
};

struct DecompressItem {
    const uint8_t *in;
    uint16_t *out;
    uint64_t n_elems;
    uint64_t payload_base;
    uint64_t payload_bytes; // total_bytes - payload_base
    uint64_t tail_base;     // fp32: where the lower halves of the elements are
    uint32_t nb, first;
    uint32_t b, mode;       // mode 0: plain byte subtract is exact; 1: borrow-safe subtract
    uint32_t hdr[10];       // first 40 bytes of the expected header
    uint32_t *status;       // device-accessible or null: set to 7 (format error) when a block is left undecoded
};

struct DecompressArgs {
    uint32_t B, logB;
    uint32_t total;
    uint32_t n_items;
    DecompressItem item[MAX_BATCH];
};

// ---------------------------------------------------------------------------------
// a5: one record per masked group (Sec. V-B: the high n - m bits of a group that needs them, packed by
// Alg. 2 with N = L), written into the LDS image at the group's rank among the block's masked groups.
// HI[t][h] = high parts of this thread's eight elements of row t in byte lanes; my_word / my_excl = the
// wave's copy of the mask words and of their exclusive popcount prefix.  Shared by the kernels for one
// tuple per tensor and for one tuple per data block.
// ---------------------------------------------------------------------------------
template <int A, int LPG>
__device__ __forceinline__ void pack_records(const uint32_t (&HI)[8][2], uint32_t my_word, uint32_t my_excl,
                                             uint8_t *img_high, uint32_t logC, uint32_t tid, bool active)
{
    constexpr HHTable TH = HH<A>::table;
    constexpr uint32_t RB = A * LPG;                     // bytes of one record: (n - m) L / 8
    if constexpr (LPG == 1) {
        // A group is this lane's 8 elements of a row, and Alg. 2 with N = 8 is the column map
        // itself.  The lane's 8 x 8 bytes (row = group, byte = element) are transposed, so that
        // one register holds the same element of four groups and the eight groups are packed at
        // once in byte lanes; A normalized bytes per group are then joined (byte i with byte
        // i + ceil(A/2)), the pad byte of an odd count is dropped.
        constexpr int HALF = (A + 1) / 2;
        uint32_t T[8][2];                 // T[element][k]: groups 4k .. 4k+3
#pragma unroll
        for (int k = 0; k < 2; ++k)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t r0 = HI[4 * k][h], r1 = HI[4 * k + 1][h], r2 = HI[4 * k + 2][h], r3 = HI[4 * k + 3][h];
                const uint32_t lo01 = byte_perm(r1, r0, 0x05010400u), hi01 = byte_perm(r1, r0, 0x07030602u);
                const uint32_t lo23 = byte_perm(r3, r2, 0x05010400u), hi23 = byte_perm(r3, r2, 0x07030602u);
                T[4 * h][k] = byte_perm(lo23, lo01, 0x05040100u);
                T[4 * h + 1][k] = byte_perm(lo23, lo01, 0x07060302u);
                T[4 * h + 2][k] = byte_perm(hi23, hi01, 0x05040100u);
                T[4 * h + 3][k] = byte_perm(hi23, hi01, 0x07060302u);
            }
        uint32_t P[A + 1][2];            // normalized byte q of groups 4k .. 4k+3 (P[A] = the pad)
#pragma unroll
        for (int q = 0; q <= A; ++q) P[q][0] = P[q][1] = 0;
#pragma unroll
        for (int f = 0; f < TH.count; ++f)
#pragma unroll
            for (int k = 0; k < 2; ++k)
                P[TH.plane[f]][k] |= shl_or_shr(T[TH.row[f]][k], TH.shift[f]) & (TH.dmask[f] * 0x01010101u);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint32_t g = ((uint32_t)t << (logC - 3)) + tid;
            const uint32_t wv = mask_word_lane<LPG>(my_word, g >> 5);
            const uint32_t pre = mask_word_lane<LPG>(my_excl, g >> 5);
            if (active && ((wv >> (g & 31u)) & 1u)) {
                const uint32_t rank = pre + __popc(wv & ((1u << (g & 31u)) - 1u));
                uint8_t *dst = img_high + RB * rank;
#pragma unroll
                for (int j = 0; j < A; ++j)
                    dst[j] = (uint8_t)(P[(j & 1) ? (j >> 1) + HALF : (j >> 1)][t >> 2] >> (8 * (t & 3)));
            }
        }
    } else if constexpr (LPG == 2) {
        const uint32_t par = tid & 1u;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // even lanes pack the group of row 2u, odd lanes the group of row 2u+1
            const uint32_t own0 = par ? HI[2 * u + 1][0] : HI[2 * u][0];
            const uint32_t own1 = par ? HI[2 * u + 1][1] : HI[2 * u][1];
            const uint32_t snd0 = par ? HI[2 * u][0] : HI[2 * u + 1][0];
            const uint32_t snd1 = par ? HI[2 * u][1] : HI[2 * u + 1][1];
            const uint32_t rcv0 = swap_pair(snd0);
            const uint32_t rcv1 = swap_pair(snd1);
            uint32_t F[4];
            F[0] = par ? rcv0 : own0;
            F[1] = par ? rcv1 : own1;
            F[2] = par ? own0 : rcv0;
            F[3] = par ? own1 : rcv1;
            const uint32_t g = ((2u * u + par) << (logC - 4)) + (tid >> 1);
            // even and odd lanes look at the groups of two rows: two wave-uniform word indices
            const uint32_t w_even = (((2u * u) << (logC - 4)) + (tid >> 1)) >> 5;
            const uint32_t w_odd = (((2u * u + 1u) << (logC - 4)) + (tid >> 1)) >> 5;
            const uint32_t wv_e = mask_word_lane<LPG>(my_word, w_even), wv_o = mask_word_lane<LPG>(my_word, w_odd);
            const uint32_t pre_e = mask_word_lane<LPG>(my_excl, w_even), pre_o = mask_word_lane<LPG>(my_excl, w_odd);
            const uint32_t wv = par ? wv_o : wv_e;
            const uint32_t pre = par ? pre_o : pre_e;
            const uint32_t bit = (wv >> (g & 31u)) & 1u;
            if (active && bit) {
                const uint32_t rank = pre + __popc(wv & ((1u << (g & 31u)) - 1u));
                // the group's 16 values are 2 columns of 8 rows: row r = bytes (2r, 2r+1)
                uint32_t P[A];
#pragma unroll
                for (int q = 0; q < A; ++q) P[q] = 0;
#pragma unroll
                for (int f = 0; f < TH.count; ++f) {
                    const int r = TH.row[f];
                    const uint32_t s = shl_or_shr(F[r >> 1], TH.shift[f] - 16 * (r & 1));
                    P[TH.plane[f]] |= s & (TH.dmask[f] * 0x0101u);
                }
                // normalized byte j = byte (j & 1) of P[j >> 1]; stream word i = nb[i] | nb[i + A] << 8
                uint16_t *dst = reinterpret_cast<uint16_t *>(img_high + 2u * A * rank);
#pragma unroll
                for (int i = 0; i < A; ++i) {
                    const uint32_t lo = (P[i >> 1] >> (8 * (i & 1))) & 0xFFu;
                    const uint32_t hi = (P[(i + A) >> 1] >> (8 * ((i + A) & 1))) & 0xFFu;
                    dst[i] = (uint16_t)(lo | (hi << 8));
                }
            }
        }
    } else {
        // a group is the 32 elements of a quad: seen as 8 rows of 4 columns (element i = row i / 4,
        // column i % 4) Alg. 2's folds again stay inside a column; lane j holds rows 2j and 2j+1
        const uint32_t j = tid & 3u;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint32_t g = ((uint32_t)t << (logC - 5)) + (tid >> 2);
            const uint32_t wv = mask_word_lane<LPG>(my_word, g >> 5);
            const uint32_t pre = mask_word_lane<LPG>(my_excl, g >> 5);
            if (active && ((wv >> (g & 31u)) & 1u)) {
                const uint32_t rank = pre + __popc(wv & ((1u << (g & 31u)) - 1u));
                uint32_t P[A];
#pragma unroll
                for (int q = 0; q < A; ++q) P[q] = 0;
#pragma unroll
                for (int f = 0; f < TH.count; ++f) {
                    const int r = TH.row[f];
                    const uint32_t c = shl_or_shr(HI[t][r & 1], TH.shift[f]) & (TH.dmask[f] * 0x01010101u);
                    P[TH.plane[f]] |= ((uint32_t)(r >> 1) == j) ? c : 0u;
                }
#pragma unroll
                for (int q = 0; q < A; ++q) P[q] = quad_or(P[q]);
                if (j == 0) {
                    // normalized byte 4q + c = byte c of P[q]; stream word i = nb[i] | nb[i + 2A] << 8
                    uint32_t *dst = reinterpret_cast<uint32_t *>(img_high + RB * rank);
#pragma unroll
                    for (int k = 0; k < A; ++k) {
                        const int i0 = 2 * k, i1 = 2 * k + 1, h0 = i0 + 2 * A, h1 = i1 + 2 * A;
                        const uint32_t b0 = (P[i0 >> 2] >> (8 * (i0 & 3))) & 0xFFu;
                        const uint32_t b1 = (P[h0 >> 2] >> (8 * (h0 & 3))) & 0xFFu;
                        const uint32_t b2 = (P[i1 >> 2] >> (8 * (i1 & 3))) & 0xFFu;
                        const uint32_t b3 = (P[h1 >> 2] >> (8 * (h1 & 3))) & 0xFFu;
                        dst[k] = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
                    }
                }
            }
        }
    }
}

// d3: the inverse for row t: the high parts of this thread's eight elements (zero if the group has no record)
template <int A, int LPG>
__device__ __forceinline__ void unpack_record_row(const uint8_t *img_high, uint32_t my_word, uint32_t my_excl,
                                                  uint32_t logC, uint32_t tid, int t, uint32_t &h0, uint32_t &h1)
{
    constexpr HHTable TH = HH<A>::table;
    constexpr int LOG_LPG = LPG == 4 ? 2 : LPG - 1;
    constexpr uint32_t RB = A * LPG;
    h0 = h1 = 0;
    const uint32_t g = ((uint32_t)t << (logC - 3 - LOG_LPG)) + (tid >> LOG_LPG);
    const uint32_t wv = mask_word_lane<LPG>(my_word, g >> 5);
    const uint32_t pre = mask_word_lane<LPG>(my_excl, g >> 5);
    if ((wv >> (g & 31u)) & 1u) {
        const uint32_t rank = pre + __popc(wv & ((1u << (g & 31u)) - 1u));
        const uint8_t *rec8 = img_high + RB * rank;
        if constexpr (LPG == 1) {
            // this lane's 8 elements are the group: stream byte j is normalized byte j/2
            // (even j) or j/2 + ceil(A/2) (odd j), the dropped pad byte is zero
            constexpr int HALF = (A + 1) / 2;
            uint32_t P[A + 1];
#pragma unroll
            for (int q = 0; q <= A; ++q) P[q] = 0;
#pragma unroll
            for (int j = 0; j < A; ++j) P[(j & 1) ? (j >> 1) + HALF : (j >> 1)] = rec8[j];
            uint32_t h[2] = {0u, 0u};
#pragma unroll
            for (int f = 0; f < TH.count; ++f) {
                const int r = TH.row[f];
                const uint32_t smask = TH.shift[f] >= 0 ? (TH.dmask[f] >> TH.shift[f])
                                                        : (TH.dmask[f] << (-TH.shift[f]));
                h[r >> 2] |= (shl_or_shr(P[TH.plane[f]], -TH.shift[f]) & smask) << (8 * (r & 3));
            }
            h0 = h[0];
            h1 = h[1];
        } else if constexpr (LPG == 2) {
            const uint32_t par = tid & 1u;
            const uint16_t *rec = reinterpret_cast<const uint16_t *>(rec8);
            uint32_t nbyte[2 * A];
#pragma unroll
            for (int i = 0; i < A; ++i) {
                const uint32_t w = rec[i];
                nbyte[i] = w & 0xFFu;
                nbyte[i + A] = w >> 8;
            }
            uint32_t P[A];
#pragma unroll
            for (int q = 0; q < A; ++q) P[q] = 0;
#pragma unroll
            for (int j = 0; j < 2 * A; ++j) P[j >> 1] |= nbyte[j] << (8 * (j & 1));
            uint32_t E[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) E[r] = 0;
#pragma unroll
            for (int f = 0; f < TH.count; ++f) {
                const uint32_t smask = (TH.shift[f] >= 0 ? (TH.dmask[f] >> TH.shift[f])
                                                        : (TH.dmask[f] << (-TH.shift[f]))) * 0x0101u;
                E[TH.row[f]] |= shl_or_shr(P[TH.plane[f]], -TH.shift[f]) & smask;
            }
            // this lane's 8 elements are rows 4*par .. 4*par+3 of the two-column view
            h0 = par ? (E[4] | (E[5] << 16)) : (E[0] | (E[1] << 16));
            h1 = par ? (E[6] | (E[7] << 16)) : (E[2] | (E[3] << 16));
        } else {
            // the quad's group as 8 rows of 4 columns: stream word i = normalized byte i |
            // normalized byte i + 2A << 8, normalized byte 4q + c = byte c of plane q
            const uint32_t *rec = reinterpret_cast<const uint32_t *>(rec8);
            uint32_t nbyte[4 * A];
#pragma unroll
            for (int k = 0; k < A; ++k) {
                const uint32_t w = rec[k];
                nbyte[2 * k] = w & 0xFFu;
                nbyte[2 * k + 2 * A] = (w >> 8) & 0xFFu;
                nbyte[2 * k + 1] = (w >> 16) & 0xFFu;
                nbyte[2 * k + 1 + 2 * A] = w >> 24;
            }
            uint32_t P[A];
#pragma unroll
            for (int q = 0; q < A; ++q)
                P[q] = nbyte[4 * q] | (nbyte[4 * q + 1] << 8) | (nbyte[4 * q + 2] << 16) | (nbyte[4 * q + 3] << 24);
            uint32_t E[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) E[r] = 0;
#pragma unroll
            for (int f = 0; f < TH.count; ++f) {
                const uint32_t smask = (TH.shift[f] >= 0 ? (TH.dmask[f] >> TH.shift[f])
                                                        : (TH.dmask[f] << (-TH.shift[f]))) * 0x01010101u;
                E[TH.row[f]] |= shl_or_shr(P[TH.plane[f]], -TH.shift[f]) & smask;
            }
            // lane j of the quad holds rows 2j and 2j+1
            const uint32_t j = tid & 3u;
            h0 = j == 0 ? E[0] : (j == 1 ? E[2] : (j == 2 ? E[4] : E[6]));
            h1 = j == 0 ? E[1] : (j == 1 ? E[3] : (j == 2 ? E[5] : E[7]));
        }
    }
}

// a1: 128-bit loads of the 8 rows of data block k (pad elements beyond the tensor's end); a
// thread's 8 elements of a row are one vector (16-bit formats) or two (fp32)
template <int DT>
__device__ __forceinline__ void load_block_rows(const CompressItem &p, uint32_t B, uint32_t logB, uint32_t k,
                                                uint32_t tid, bool active, uint32_t logC,
                                                uint4 (&raw)[DT == DT_FP32 ? 16 : 8])
{
    const uint64_t blk0 = (uint64_t)k << logB;
    // a pad element has exponent b and nothing else: y = 0, raw byte 0, no left-over bits
    const uint32_t padw = DT == DT_FP32 ? (p.b << 23) : (p.b << (DT == DT_FP16 ? 10 : 7)) * 0x00010001u;
    if constexpr (DT == DT_FP32) {
        const uint32_t *in = reinterpret_cast<const uint32_t *>(p.in);
        if (blk0 + B <= p.n_elems) {
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const uint4 *src = reinterpret_cast<const uint4 *>(in + blk0 + ((uint64_t)t << logC) + 8u * tid);
                raw[2 * t] = active ? src[0] : make_uint4(padw, padw, padw, padw);
                raw[2 * t + 1] = active ? src[1] : make_uint4(padw, padw, padw, padw);
            }
            return;
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint64_t e0 = blk0 + ((uint64_t)t << logC) + 8u * tid;
            uint32_t d[8] = {padw, padw, padw, padw, padw, padw, padw, padw};
            if (active && e0 < p.n_elems) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (e0 + i < p.n_elems) d[i] = in[e0 + i];
            }
            raw[2 * t] = make_uint4(d[0], d[1], d[2], d[3]);
            raw[2 * t + 1] = make_uint4(d[4], d[5], d[6], d[7]);
        }
    } else {
        if (blk0 + B <= p.n_elems) {               // whole block inside the tensor: no per-row tests
#pragma unroll
            for (int t = 0; t < 8; ++t)
                raw[t] = active ? *reinterpret_cast<const uint4 *>(p.in + blk0 + ((uint64_t)t << logC) + 8u * tid)
                                : make_uint4(padw, padw, padw, padw);
            return;
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint64_t e0 = blk0 + ((uint64_t)t << logC) + 8u * tid;
            uint32_t d[4] = {padw, padw, padw, padw};
            if (active && e0 < p.n_elems) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (e0 + i < p.n_elems) {
                        const uint32_t v = p.in[e0 + i];
                        d[i >> 1] = (i & 1) ? ((d[i >> 1] & 0x0000FFFFu) | (v << 16))
                                            : ((d[i >> 1] & 0xFFFF0000u) | v);
                    }
            }
            raw[t] = make_uint4(d[0], d[1], d[2], d[3]);
        }
    }
}

// ---------------------------------------------------------------------------------
// compression: split, transform, group test, packing, inter-block scan, store
// (Sec. V-A compression path; Sec. V-B; Sec. V-C; Fig. 4)
// ---------------------------------------------------------------------------------
template <int M, int A, int DT, int LPG>
__global__ void __launch_bounds__(512) ENEC_COMPRESS_OCCUPANCY compress_kernel(const CompressArgs p)
{
    constexpr int N = M + A;
    constexpr int LOG_LPG = LPG == 4 ? 2 : LPG - 1;
    constexpr uint32_t RB = A * LPG;                     // bytes of one high record: (n - m) L / 8
    constexpr int LM = low_plane_bits(M, DT);            // width of the low plane
    constexpr uint32_t NMASK = ((1u << N) - 1u) * 0x01010101u;
    constexpr uint32_t LMASK = ((1u << M) - 1u) * 0x01010101u;
    constexpr uint32_t AMASK = ((1u << A) - 1u) * 0x01010101u;
    constexpr uint32_t SREP = (1u << (N - 1)) * 0x01010101u;
    constexpr int MP = LM > 0 ? LM : 1;
    constexpr int AP = A > 0 ? A : 1;
    constexpr int RW = DT == DT_FP32 ? 16 : 8;           // 128-bit vectors of one block per thread

    // two LDS images of the packed part of a payload: mask | low plane (as normalized bytes,
    // interleaved on the way out) | high records
    extern __shared__ __align__(16) uint8_t smem[];
    __shared__ uint32_t s_k[2];                // block index of this / the next iteration
    __shared__ unsigned long long s_tag;       // tag of this call
    __shared__ unsigned long long s_off;       // start of the block being stored, bytes
    __shared__ uint32_t s_status;              // header status found by the scan for that block
    __shared__ uint32_t s_err[2];              // range error in the block of image 0 / 1

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t B = p.B, logC = p.logB - 3u;
    const uint32_t nact = B >> 6;
    const bool active = tid < nact;
    const uint32_t acc_tid = blockDim.x > 64u ? 64u : 0u;   // the lane that talks to the group accumulators
    const uint32_t mask_bytes = (B >> 6) >> LOG_LPG;                  // B / (8 L)
    const uint32_t img_bytes = mask_bytes + (((uint32_t)(LM + A) * B) >> 3);
    const uint32_t fixed = B + mask_bytes + ((LM * B) >> 3);

    // ---- control record of this workgroup's class (thread 0) ---------------------------
    const uint32_t home = blockIdx.x % p.ncls;
    uint32_t *ctl = p.ws_ctl + WS_STRIDE * home;
    const uint32_t class_blocks = home < p.total ? (p.total - home + p.ncls - 1u) / p.ncls : 0u;
    const uint32_t class_wgs = (gridDim.x - home + p.ncls - 1u) / p.ncls;
    uint32_t ticket_base = 0, zero = 0;
    uint64_t tag0 = 0;
    bool drawing = true;
    // decode a draw; the last draw of the class hands the record over to the next call
    auto decode_draw = [&](uint32_t raw) -> uint32_t {
        const uint32_t t = raw - ticket_base;
        if (t == class_blocks + class_wgs - 1u) {
            ctl[1] = raw + 1u;
            for (uint32_t c = home; c < WS_CLASSES; c += p.ncls)
                *reinterpret_cast<uint64_t *>(p.ws_ctl + WS_STRIDE * c + 2) = tag0;
        }
        if (t >= class_blocks) { drawing = false; return NO_BLOCK; }
        return t * p.ncls + home;
    };
    uint32_t slot = 0;
    // tensor that global block kg belongs to, searching upwards from item c
    auto item_of = [&](uint32_t kg, uint32_t c) -> uint32_t {
        while (c + 1u < p.n_items && kg >= p.item[c + 1u].first) ++c;
        return c;
    };
    // Every block is drawn, also the first one: a workgroup that is dispatched late (the device may
    // be shared with other kernels) must not own a block that running workgroups wait for.  When all
    // workgroups start together, workgroup w draws block w, so its rows are requested on that guess
    // while the control record and the draw are still travelling.
    const uint32_t guess = blockIdx.x;                       // the grid never exceeds the number of blocks
    uint32_t ci = item_of(guess, 0);
    uint4 raw[RW];
    load_block_rows<DT>(p.item[ci], B, p.logB, guess - p.item[ci].first, tid, active, logC, raw);
    if (tid == 0) {
        ticket_base = ctl[1];
        tag0 = *reinterpret_cast<const uint64_t *>(ctl + 2) + 1u;
        // the record must have been read before this workgroup's first draw can be counted
        zero = ticket_base ^ (uint32_t)tag0;
        asm volatile("v_and_b32 %0, 0, %0" : "+v"(zero));
        s_k[0] = decode_draw(atomicAdd(ctl + zero, 1u));
        s_tag = tag0;
        s_err[0] = s_err[1] = 0;
        s_status = 0;
    }
    __syncthreads();
    uint32_t k = __builtin_amdgcn_readfirstlane(s_k[0]);     // global block index
    if (k != guess && k != NO_BLOCK) {                       // the guess was wrong: ask again
        ci = item_of(k, 0);
        load_block_rows<DT>(p.item[ci], B, p.logB, k - p.item[ci].first, tid, active, logC, raw);
    }
    const uint64_t tag = (uint64_t)s_tag << 24;
    constexpr HHTable TL = HH<MP>::table;

    // wave 0 carries the scan of one tensor: sum of its group words [0, groups_summed) and what
    // went wrong so far (bit 1 range error in an earlier block, bit 2 gave up waiting)
    uint64_t groups_sum = 0;
    uint32_t groups_summed = 0, scan_flags = 0, scan_item = NO_BLOCK;

    // sum of the (valid) words base[0 .. count), count <= 64, one word per lane; `v` may hold a
    // copy read earlier (have = true), words that were not valid yet are read again until they are
    auto sum_words = [&](const uint64_t *base, uint32_t count, bool have, uint64_t v, uint32_t &flags) -> uint64_t {
        const bool need = lane < count;
        bool ok = !need || (have && (v & ~0xFFFFFFull) == tag);
        uint32_t spins = 0;
        while (__builtin_amdgcn_ballot_w64(!ok) != 0) {
            if (!ok) {
                v = ld_state(base + lane);
                ok = (v & ~0xFFFFFFull) == tag;
            }
            if (__builtin_amdgcn_ballot_w64(!ok) == 0) break;
            if (++spins > p.spin_limit) {                                      // never hang
                flags |= 4u;
                v = 0;
                if (lane == 0) st_state(reinterpret_cast<uint64_t *>(p.ws_ctl + 4), tag);
                break;
            }
            spin_pause(spins);
        }
        if (__builtin_amdgcn_ballot_w64(need && (v & ST_ERR))) flags |= 2u;
        // at most 64 sizes below 2^23 units of 16 bytes: the sum fits 32 bits
        return wave_sum32(need ? (uint32_t)(v & ST_VALUE) : 0u);
    };
    // start of block kb (wave 0; early_g / early_b = copies of the first needed group words / of
    // the earlier block words of its group, read ahead of time)
    auto block_start = [&](const CompressItem &it, uint32_t kb, bool early, uint64_t early_g, uint64_t early_b) -> uint64_t {
        const uint32_t g = kb >> GROUP_LOG;
        while (groups_summed < g) {
            const uint32_t c = g - groups_summed < 64u ? g - groups_summed : 64u;
            groups_sum += sum_words(it.ws_group + groups_summed, c, early, early_g, scan_flags);
            groups_summed += c;
            early = false;
        }
        const uint64_t own_group = sum_words(it.ws_block + ((uint64_t)g << GROUP_LOG), kb & (GROUP - 1u), early_b != 0, early_b, scan_flags);
        return (groups_sum + own_group) << 4;
    };

    // the block waiting to be stored
    uint32_t pend = NO_BLOCK, pend_item = 0, pend_cnt = 0, pend_S = 0, pend_err = 0;   // pend: index inside its tensor
    // its sign/mantissa bytes wait in LDS behind the two images, every thread's own 64 bytes (in
    // registers they were what the compiler spilled); the instances built for two waves per SIMD have
    // the registers and keep them there
    constexpr bool SM_IN_LDS = compress_sm_in_lds(DT, LPG);
    uint8_t *sm_wait = smem + 2u * img_bytes;
    uint32_t SMp[SM_IN_LDS ? 1 : 8][2];

    // stores block `kb` whose packed part sits in image `img` and whose sign/mantissa bytes sit in sm_wait
    auto store_block = [&](const CompressItem &it, uint32_t kb, uint32_t cnt, uint32_t S, const uint8_t *img,
                           uint32_t err_own) {
        const uint64_t off = s_off;
        uint8_t *dst = it.out + it.payload_base + off;
        if constexpr (SM_IN_LDS) {
            // the plane waits in LDS in element order and leaves as 128-bit vectors (four per thread
            // instead of eight 64-bit stores of the thread's own bytes; measured neutral, within 1 %)
            for (uint32_t v = tid; v < (B >> 4); v += blockDim.x)
                *reinterpret_cast<uint4 *>(dst + 16u * v) = *reinterpret_cast<const uint4 *>(sm_wait + 16u * v);
        } else if (active) {
#pragma unroll
            for (int t = 0; t < 8; ++t)
                *reinterpret_cast<uint2 *>(dst + ((size_t)t << logC) + 8u * tid) = make_uint2(SMp[t][0], SMp[t][1]);
        }
        for (uint32_t v = tid; v < (mask_bytes >> 4); v += blockDim.x)
            *reinterpret_cast<uint4 *>(dst + B + 16u * v) = *reinterpret_cast<const uint4 *>(img + 16u * v);
        if (LM > 0) {
            const uint8_t *ilow = img + mask_bytes;
            uint8_t *dlow = dst + B + mask_bytes;
            const uint32_t T2 = (LM * B) >> 4;                // half of the plane's length
            for (uint32_t v = tid; v < (T2 >> 3); v += blockDim.x) {
                const uint2 a = *reinterpret_cast<const uint2 *>(ilow + 8u * v);
                const uint2 c = *reinterpret_cast<const uint2 *>(ilow + 8u * v + T2);
                uint4 o;   // stream byte 2i = normalized byte i, stream byte 2i+1 = normalized byte i + T/2
                o.x = byte_perm(c.x, a.x, 0x05010400u);
                o.y = byte_perm(c.x, a.x, 0x07030602u);
                o.z = byte_perm(c.y, a.y, 0x05010400u);
                o.w = byte_perm(c.y, a.y, 0x07030602u);
                *reinterpret_cast<uint4 *>(dlow + 16u * v) = o;
            }
        }
        if (A > 0) {
            const uint8_t *ihigh = img + mask_bytes + ((LM * B) >> 3);
            uint8_t *dhigh = dst + fixed;
            const uint32_t hbytes = RB * cnt;
            for (uint32_t v = tid; 16u * v < hbytes; v += blockDim.x) {
                uint4 o = *reinterpret_cast<const uint4 *>(ihigh + 16u * v);
                uint32_t w[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {                 // zero the padding behind the last record
                    const uint32_t at = 16u * v + 4u * i;
                    if (at >= hbytes) w[i] = 0;
                    else if (at + 4u > hbytes) w[i] &= (1u << (8u * (hbytes - at))) - 1u;
                }
                *reinterpret_cast<uint4 *>(dhigh + 16u * v) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
        if (tid == 0) {
            uint64_t *table = reinterpret_cast<uint64_t *>(it.out + 64);
            table[kb] = off;
            if (kb == it.nb - 1u) {
                const uint64_t end = off + S;
                uint32_t fl = s_status | err_own;
                if (ld_state(reinterpret_cast<const uint64_t *>(p.ws_ctl + 4)) == tag) fl |= 4u;   // somebody gave up
                const uint32_t status = (fl & 4u) ? 8u : ((fl & 3u) ? 6u : 0u);
                const uint64_t total = status ? 0ull : it.payload_base + end;
                table[it.nb] = end;
                if (((uint64_t)(it.nb + 1u) & 1ull)) table[it.nb + 1u] = 0;   // pad up to the payload base
                uint32_t *h = reinterpret_cast<uint32_t *>(it.out);
                h[0] = 0x43454E45u;                              // "ENEC"
                h[1] = 1u | ((uint32_t)DT << 16) | ((8u * LPG) << 24);   // version, dtype, L
                h[2] = (uint32_t)it.n_elems; h[3] = (uint32_t)(it.n_elems >> 32);
                h[4] = B; h[5] = it.nb;
                h[6] = it.b | ((uint32_t)N << 8) | ((uint32_t)M << 16) | (exponent_bits(DT) << 24);
                h[7] = status;
                h[8] = (uint32_t)total; h[9] = (uint32_t)(total >> 32);
#pragma unroll
                for (int i = 10; i < 16; ++i) h[i] = 0;
                if (it.out_bytes) *it.out_bytes = total;
            }
        }
    };

    while (k != NO_BLOCK) {
        uint8_t *img = smem + slot * img_bytes;
        uint32_t *img_maskw = reinterpret_cast<uint32_t *>(img);
        uint8_t *img_low = img + mask_bytes;
        uint8_t *img_high = img_low + (((size_t)LM * B) >> 3);

        // wave 0 reads the scan state for the block stored in this iteration now and uses it
        // after the arithmetic: published an iteration ago, it is normally all there
        const CompressItem &it = p.item[ci];
        const uint32_t kl = k - it.first;                    // index of the block inside its tensor
        const uint32_t crep = ((it.b + (1u << (N - 1))) & 0xFFu) * 0x01010101u;
        const uint32_t xlo = it.b + 1u > (1u << (N - 1)) ? it.b + 1u - (1u << (N - 1)) : 0u;
        const uint32_t xhi = it.b + (1u << (N - 1)) < 255u ? it.b + (1u << (N - 1)) : 255u;
        const uint32_t mode = it.mode;
        uint64_t early_g = 0, early_b = 0;
        if (wave == 0 && pend != NO_BLOCK) {
            if (scan_item != pend_item) { scan_item = pend_item; groups_sum = 0; groups_summed = 0; scan_flags = 0; }
            const CompressItem &pit = p.item[pend_item];
            const uint32_t pg = pend >> GROUP_LOG;
            if (groups_summed + lane < pg) early_g = ld_state(pit.ws_group + groups_summed + lane);
            if (lane < (pend & (GROUP - 1u))) early_b = ld_state(pit.ws_block + ((uint64_t)pg << GROUP_LOG) + lane);
        }

        // the ticket for the following block is drawn now and looked at after the arithmetic
        uint32_t next_raw = 0;
        const bool draw_now = tid == 0 && p.lookahead && drawing;
        if (draw_now) next_raw = atomicAdd(ctl + zero, 1u);

        uint32_t SMc[8][2], HI[8][2], accP[MP][2], mw[8], mw_hi[LPG == 1 ? 8 : 1];
        uint32_t err_acc = 0;
        bool bad = false;
#pragma unroll
        for (int q = 0; q < MP; ++q) accP[q][0] = accP[q][1] = 0;

        const uint64_t row0 = ((uint64_t)kl << p.logB) + 8u * tid;   // this thread's first element of row 0
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            uint32_t gor = 0;
            uint4 r16;                           // the row's eight 16-bit words
            if constexpr (DT == DT_FP32) {
                // upper halves go on as bf16 words, lower halves leave at once
                const uint4 u = raw[2 * t], v = raw[2 * t + 1];
                r16 = make_uint4(byte_perm(u.y, u.x, 0x07060302u), byte_perm(u.w, u.z, 0x07060302u),
                                 byte_perm(v.y, v.x, 0x07060302u), byte_perm(v.w, v.z, 0x07060302u));
                const uint64_t e0 = row0 + ((uint64_t)t << logC);
                if (active && e0 < it.n_elems)   // elements past the end are pads with zero lower halves
                    *reinterpret_cast<uint4 *>(it.out + it.tail_base + 2u * e0) =
                        make_uint4(byte_perm(u.y, u.x, 0x05040100u), byte_perm(u.w, u.z, 0x05040100u),
                                   byte_perm(v.y, v.x, 0x05040100u), byte_perm(v.w, v.z, 0x05040100u));
            } else {
                r16 = raw[t];
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t d0 = h ? r16.z : r16.x;
                const uint32_t d1 = h ? r16.w : r16.y;
                // a1 split: low / high bytes of four 16-bit words
                const uint32_t Lb = byte_perm(d1, d0, 0x06040200u);
                const uint32_t Hb = byte_perm(d1, d0, 0x07050301u);
                uint32_t X, T3 = 0;
                if constexpr (DT == DT_FP16) {
                    SMc[t][h] = (Hb & 0x80808080u) | ((Hb & 0x03030303u) << 5) | ((Lb >> 3) & 0x1F1F1F1Fu);
                    X = (Hb >> 2) & 0x1F1F1F1Fu;
                    T3 = Lb & 0x07070707u;
                } else {
                    SMc[t][h] = bfi(0x7F7F7F7Fu, Lb, Hb);
                    X = bfi(0xFEFEFEFEu, Hb << 1, Lb >> 7);
                }
                // a2 transform: z = (b + 2^(n-1) - x) mod 256 per byte, y = z with the sign bit flipped
                uint32_t Z;
                if (mode == 0) {
                    Z = crep - X;
                    if (N < 8) err_acc |= Z;
                } else {
                    Z = bytesub_safe(crep, X);
                    if (mode == 2) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const uint32_t xb = (X >> (8 * i)) & 0xFFu;
                            bad |= (xb < xlo) | (xb > xhi);
                        }
                    }
                }
                uint32_t Y = Z ^ SREP;
                if (N < 8) Y &= NMASK;
                // a3: high parts decide the group; a4: low parts go to the column packer
                const uint32_t hi = A > 0 ? ((Y >> M) & AMASK) : 0u;
                HI[t][h] = hi;
                gor |= hi;
                if (LM > 0) {
                    const uint32_t low = (Y & LMASK) | (T3 << M);
#pragma unroll
                    for (int f = 0; f < TL.count; ++f)
                        if (TL.row[f] == t) {
                            uint32_t s = shl_or_shr(low, TL.shift[f]);
                            if (!TL.clean[f]) s &= TL.dmask[f] * 0x01010101u;
                            accP[TL.plane[f]][h] |= s;
                        }
                }
            }
            // a3: OR over the lanes that share a group, one mask bit per group
            if constexpr (LPG == 2) gor |= swap_pair(gor);
            if constexpr (LPG == 4) gor = quad_or(gor);
            const uint64_t flagged = __builtin_amdgcn_ballot_w64(gor != 0);
            if constexpr (LPG == 1) { mw[t] = (uint32_t)flagged; mw_hi[t] = (uint32_t)(flagged >> 32); }
            else if constexpr (LPG == 2) mw[t] = compact_even_bits(flagged);
            else mw[t] = compact_fourth_bits(flagged);
        }
        if (N < 8 && mode == 0) bad = (err_acc & ~NMASK) != 0;
        if (__builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) atomicOr(&s_err[slot], 1u);

        // a wave holds 64 / LPG mask bits of every row (nact / LPG when the block has 2048 elements
        // and the only wave is half empty); group order = row-major
        if (lane == 0 && 64u * wave < nact) {
            if constexpr (LPG == 1) {
                if (logC >= 9) {
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        img_maskw[((uint32_t)t << (logC - 8)) + 2u * wave] = mw[t];
                        img_maskw[((uint32_t)t << (logC - 8)) + 2u * wave + 1u] = mw_hi[t];
                    }
                } else {  // B = 2048: 32 groups per row
#pragma unroll
                    for (int t = 0; t < 8; ++t) img_maskw[t] = mw[t];
                }
            } else if constexpr (LPG == 2) {
                if (logC >= 9) {
#pragma unroll
                    for (int t = 0; t < 8; ++t) img_maskw[((uint32_t)t << (logC - 9)) + wave] = mw[t];
                } else {  // B = 2048: 16 groups per row, one wave
#pragma unroll
                    for (int u = 0; u < 4; ++u) img_maskw[u] = mw[2 * u] | (mw[2 * u + 1] << 16);
                }
            } else {      // 16 bits per wave and row (B >= 4096)
                uint16_t *img_mask16 = reinterpret_cast<uint16_t *>(img);
#pragma unroll
                for (int t = 0; t < 8; ++t) img_mask16[((uint32_t)t << (logC - 9)) + wave] = (uint16_t)mw[t];
            }
        }
        if (LM > 0 && active) {
#pragma unroll
            for (int q = 0; q < LM; ++q)
                *reinterpret_cast<uint2 *>(img_low + ((size_t)q << logC) + 8u * tid) =
                    make_uint2(accP[q][0], accP[q][1]);
        }
        if (tid == 0) s_k[slot ^ 1u] = draw_now ? decode_draw(next_raw) : NO_BLOCK;
        __syncthreads();                                                     // barrier 1

        // ---- a5 (positions): exclusive popcount prefix over the block's mask words; every wave
        // computes it for itself (a wave scan of at most 64 words) -----------------------
        const uint32_t nwords = (B >> 8) >> LOG_LPG;          // 32-bit words of the mask (at most 64)
        const uint32_t my_word = lane < nwords ? img_maskw[lane] : 0u;
        const uint32_t my_pc = __popc(my_word);
        const uint32_t my_incl = wave_incl_scan(my_pc, lane);
        const uint32_t my_excl = my_incl - my_pc;
        const uint32_t cnt = (uint32_t)__builtin_amdgcn_readlane((int)my_incl, 63);
        const uint32_t own_err = s_err[slot] & 1u;
        const uint32_t S = (fixed + RB * cnt + 15u) & ~15u;

        // ---- a6: publish this block's size at once, and add it to its group's accumulator
        // [blocks:16 | blocks with a range error:16 | sum of sizes:32]; what the addition returns
        // is looked at after barrier 2, when it has had time to travel ---------------------
        if (tid == 0) st_state(it.ws_block + kl, tag | (own_err ? ST_ERR : 0ull) | (uint64_t)(S >> 4));
        // (a group of one block, e.g. a tensor of one block, is complete with its only member)
        const uint32_t grp = kl >> GROUP_LOG;
        const uint32_t members = it.nb - (grp << GROUP_LOG) < GROUP ? it.nb - (grp << GROUP_LOG) : GROUP;
        uint64_t acc_old = 0;
        if (tid == acc_tid && members > 1u)
            acc_old = __hip_atomic_fetch_add(it.ws_acc + grp, (1ull << 48) | ((uint64_t)own_err << 32) | (uint64_t)(S >> 4),
                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

        // ---- a5: one record per masked group ------------------------------------------
        if constexpr (A > 0) pack_records<A, LPG>(HI, my_word, my_excl, img_high, logC, tid, active);

        // ---- a6 (wave 0): the start of the block stored in this iteration -----------------
        if (wave == 0 && pend != NO_BLOCK) {
            const uint64_t off = block_start(p.item[pend_item], pend, true, early_g, early_b);
            if (lane == 0) { s_off = off; s_status = scan_flags; }
        }
        __syncthreads();                                                     // barrier 2
        if (tid == 0) s_err[slot] = 0;          // read by everybody before barrier 2; next use in two iterations

        // ---- a6: whoever completes a group publishes its word and clears the accumulator for
        // the next call; nobody ever waits for blocks of its own generation ------------------
        if (tid == acc_tid) {
            if ((uint32_t)(acc_old >> 48) == members - 1u) {
                const uint64_t sum = (acc_old & 0xFFFFFFFFull) + (S >> 4);
                const bool any_err = ((acc_old >> 32) & 0xFFFFull) != 0 || own_err;
                st_state(it.ws_group + grp, tag | (any_err ? ST_ERR : 0ull) | sum);
                if (members > 1u) st_state(it.ws_acc + grp, 0ull);
            }
        }

        // the following block's rows start to travel while the previous block is stored
        const uint32_t knext = __builtin_amdgcn_readfirstlane(s_k[slot ^ 1u]);
        uint32_t cnext = ci;
        if (knext != NO_BLOCK) {
            cnext = item_of(knext, ci);
            load_block_rows<DT>(p.item[cnext], B, p.logB, knext - p.item[cnext].first, tid, active, logC, raw);
        }

        // ---- a7: stores of the previous block ----------------------------------------------
        if (pend != NO_BLOCK)
            store_block(p.item[pend_item], pend, pend_cnt, pend_S, smem + (slot ^ 1u) * img_bytes, pend_err);
        __syncthreads();                                                     // barrier 3: other image free

        // this block becomes the pending one
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if constexpr (SM_IN_LDS) {
                if (active)
                    *reinterpret_cast<uint2 *>(sm_wait + ((size_t)t << logC) + 8u * tid) = make_uint2(SMc[t][0], SMc[t][1]);
            } else {
                SMp[t][0] = SMc[t][0];
                SMp[t][1] = SMc[t][1];
            }
        }
        pend = kl; pend_item = ci; pend_cnt = cnt; pend_S = S; pend_err = own_err;
        slot ^= 1u;
        k = knext;
        ci = cnext;
        if (k == NO_BLOCK && !p.lookahead) {           // without lookahead the next ticket is drawn only now
            if (tid == 0) s_k[slot] = drawing ? decode_draw(atomicAdd(ctl + zero, 1u)) : NO_BLOCK;
            __syncthreads();
            k = __builtin_amdgcn_readfirstlane(s_k[slot]);
            if (k != NO_BLOCK) {
                ci = item_of(k, ci);
                load_block_rows<DT>(p.item[ci], B, p.logB, k - p.item[ci].first, tid, active, logC, raw);
            }
        }
    }

    // ---- drain: the last block of this workgroup ---------------------------------------------
    if (pend != NO_BLOCK) {
        if (wave == 0) {
            if (scan_item != pend_item) { scan_item = pend_item; groups_sum = 0; groups_summed = 0; scan_flags = 0; }
            const uint64_t off = block_start(p.item[pend_item], pend, false, 0, 0);
            if (lane == 0) { s_off = off; s_status = scan_flags; }
        }
        __syncthreads();
        store_block(p.item[pend_item], pend, pend_cnt, pend_S, smem + (slot ^ 1u) * img_bytes, pend_err);
    }
}

// ---------------------------------------------------------------------------------
// decompression: offset lookup, mask prefix, unpack, inverse transform, recombine
// (Sec. V-A decompression path; Alg. 1 decompression part)
//
// Persistent grid, block k handled by workgroup k mod gridDim (blocks are independent, so no
// tickets are needed).  While block k is unpacked and stored, the payload of the workgroup's
// next block is already travelling: its sign/mantissa bytes into registers, its packed part
// (mask | low plane | high records, exactly as in the stream) into the other of two LDS images.
// ---------------------------------------------------------------------------------
template <int M, int A, int DT, int LPG>
__global__ void __launch_bounds__(512) decompress_kernel(const DecompressArgs p)
{
    constexpr int N = M + A;
    constexpr int LOG_LPG = LPG == 4 ? 2 : LPG - 1;
    constexpr uint32_t RB = A * LPG;                     // bytes of one high record: (n - m) L / 8
    constexpr int LM = low_plane_bits(M, DT);            // width of the low plane
    constexpr uint32_t SREP = (1u << (N - 1)) * 0x01010101u;
    constexpr uint32_t LMASK = ((1u << M) - 1u) * 0x01010101u;
    constexpr int MP = LM > 0 ? LM : 1;
    constexpr int AP = A > 0 ? A : 1;
    constexpr int VMAX = (LM + A) / 2 + 1;   // 16-byte vectors of packed payload per thread

    extern __shared__ __align__(16) uint8_t smem[];

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t B = p.B, logC = p.logB - 3u, C = 1u << logC;
    const uint32_t nact = B >> 6;
    const bool active = tid < nact;
    const uint32_t mask_bytes = (B >> 6) >> LOG_LPG;                  // B / (8 L)
    const uint32_t img_bytes = mask_bytes + (((uint32_t)(LM + A) * B) >> 3);
    const uint32_t fixed = B + mask_bytes + ((LM * B) >> 3);

    // tensor that global block kg belongs to, searching upwards from item c
    auto item_of = [&](uint32_t kg, uint32_t c) -> uint32_t {
        while (c + 1u < p.n_items && kg >= p.item[c + 1u].first) ++c;
        return c;
    };
    // d1: the header in memory must be the one the launch was configured from (the host has
    // checked that header and table lie inside the buffer); otherwise the tensor is not touched
    uint32_t hdr_ok = 0, hdr_seen = 0;                       // one bit per item
    auto header_matches = [&](uint32_t c) -> bool {
        if (!((hdr_seen >> c) & 1u)) {
            const uint32_t *h = reinterpret_cast<const uint32_t *>(p.item[c].in);
            bool same = true;
#pragma unroll
            for (int i = 0; i < 10; ++i) same &= (h[i] == p.item[c].hdr[i]);
            hdr_seen |= 1u << c;
            if (same) hdr_ok |= 1u << c;
        }
        return (hdr_ok >> c) & 1u;
    };
    // d1: offset lookup, in two steps so that the loads can be issued well before they are used;
    // a block whose table entries point outside the stream is skipped.  kg = global block index.
    auto fetch = [&](uint32_t kg, uint32_t c, uint64_t &t0, uint64_t &t1) {
        if (kg < p.total) {
            const uint64_t *table = reinterpret_cast<const uint64_t *>(p.item[c].in + 64);
            const uint32_t kb = kg - p.item[c].first;
            t0 = table[kb];
            t1 = table[kb + 1];
        }
    };
    auto check = [&](uint32_t kg, uint32_t c, uint64_t t0, uint64_t t1, uint64_t &off, uint32_t &size) -> bool {
        if (kg >= p.total) return false;
        const uint64_t sz = t1 - t0;
        off = t0;
        size = (uint32_t)sz;
        return header_matches(c) &&
               !(sz < fixed || sz > fixed + RB * ((B >> 3) >> LOG_LPG) + 15u || (sz & 15u) || t0 > p.item[c].payload_bytes ||
                 sz > p.item[c].payload_bytes - t0);
    };
    // issue the loads of one block: sign/mantissa rows and the packed part
    auto issue = [&](uint32_t c, uint64_t off, uint32_t size, uint2 (&smv)[8], uint4 (&vec)[VMAX]) {
        const uint8_t *src = p.item[c].in + p.item[c].payload_base + off;
#pragma unroll
        for (int t = 0; t < 8; ++t)
            smv[t] = active ? *reinterpret_cast<const uint2 *>(src + ((size_t)t << logC) + 8u * tid) : make_uint2(0, 0);
        const uint32_t nvec = (size - B) >> 4;
#pragma unroll
        for (int i = 0; i < VMAX; ++i) {
            const uint32_t v = tid + (uint32_t)i * blockDim.x;
            vec[i] = v < nvec ? *reinterpret_cast<const uint4 *>(src + B + 16u * v) : make_uint4(0, 0, 0, 0);
        }
    };
    auto to_image = [&](uint8_t *img, const uint4 (&vec)[VMAX]) {
#pragma unroll
        for (int i = 0; i < VMAX; ++i) {
            const uint32_t v = tid + (uint32_t)i * blockDim.x;
            if (16u * v < img_bytes) *reinterpret_cast<uint4 *>(img + 16u * v) = vec[i];
        }
    };

    uint32_t k = blockIdx.x;                                // global block index
    if (k >= p.total) return;
    // A block that fails these tests is skipped and its part of the output stays as it was.  For the
    // tensors that come with a status word, the last workgroup looks at the header and at every table
    // entry once more before its own work and tells the caller if any block will be skipped.  (Done
    // here, outside the loop below: a store inside that loop cost 5 % of the kernel's time.)
    if (blockIdx.x == gridDim.x - 1u) {
        for (uint32_t c = 0; c < p.n_items; ++c) {
            if (!p.item[c].status) continue;
            const uint64_t *table = reinterpret_cast<const uint64_t *>(p.item[c].in + 64);
            bool bad = !header_matches(c);
            for (uint32_t e = tid; e < p.item[c].nb && !bad; e += blockDim.x) {
                const uint64_t t0 = table[e], sz = table[e + 1] - t0;
                bad = sz < fixed || sz > fixed + RB * ((B >> 3) >> LOG_LPG) + 15u || (sz & 15u) || t0 > p.item[c].payload_bytes ||
                      sz > p.item[c].payload_bytes - t0;
            }
            if (bad) *p.item[c].status = 7u;
        }
    }
    uint32_t ci = item_of(k, 0);
    uint32_t cn = item_of(k + gridDim.x, ci);               // item of the next block (if there is one)
    uint64_t off = 0, offn = 0;
    uint32_t size = 0, sizen = 0;
    uint64_t ta = 0, tb = 0, tc = 0, td = 0;
    fetch(k, ci, ta, tb);
    fetch(k + gridDim.x, cn, tc, td);                       // the table is read one block ahead
    bool valid = check(k, ci, ta, tb, off, size);
    bool validn = check(k + gridDim.x, cn, tc, td, offn, sizen);
    uint2 smc[8], smn[8];
    uint4 vec[VMAX];
    if (valid) {
        issue(ci, off, size, smc, vec);
        to_image(smem, vec);
    }
    uint32_t slot = 0;
    constexpr HHTable TL = HH<MP>::table;

    while (k < p.total) {
        __syncthreads();            // image[slot] is complete, image[slot ^ 1] is free
        // the next block's loads start now and are consumed at the end of the iteration
        const uint32_t kn = k + gridDim.x;
        if (validn) issue(cn, offn, sizen, smn, vec);
        const uint32_t c2 = item_of(kn + gridDim.x, cn);
        fetch(kn + gridDim.x, c2, ta, tb);
        const DecompressItem &it = p.item[ci];
        const uint32_t crep = ((it.b + (1u << (N - 1))) & 0xFFu) * 0x01010101u;

        if (valid && active) {
            const uint8_t *img = smem + slot * img_bytes;
            const uint8_t *img_low = img + mask_bytes;
            const uint8_t *img_high = img_low + (((size_t)LM * B) >> 3);
            const uint64_t blk0 = (uint64_t)(k - it.first) << p.logB;
            // fp32: the lower halves of this thread's elements, straight from the stream
            uint4 tl[DT == DT_FP32 ? 8 : 1];
            if constexpr (DT == DT_FP32) {
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const uint64_t e0 = blk0 + ((uint64_t)t << logC) + 8u * tid;
                    tl[t] = e0 < it.n_elems ? *reinterpret_cast<const uint4 *>(it.in + it.tail_base + 2u * e0)
                                            : make_uint4(0, 0, 0, 0);
                }
            }
            // d2: mask words and their exclusive popcount prefix (a wave scan per wave)
            const uint32_t nwords = (B >> 8) >> LOG_LPG;
            const uint32_t my_word = lane < nwords ? reinterpret_cast<const uint32_t *>(img)[lane] : 0u;
            const uint32_t my_pc = __popc(my_word);
            const uint32_t my_excl = wave_incl_scan(my_pc, lane) - my_pc;

            // low plane: the 8 normalized bytes of plane q for this thread's columns are every
            // other byte of one 16-byte span of the stream (undoing the final join of Alg. 2)
            uint32_t Pl[MP][2];
#pragma unroll
            for (int q = 0; q < MP; ++q) {
                if (LM > 0) {
                    const uint32_t T2 = (LM * B) >> 4;
                    const uint32_t i = ((uint32_t)q << logC) + 8u * tid;
                    const bool even = i < T2;
                    const uint4 sp = *reinterpret_cast<const uint4 *>(img_low + 2u * (even ? i : i - T2));
                    const uint32_t sel = even ? 0x06040200u : 0x07050301u;
                    Pl[q][0] = byte_perm(sp.y, sp.x, sel);
                    Pl[q][1] = byte_perm(sp.w, sp.z, sel);
                } else {
                    Pl[q][0] = Pl[q][1] = 0;
                }
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                uint32_t Y[2] = {0u, 0u}, T3[2] = {0u, 0u};
                // d3: low-plane values of the 8 columns of this row: the low m bits of y (fp16:
                // with the last three mantissa bits on top)
                if (LM > 0) {
#pragma unroll
                    for (int f = 0; f < TL.count; ++f)
                        if (TL.row[f] == t) {
                            const uint32_t smask = (TL.shift[f] >= 0 ? (TL.dmask[f] >> TL.shift[f])
                                                                    : (TL.dmask[f] << (-TL.shift[f]))) * 0x01010101u;
#pragma unroll
                            for (int h = 0; h < 2; ++h)
                                Y[h] |= shl_or_shr(Pl[TL.plane[f]][h], -TL.shift[f]) & smask;
                        }
                    if constexpr (DT == DT_FP16) {
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            T3[h] = (Y[h] >> M) & 0x07070707u;
                            Y[h] &= LMASK;
                        }
                    }
                }
                // d2/d3: high bits of masked groups, found through the mask prefix
                if constexpr (A > 0) {
                    uint32_t h0, h1;
                    unpack_record_row<A, LPG>(img_high, my_word, my_excl, logC, tid, t, h0, h1);
                    Y[0] |= h0 << M;
                    Y[1] |= h1 << M;
                }
                // d4: x = b - sext_n(y) = (b + 2^(n-1)) - (y ^ 2^(n-1)); recombine with sign/mantissa
                uint32_t o[4];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t Z = Y[h] ^ SREP;
                    const uint32_t X = it.mode == 0 ? crep - Z : bytesub_safe(crep, Z);
                    const uint32_t sm = h ? smc[t].y : smc[t].x;
                    uint32_t Hi, Lo;         // high / low bytes of four 16-bit words
                    if constexpr (DT == DT_FP16) {
                        Hi = (sm & 0x80808080u) | ((X & 0x1F1F1F1Fu) << 2) | ((sm >> 5) & 0x03030303u);
                        Lo = ((sm & 0x1F1F1F1Fu) << 3) | T3[h];
                    } else {
                        Hi = bfi(0x7F7F7F7Fu, X >> 1, sm);
                        Lo = bfi(0x7F7F7F7Fu, sm, X << 7);
                    }
                    o[2 * h] = byte_perm(Hi, Lo, 0x05010400u);
                    o[2 * h + 1] = byte_perm(Hi, Lo, 0x07030602u);
                }
                const uint64_t e0 = blk0 + ((uint64_t)t << logC) + 8u * tid;
                if constexpr (DT == DT_FP32) {
                    // element = lower half | bf16 word << 16
                    const uint32_t lo[4] = {tl[t].x, tl[t].y, tl[t].z, tl[t].w};
                    uint32_t w[8];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        w[2 * i] = byte_perm(o[i], lo[i], 0x05040100u);
                        w[2 * i + 1] = byte_perm(o[i], lo[i], 0x07060302u);
                    }
                    uint32_t *out32 = reinterpret_cast<uint32_t *>(it.out);
                    if (e0 + 8 <= it.n_elems) {
                        *reinterpret_cast<uint4 *>(out32 + e0) = make_uint4(w[0], w[1], w[2], w[3]);
                        *reinterpret_cast<uint4 *>(out32 + e0 + 4) = make_uint4(w[4], w[5], w[6], w[7]);
                    } else if (e0 < it.n_elems) {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (e0 + i < it.n_elems) out32[e0 + i] = w[i];
                    }
                } else if (e0 + 8 <= it.n_elems) {
                    *reinterpret_cast<uint4 *>(it.out + e0) = make_uint4(o[0], o[1], o[2], o[3]);
                } else if (e0 < it.n_elems) {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (e0 + i < it.n_elems) it.out[e0 + i] = (uint16_t)(o[i >> 1] >> (16 * (i & 1)));
                }
            }
        }
        // the next block's packed part goes to the other image
        if (validn) {
            to_image(smem + (slot ^ 1u) * img_bytes, vec);
#pragma unroll
            for (int t = 0; t < 8; ++t) smc[t] = smn[t];
        }
        valid = validn;
        validn = check(kn + gridDim.x, c2, ta, tb, offn, sizen);
        k = kn;
        ci = cn;
        cn = c2;
        slot ^= 1u;
    }
}

// ---------------------------------------------------------------------------------
// exponent histogram (Sec. V-E phase 1), of the whole tensor (every = 1) or of a sample of it
// ---------------------------------------------------------------------------------
constexpr uint32_t SAMPLE_CHUNK = 4096;     // elements; the sample is taken in whole chunks

struct HistogramItem {          // one tensor of a launch
    const void *in;
    uint64_t n_elems;
    unsigned long long *hist;   // 256 counters, zero at launch
    uint32_t first, count;      // its workgroups: first .. first + count - 1
};
struct HistogramArgs {
    HistogramItem item[MAX_BATCH];
    uint32_t n_items, every;
};

template <int DT>
__global__ void __launch_bounds__(256) histogram_kernel(const HistogramArgs p)
{
    uint32_t ti = 0;
    for (uint32_t i = 1; i < p.n_items; ++i)
        if (blockIdx.x >= p.item[i].first) ti = i;
    const void *in_ = p.item[ti].in;
    const uint64_t n_elems = p.item[ti].n_elems;
    unsigned long long *hist = p.item[ti].hist;
    const uint32_t every = p.every;
    const uint32_t wg = blockIdx.x - p.item[ti].first, wgs = p.item[ti].count;    // this tensor's share of the grid
    // 32 copies of the histogram, lane i of every wave counts into copy i mod 32: lanes with equal
    // exponents, the normal case, would otherwise queue up on one LDS word; the copies are 257 words
    // apart, which puts the same bin of all copies into different banks.  (Measured on this machine:
    // LDS atomics run at 7.2 lanes per clock and CU when no two lanes of an instruction share a bank
    // beyond the two that must, 4.6 with sixteen copies and Gaussian weights, 0.5 on one address.)
    constexpr uint32_t COPIES = 32, STRIDE = 257;
    __shared__ uint32_t s_h[COPIES * STRIDE];
    const uint32_t tid = threadIdx.x;
    for (uint32_t i = tid; i < COPIES * STRIDE; i += 256) s_h[i] = 0;
    __syncthreads();
    uint32_t *mine = s_h + (tid & (COPIES - 1u)) * STRIDE;
    constexpr uint32_t PER_VEC = DT == DT_FP32 ? 4u : 8u;        // elements in 16 bytes
    const uint64_t nvec = n_elems / PER_VEC;
    const uint64_t stride = (uint64_t)wgs * 256u;
    // the LDS counters cannot overflow: a workgroup counts at most 2^34 / 512 elements
    // the sample: chunks of SAMPLE_CHUNK elements whose number is a multiple of `every`
    constexpr uint32_t LOG_VPC = DT == DT_FP32 ? 10u : 9u;      // 16-byte vectors in a chunk
    const uint64_t chunks = (nvec + (1u << LOG_VPC) - 1u) >> LOG_VPC;
    const uint64_t picked = ((chunks + every - 1u) / every) << LOG_VPC;
    auto count = [&](const uint4 q) {
        const uint32_t d[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (DT == DT_FP32) {
                atomicAdd(&mine[(d[i] >> 23) & 0xFFu], 1u);
            } else if constexpr (DT == DT_FP16) {
                atomicAdd(&mine[(d[i] >> 10) & 0x1Fu], 1u);
                atomicAdd(&mine[(d[i] >> 26) & 0x1Fu], 1u);
            } else {
                atomicAdd(&mine[(d[i] >> 7) & 0xFFu], 1u);
                atomicAdd(&mine[(d[i] >> 23) & 0xFFu], 1u);
            }
        }
    };
    auto vec_of = [&](uint64_t sv) { return (((sv >> LOG_VPC) * every) << LOG_VPC) + (sv & ((1u << LOG_VPC) - 1u)); };
    // four vectors of a thread travel together
    uint64_t sv = (uint64_t)wg * 256u + tid;
    for (; sv + 3u * stride < picked; sv += 4u * stride) {
        uint4 q[4];
        bool ok[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint64_t v = vec_of(sv + u * stride);
            ok[u] = v < nvec;
            q[u] = ok[u] ? reinterpret_cast<const uint4 *>(in_)[v] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (ok[u]) count(q[u]);
    }
    for (; sv < picked; sv += stride) {
        const uint64_t v = vec_of(sv);
        if (v >= nvec) continue;
        count(reinterpret_cast<const uint4 *>(in_)[v]);
    }
    if (wg == 0 && tid < (uint32_t)(n_elems % PER_VEC) && ((nvec * PER_VEC) / SAMPLE_CHUNK) % every == 0) {
        const uint64_t e = nvec * PER_VEC + tid;
        uint32_t x;
        if constexpr (DT == DT_FP32) x = (reinterpret_cast<const uint32_t *>(in_)[e] >> 23) & 0xFFu;
        else if constexpr (DT == DT_FP16) x = (reinterpret_cast<const uint16_t *>(in_)[e] >> 10) & 0x1Fu;
        else x = (reinterpret_cast<const uint16_t *>(in_)[e] >> 7) & 0xFFu;
        atomicAdd(&mine[x], 1u);
    }
    __syncthreads();
    uint32_t c = 0;
#pragma unroll
    for (uint32_t i = 0; i < COPIES; ++i) c += s_h[i * STRIDE + tid];
    if (c) atomicAdd(&hist[tid], (unsigned long long)c);
}

}  // namespace enec
