// ENEC streams with one (b, n, m) per data block: the search of Sec. V-E (Eq. 1-4) runs inside the
// compress kernel on the exponents of each block's own elements, so a tensor whose blocks differ
// (zeros, constants, weights of several scales, noise) is coded block by block with the tuple
// that fits.  One workgroup per data block, one pass over the tensor:
//   ticket -> rows -> split -> LDS histogram -> (b, n) by Eq. 1-3 -> m by Eq. 4 -> transform ->
//   group test -> size (published) -> packing (Alg. 2, widths chosen at run time from the template
//   instances) -> look-back over the earlier blocks' sizes -> stores.
// The widths are run-time values here, so the packers are reached through a switch; the kernels
// of enec_device.hpp, which know their widths at compile time, stay the fast path for one tuple
// per tensor.
#pragma once
#include "enec_kernels.hpp"

namespace enec {

// look-back word of a block: zero = nothing yet
constexpr uint64_t PB_PREFIX = 1ull << 63;     // [60:0] = end of this block's payload (inclusive prefix), / 16
constexpr uint64_t PB_SIZE = 1ull << 62;       // [60:0] = size of this block's payload, / 16
constexpr uint64_t PB_GAVE_UP = 1ull << 61;    // somebody before (or this block) stopped waiting
constexpr uint64_t PB_VALUE = (1ull << 61) - 1;
constexpr int PB_WINDOW = 256;                  // blocks one look-back step covers (4 words per lane)

// the inverse: plane values of the thread's 8 rows from the stream's low plane (already joined
// pairwise by Alg. 2's last step: stream byte 2i = normalized byte i, 2i+1 = normalized byte i + T/2)
template <int LM>
__device__ __forceinline__ void pb_unpack_low(const uint8_t *img_low, uint32_t B, uint32_t logC, uint32_t tid,
                                              uint32_t (&LOW)[8][2])
{
    constexpr HHTable TL = HH<LM>::table;
    uint32_t Pl[LM][2];
    const uint32_t T2 = (LM * B) >> 4;
#pragma unroll
    for (int q = 0; q < LM; ++q) {
        const uint32_t i = ((uint32_t)q << logC) + 8u * tid;
        const bool even = i < T2;
        const uint4 sp = *reinterpret_cast<const uint4 *>(img_low + 2u * (even ? i : i - T2));
        const uint32_t sel = even ? 0x06040200u : 0x07050301u;
        Pl[q][0] = byte_perm(sp.y, sp.x, sel);
        Pl[q][1] = byte_perm(sp.w, sp.z, sel);
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) LOW[t][0] = LOW[t][1] = 0;
#pragma unroll
    for (int f = 0; f < TL.count; ++f) {
        const uint32_t smask = (TL.shift[f] >= 0 ? (TL.dmask[f] >> TL.shift[f]) : (TL.dmask[f] << (-TL.shift[f]))) * 0x01010101u;
#pragma unroll
        for (int h = 0; h < 2; ++h) LOW[TL.row[f]][h] |= shl_or_shr(Pl[TL.plane[f]][h], -TL.shift[f]) & smask;
    }
}

// The records of the masked groups are packed and unpacked by pack_records / unpack_record_row of
// enec_device.hpp, the functions the kernels for one tuple per tensor use.
template <int A, int LPG>
__device__ __forceinline__ void pb_unpack_records(const uint8_t *img_high, uint32_t my_word, uint32_t my_excl,
                                                  uint32_t logC, uint32_t tid, uint32_t (&HI)[8][2])
{
#pragma unroll
    for (int t = 0; t < 8; ++t) unpack_record_row<A, LPG>(img_high, my_word, my_excl, logC, tid, t, HI[t][0], HI[t][1]);
}


// Eq. 1: bits needed for the window [l, h] around b, capped by the exponent field
__device__ __forceinline__ uint32_t pb_width_for(uint32_t b, uint32_t l, uint32_t h, uint32_t E)
{
    const uint32_t pos = 32u - __clz(b - l);                          // bit length, 0 for 0
    const uint32_t neg = h > b ? 32u - __clz(h - b - 1u) : 0u;
    const uint32_t w = (pos > neg ? pos : neg) + 1u;
    return w < E ? w : E;
}

// a1: the 8 rows of data block k as 128-bit vectors (a thread's 8 elements of a row are one vector,
// two for fp32); elements beyond the tensor's end read as zero words
template <int DT>
__device__ __forceinline__ void pb_load_rows(const void *src, uint64_t n_elems, uint32_t B, uint32_t logB, uint32_t k, uint32_t tid, bool active,
                                             uint32_t logC, uint4 (&raw)[DT == DT_FP32 ? 16 : 8])
{
    const uint64_t blk0 = (uint64_t)k << logB;
    const uint32_t real = n_elems - blk0 < B ? (uint32_t)(n_elems - blk0) : B;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const uint32_t at = ((uint32_t)t << logC) + 8u * tid;         // first element of the thread in this row
        if constexpr (DT == DT_FP32) {
            uint4 u = make_uint4(0, 0, 0, 0), v = make_uint4(0, 0, 0, 0);
            if (active && at < real) {
                const uint32_t *in = reinterpret_cast<const uint32_t *>(src) + blk0 + at;
                if (at + 8u <= real) {
                    u = *reinterpret_cast<const uint4 *>(in);
                    v = *reinterpret_cast<const uint4 *>(in + 4);
                } else {
                    uint32_t d[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (at + i < real) d[i] = in[i];
                    u = make_uint4(d[0], d[1], d[2], d[3]);
                    v = make_uint4(d[4], d[5], d[6], d[7]);
                }
            }
            raw[2 * t] = u;
            raw[2 * t + 1] = v;
        } else {
            uint4 r = make_uint4(0, 0, 0, 0);
            if (active && at < real) {
                const uint16_t *in = reinterpret_cast<const uint16_t *>(src) + blk0 + at;
                if (at + 8u <= real) {
                    r = *reinterpret_cast<const uint4 *>(in);
                } else {
                    uint32_t d[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (at + i < real) d[i >> 1] |= (uint32_t)in[i] << (16 * (i & 1));
                    r = make_uint4(d[0], d[1], d[2], d[3]);
                }
            }
            raw[t] = r;
        }
    }
}

// Alg. 2 over the low plane of the thread's 8 rows, taken straight from the transformed bytes Y (bits
// below m; fp16 adds the three left-over mantissa bits kept in bits 5..7 of Y's bytes): the plane
// value of a row exists only while that row is folded into the normalized bytes
template <int LM, int DT>
__device__ __forceinline__ void pb_pack_low_from_y(const uint32_t (&Y)[8][2], uint32_t lrep, uint32_t m,
                                                   uint8_t *img_low, uint32_t logC, uint32_t tid)
{
    constexpr HHTable TL = HH<LM>::table;
    uint32_t acc[LM][2];
#pragma unroll
    for (int q = 0; q < LM; ++q) acc[q][0] = acc[q][1] = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t low = Y[t][h] & lrep;
            if constexpr (DT == DT_FP16) low |= ((Y[t][h] >> 5) & 0x07070707u) << m;
#pragma unroll
            for (int f = 0; f < TL.count; ++f)
                if (TL.row[f] == t) {
                    uint32_t s = shl_or_shr(low, TL.shift[f]);
                    if (!TL.clean[f]) s &= TL.dmask[f] * 0x01010101u;
                    acc[TL.plane[f]][h] |= s;
                }
        }
#pragma unroll
    for (int q = 0; q < LM; ++q)
        *reinterpret_cast<uint2 *>(img_low + ((size_t)q << logC) + 8u * tid) = make_uint2(acc[q][0], acc[q][1]);
}

template <int A, int LPG>
__device__ __forceinline__ void pb_pack_records_from_y(const uint32_t (&Y)[8][2], uint32_t m, uint32_t arep,
                                                       uint32_t my_word, uint32_t my_excl, uint8_t *img_high,
                                                       uint32_t logC, uint32_t tid, bool active)
{
    uint32_t HI[8][2];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        HI[t][0] = (Y[t][0] >> m) & arep;
        HI[t][1] = (Y[t][1] >> m) & arep;
    }
    pack_records<A, LPG>(HI, my_word, my_excl, img_high, logC, tid, active);
}

// minimum over the 64 lanes, in every lane
__device__ __forceinline__ uint32_t wave_min32(uint32_t v)
{
    auto mn = [](uint32_t a, uint32_t b) { return a < b ? a : b; };
    v = mn(v, (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)v, 0x111 /* row_shr:1 */, 0xF, 0xF, false));
    v = mn(v, (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)v, 0x112 /* row_shr:2 */, 0xF, 0xF, false));
    v = mn(v, (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)v, 0x114 /* row_shr:4 */, 0xF, 0xF, false));
    v = mn(v, (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)v, 0x118 /* row_shr:8 */, 0xF, 0xF, false));
    v = mn(v, (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)v, 0x142 /* row_bcast:15 */, 0xA, 0xF, false));
    v = mn(v, (uint32_t)__builtin_amdgcn_update_dpp(-1, (int)v, 0x143 /* row_bcast:31 */, 0xC, 0xF, false));
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// waves per SIMD the compress kernel is built for: six where the instance fits 80 registers without
// spilling (fp16, and bf16 with groups of 16), five elsewhere: a spill here parks raw bytes in scratch
// memory, and they are reloaded when the block is stored, after they have left the L2
#define PB_COMPRESS_WAVES ((DT == DT_FP32 || (DT == DT_BF16 && LPG != 2)) ? 5 : 6)

template <int DT, int LPG>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(PB_COMPRESS_WAVES, PB_COMPRESS_WAVES)))
compress_per_block_kernel(const PbCompressArgs p)
{
    constexpr uint32_t E = exponent_bits(DT);
    constexpr int RW = DT == DT_FP32 ? 16 : 8;
    constexpr int LOG_LPG = LPG == 4 ? 2 : LPG - 1;

    extern __shared__ __align__(16) uint8_t smem[];      // mask | low plane (normalized bytes) | high records
    __shared__ uint32_t s_hist[256];
    __shared__ unsigned long long s_best;                // Eq. 3 cost << 16 | n << 8 | b of the best candidate
    __shared__ uint32_t s_ticket, s_m, s_flags;
    __shared__ unsigned long long s_present[4];          // exponent values that occur, one bit each
    __shared__ unsigned long long s_off;

    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t B = p.B, logC = p.logB - 3u;
    const uint32_t nact = B >> 6;
    const bool active = tid < nact;
    const uint32_t mask_bytes = (B >> 6) >> LOG_LPG;                  // B / (8 L)

    // Blocks are taken in the order in which workgroups start (tickets), not by blockIdx: a block then
    // only waits for blocks that running workgroups hold or that the next workgroups to start will
    // draw, and every workgroup publishes its size before it waits for anything, so the look-back
    // makes progress whatever part of the grid is resident (every wait is bounded by the spin limit
    // as well).  There are PB_TICKET_CLASSES counters: the blocks of a call's launches are numbered
    // through, workgroup w of a launch draws from counter (the launch's first block + w) mod 8, the
    // t-th draw from counter c is block 8 t + c, and every launch has as many workgroups of a class
    // as blocks of it (the counters go on counting from one launch of the call to the next).
    // Returning atomics on one address are serialised at the memory side; with eight addresses the
    // kernel measured 5 % faster than with one.
    const uint32_t cls = (p.first_block + blockIdx.x) & (PB_TICKET_CLASSES - 1u);
    uint32_t ticket = 0;
    if (tid == 0) {
        ticket = atomicAdd(p.ticket + PB_TICKET_STRIDE * cls, 1u);
        s_best = ~0ull;
        s_flags = 0u;
    }
    // Phase 1 counts into PB_HIST_COPIES copies of the histogram (lane i uses copy i mod 16), so that
    // lanes with equal exponents, the normal case, do not queue up on one LDS word; the copies are
    // PB_HIST_STRIDE words apart, which spreads one bin of all copies over the banks.  They share
    // the dynamic LDS with the payload image, which is written only after the search.  They are
    // cleared while the ticket travels.
    uint32_t *hcopy = reinterpret_cast<uint32_t *>(smem);
    for (uint32_t i = tid; i < PB_HIST_COPIES * PB_HIST_STRIDE / 4u; i += blockDim.x)
        reinterpret_cast<uint4 *>(hcopy)[i] = make_uint4(0, 0, 0, 0);
    if (tid == 0) s_ticket = ticket;
    __syncthreads();
    // the tensor this block belongs to (the blocks of the call's tensors are numbered through)
    const uint32_t kg = __builtin_amdgcn_readfirstlane(s_ticket * PB_TICKET_CLASSES + cls);
    if (kg - p.first_block >= p.n_blocks) return;        // (never: a class has as many workgroups as blocks)
    uint32_t ti = 0;
    for (uint32_t i = 1; i < p.n_items; ++i)
        if (kg >= p.item[i].first) ti = i;
    const PbCompressItem &it = p.item[ti];
    const uint32_t k = kg - it.first;
    uint4 raw[RW];
    pb_load_rows<DT>(it.in, it.n_elems, B, p.logB, k, tid, active, logC, raw);
    uint32_t *mine = hcopy + (lane & (PB_HIST_COPIES - 1u)) * PB_HIST_STRIDE;
    const uint64_t blk0 = (uint64_t)k << p.logB;
    const uint32_t real = it.n_elems - blk0 < B ? (uint32_t)(it.n_elems - blk0) : B;   // elements that are not pads
    const bool full = real == B && nact >= 64u;          // no pads and no idle lanes (uniform)

    // ---- a1: rows, split into exponent bytes X and raw bytes SM; fp16's three left-over mantissa bits
    // travel in bits 5..7 of X's bytes (its exponents have five bits) ----
    uint32_t X[8][2], SM[PB_SM_REG_ROWS][2];
    // The raw bytes wait for the block's offset from here to the very end.  Rows PB_SM_REG_ROWS .. 7
    // wait in LDS behind the image (8 bytes per thread and row), the others in registers: with all
    // eight in registers the kernel needs 90 of them, five workgroups fit a CU; with four parked it
    // needs 77 and six fit (LDS: 16.4 KB of image + 8 KB), which measured 5 to 14 % faster.
    uint8_t *sm_park = smem + p.park_at;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const uint32_t at = ((uint32_t)t << logC) + 8u * tid;         // first element of the thread in this row
        uint4 r16;
        if constexpr (DT == DT_FP32) {
            const uint4 u = raw[2 * t], v = raw[2 * t + 1];
            r16 = make_uint4(byte_perm(u.y, u.x, 0x07060302u), byte_perm(u.w, u.z, 0x07060302u),
                             byte_perm(v.y, v.x, 0x07060302u), byte_perm(v.w, v.z, 0x07060302u));
            // the lower halves leave at once (pads have zero lower halves; the region is padded to 16 bytes)
            if (active && at < real)
                *reinterpret_cast<uint4 *>(it.out + it.tail_base + 2u * (blk0 + at)) =
                    make_uint4(byte_perm(u.y, u.x, 0x05040100u), byte_perm(u.w, u.z, 0x05040100u),
                               byte_perm(v.y, v.x, 0x05040100u), byte_perm(v.w, v.z, 0x05040100u));
        } else {
            r16 = raw[t];
        }
        uint32_t sm2[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t d0 = h ? r16.z : r16.x;
            const uint32_t d1 = h ? r16.w : r16.y;
            const uint32_t Lb = byte_perm(d1, d0, 0x06040200u);
            const uint32_t Hb = byte_perm(d1, d0, 0x07050301u);
            uint32_t x;
            if constexpr (DT == DT_FP16) {
                sm2[h] = (Hb & 0x80808080u) | ((Hb & 0x03030303u) << 5) | ((Lb >> 3) & 0x1F1F1F1Fu);
                x = (Hb >> 2) & 0x1F1F1F1Fu;
                X[t][h] = x | ((Lb & 0x07070707u) << 5);
            } else {
                sm2[h] = bfi(0x7F7F7F7Fu, Lb, Hb);
                x = bfi(0xFEFEFEFEu, Hb << 1, Lb >> 7);
                X[t][h] = x;
            }
            // ---- Sec. V-E phase 1: exponent counts of the block's own elements ----
            if (full) {
                if (active) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) atomicAdd(&mine[(x >> (8 * i)) & 0xFFu], 1u);
                }
            } else if (active) {
                const uint32_t e = at + 4u * h;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (e + i < real) atomicAdd(&mine[(x >> (8 * i)) & 0xFFu], 1u);
            }
        }
        if (t < PB_SM_REG_ROWS) { SM[t % PB_SM_REG_ROWS][0] = sm2[0]; SM[t % PB_SM_REG_ROWS][1] = sm2[1]; }
        else *reinterpret_cast<uint2 *>(sm_park + (((uint32_t)(t - PB_SM_REG_ROWS) * blockDim.x + tid) << 3)) = make_uint2(sm2[0], sm2[1]);
    }
    __syncthreads();

    // ---- phase 2: the counts of the 256 exponent values, lowest and highest value present ----
    for (uint32_t x = tid; x < 256u; x += blockDim.x) {
        uint32_t c = 0;
#pragma unroll 8
        for (uint32_t i = 0; i < PB_HIST_COPIES; ++i) c += hcopy[i * PB_HIST_STRIDE + x];
        s_hist[x] = c;
        const uint64_t present = __builtin_amdgcn_ballot_w64(c != 0);       // x / 64 is the same for the whole wave
        if (lane == 0) s_present[x >> 6] = present;
    }
    __syncthreads();
    uint32_t xl = 255u, xh = 0u;
#pragma unroll
    for (int c = 3; c >= 0; --c) {
        const uint64_t z = s_present[c];
        if (z) xl = 64u * c + (uint32_t)__builtin_ctzll(z);
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint64_t z = s_present[c];
        if (z) xh = 64u * c + 63u - (uint32_t)__builtin_clzll(z);
    }
    xl = __builtin_amdgcn_readfirstlane(xl);
    xh = __builtin_amdgcn_readfirstlane(xh);
    // Eq. 4 for every m (lane m holds the count of elements whose y fits m bits) with the group length
    // the block is coded with, 1/L + n + (m - n) p^L, in IEEE double, p^L by three to five squarings;
    // the smallest value wins, ties go to the smaller m (one wave)
    auto choose_m = [&](uint32_t cnt, uint32_t n) -> uint32_t {
        const double q = (double)cnt / (double)real;
        const double q2 = q * q, q4 = q2 * q2;
        double qL = q4 * q4;                                   // p^8
        if constexpr (LPG >= 2) qL = qL * qL;                  // p^16
        if constexpr (LPG == 4) qL = qL * qL;                  // p^32
        const double bexp = (1.0 / (double)(8 * LPG) + (double)n) + ((double)lane - (double)n) * qL;
        const unsigned long long bits = (unsigned long long)__double_as_longlong(bexp);
        uint32_t best_m = 0;
        double best = __longlong_as_double((long long)(((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(bits >> 32), 0) << 32) |
                                                       (uint32_t)__builtin_amdgcn_readlane((int)bits, 0)));
        for (uint32_t j = 1; j <= n; ++j) {
            const double cand = __longlong_as_double((long long)(((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(bits >> 32), (int)j) << 32) |
                                                                 (uint32_t)__builtin_amdgcn_readlane((int)bits, (int)j)));
            if (cand < best) { best = cand; best_m = j; }                 // ties: smaller m
        }
        return best_m;
    };
    if (xh - xl < 64u) {
        // The usual case, at most 64 values between the lowest and the highest: wave 0 does the whole
        // search in registers.  Lane j holds the count of value xl + j and is candidate b = xl + j.
        if (wave == 0) {
            const uint32_t R = xh - xl + 1u;
            const bool valid = lane < R;
            const uint32_t v = valid ? s_hist[xl + lane] : 0u;
            // every b with Eq. 1's n and Eq. 3's cost; ties: smaller n, then smaller b
            const uint32_t nb_ = pb_width_for(xl + lane, xl, xh, E);
            const uint32_t nmask_b = (1u << nb_) - 1u;
            uint32_t D = 0;                                   // at most 2^15 elements * 255
            for (uint32_t i = 0; i < R; ++i)
                D += __umul24((uint32_t)__builtin_amdgcn_readlane((int)v, (int)i), (lane - i) & nmask_b);
            const uint32_t Dmin = wave_min32(valid ? D : 0xFFFFFFFFu);
            const uint32_t pick = wave_min32(valid && D == Dmin ? (nb_ << 8) | (xl + lane) : 0xFFFFFFFFu);
            const uint32_t b = pick & 0xFFu, n = pick >> 8;
            // phase 3: lane m counts the elements whose y fits m bits
            const uint32_t y = (b - (xl + lane)) & ((1u << n) - 1u);
            const uint32_t ybits = 32u - (uint32_t)__clz(y);           // y < 2^m  <=>  ybits <= m
            uint32_t cnt = 0;
            for (uint32_t j = 0; j <= n; ++j) {
                const uint32_t s = wave_sum32(valid && ybits <= j ? v : 0u);
                if (lane == j) cnt = s;
            }
            const uint32_t best_m = choose_m(cnt, n);
            if (lane == 0) {
                s_best = ((unsigned long long)n << 8) | b;
                s_m = best_m;
            }
        }
        __syncthreads();
    } else {
        // A block whose exponents spread over more than 64 values.  Lane j of a wave holds the counts of
        // the values j, 64 + j, 128 + j and 192 + j; wave w takes the candidates b = xl + 64 w + j (and
        // further ones if the workgroup has fewer than four waves); the waves' best meet in s_best.
        // Eq. 1 gives n = 7 or 8 for every b of such a block (the wider side of the window has at least
        // 32 values).  With n fixed, Eq. 3's cost D_n(b) = sum_x count[x] ((b - x) mod 2^n) obeys
        //   D_n(b + 1) - D_n(b) = N - 2^n H_n[(b + 1) mod 2^n],   H_n = the counts folded modulo 2^n,
        // (every term grows by one, the ones that wrap fall by 2^n - 1), so the 64 costs of a wave come
        // from D_n of its first candidate, a sum over the lanes, and a prefix sum of H_n over the lanes.
        uint32_t hv[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) hv[c] = s_hist[64 * c + lane];
        for (uint32_t b0 = xl + 64u * wave; b0 <= xh; b0 += blockDim.x) {
            const uint32_t bb = b0 + lane;
            const bool valid = bb <= xh;
            const uint32_t nb_ = pb_width_for(bb, xl, xh, E);
            const uint32_t h0 = s_hist[bb & 255u], h1 = s_hist[(bb + 128u) & 255u];
            uint32_t D = 0xFFFFFFFFu;                         // costs are at most 2^15 elements * 255
#pragma unroll
            for (uint32_t nn = 7; nn <= 8; ++nn) {
                const uint32_t mask = (1u << nn) - 1u;
                uint32_t t = 0;
#pragma unroll
                for (int c = 0; c < 4; ++c) t += __umul24(hv[c], (b0 - (64u * c + lane)) & mask);
                const uint32_t first = wave_sum32(t);                       // D_nn(b0)
                const uint32_t g = nn == 8 ? h0 : h0 + h1;                  // H_nn[b mod 2^nn]
                const uint32_t upto = wave_incl_scan(g, lane) - (uint32_t)__builtin_amdgcn_readlane((int)g, 0);
                if (nb_ == nn) D = first + lane * real - (upto << nn);
            }
            const uint32_t Dmin = wave_min32(valid ? D : 0xFFFFFFFFu);
            const uint32_t pick = wave_min32(valid && D == Dmin ? (nb_ << 8) | bb : 0xFFFFFFFFu);
            if (lane == 0) atomicMin(&s_best, ((unsigned long long)Dmin << 16) | pick);   // ties: smaller n, then smaller b
        }
        __syncthreads();
        if (wave == 0) {
            const uint32_t b = (uint32_t)s_best & 0xFFu, n = ((uint32_t)s_best >> 8) & 0xFFu;
            uint32_t ybits[4];                                     // y < 2^m  <=>  ybits <= m
#pragma unroll
            for (int c = 0; c < 4; ++c) ybits[c] = 32u - (uint32_t)__clz((b - (64u * c + lane)) & ((1u << n) - 1u));
            uint32_t cnt = 0;
            for (uint32_t j = 0; j <= n; ++j) {
                uint32_t t = 0;
#pragma unroll
                for (int c = 0; c < 4; ++c) t += ybits[c] <= j ? hv[c] : 0u;
                const uint32_t s = wave_sum32(t);
                if (lane == j) cnt = s;
            }
            const uint32_t best_m = choose_m(cnt, n);
            if (lane == 0) s_m = best_m;
        }
        __syncthreads();
    }
    const uint32_t b = (uint32_t)s_best & 0xFFu, n = ((uint32_t)s_best >> 8) & 0xFFu;
    const uint32_t m = s_m, a = n - m;
    const uint32_t lm = m + (DT == DT_FP16 ? 3u : 0u);

    uint8_t *img = smem;
    uint32_t *img_maskw = reinterpret_cast<uint32_t *>(img);
    uint8_t *img_low = img + mask_bytes;
    uint8_t *img_high = img_low + ((lm * B) >> 3);
    const uint32_t fixed = B + mask_bytes + ((lm * B) >> 3);

    // ---- a2 transform (in place: X becomes y, fp16 keeps its three bits above), a3 group test ----
    const uint32_t crep = ((b + (1u << (n - 1))) & 0xFFu) * 0x01010101u;
    const uint32_t brep = b * 0x01010101u;
    const uint32_t srep = (1u << (n - 1)) * 0x01010101u;
    const uint32_t nrep = ((1u << n) - 1u) * 0x01010101u;
    const uint32_t lrep = ((1u << m) - 1u) * 0x01010101u;
    const uint32_t arep = ((1u << a) - 1u) * 0x01010101u;
    const bool mask_writer = lane == 0 && 64u * wave < nact;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        uint32_t gor = 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t x = X[t][h];
            if constexpr (DT == DT_FP16) x &= 0x1F1F1F1Fu;
            if (!full) {      // pads behave like exponent b: y = 0
                const int32_t left = (int32_t)real - (int32_t)(((uint32_t)t << logC) + 8u * tid + 4u * h);
                const uint32_t padm = !active || left <= 0 ? 0xFFFFFFFFu : (left >= 4 ? 0u : 0xFFFFFFFFu << (8 * left));
                x = bfi(padm, brep, x);
            }
            const uint32_t Y = (bytesub_safe(crep, x) ^ srep) & nrep;
            gor |= (Y >> m) & arep;
            if constexpr (DT == DT_FP16) X[t][h] = Y | (X[t][h] & 0xE0E0E0E0u);
            else X[t][h] = Y;
        }
        // a3: OR over the lanes that share a group, one mask bit per group; a wave holds 64 / LPG mask
        // bits of every row, group order = row-major
        if constexpr (LPG == 2) gor |= swap_pair(gor);
        if constexpr (LPG == 4) gor = quad_or(gor);
        const uint64_t flagged = __builtin_amdgcn_ballot_w64(gor != 0);
        if constexpr (LPG == 1) {
            if (mask_writer) {
                if (logC >= 9) {
                    img_maskw[((uint32_t)t << (logC - 8)) + 2u * wave] = (uint32_t)flagged;
                    img_maskw[((uint32_t)t << (logC - 8)) + 2u * wave + 1u] = (uint32_t)(flagged >> 32);
                } else {      // B = 2048: 32 groups per row
                    img_maskw[t] = (uint32_t)flagged;
                }
            }
        } else if constexpr (LPG == 2) {
            const uint32_t mw = compact_even_bits(flagged);
            if (mask_writer) {
                if (logC >= 9) img_maskw[((uint32_t)t << (logC - 9)) + wave] = mw;
                else reinterpret_cast<uint16_t *>(img)[t] = (uint16_t)mw;      // B = 2048: 16 groups per row, one wave
            }
        } else {              // 16 bits per wave and row (B >= 4096)
            const uint32_t mw = compact_fourth_bits(flagged);
            if (mask_writer) reinterpret_cast<uint16_t *>(img)[((uint32_t)t << (logC - 9)) + wave] = (uint16_t)mw;
        }
    }
    __syncthreads();

    // ---- a5 positions: exclusive popcount prefix over the mask words (a wave scan per wave) ----
    const uint32_t nwords = (B >> 8) >> LOG_LPG;          // 32-bit words of the mask (at most 64)
    const uint32_t my_word = lane < nwords ? img_maskw[lane] : 0u;
    const uint32_t my_pc = __popc(my_word);
    const uint32_t my_incl = wave_incl_scan(my_pc, lane);
    const uint32_t my_excl = my_incl - my_pc;
    const uint32_t cnt = __shfl(my_incl, 63, 64);
    const uint32_t S = (fixed + (uint32_t)LPG * a * cnt + 15u) & ~15u;
    // ---- a6: the size is known: publish it before anything else ----
    if (tid == 0) st_state(it.words + k, PB_SIZE | (uint64_t)(S >> 4));

    // ---- a4 low plane ----
    if (active) {
        switch (lm) {
        case 1: pb_pack_low_from_y<1, DT>(X, lrep, m, img_low, logC, tid); break;
        case 2: pb_pack_low_from_y<2, DT>(X, lrep, m, img_low, logC, tid); break;
        case 3: pb_pack_low_from_y<3, DT>(X, lrep, m, img_low, logC, tid); break;
        case 4: pb_pack_low_from_y<4, DT>(X, lrep, m, img_low, logC, tid); break;
        case 5: pb_pack_low_from_y<5, DT>(X, lrep, m, img_low, logC, tid); break;
        case 6: pb_pack_low_from_y<6, DT>(X, lrep, m, img_low, logC, tid); break;
        case 7: pb_pack_low_from_y<7, DT>(X, lrep, m, img_low, logC, tid); break;
        case 8: pb_pack_low_from_y<8, DT>(X, lrep, m, img_low, logC, tid); break;
        default: break;
        }
    }
    switch (a) {
    case 1: pb_pack_records_from_y<1, LPG>(X, m, arep, my_word, my_excl, img_high, logC, tid, active); break;
    case 2: pb_pack_records_from_y<2, LPG>(X, m, arep, my_word, my_excl, img_high, logC, tid, active); break;
    case 3: pb_pack_records_from_y<3, LPG>(X, m, arep, my_word, my_excl, img_high, logC, tid, active); break;
    case 4: pb_pack_records_from_y<4, LPG>(X, m, arep, my_word, my_excl, img_high, logC, tid, active); break;
    case 5: pb_pack_records_from_y<5, LPG>(X, m, arep, my_word, my_excl, img_high, logC, tid, active); break;
    case 6: pb_pack_records_from_y<6, LPG>(X, m, arep, my_word, my_excl, img_high, logC, tid, active); break;
    case 7: pb_pack_records_from_y<7, LPG>(X, m, arep, my_word, my_excl, img_high, logC, tid, active); break;
    case 8: pb_pack_records_from_y<8, LPG>(X, m, arep, my_word, my_excl, img_high, logC, tid, active); break;
    default: break;
    }

    // ---- a6 (wave 0): look back over the earlier blocks, PB_WINDOW at a time (lane i reads blocks
    // top - i, top - 64 - i, ...), until one of them carries its inclusive prefix.  A lower block is held
    // by a workgroup that publishes its size before it waits for anything (see above), so every wait
    // ends; the spin limit is a safety net. ----
    if (wave == 0) {
        uint64_t sum = 0;
        uint32_t flags = 0;
        int64_t top = (int64_t)k - 1;                    // highest block of the current window
        while (top >= 0) {
            uint64_t v[PB_WINDOW / 64];
            bool ok[PB_WINDOW / 64];
#pragma unroll
            for (int w = 0; w < PB_WINDOW / 64; ++w) { v[w] = 0; ok[w] = top - 64 * w - (int64_t)lane < 0; }
            uint32_t spins = 0, first_w = PB_WINDOW / 64, first_lane = 64;
            for (;;) {
#pragma unroll
                for (int w = 0; w < PB_WINDOW / 64; ++w)
                    if (!ok[w]) v[w] = ld_state(it.words + (top - 64 * w - (int64_t)lane));
                // the nearest block with a prefix; everything above it must be there
                bool missing = false;
                first_w = PB_WINDOW / 64;
                first_lane = 64;
#pragma unroll
                for (int w = 0; w < PB_WINDOW / 64; ++w) {
                    if (!ok[w]) ok[w] = v[w] != 0;
                    if (first_w == PB_WINDOW / 64) {
                        const uint64_t stop = __builtin_amdgcn_ballot_w64((v[w] & PB_PREFIX) != 0);
                        const uint64_t need = stop ? ((stop & (~stop + 1ull)) << 1) - 1ull : ~0ull;
                        if (__builtin_amdgcn_ballot_w64(!ok[w]) & need) missing = true;
                        if (stop) { first_w = w; first_lane = (uint32_t)__builtin_ctzll(stop); }
                    }
                }
                if (!missing) break;
                if (++spins > p.spin_limit) { flags |= 4u; break; }
                spin_pause(spins);
            }
            if (flags & 4u) break;
            uint64_t part = 0;
            bool gave_up = false;
#pragma unroll
            for (int w = 0; w < PB_WINDOW / 64; ++w) {
                const bool use = top - 64 * w - (int64_t)lane >= 0 &&
                                 ((uint32_t)w < first_w || ((uint32_t)w == first_w && lane <= first_lane));
                if (use) { part += v[w] & PB_VALUE; gave_up |= (v[w] & PB_GAVE_UP) != 0; }
            }
            if (__builtin_amdgcn_ballot_w64(gave_up)) flags |= 4u;
            sum += wave_sum(part);
            if (first_w != PB_WINDOW / 64) break;
            top -= PB_WINDOW;
        }
        if (lane == 0) {
            s_off = sum << 4;
            s_flags = flags;
            st_state(it.words + k, PB_PREFIX | ((flags & 4u) ? PB_GAVE_UP : 0ull) | (sum + (S >> 4)));
        }
    }
    __syncthreads();

    // ---- a7: stores ----
    const uint64_t off = s_off;
    uint8_t *dst = it.out + it.payload_base + off;
    if (active) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            // pads have zero raw bytes already (their words were loaded as zero)
            const uint2 sm = t < PB_SM_REG_ROWS ? make_uint2(SM[t % PB_SM_REG_ROWS][0], SM[t % PB_SM_REG_ROWS][1])
                                                : *reinterpret_cast<const uint2 *>(sm_park + (((uint32_t)(t - PB_SM_REG_ROWS) * blockDim.x + tid) << 3));
            *reinterpret_cast<uint2 *>(dst + ((size_t)t << logC) + 8u * tid) = sm;
        }
    }
    for (uint32_t v = tid; v < (mask_bytes >> 4); v += blockDim.x)
        *reinterpret_cast<uint4 *>(dst + B + 16u * v) = *reinterpret_cast<const uint4 *>(img + 16u * v);
    if (lm > 0) {
        uint8_t *dlow = dst + B + mask_bytes;
        const uint32_t T2 = (lm * B) >> 4;               // half of the plane's length
        for (uint32_t v = tid; v < (T2 >> 3); v += blockDim.x) {
            const uint2 lo = *reinterpret_cast<const uint2 *>(img_low + 8u * v);
            const uint2 hi = *reinterpret_cast<const uint2 *>(img_low + 8u * v + T2);
            uint4 o;   // stream byte 2i = normalized byte i, stream byte 2i+1 = normalized byte i + T/2
            o.x = byte_perm(hi.x, lo.x, 0x05010400u);
            o.y = byte_perm(hi.x, lo.x, 0x07030602u);
            o.z = byte_perm(hi.y, lo.y, 0x05010400u);
            o.w = byte_perm(hi.y, lo.y, 0x07030602u);
            *reinterpret_cast<uint4 *>(dlow + 16u * v) = o;
        }
    }
    if (a > 0) {
        uint8_t *dhigh = dst + fixed;
        const uint32_t hbytes = (uint32_t)LPG * a * cnt;
        for (uint32_t v = tid; 16u * v < hbytes; v += blockDim.x) {
            const uint4 o = *reinterpret_cast<const uint4 *>(img_high + 16u * v);
            uint32_t w[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {                // zero the padding behind the last record
                const uint32_t at = 16u * v + 4u * i;
                if (at >= hbytes) w[i] = 0;
                else if (at + 4u > hbytes) w[i] &= (1u << (8u * (hbytes - at))) - 1u;
            }
            *reinterpret_cast<uint4 *>(dhigh + 16u * v) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
    if (tid == 0) {
        uint64_t *table = reinterpret_cast<uint64_t *>(it.out + 64);
        table[k] = off;
        *reinterpret_cast<uint32_t *>(it.out + it.tuples_at + 4u * k) = b | (n << 8) | (m << 16);
        if (k == it.nb - 1u) {
            const uint64_t end = off + S;
            const uint32_t status = (s_flags & 4u) ? 8u : 0u;
            const uint64_t total = status ? 0ull : it.payload_base + end;
            table[it.nb] = end;
            if (((uint64_t)(it.nb + 1u) & 1ull)) table[it.nb + 1u] = 0;          // pad up to the tuple table
            for (uint32_t i = it.nb; i < ((it.nb + 3u) & ~3u); ++i)              // pad behind the tuple table
                *reinterpret_cast<uint32_t *>(it.out + it.tuples_at + 4u * i) = 0;
            uint32_t *h = reinterpret_cast<uint32_t *>(it.out);
            h[0] = 0x43454E45u;                                                // "ENEC"
            h[1] = 1u | ((uint32_t)DT << 16) | ((8u * LPG) << 24);             // version, dtype, L
            h[2] = (uint32_t)it.n_elems; h[3] = (uint32_t)(it.n_elems >> 32);
            h[4] = B; h[5] = it.nb;
            h[6] = E << 24;                                                    // (b, n, m) = 0: see the tuple table
            h[7] = status;
            h[8] = (uint32_t)total; h[9] = (uint32_t)(total >> 32);
            h[10] = 1u;                                                        // one tuple per block
#pragma unroll
            for (int i = 11; i < 16; ++i) h[i] = 0;
            if (it.out_bytes) *it.out_bytes = total;
        }
    }
}

// ---------------------------------------------------------------------------------
// decompression of such a stream: one workgroup per data block; tuple and offsets come from the
// stream, every size is checked against the tuple before anything is read or written
// ---------------------------------------------------------------------------------
template <int DT, int LPG>
__global__ void __launch_bounds__(512) decompress_per_block_kernel(const PbDecompressArgs p)
{
    constexpr uint32_t E = exponent_bits(DT);
    constexpr int LOG_LPG = LPG == 4 ? 2 : LPG - 1;
    extern __shared__ __align__(16) uint8_t smem[];      // the packed part as it is in the stream
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t B = p.B, logC = p.logB - 3u;
    const uint32_t nact = B >> 6;
    const bool active = tid < nact;
    const uint32_t mask_bytes = (B >> 6) >> LOG_LPG;                  // B / (8 L)
    // the stream this block belongs to (the blocks of the launch's streams are numbered through)
    if (blockIdx.x >= p.n_blocks) return;
    uint32_t ti = 0;
    for (uint32_t i = 1; i < p.n_items; ++i)
        if (blockIdx.x >= p.item[i].first) ti = i;
    const PbDecompressItem &it = p.item[ti];
    const uint32_t k = blockIdx.x - it.first;

    // d1: header as configured, tuple, offsets
    const uint32_t *hd = reinterpret_cast<const uint32_t *>(it.in);
    bool same = true;
#pragma unroll
    for (int i = 0; i < 11; ++i) same &= (hd[i] == it.hdr[i]);
    const uint32_t tup = *reinterpret_cast<const uint32_t *>(it.in + it.tuples_at + 4u * k);
    const uint32_t b = tup & 0xFFu, n = (tup >> 8) & 0xFFu, m = (tup >> 16) & 0xFFu;
    const uint64_t *table = reinterpret_cast<const uint64_t *>(it.in + 64);
    const uint64_t t0 = table[k], t1 = table[k + 1];
    // a block that is skipped (damaged header, tuple or table entry) leaves its part of the output
    // untouched: the caller is told through the status word
    const uint32_t a = n - m, lm = m + (DT == DT_FP16 ? 3u : 0u);
    const uint32_t fixed = B + mask_bytes + ((lm * B) >> 3);
    const uint64_t sz = t1 - t0;
    if (!same || n < 1u || n > E || m > n || b >= (1u << E) ||
        sz < fixed || sz > fixed + (uint32_t)LPG * a * ((B >> 3) >> LOG_LPG) + 15u || ((sz | t0) & 15u) || t0 > it.payload_bytes || sz > it.payload_bytes - t0) {
        if (tid == 0 && it.status) *it.status = 7u;
        return;
    }
    const uint8_t *src = it.in + it.payload_base + t0;
    const uint32_t nvec = ((uint32_t)sz - B) >> 4;
    for (uint32_t v = tid; v < nvec; v += blockDim.x)
        *reinterpret_cast<uint4 *>(smem + 16u * v) = *reinterpret_cast<const uint4 *>(src + B + 16u * v);
    uint2 smv[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
        smv[t] = active ? *reinterpret_cast<const uint2 *>(src + ((size_t)t << logC) + 8u * tid) : make_uint2(0, 0);
    __syncthreads();
    if (!active) return;

    const uint8_t *img_low = smem + mask_bytes;
    const uint8_t *img_high = img_low + ((lm * B) >> 3);
    const uint32_t nwords = (B >> 8) >> LOG_LPG;
    const uint32_t my_word = lane < nwords ? reinterpret_cast<const uint32_t *>(smem)[lane] : 0u;
    const uint32_t my_pc = __popc(my_word);
    const uint32_t my_excl = wave_incl_scan(my_pc, lane) - my_pc;

    uint32_t LOW[8][2], HI[8][2];
    switch (lm) {
    case 1: pb_unpack_low<1>(img_low, B, logC, tid, LOW); break;
    case 2: pb_unpack_low<2>(img_low, B, logC, tid, LOW); break;
    case 3: pb_unpack_low<3>(img_low, B, logC, tid, LOW); break;
    case 4: pb_unpack_low<4>(img_low, B, logC, tid, LOW); break;
    case 5: pb_unpack_low<5>(img_low, B, logC, tid, LOW); break;
    case 6: pb_unpack_low<6>(img_low, B, logC, tid, LOW); break;
    case 7: pb_unpack_low<7>(img_low, B, logC, tid, LOW); break;
    case 8: pb_unpack_low<8>(img_low, B, logC, tid, LOW); break;
    default:
#pragma unroll
        for (int t = 0; t < 8; ++t) LOW[t][0] = LOW[t][1] = 0;
        break;
    }
    switch (a) {
    case 1: pb_unpack_records<1, LPG>(img_high, my_word, my_excl, logC, tid, HI); break;
    case 2: pb_unpack_records<2, LPG>(img_high, my_word, my_excl, logC, tid, HI); break;
    case 3: pb_unpack_records<3, LPG>(img_high, my_word, my_excl, logC, tid, HI); break;
    case 4: pb_unpack_records<4, LPG>(img_high, my_word, my_excl, logC, tid, HI); break;
    case 5: pb_unpack_records<5, LPG>(img_high, my_word, my_excl, logC, tid, HI); break;
    case 6: pb_unpack_records<6, LPG>(img_high, my_word, my_excl, logC, tid, HI); break;
    case 7: pb_unpack_records<7, LPG>(img_high, my_word, my_excl, logC, tid, HI); break;
    case 8: pb_unpack_records<8, LPG>(img_high, my_word, my_excl, logC, tid, HI); break;
    default:
#pragma unroll
        for (int t = 0; t < 8; ++t) HI[t][0] = HI[t][1] = 0;
        break;
    }

    const uint32_t crep = ((b + (1u << (n - 1))) & 0xFFu) * 0x01010101u;
    const uint32_t srep = (1u << (n - 1)) * 0x01010101u;
    const uint32_t lrep = ((1u << m) - 1u) * 0x01010101u;
    const uint32_t erep = ((1u << E) - 1u) * 0x01010101u;
    const uint64_t blk0 = (uint64_t)k << p.logB;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const uint64_t e0 = blk0 + ((uint64_t)t << logC) + 8u * tid;
        uint32_t o[4];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t Y = (LOW[t][h] & lrep) | (HI[t][h] << m);
            // d4: x = b - sext_n(y) = (b + 2^(n-1)) - (y ^ 2^(n-1)), modulo the exponent field
            const uint32_t Xv = bytesub_safe(crep, Y ^ srep) & erep;
            const uint32_t sm = h ? smv[t].y : smv[t].x;
            uint32_t Hi, Lo;
            if constexpr (DT == DT_FP16) {
                const uint32_t T3 = (LOW[t][h] >> m) & 0x07070707u;
                Hi = (sm & 0x80808080u) | (Xv << 2) | ((sm >> 5) & 0x03030303u);
                Lo = ((sm & 0x1F1F1F1Fu) << 3) | T3;
            } else {
                Hi = bfi(0x7F7F7F7Fu, Xv >> 1, sm);
                Lo = bfi(0x7F7F7F7Fu, sm, Xv << 7);
            }
            o[2 * h] = byte_perm(Hi, Lo, 0x05010400u);
            o[2 * h + 1] = byte_perm(Hi, Lo, 0x07030602u);
        }
        if constexpr (DT == DT_FP32) {
            if (e0 < it.n_elems) {
                const uint4 tl = *reinterpret_cast<const uint4 *>(it.in + it.tail_base + 2u * e0);   // region padded to 16 bytes
                const uint32_t lo[4] = {tl.x, tl.y, tl.z, tl.w};
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
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (e0 + i < it.n_elems) out32[e0 + i] = w[i];
                }
            }
        } else {
            uint16_t *out16 = reinterpret_cast<uint16_t *>(it.out);
            if (e0 + 8 <= it.n_elems) {
                *reinterpret_cast<uint4 *>(out16 + e0) = make_uint4(o[0], o[1], o[2], o[3]);
            } else if (e0 < it.n_elems) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (e0 + i < it.n_elems) out16[e0 + i] = (uint16_t)(o[i >> 1] >> (16 * (i & 1)));
            }
        }
    }
}

}  // namespace enec
