/*
 * ENEC lossless weight codec (bf16, fp16, fp32) -- CPU ORACLE.
 *
 * THIS FILE IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * single-threaded scalar C implementation of the codec exactly as the paper
 * states it, used only to check the GPU library and to be timed beside it as
 * a host baseline.  It shares no code, header, table or helper with the HIP
 * path and must never be linked into or called from it.
 *
 * Parity status: every function here is pinned by the CPU test-suite
 * (paper's worked numbers, hand-worked vectors, closed forms, brute force,
 * an independent pure-Python twin).  The one thing that cannot be pinned
 * without the paper's checkpoints is the compression ratio on real model
 * weights ("parity unpinned"; only the paper's 1.35-1.38 band is checked on
 * Gaussian stand-ins).
 *
 * What is computed, with the passages followed:
 *   split      bf16 -> 8-bit exponent x, and sign+7-bit mantissa kept raw
 *              (Sec. IV-B, Alg. 1 "Split"; Sec. V-A step 1); fp16 (5-bit
 *              exponent) and fp32 (8-bit exponent) are split the same way
 *              (Alg. 1 input line; Sec. VI-B: mantissas are never coded), the
 *              mantissa bits beyond the first seven are kept raw as well, see
 *              orc_compress_dt for where they go
 *   transform  y = (b - x) mod 2^n               (Sec. V-C; Sec. V-E Eq. 2)
 *   group test OR of the L=16 values of a group; group is "anomalous"
 *              (mask bit 1, stored with n bits) iff OR >= 2^m, else stored
 *              with m bits                        (Sec. V-B)
 *   packing    hierarchical-halving bit-packing with byte normalisation
 *              (Sec. V-B, Alg. 2), used for the low-m-bit plane of a whole
 *              data block and for the high (n-m) bits of each anomalous group
 *   placement  prefix sum of per-block compressed sizes -> start of every
 *              block's payload                    (Fig. 4 caption)
 *   inverse    mask -> {0,1} -> exclusive prefix sum -> position of each
 *              anomalous group's high bits; unpack; OR; x = b - sext_n(y);
 *              recombine                          (Sec. IV-B Alg. 1
 *              decompression part; Sec. V-A last paragraph)
 *   tuning     histogram -> b,n by Eq. 1-3 -> m by Eq. 4 with L = 16
 *              (Sec. V-E phases 1-3)
 *
 * Readings where the paper is silent or inconsistent are listed in the
 * repository's design notes; the ones that matter for the bytes are repeated
 * at the function that takes them.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

enum {
    ORC_OK = 0,
    ORC_E_ARG = 1,
    ORC_E_DTYPE = 2,
    ORC_E_BLOCK = 3,
    ORC_E_PARAMS = 4,
    ORC_E_CAPACITY = 5,
    ORC_E_RANGE = 6,
    ORC_E_FORMAT = 7
};

#define ORC_L 16u          /* default group length, Sec. VI-D "Group Length" / Table VI */

/* Group lengths the container accepts: Eq. 4 searches L jointly with m; the paper's hardware
 * forces L >= 16 and L = 16 always wins there (Sec. V-E phase 3, Sec. VI-D). */
static int group_ok(unsigned L) { return L == 8u || L == 16u || L == 32u; }
#define ORC_HEADER 64u

/* ------------------------------------------------------------------ */
/* Alg. 2: hierarchical halving bit-packing with byte normalisation.   */
/* ------------------------------------------------------------------ */

/* Packs N values (each < 2^a, N a power of two, 0 < a <= 8) held in 16-bit
 * lanes.  Writes the byte stream to out, returns its length.  The steps are
 * those of Alg. 2 in its order: fold while the lane width is below 8, peel
 * the low byte of every live lane, continue on the overflow, pad to an even
 * count, then join byte i with byte i + total/2 into little-endian words. */
size_t orc_hh_pack(const uint16_t *data_in, size_t N, int a, uint8_t *out)
{
    uint16_t *data = (uint16_t *)malloc((N ? N : 1) * sizeof(uint16_t));
    uint8_t *normalized = (uint8_t *)malloc(N * 2 + 2);
    size_t total_length = 0, length = N, i, j;
    int width = a;
    memcpy(data, data_in, N * sizeof(uint16_t));

    while (width > 0) {
        while (length > 1 && width < 8) {
            length = length / 2;
            for (i = 0; i < length; i++)
                data[i] = (uint16_t)(data[i] | (uint16_t)(data[i + length] << width));
            width = width * 2;
        }
        for (j = 0; j < length; j++) {
            normalized[total_length + j] = (uint8_t)(data[j] & 0xFFu);
            data[j] = (uint16_t)(data[j] >> 8);
        }
        width = width - 8;
        total_length = total_length + length;
    }
    if (total_length % 2 != 0) {
        normalized[total_length] = 0;
        total_length = total_length + 1;
    }
    for (i = 0; i < total_length / 2; i++) {
        uint16_t word = (uint16_t)(normalized[i] | (normalized[i + total_length / 2] << 8));
        out[2 * i] = (uint8_t)(word & 0xFFu);        /* words are little-endian */
        out[2 * i + 1] = (uint8_t)(word >> 8);
    }
    free(data);
    free(normalized);
    return total_length;
}

/* Inverse of orc_hh_pack ("the bit-unpacking process is precisely the inverse
 * of the bit-packing process", Sec. V-B): the forward schedule of folds and
 * peels is replayed to learn its shape, then undone last step first. */
size_t orc_hh_unpack(const uint8_t *in, size_t N, int a, uint16_t *data)
{
    enum { MAXOPS = 64 };
    int op_kind[MAXOPS];         /* 0 = fold, 1 = peel */
    size_t op_len[MAXOPS];       /* live lanes after the fold / during the peel */
    int op_width[MAXOPS];        /* lane width before the fold */
    size_t op_off[MAXOPS];       /* peel: offset of its bytes in the normalised vector */
    int nops = 0, width = a, k;
    size_t length = N, total_length = 0, i;
    uint8_t *normalized;

    while (width > 0) {
        while (length > 1 && width < 8) {
            length = length / 2;
            op_kind[nops] = 0; op_len[nops] = length; op_width[nops] = width; op_off[nops] = 0;
            nops++;
            width = width * 2;
        }
        op_kind[nops] = 1; op_len[nops] = length; op_width[nops] = width; op_off[nops] = total_length;
        nops++;
        width = width - 8;
        total_length = total_length + length;
    }
    if (total_length % 2 != 0) total_length = total_length + 1;

    normalized = (uint8_t *)malloc(total_length + 1);
    for (i = 0; i < total_length / 2; i++) {
        normalized[i] = in[2 * i];
        normalized[i + total_length / 2] = in[2 * i + 1];
    }
    for (i = 0; i < N; i++) data[i] = 0;
    for (k = nops - 1; k >= 0; k--) {
        if (op_kind[k] == 1) {
            for (i = 0; i < op_len[k]; i++)
                data[i] = (uint16_t)((data[i] << 8) | normalized[op_off[k] + i]);
        } else {
            uint16_t keep = (uint16_t)((1u << op_width[k]) - 1u);
            for (i = 0; i < op_len[k]; i++) {
                data[i + op_len[k]] = (uint16_t)(data[i] >> op_width[k]);
                data[i] = (uint16_t)(data[i] & keep);
            }
        }
    }
    free(normalized);
    return total_length;
}

/* ------------------------------------------------------------------ */
/* Sec. V-C / Eq. 2: the branch-free integer transformation.           */
/* ------------------------------------------------------------------ */

/* n is the TOTAL stored width (the n of Sec. V-E and Table VI; Sec. V-C
 * counts the sign bit separately, so its "n" is this n minus one).
 * Returns y = (b - x) mod 2^n in [0, 2^n). */
unsigned orc_transform(unsigned x, unsigned b, unsigned n)
{
    int d = (int)b - (int)x;
    int mod = 1 << n;
    int y = d % mod;
    if (y < 0) y += mod;
    return (unsigned)y;
}

/* 1 iff x can be represented: n == 8 (the map is a bijection of all 8-bit
 * exponents) or b - x lies in the signed n-bit range. */
int orc_in_range(unsigned x, unsigned b, unsigned n)
{
    int d = (int)b - (int)x;
    if (n >= 8) return 1;
    return d >= -(1 << (n - 1)) && d <= (1 << (n - 1)) - 1;
}

/* Inverse: sign-extend y from n bits, x = (b - s) mod 256. */
unsigned orc_inverse_transform(unsigned y, unsigned b, unsigned n)
{
    int s = (int)y;
    if (y >= (1u << (n - 1))) s -= (1 << n);
    return (unsigned)(((int)b - s) & 0xFF);
}

/* The same two for an exponent field of E bits (8 for bf16 and fp32, 5 for
 * fp16): at n = E the map is a bijection of all E-bit exponents. */
int orc_in_range_e(unsigned x, unsigned b, unsigned n, unsigned E)
{
    int d = (int)b - (int)x;
    if (n >= E) return 1;
    return d >= -(1 << (n - 1)) && d <= (1 << (n - 1)) - 1;
}

unsigned orc_inverse_transform_e(unsigned y, unsigned b, unsigned n, unsigned E)
{
    int s = (int)y;
    if (y >= (1u << (n - 1))) s -= (1 << n);
    return (unsigned)(((int)b - s) & ((1 << E) - 1));
}

/* ------------------------------------------------------------------ */
/* Sec. V-E: parameter tuning.                                         */
/* ------------------------------------------------------------------ */

static unsigned bitlen(unsigned v)
{
    unsigned r = 0;
    while (v) { r++; v >>= 1; }
    return r;
}

/* Eq. 1 with its edge cases made explicit: floor(log2 v)+1 = bitlen(v) and
 * ceil(log2 v) = bitlen(v-1) wherever Eq. 1 is defined; bitlen(0)=0 covers
 * b = l and b = h; n is capped at the 8 bits an exponent has. */
unsigned orc_width_for_e(unsigned b, unsigned l, unsigned h, unsigned E)
{
    unsigned pos = bitlen(b - l);
    unsigned neg = (h > b) ? bitlen(h - b - 1) : 0;
    unsigned n = (pos > neg ? pos : neg) + 1;
    return n > E ? E : n;
}

unsigned orc_width_for(unsigned b, unsigned l, unsigned h) { return orc_width_for_e(b, l, h, 8); }

/* Element formats.  dtype 0 = bf16 (1|8|7), 1 = fp16 (1|5|10), 2 = fp32 (1|8|23). */
enum { ORC_BF16 = 0, ORC_FP16 = 1, ORC_FP32 = 2 };

static int dtype_ok(int dtype) { return dtype == ORC_BF16 || dtype == ORC_FP16 || dtype == ORC_FP32; }
unsigned orc_exp_bits(int dtype) { return dtype == ORC_FP16 ? 5u : 8u; }
unsigned orc_elem_bytes(int dtype) { return dtype == ORC_FP32 ? 4u : 2u; }

/* Element e of a tensor as an unsigned integer (little-endian words in memory). */
static uint32_t load_elem(const void *in, size_t e, int dtype)
{
    if (dtype == ORC_FP32) return ((const uint32_t *)in)[e];
    return ((const uint16_t *)in)[e];
}

/* Split (Alg. 1 "Split"): exponent field, the raw byte sign<<7 | first seven
 * mantissa bits, and the mantissa bits that are left over (none for bf16,
 * 3 for fp16, 16 for fp32). */
static void split_elem(uint32_t w, int dtype, unsigned *x, unsigned *sm, unsigned *rest)
{
    if (dtype == ORC_FP32) {
        *x = (w >> 23) & 0xFFu;
        *sm = ((w >> 24) & 0x80u) | ((w >> 16) & 0x7Fu);
        *rest = w & 0xFFFFu;
    } else if (dtype == ORC_FP16) {
        *x = (w >> 10) & 0x1Fu;
        *sm = ((w >> 8) & 0x80u) | ((w >> 3) & 0x7Fu);
        *rest = w & 0x7u;
    } else {
        *x = (w >> 7) & 0xFFu;
        *sm = ((w >> 8) & 0x80u) | (w & 0x7Fu);
        *rest = 0;
    }
}

static uint32_t join_elem(unsigned x, unsigned sm, unsigned rest, int dtype)
{
    if (dtype == ORC_FP32) return ((uint32_t)(sm & 0x80u) << 24) | ((uint32_t)x << 23) | ((uint32_t)(sm & 0x7Fu) << 16) | rest;
    if (dtype == ORC_FP16) return ((sm & 0x80u) << 8) | (x << 10) | ((sm & 0x7Fu) << 3) | rest;
    return ((sm & 0x80u) << 8) | (x << 7) | (sm & 0x7Fu);
}

void orc_histogram_dt(const void *w, size_t n_elems, int dtype, uint64_t hist[256])
{
    size_t i;
    memset(hist, 0, 256 * sizeof(uint64_t));
    for (i = 0; i < n_elems; i++) {
        unsigned x, sm, rest;
        split_elem(load_elem(w, i, dtype), dtype, &x, &sm, &rest);
        hist[x]++;
    }
}

void orc_histogram(const uint16_t *w, size_t n_elems, uint64_t hist[256])
{
    orc_histogram_dt(w, n_elems, ORC_BF16, hist);
}

/* Phases 2 and 3 on a given histogram.  out_D receives the integer cost
 * sum_x c[x]*y (Eq. 3 times N), out_bexp the value of Eq. 4 at the optimum.
 * Ties: smaller D wins, then smaller n, then smaller b; for m the smaller m.
 * L is fixed to 16.  An empty histogram gives (0, 1, 0). */
void orc_tune_hist_e(const uint64_t hist[256], unsigned E, uint8_t params[4], uint64_t *out_D, double *out_bexp)
{
    unsigned l = 256, h = 0, x, b, best_b = 0, best_n = 1, m, best_m = 0;
    uint64_t total = 0, best_D = 0;
    double best_bexp = 0.0;
    int have = 0;

    for (x = 0; x < 256; x++)
        if (hist[x]) { if (x < l) l = x; h = x; total += hist[x]; }
    if (total == 0) {
        params[0] = 0; params[1] = 1; params[2] = 0; params[3] = ORC_L;
        if (out_D) *out_D = 0;
        if (out_bexp) *out_bexp = 1.0 / 16.0;
        return;
    }
    for (b = l; b <= h; b++) {
        unsigned n = orc_width_for_e(b, l, h, E);
        uint64_t D = 0;
        for (x = l; x <= h; x++) D += hist[x] * (uint64_t)orc_transform(x, b, n);
        if (!have || D < best_D || (D == best_D && n < best_n)) {
            have = 1; best_D = D; best_n = n; best_b = b;
        }
    }
    have = 0;
    for (m = 0; m <= best_n; m++) {
        uint64_t cnt = 0;
        double p, p2, p4, p8, p16, bexp;
        for (x = l; x <= h; x++)
            if (orc_transform(x, best_b, best_n) < (1u << m)) cnt += hist[x];
        p = (double)cnt / (double)total;
        p2 = p * p; p4 = p2 * p2; p8 = p4 * p4; p16 = p8 * p8;
        bexp = (1.0 / 16.0 + (double)best_n) + ((double)m - (double)best_n) * p16;
        if (!have || bexp < best_bexp) { have = 1; best_bexp = bexp; best_m = m; }
    }
    params[0] = (uint8_t)best_b; params[1] = (uint8_t)best_n;
    params[2] = (uint8_t)best_m; params[3] = ORC_L;
    if (out_D) *out_D = best_D;
    if (out_bexp) *out_bexp = best_bexp;
}

void orc_tune_hist(const uint64_t hist[256], uint8_t params[4], uint64_t *out_D, double *out_bexp)
{
    orc_tune_hist_e(hist, 8, params, out_D, out_bexp);
}

/* Phase 3 as Eq. 4 states it, with the group length searched jointly with m over the lengths
 * whose bits are set in `lengths` (8 | 16 | 32): B_exp(m, L) = 1/L + n + (m - n) p(m)^L, the power
 * by repeated squaring.  (b, n) come from phase 2 as above.  Ties: smaller m, then smaller L. */
void orc_tune_hist_groups(const uint64_t hist[256], unsigned E, unsigned lengths, uint8_t params[4],
                          uint64_t *out_D, double *out_bexp)
{
    unsigned l = 256, h = 0, x, m, L, best_m = 0, best_L = 0, b, n;
    uint64_t total = 0;
    double best = 0.0;
    int have = 0;
    orc_tune_hist_e(hist, E, params, out_D, NULL);
    b = params[0]; n = params[1];
    for (x = 0; x < 256; x++)
        if (hist[x]) { if (x < l) l = x; h = x; total += hist[x]; }
    for (m = 0; m <= n; m++) {
        uint64_t cnt = 0;
        double p, pw;
        if (total) {
            for (x = l; x <= h; x++)
                if (orc_transform(x, b, n) < (1u << m)) cnt += hist[x];
            p = (double)cnt / (double)total;
        } else {
            p = 1.0;
        }
        pw = p * p; pw = pw * pw; pw = pw * pw;          /* p^8 */
        for (L = 8; L <= 32; L *= 2) {
            if (lengths & L) {
                double bexp = (1.0 / (double)L + (double)n) + ((double)m - (double)n) * pw;
                if (!have || bexp < best) { have = 1; best = bexp; best_m = m; best_L = L; }
            }
            pw = pw * pw;                                /* p^16, p^32 */
        }
    }
    if (have) { params[2] = (uint8_t)best_m; params[3] = (uint8_t)best_L; }
    if (out_bexp) *out_bexp = best;
}

void orc_tune(const uint16_t *w, size_t n_elems, uint8_t params[4], uint64_t *out_D, double *out_bexp)
{
    uint64_t hist[256];
    orc_histogram(w, n_elems, hist);
    orc_tune_hist(hist, params, out_D, out_bexp);
}

void orc_tune_dt(const void *w, size_t n_elems, int dtype, uint8_t params[4], uint64_t *out_D, double *out_bexp)
{
    uint64_t hist[256];
    orc_histogram_dt(w, n_elems, dtype, hist);
    orc_tune_hist_e(hist, orc_exp_bits(dtype), params, out_D, out_bexp);
}

/* ------------------------------------------------------------------ */
/* Container.                                                          */
/* ------------------------------------------------------------------ */

static size_t align16(size_t v) { return (v + 15u) & ~(size_t)15u; }

static int block_ok(uint32_t B)
{
    return B >= 128u && B <= 32768u && (B & (B - 1u)) == 0;
}

/* Default data-block size: 16384 (Sec. VI-D "Data Block Size"); a tensor
 * shorter than that takes the largest power of two not above its length,
 * but never below 2048. */
uint32_t orc_default_block(size_t n_elems)
{
    uint32_t B = 16384u;
    if (n_elems >= B) return B;
    while (B > 2048u && B > n_elems) B >>= 1;
    return B;
}

size_t orc_num_blocks(size_t n_elems, uint32_t B) { return (n_elems + B - 1) / B; }

/* End of header + offset table, rounded up to 16. */
size_t orc_table_end(size_t n_elems, uint32_t B)
{
    return align16(ORC_HEADER + 8u * (orc_num_blocks(n_elems, B) + 1u));
}

/* Where the block payloads start.  An fp32 stream keeps the low 16 mantissa
 * bits of all elements between the table and the payloads. */
size_t orc_payload_base_dt(size_t n_elems, uint32_t B, int dtype)
{
    size_t base = orc_table_end(n_elems, B);
    if (dtype == ORC_FP32) base += align16(2u * n_elems);
    return base;
}

size_t orc_payload_base(size_t n_elems, uint32_t B) { return orc_payload_base_dt(n_elems, B, ORC_BF16); }

/* A stream with one tuple per data block keeps them, four bytes each (b, n, m, 0),
 * block order, zeros to a multiple of 16, right behind the offset table; the fp32
 * region and the payloads follow. */
size_t orc_tuple_table_bytes(size_t n_elems, uint32_t B)
{
    return align16(4u * orc_num_blocks(n_elems, B));
}

size_t orc_payload_base_pb(size_t n_elems, uint32_t B, int dtype)
{
    return orc_payload_base_dt(n_elems, B, dtype) + orc_tuple_table_bytes(n_elems, B);
}

/* Worst case for any group length: every group anomalous with n = 8 (bf16, fp32:
 * B raw bytes + B bytes of planes) or n = 5 (fp16: B raw bytes + (5+3)B/8
 * bytes of planes), and the longest mask (L = 8: B/64 bytes). */
size_t orc_compress_bound_dt(size_t n_elems, uint32_t B, int dtype)
{
    size_t nb = orc_num_blocks(n_elems, B);
    size_t per_block = align16((size_t)B + B / 64u + (size_t)B);
    return orc_payload_base_dt(n_elems, B, dtype) + nb * per_block;
}

size_t orc_compress_bound(size_t n_elems, uint32_t B) { return orc_compress_bound_dt(n_elems, B, ORC_BF16); }

size_t orc_compress_bound_pb(size_t n_elems, uint32_t B, int dtype)
{
    return orc_compress_bound_dt(n_elems, B, dtype) + orc_tuple_table_bytes(n_elems, B);
}

static void put_u16(uint8_t *p, uint16_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static void put_u32(uint8_t *p, uint32_t v) { int i; for (i = 0; i < 4; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static void put_u64(uint8_t *p, uint64_t v) { int i; for (i = 0; i < 8; i++) p[i] = (uint8_t)(v >> (8 * i)); }
static uint16_t get_u16(const uint8_t *p) { return (uint16_t)(p[0] | (p[1] << 8)); }
static uint32_t get_u32(const uint8_t *p) { uint32_t v = 0; int i; for (i = 3; i >= 0; i--) v = (v << 8) | p[i]; return v; }
static uint64_t get_u64(const uint8_t *p) { uint64_t v = 0; int i; for (i = 7; i >= 0; i--) v = (v << 8) | p[i]; return v; }

static void write_header(uint8_t *out, size_t n_elems, int dtype, uint32_t B, size_t nb,
                         const uint8_t params[4], uint32_t status, uint64_t total)
{
    memset(out, 0, ORC_HEADER);
    out[0] = 'E'; out[1] = 'N'; out[2] = 'E'; out[3] = 'C';
    put_u16(out + 4, 1);
    out[6] = (uint8_t)dtype;
    out[7] = params[3];
    put_u64(out + 8, (uint64_t)n_elems);
    put_u32(out + 16, B);
    put_u32(out + 20, (uint32_t)nb);
    out[24] = params[0]; out[25] = params[1]; out[26] = params[2];
    out[27] = (uint8_t)orc_exp_bits(dtype);
    put_u32(out + 28, status);
    put_u64(out + 32, total);
}

/* Compresses n_elems values of the given dtype (little-endian words) with
 * data-block size B and parameters (b, n, m, L), L one of 8, 16, 32 with
 * B >= 8 L; n is at most the width of the dtype's exponent field.
 *
 * Per data block (Sec. V-A, V-B; stream layout after the Fig. 4 caption):
 *   payload = raw bytes (sign<<7 | first seven mantissa bits) of the B elements,
 *             element order
 *           | group bit mask, B/(8L) bytes, group g = bit (g mod 8), LSB first,
 *             of byte (g div 8); 1 = anomalous
 *           | Alg. 2 over the low plane of all B values
 *               bf16, fp32: the low m bits of y                     (m*B/8 bytes)
 *               fp16: the low m bits of y with the element's last three
 *                     mantissa bits on top, (y mod 2^m) | (w & 7) << m
 *                                                                   ((m+3)*B/8 bytes)
 *           | for each anomalous group in group order, Alg. 2 over the
 *             high n-m bits of its L values; the zero byte Alg. 2 appends to an
 *             odd byte count (only L = 8 with odd n-m) is not stored
 *                                                                   ((n-m)L/8 bytes each)
 *           | zeros up to a multiple of 16
 * The last block is completed with elements that encode as y = 0 and zero raw
 * bits.  Groups are runs of L consecutive elements.
 * Stream = 64-byte header | (nb+1) u64 block offsets (exclusive prefix sums
 * of payload sizes, last = sum) | zeros to a multiple of 16
 *        | fp32 only: the low 16 bits of every element, element order, little
 *          endian, then zeros to a multiple of 16
 *        | payloads.
 * The paper codes exponents only and leaves the storage of the remaining
 * mantissa bits open (Sec. VI-B "we avoid compressing the mantissa"): fp16's
 * three bits ride in the low plane because 11 raw bits are no whole number of
 * bytes and m + 3 <= 8 always fits Alg. 2; fp32's two bytes per element sit at
 * a position that does not depend on any compressed size.
 *
 * A value outside the representable window gives ORC_E_RANGE: the header is
 * still written, with status = ORC_E_RANGE and total_bytes = 0, *out_bytes = 0.
 */
static int compress_core(const void *in, size_t n_elems, int dtype, uint32_t B, const uint8_t params[4],
                         int per_block, uint8_t *out, size_t capacity, size_t *out_bytes)
{
    unsigned b, n, m, a, E, lowbits, L;
    size_t nb, base, k, off = 0, G, e, rb;
    uint8_t *sm, *maskbytes, rec[80], *tuples = NULL;
    uint16_t *y, *rest, *tmp;
    int range_error = 0;

    if (!out || !out_bytes || !params || (!in && n_elems)) return ORC_E_ARG;
    if (!dtype_ok(dtype)) return ORC_E_DTYPE;
    if (!block_ok(B)) return ORC_E_BLOCK;
    E = orc_exp_bits(dtype);
    b = params[0]; n = params[1]; m = params[2]; L = params[3];
    if (!group_ok(L) || B < 8u * L) return ORC_E_PARAMS;
    if (!per_block && (n < 1 || n > E || m > n || b >= (1u << E))) return ORC_E_PARAMS;
    if (capacity < (per_block ? orc_compress_bound_pb(n_elems, B, dtype) : orc_compress_bound_dt(n_elems, B, dtype)))
        return ORC_E_CAPACITY;
    nb = orc_num_blocks(n_elems, B);
    base = per_block ? orc_payload_base_pb(n_elems, B, dtype) : orc_payload_base_dt(n_elems, B, dtype);
    G = B / L;
    memset(out, 0, base);
    if (per_block) tuples = out + orc_table_end(n_elems, B);
    if (dtype == ORC_FP32 && per_block) {
        uint8_t *t = out + orc_table_end(n_elems, B) + orc_tuple_table_bytes(n_elems, B);
        for (e = 0; e < n_elems; e++) put_u16(t + 2 * e, (uint16_t)(load_elem(in, e, dtype) & 0xFFFFu));
    }

    if (dtype == ORC_FP32 && !per_block) {
        uint8_t *t = out + orc_table_end(n_elems, B);
        for (e = 0; e < n_elems; e++) put_u16(t + 2 * e, (uint16_t)(load_elem(in, e, dtype) & 0xFFFFu));
    }

    sm = (uint8_t *)malloc(B);
    maskbytes = (uint8_t *)malloc(G / 8 ? G / 8 : 1);
    y = (uint16_t *)malloc(B * sizeof(uint16_t));
    rest = (uint16_t *)malloc(B * sizeof(uint16_t));
    tmp = (uint16_t *)malloc(B * sizeof(uint16_t));

    for (k = 0; k < nb; k++) {
        uint8_t *p = out + base + off;
        size_t pos = 0, i, g;
        if (per_block) {
            /* Sec. V-E on the exponents of this block's own elements */
            uint8_t t[4];
            size_t first = k * (size_t)B, count = n_elems - first < B ? n_elems - first : B;
            uint64_t hist[256];
            const uint8_t *src = (const uint8_t *)in + first * orc_elem_bytes(dtype);
            orc_histogram_dt(src, count, dtype, hist);
            /* phase 3 with the group length the block is coded with: Eq. 4 is 1/L + n + (m - n) p(m)^L */
            orc_tune_hist_groups(hist, E, L, t, NULL, NULL);
            b = t[0]; n = t[1]; m = t[2];
            tuples[4 * k] = t[0]; tuples[4 * k + 1] = t[1]; tuples[4 * k + 2] = t[2];
        }
        a = n - m;
        rb = (size_t)a * L / 8u;                 /* bytes of one high record */
        lowbits = m + (dtype == ORC_FP16 ? 3u : 0u);
        /* split + transform */
        for (i = 0; i < B; i++) {
            e = k * (size_t)B + i;
            if (e < n_elems) {
                unsigned x, s, r;
                split_elem(load_elem(in, e, dtype), dtype, &x, &s, &r);
                sm[i] = (uint8_t)s;
                rest[i] = (uint16_t)r;
                if (!orc_in_range_e(x, b, n, E)) range_error = 1;
                y[i] = (uint16_t)orc_transform(x, b, n);
            } else {
                sm[i] = 0;
                rest[i] = 0;
                y[i] = 0;
            }
        }
        /* group test by bitwise OR */
        memset(maskbytes, 0, G / 8 ? G / 8 : 1);
        for (g = 0; g < G; g++) {
            unsigned o = 0;
            for (i = 0; i < L; i++) o |= y[g * L + i];
            if (o >= (1u << m)) maskbytes[g / 8] |= (uint8_t)(1u << (g % 8));
        }
        memcpy(p + pos, sm, B); pos += B;
        memcpy(p + pos, maskbytes, G / 8); pos += G / 8;
        /* low plane */
        if (lowbits > 0) {
            for (i = 0; i < B; i++) {
                unsigned v = y[i] & ((1u << m) - 1u);
                if (dtype == ORC_FP16) v |= (unsigned)rest[i] << m;
                tmp[i] = (uint16_t)v;
            }
            pos += orc_hh_pack(tmp, B, (int)lowbits, p + pos);
        }
        /* high plane: one record per anomalous group */
        for (g = 0; g < G; g++) {
            if (maskbytes[g / 8] & (1u << (g % 8))) {
                for (i = 0; i < L; i++) tmp[i] = (uint16_t)(y[g * L + i] >> m);
                orc_hh_pack(tmp, L, (int)a, rec);
                memcpy(p + pos, rec, rb);
                pos += rb;
            }
        }
        while (pos % 16) p[pos++] = 0;
        put_u64(out + ORC_HEADER + 8 * k, (uint64_t)off);
        off += pos;
    }
    put_u64(out + ORC_HEADER + 8 * nb, (uint64_t)off);
    free(sm); free(maskbytes); free(y); free(rest); free(tmp);

    if (range_error) {
        write_header(out, n_elems, dtype, B, nb, params, ORC_E_RANGE, 0);
        *out_bytes = 0;
        return ORC_E_RANGE;
    }
    write_header(out, n_elems, dtype, B, nb, params, ORC_OK, (uint64_t)(base + off));
    if (per_block) out[40] = 1;
    *out_bytes = base + off;
    return ORC_OK;
}

int orc_compress_dt(const void *in, size_t n_elems, int dtype, uint32_t B, const uint8_t params[4],
                    uint8_t *out, size_t capacity, size_t *out_bytes)
{
    return compress_core(in, n_elems, dtype, B, params, 0, out, capacity, out_bytes);
}

/* One tuple per data block: block k is coded with the (b, n, m) that Sec. V-E's
 * search returns for the exponents of its own elements (the pad elements of the
 * last block are not counted), so no exponent is ever out of range.  Header:
 * byte 40 = 1, and (b, n, m) = (0, 0, 0); n = 0 occurs in no other stream.
 * The tuples sit behind the offset table (see orc_tuple_table_bytes). */
int orc_compress_pb(const void *in, size_t n_elems, int dtype, uint32_t B, unsigned L,
                    uint8_t *out, size_t capacity, size_t *out_bytes)
{
    uint8_t params[4] = {0, 0, 0, 0};
    params[3] = (uint8_t)L;
    return compress_core(in, n_elems, dtype, B, params, 1, out, capacity, out_bytes);
}

int orc_compress(const uint16_t *in, size_t n_elems, uint32_t B, const uint8_t params[4],
                 uint8_t *out, size_t capacity, size_t *out_bytes)
{
    return orc_compress_dt(in, n_elems, ORC_BF16, B, params, out, capacity, out_bytes);
}

/* Reads the fixed header.  Any output may be NULL. */
int orc_stream_info_dt(const uint8_t *hdr, uint8_t params[4], uint64_t *n_elems, uint32_t *B,
                       uint64_t *total, uint32_t *status, int *dtype)
{
    if (!hdr) return ORC_E_ARG;
    if (hdr[0] != 'E' || hdr[1] != 'N' || hdr[2] != 'E' || hdr[3] != 'C') return ORC_E_FORMAT;
    if (get_u16(hdr + 4) != 1) return ORC_E_FORMAT;
    if (!dtype_ok(hdr[6])) return ORC_E_DTYPE;
    if (!group_ok(hdr[7]) || hdr[27] != orc_exp_bits(hdr[6])) return ORC_E_FORMAT;
    if (params) { params[0] = hdr[24]; params[1] = hdr[25]; params[2] = hdr[26]; params[3] = hdr[7]; }
    if (n_elems) *n_elems = get_u64(hdr + 8);
    if (B) *B = get_u32(hdr + 16);
    if (total) *total = get_u64(hdr + 32);
    if (status) *status = get_u32(hdr + 28);
    if (dtype) *dtype = hdr[6];
    return ORC_OK;
}

/* 1 if the stream carries one tuple per data block, 0 if one tuple for all. */
int orc_stream_per_block(const uint8_t *hdr) { return hdr && hdr[40] == 1; }

/* The bf16-only form: any other dtype in the header is ORC_E_DTYPE. */
int orc_stream_info(const uint8_t *hdr, uint8_t params[4], uint64_t *n_elems, uint32_t *B,
                    uint64_t *total, uint32_t *status)
{
    int dtype = 0, rc = orc_stream_info_dt(hdr, params, n_elems, B, total, status, &dtype);
    if (rc == ORC_OK && dtype != ORC_BF16) return ORC_E_DTYPE;
    return rc;
}

/* Decompresses a stream made by orc_compress_dt into n_elems values of the
 * dtype its header names (u16 or u32 words). */
int orc_decompress_dt(const uint8_t *in, size_t in_bytes, void *out, size_t n_elems)
{
    uint8_t params[4];
    uint64_t hdr_n, total;
    uint32_t B, status;
    unsigned b, n, m, a, E, lowbits, L;
    size_t nb, base, k, G, rb;
    uint16_t *low, *high, *prefix;
    uint8_t rec[80];
    const uint8_t *tail16, *tuples;
    int rc, dtype, per_block;

    if (!in || (!out && n_elems) || in_bytes < ORC_HEADER) return ORC_E_ARG;
    rc = orc_stream_info_dt(in, params, &hdr_n, &B, &total, &status, &dtype);
    if (rc != ORC_OK) return rc;
    if (status != ORC_OK || hdr_n != (uint64_t)n_elems || !block_ok(B)) return ORC_E_FORMAT;
    E = orc_exp_bits(dtype);
    per_block = orc_stream_per_block(in);
    b = params[0]; n = params[1]; m = params[2]; L = params[3];
    if (B < 8u * L) return ORC_E_FORMAT;
    if (!per_block && (n < 1 || n > E || m > n)) return ORC_E_FORMAT;
    nb = orc_num_blocks(n_elems, B);
    base = per_block ? orc_payload_base_pb(n_elems, B, dtype) : orc_payload_base_dt(n_elems, B, dtype);
    if (get_u32(in + 20) != (uint32_t)nb || total > in_bytes || total < base) return ORC_E_FORMAT;
    G = B / L;
    tuples = in + orc_table_end(n_elems, B);
    tail16 = tuples + (per_block ? orc_tuple_table_bytes(n_elems, B) : 0);
    if (per_block)
        for (k = 0; k < nb; k++)
            if (tuples[4 * k + 1] < 1 || tuples[4 * k + 1] > E || tuples[4 * k + 2] > tuples[4 * k + 1])
                return ORC_E_FORMAT;

    low = (uint16_t *)malloc(B * sizeof(uint16_t));
    high = (uint16_t *)malloc(L * sizeof(uint16_t));
    prefix = (uint16_t *)malloc((G + 1) * sizeof(uint16_t));

    for (k = 0; k < nb; k++) {
        uint64_t off = get_u64(in + ORC_HEADER + 8 * k);
        const uint8_t *p = in + base + off;
        const uint8_t *sm = p;
        const uint8_t *maskbytes = p + B;
        const uint8_t *lowplane = maskbytes + G / 8;
        const uint8_t *highplane;
        size_t i, g;
        if (per_block) { b = tuples[4 * k]; n = tuples[4 * k + 1]; m = tuples[4 * k + 2]; }
        a = n - m;
        rb = (size_t)a * L / 8u;
        lowbits = m + (dtype == ORC_FP16 ? 3u : 0u);
        highplane = lowplane + (size_t)lowbits * B / 8;
        /* mask bits -> {0,1} integers -> exclusive prefix sum = record index */
        prefix[0] = 0;
        for (g = 0; g < G; g++)
            prefix[g + 1] = (uint16_t)(prefix[g] + ((maskbytes[g / 8] >> (g % 8)) & 1u));
        if (lowbits > 0) orc_hh_unpack(lowplane, B, (int)lowbits, low);
        else for (i = 0; i < B; i++) low[i] = 0;
        for (g = 0; g < G; g++) {
            int anomalous = (maskbytes[g / 8] >> (g % 8)) & 1u;
            if (anomalous) {
                memset(rec, 0, sizeof rec);             /* the pad byte Alg. 2 expects after an odd count */
                memcpy(rec, highplane + rb * prefix[g], rb);
                orc_hh_unpack(rec, L, (int)a, high);
            }
            for (i = 0; i < L; i++) {
                size_t e = k * (size_t)B + g * L + i;
                unsigned yv, x, s, r = 0;
                uint32_t w;
                if (e >= n_elems) break;
                yv = low[g * L + i] & ((1u << m) - 1u);
                if (dtype == ORC_FP16) r = low[g * L + i] >> m;
                if (dtype == ORC_FP32) r = get_u16(tail16 + 2 * e);
                if (anomalous) yv |= (unsigned)high[i] << m;
                x = orc_inverse_transform_e(yv, b, n, E);
                s = sm[g * L + i];
                w = join_elem(x, s, r, dtype);
                if (dtype == ORC_FP32) ((uint32_t *)out)[e] = w;
                else ((uint16_t *)out)[e] = (uint16_t)w;
            }
        }
    }
    free(low); free(high); free(prefix);
    return ORC_OK;
}

/* The bf16-only form. */
int orc_decompress(const uint8_t *in, size_t in_bytes, uint16_t *out, size_t n_elems)
{
    if (in && in_bytes >= ORC_HEADER && in[6] != ORC_BF16 && in[0] == 'E') {
        int rc = orc_stream_info(in, NULL, NULL, NULL, NULL, NULL);
        if (rc != ORC_OK) return rc;
    }
    return orc_decompress_dt(in, in_bytes, out, n_elems);
}
