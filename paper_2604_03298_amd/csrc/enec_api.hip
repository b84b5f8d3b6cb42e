// Host side of libenec: argument checks, kernel dispatch, the parameter search.
// See include/enec.h for the contract of every entry point.
#include "enec.h"
#include "enec_kernels.hpp"

#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <tuple>
#include <vector>

namespace enec {

// kernels that exist once: the header-only stream of an empty tensor, zero fill, plain copy
__global__ void compress_empty_kernel(uint8_t *out, uint64_t *out_bytes, uint32_t B, uint32_t b, uint32_t n, uint32_t m,
                                      uint32_t dtype, uint32_t L)
{
    if (threadIdx.x != 0) return;
    uint32_t *h = reinterpret_cast<uint32_t *>(out);
    h[0] = 0x43454E45u;
    h[1] = 1u | (dtype << 16) | ((L & 0xFFu) << 24);
    h[2] = h[3] = 0;
    h[4] = B; h[5] = 0;
    h[6] = b | (n << 8) | (m << 16) | (exponent_bits((int)dtype) << 24);
    h[7] = 0;
    h[8] = 80; h[9] = 0;
    h[10] = L >> 8;                           // 1 = a stream with one tuple per data block
    for (int i = 11; i < 16; ++i) h[i] = 0;
    h[16] = h[17] = h[18] = h[19] = 0;      // table[0] = 0 and the pad to 80 bytes
    if (out_bytes) *out_bytes = 80;
}

__global__ void __launch_bounds__(256) fill_zero_kernel(uint4 *p, uint64_t nvec)
{
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t v = (uint64_t)blockIdx.x * 256u + threadIdx.x; v < nvec; v += stride)
        p[v] = make_uint4(0, 0, 0, 0);
}

__global__ void __launch_bounds__(256) copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, uint64_t nvec)
{
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t v = (uint64_t)blockIdx.x * 256u + threadIdx.x; v < nvec; v += stride) dst[v] = src[v];
}

}  // namespace enec

namespace {

using namespace enec;

// workspace: [0, 1024) control records of the block classes | [1024, 33792) sixteen histograms |
// group words | block words (the last two sized by the call's block count)
constexpr size_t WS_CTL = 0, WS_HIST = 1024, WS_HIST_SLOTS = MAX_BATCH, WS_STATE = WS_HIST + WS_HIST_SLOTS * 256 * 8;
inline size_t ws_groups(size_t nb) { return (nb + GROUP - 1) / GROUP; }
// The state words behind WS_STATE: first the group accumulators, which every call leaves zero, in
// a region whose length depends only on the size of the workspace (1/9 of the words), then the
// tagged group and block words, handed out anew by every launch.
inline size_t ws_state_words(size_t workspace_bytes) { return workspace_bytes < WS_STATE ? 0 : (workspace_bytes - WS_STATE) / 8; }
inline size_t ws_acc_words(size_t workspace_bytes) { return ws_state_words(workspace_bytes) / 9; }
constexpr size_t MAX_ELEMS = (size_t)1 << 34;      // keeps every offset below 2^36 bytes

inline size_t align16(size_t v) { return (v + 15) & ~(size_t)15; }
inline bool block_ok(uint32_t B) { return B >= 2048 && B <= 32768 && (B & (B - 1)) == 0; }
inline uint32_t ilog2(uint32_t v) { uint32_t r = 0; while ((1u << r) < v) ++r; return r; }
inline size_t num_blocks(size_t n, uint32_t B) { return (n + B - 1) / B; }
inline bool dtype_ok(int dtype) { return dtype == ENEC_BF16 || dtype == ENEC_FP16 || dtype == ENEC_FP32; }
inline unsigned exp_bits(int dtype) { return dtype == ENEC_FP16 ? 5u : 8u; }
inline size_t elem_bytes(int dtype) { return dtype == ENEC_FP32 ? 4 : 2; }
// end of header + offset table; an fp32 stream keeps the lower halves of its elements from here on
inline size_t table_end(size_t n, uint32_t B) { return align16(ENEC_HEADER_BYTES + 8 * (num_blocks(n, B) + 1)); }
inline size_t payload_base(size_t n, uint32_t B, int dtype)
{
    return table_end(n, B) + (dtype == ENEC_FP32 ? align16(2 * n) : 0);
}
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
// a stream with one tuple per data block keeps them (4 bytes each) right behind the offset table
inline size_t tuple_table_bytes(size_t n, uint32_t B) { return align16(4 * num_blocks(n, B)); }

inline bool group_ok(unsigned L) { return L == 8 || L == 16 || L == 32; }

inline CompressFn pick_compress(int m, int a, int dtype, unsigned L)
{
#define ENEC_ROW(dt) (L == 8 ? pick_compress_##dt##_lpg1(m, a) : L == 16 ? pick_compress_##dt##_lpg2(m, a) : pick_compress_##dt##_lpg4(m, a))
    if (dtype == ENEC_FP16) return ENEC_ROW(dt1);
    if (dtype == ENEC_FP32) return ENEC_ROW(dt2);
    return ENEC_ROW(dt0);
#undef ENEC_ROW
}
inline DecompressFn pick_decompress(int m, int a, int dtype, unsigned L)
{
#define ENEC_ROW(dt) (L == 8 ? pick_decompress_##dt##_lpg1(m, a) : L == 16 ? pick_decompress_##dt##_lpg2(m, a) : pick_decompress_##dt##_lpg4(m, a))
    if (dtype == ENEC_FP16) return ENEC_ROW(dt1);
    if (dtype == ENEC_FP32) return ENEC_ROW(dt2);
    return ENEC_ROW(dt0);
#undef ENEC_ROW
}

// A group length needs whole 16-byte vectors of mask per block (B >= 128 L) and at most 64 mask
// words per block (the kernels scan them with one wave: B / L <= 2048).
inline bool group_fits_block(unsigned L, uint32_t B) { return B >= 128u * L && B / L <= 2048u; }

// how the kernels subtract exponents in byte lanes: 0 = plain subtract (no byte can borrow for
// an exponent inside the window), 1 = borrow-safe subtract, the window is the whole exponent
// range, 2 = borrow-safe subtract plus an explicit window test (the window of an 8-bit exponent
// touches 0 or 255, where a plain subtract could wrap back into the window)
inline unsigned subtract_mode(unsigned b, unsigned n, int dtype)
{
    if (n == exp_bits(dtype)) return 1u;
    if (dtype == ENEC_FP16) return 0u;           // 5-bit exponents in byte lanes cannot wrap
    const unsigned cc = b + (1u << (n - 1));
    return (cc <= 255 && cc >= (1u << n) - 1u) ? 0u : 2u;
}

bool device_accessible(const void *p)
{
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeHost ||
           attr.type == hipMemoryTypeManaged;
}

// Number of workgroups of `fn` the current device holds at once.  The figure depends only on the
// kernel, its launch shape and the device, so it is looked up once per such combination and kept (a
// map under a mutex: there are several hundred kernel instances); a call whose combination is known
// makes no HIP call here, which also keeps it usable under stream capture once warmed up.
unsigned resident_workgroups(const void *fn, unsigned threads, size_t lds)
{
    static std::map<std::tuple<const void *, unsigned, size_t, int>, unsigned> cache;
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    std::lock_guard<std::mutex> lock(mu);
    const auto key = std::make_tuple(fn, threads, lds, dev);
    const auto hit = cache.find(key);
    if (hit != cache.end()) return hit->second;
    if (lds > 65536 &&
        hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return 0;
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, (int)threads, lds) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || per_cu < 1 || cus < 1)
        return 0;
    const unsigned value = (unsigned)per_cu * (unsigned)cus;
    cache.emplace(key, value);
    return value;
}

// A persistent grid for `total` blocks on a device that holds `resident` workgroups.  (Shrinking the
// grid until every round of blocks is full, e.g. 727 instead of 768 workgroups for 12352 blocks, was
// measured and lost 1.5 % on compression and 4 % on decompression of the 7B layer: the last, nearly
// empty round costs less than the parallelism given up in all the others.)
unsigned persistent_grid(unsigned total, unsigned resident)
{
    return total < resident ? total : resident;
}

// polls after which a waiting workgroup gives up; builds with ENEC_TEST_HOOKS (the test library) let
// the environment lower it so that a test can watch a scan give up without waiting for seconds
uint32_t spin_limit()
{
#ifdef ENEC_TEST_HOOKS
    if (const char *e = std::getenv("ENEC_SPIN_LIMIT")) {
        const long v = std::atol(e);
        if (v > 0 && v < (long)SPIN_LIMIT) return (uint32_t)v;
    }
#endif
    return SPIN_LIMIT;
}

unsigned bit_length(unsigned v) { unsigned r = 0; for (; v; v >>= 1) ++r; return r; }

// ---- Sec. V-E phases 1-3 on a 256-bin exponent histogram -------------------------------------
struct Search {
    unsigned lo, hi;            // occupied exponent range [l, h] (phase 1)
    uint64_t total;             // number of elements
    unsigned b, n;              // mapping centre and stored width (phase 2)
    unsigned m, L;              // threshold width and group length (phase 3)
    uint64_t at_most[9];        // at_most[w] = elements whose y fits in w bits, w = 0 .. n
};

// Phase 2: every centre b of [l, h] with the width Eq. 1 gives it (capped at the exponent field) is
// priced by Eq. 3 in exact integers, sum of count * y with y from Eq. 2; the cheapest wins, then the
// narrower, then the smaller centre.  Afterwards the elements are counted by the bit length of their y,
// which is all phase 3 needs.  False for an empty histogram.
bool centre_and_width(const uint64_t *hist, unsigned nmax, Search &r)
{
    r.lo = 256; r.hi = 0; r.total = 0;
    for (unsigned x = 0; x < 256; ++x) {
        if (!hist[x]) continue;
        if (r.lo == 256) r.lo = x;
        r.hi = x;
        r.total += hist[x];
    }
    if (r.total == 0) return false;
    auto key_of = [&](unsigned b) {
        const unsigned need_below = bit_length(b - r.lo);                       // y = b - x, largest for x = l
        const unsigned need_above = r.hi > b ? bit_length(r.hi - b - 1u) : 0u;  // y = 2^n - (x - b)
        unsigned n = (need_below > need_above ? need_below : need_above) + 1u;
        if (n > nmax) n = nmax;
        uint64_t cost = 0;
        for (unsigned x = r.lo; x <= r.hi; ++x) cost += hist[x] * (uint64_t)((b - x) & ((1u << n) - 1u));
        return std::make_tuple(cost, n, b);
    };
    auto best = key_of(r.lo);
    for (unsigned b = r.lo + 1; b <= r.hi; ++b) {
        const auto k = key_of(b);
        if (k < best) best = k;                   // lexicographic: cost, then width, then centre
    }
    r.n = std::get<1>(best);
    r.b = std::get<2>(best);
    uint64_t by_length[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    for (unsigned x = r.lo; x <= r.hi; ++x) by_length[bit_length((r.b - x) & ((1u << r.n) - 1u))] += hist[x];
    uint64_t run = 0;
    for (unsigned w = 0; w <= r.n; ++w) { run += by_length[w]; r.at_most[w] = run; }
    return true;
}

// Phase 3, Eq. 4: expected exponent bits per element 1/L + n + (m - n) p(m)^L over m in [0, n] and the
// candidate group lengths (OR of 8, 16, 32), p(m) = share of elements with y < 2^m.  Evaluated in IEEE
// double, p^L by log2 L squarings, as (1/L + n) + (m - n) p^L; the smallest wins, then the smaller m,
// then the smaller L.  (The build keeps the compiler from fusing the multiply and the add.)
void threshold_and_length(Search &r, uint32_t lengths)
{
    bool have = false;
    double least = 0.0;
    for (unsigned L = 8, squarings = 3; L <= 32; L *= 2, ++squarings) {
        if (!(lengths & L)) continue;
        for (unsigned m = 0; m <= r.n; ++m) {
            double q = (double)r.at_most[m] / (double)r.total;
            for (unsigned i = 0; i < squarings; ++i) q = q * q;
            const double bits = (1.0 / (double)L + (double)r.n) + ((double)m - (double)r.n) * q;
            if (!have || bits < least || (bits == least && (m < r.m || (m == r.m && L < r.L)))) {
                have = true; least = bits; r.m = m; r.L = L;
            }
        }
    }
}

struct Header {
    enec_params prm;
    uint64_t n_elems, total;
    uint32_t B, nb, status;
    int dtype;
    bool per_block;          // one tuple per data block (header byte 40)
};

int parse_header(const void *host_header, Header *h)
{
    const uint8_t *p = static_cast<const uint8_t *>(host_header);
    if (std::memcmp(p, "ENEC", 4) != 0) return ENEC_E_FORMAT;
    uint16_t ver; std::memcpy(&ver, p + 4, 2);
    if (ver != 1 || !group_ok(p[7])) return ENEC_E_FORMAT;
    h->dtype = p[6];
    if (!dtype_ok(h->dtype)) return ENEC_E_DTYPE;
    if (p[27] != exp_bits(h->dtype)) return ENEC_E_FORMAT;
    std::memcpy(&h->n_elems, p + 8, 8);
    std::memcpy(&h->B, p + 16, 4);
    std::memcpy(&h->nb, p + 20, 4);
    h->prm.b = p[24]; h->prm.n = p[25]; h->prm.m = p[26]; h->prm.L = p[7];
    std::memcpy(&h->status, p + 28, 4);
    std::memcpy(&h->total, p + 32, 8);
    if (p[40] > 1) return ENEC_E_FORMAT;
    h->per_block = p[40] == 1;
    return ENEC_OK;
}

}  // namespace

extern "C" {

uint32_t enec_version(void) { return 1; }

const char *enec_strerror(int status)
{
    switch (status) {
    case ENEC_OK: return "ok";
    case ENEC_E_ARG: return "invalid argument (null or misaligned pointer, size out of range)";
    case ENEC_E_DTYPE: return "unsupported dtype (bf16, fp16 and fp32 are supported)";
    case ENEC_E_BLOCK: return "block_size must be a power of two in [2048, 32768]";
    case ENEC_E_PARAMS: return "invalid parameters (need 1 <= n <= exponent width, 0 <= m <= n, b inside the exponent range, L in {8, 16, 32} with 128 L <= block_size <= 2048 L)";
    case ENEC_E_CAPACITY: return "output capacity or workspace too small";
    case ENEC_E_RANGE: return "an exponent lies outside the window of (b, n)";
    case ENEC_E_FORMAT: return "not an ENEC stream or header mismatch";
    case ENEC_E_HIP: return "HIP runtime error (as a stream's status: the inter-block scan gave up on a workspace that was not in the state the last call left it in)";
    default: return "unknown status";
    }
}

uint32_t enec_default_block_size(size_t n_elems)
{
    uint32_t B = ENEC_DEFAULT_BLOCK;
    while (B > 2048 && B > n_elems) B >>= 1;
    return B;
}

size_t enec_compress_bound(size_t n_elems, int dtype, uint32_t block_size)
{
    if (!dtype_ok(dtype)) return 0;
    const uint32_t B = block_size ? block_size : enec_default_block_size(n_elems);
    if (!block_ok(B)) return 0;
    // worst case for any group length: every group anomalous at full exponent width (fp16: (5 + 3)
    // plane bits) and the longest mask (L = 8)
    return payload_base(n_elems, B, dtype) + num_blocks(n_elems, B) * align16((size_t)B + B / 64 + B);
}

size_t enec_workspace_bytes(size_t n_elems, uint32_t block_size)
{
    const uint32_t B = block_size ? block_size : enec_default_block_size(n_elems);
    if (!block_ok(B)) return 0;
    // room for the scan words of up to MAX_BATCH tensors with n_elems elements in total
    const size_t nb = num_blocks(n_elems, B) + MAX_BATCH;
    const size_t groups = ws_groups(nb) + MAX_BATCH;
    const size_t by_acc = 9 * groups, by_words = (9 * (groups + nb) + 7) / 8;
    return (WS_STATE + 8 * ((by_acc > by_words ? by_acc : by_words) + 9) + 255) & ~(size_t)255;
}

int enec_workspace_init(void *workspace, size_t bytes, void *stream)
{
    if (!workspace || !aligned16(workspace) || (bytes & 15)) return ENEC_E_ARG;
    if (bytes == 0) return ENEC_OK;
    const uint64_t nvec = bytes / 16;
    const unsigned grid = (unsigned)((nvec + 255) / 256 < 1024 ? (nvec + 255) / 256 : 1024);
    fill_zero_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(static_cast<uint4 *>(workspace), nvec);
    return hipGetLastError() == hipSuccess ? ENEC_OK : ENEC_E_HIP;
}

int enec_tune_histogram(const uint64_t *hist, int dtype, enec_params *params)
{
    return enec_tune_histogram_groups(hist, dtype, 16u, 0u, params);
}

int enec_tune_histogram_groups(const uint64_t *hist, int dtype, uint32_t group_lengths, uint32_t block_size,
                               enec_params *params)
{
    if (!dtype_ok(dtype)) return ENEC_E_DTYPE;
    if (!hist || !params) return ENEC_E_ARG;
    if (!(group_lengths & (8u | 16u | 32u)) || (group_lengths & ~(8u | 16u | 32u))) return ENEC_E_PARAMS;
    const uint32_t B = block_size ? block_size : ENEC_DEFAULT_BLOCK;
    if (!block_ok(B)) return ENEC_E_BLOCK;
    // only lengths the block size admits are candidates; 16 fits every block size and stands in if none is left
    uint32_t lengths = 0;
    for (unsigned L = 8; L <= 32; L *= 2)
        if ((group_lengths & L) && group_fits_block(L, B)) lengths |= L;
    if (!lengths) lengths = 16u;
    Search r;
    if (!centre_and_width(hist, exp_bits(dtype), r)) {          // no elements at all: (b, n) = (0, 1) and p = 1
        r.b = 0; r.n = 1; r.total = 1;
        r.at_most[0] = r.at_most[1] = 1;
    }
    threshold_and_length(r, lengths);
    *params = enec_params{(uint8_t)r.b, (uint8_t)r.n, (uint8_t)r.m, (uint8_t)r.L};
    return ENEC_OK;
}

int enec_tune_batch(const enec_tune_item *items, size_t n_items, int dtype, uint32_t every, enec_params *params,
                    uint64_t *histograms, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!dtype_ok(dtype)) return ENEC_E_DTYPE;
    if (workspace_bytes < WS_STATE) return ENEC_E_CAPACITY;
    if ((!items && n_items) || (!params && n_items) || !workspace || !aligned16(workspace) || every == 0) return ENEC_E_ARG;
    for (size_t i = 0; i < n_items; ++i)
        if ((!items[i].in && items[i].n_elems) || !aligned16(items[i].in) || items[i].n_elems > MAX_ELEMS) return ENEC_E_ARG;
    hipStream_t s = (hipStream_t)stream;
    auto *dhist = reinterpret_cast<unsigned long long *>(static_cast<uint8_t *>(workspace) + WS_HIST);
    std::vector<uint64_t> host(WS_HIST_SLOTS * 256);
    // sixteen tensors at a time: their histograms are counted into sixteen slots, copied back together,
    // and the stream is waited for once
    for (size_t first = 0; first < n_items; first += WS_HIST_SLOTS) {
        const size_t count = n_items - first < WS_HIST_SLOTS ? n_items - first : WS_HIST_SLOTS;
        fill_zero_kernel<<<(unsigned)count, 256, 0, s>>>(reinterpret_cast<uint4 *>(dhist), count * 256 * 8 / 16);
        // One launch for the sixteen: a workgroup per 256 vectors of the sample, but no more than 512
        // workgroups in all, shared out by size (every workgroup ends with one global atomic per exponent
        // value it has seen: with 2048 workgroups per tensor those few addresses were half of the time).
        HistogramArgs a;
        a.n_items = 0;
        a.every = every;
        uint64_t want_all = 0;
        for (size_t j = 0; j < count; ++j)
            want_all += (items[first + j].n_elems * elem_bytes(dtype) / 16 / every + 255) / 256;
        uint32_t grid = 0;
        for (size_t j = 0; j < count; ++j) {
            const enec_tune_item &it = items[first + j];
            if (it.n_elems == 0) continue;
            const uint64_t want = (it.n_elems * elem_bytes(dtype) / 16 / every + 255) / 256;
            uint64_t share = want_all > 512 ? want * 512 / want_all : want;
            if (share < 1) share = 1;
            HistogramItem &d = a.item[a.n_items++];
            d.in = it.in;
            d.n_elems = it.n_elems;
            d.hist = dhist + 256 * j;
            d.first = grid;
            d.count = (uint32_t)share;
            grid += d.count;
        }
        if (grid) {
            for (uint32_t j = a.n_items; j < (uint32_t)MAX_BATCH; ++j) a.item[j] = a.item[0];
            if (dtype == ENEC_FP32) histogram_kernel<DT_FP32><<<grid, 256, 0, s>>>(a);
            else if (dtype == ENEC_FP16) histogram_kernel<DT_FP16><<<grid, 256, 0, s>>>(a);
            else histogram_kernel<DT_BF16><<<grid, 256, 0, s>>>(a);
        }
        if (hipMemcpyAsync(host.data(), dhist, count * 256 * 8, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess) {
            (void)hipGetLastError();
            return ENEC_E_HIP;
        }
        for (size_t j = 0; j < count; ++j) {
            int rc = enec_tune_histogram(host.data() + 256 * j, dtype, &params[first + j]);
            if (rc != ENEC_OK) return rc;
            if (histograms) std::memcpy(histograms + 256 * (first + j), host.data() + 256 * j, 256 * 8);
        }
    }
    return ENEC_OK;
}

int enec_tune_sampled(const void *in, size_t n_elems, int dtype, uint32_t every, enec_params *params,
                      uint64_t *histogram, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!params) return ENEC_E_ARG;
    enec_tune_item it;
    it.in = in;
    it.n_elems = n_elems;
    return enec_tune_batch(&it, 1, dtype, every, params, histogram, workspace, workspace_bytes, stream);
}

int enec_tune(const void *in, size_t n_elems, int dtype, enec_params *params, uint64_t *histogram,
              void *workspace, size_t workspace_bytes, void *stream)
{
    return enec_tune_sampled(in, n_elems, dtype, 1, params, histogram, workspace, workspace_bytes, stream);
}

int enec_compress_sampled(const void *in, size_t n_elems, int dtype, uint32_t block_size, uint32_t every,
                          enec_params *params_used, void *out, size_t out_capacity, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    enec_params prm;
    int rc = enec_tune_sampled(in, n_elems, dtype, every, &prm, nullptr, workspace, workspace_bytes, stream);
    if (rc != ENEC_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    for (int attempt = 0; attempt < 2; ++attempt) {
        rc = enec_compress(in, n_elems, dtype, block_size, &prm, out, out_capacity, nullptr, workspace,
                           workspace_bytes, stream);
        if (rc != ENEC_OK) return rc;
        uint8_t head[ENEC_HEADER_BYTES];
        if (hipMemcpyAsync(head, out, sizeof head, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            return ENEC_E_HIP;
        uint32_t status = 0;
        rc = enec_stream_info(head, nullptr, nullptr, nullptr, nullptr, nullptr, &status);
        if (rc != ENEC_OK) return rc;
        if (params_used) *params_used = prm;
        if (status != (uint32_t)ENEC_E_RANGE) return (int)status;
        // an exponent outside the sample's window: the full width makes the map a bijection [Sec. V-C]
        prm.n = (uint8_t)exp_bits(dtype);
    }
    return ENEC_E_RANGE;   // not reached: the full width has no range error
}

int enec_compress_batch(const enec_compress_item *items, size_t n_items, int dtype, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    if (!dtype_ok(dtype)) return ENEC_E_DTYPE;
    if (!items || !workspace || !aligned16(workspace)) return ENEC_E_ARG;

    // ---- every check that can be made on the host, before anything is enqueued -------------
    struct Prepared { enec_params prm; uint32_t B; uint32_t nb; };
    std::vector<Prepared> prep(n_items);
    size_t state_words = 0, groups = 0;
    for (size_t i = 0; i < n_items; ++i) {
        const enec_compress_item &it = items[i];
        if (!it.out || (!it.in && it.n_elems) || !aligned16(it.in) || !aligned16(it.out) ||
            it.n_elems > MAX_ELEMS || ((uintptr_t)it.out_bytes & 7))
            return ENEC_E_ARG;
        const uint32_t B = it.block_size ? it.block_size : enec_default_block_size(it.n_elems);
        if (!block_ok(B)) return ENEC_E_BLOCK;
        prep[i].B = B;
        prep[i].nb = (uint32_t)num_blocks(it.n_elems, B);
        state_words += ws_groups(prep[i].nb) + prep[i].nb;
        groups += ws_groups(prep[i].nb);
    }
    const size_t acc_words = ws_acc_words(workspace_bytes);
    if (groups > acc_words || acc_words + state_words > ws_state_words(workspace_bytes)) return ENEC_E_CAPACITY;
    {   // tensors without a tuple are tuned first, together (one wait for the stream per sixteen of them)
        std::vector<enec_tune_item> todo;
        std::vector<size_t> who;
        for (size_t i = 0; i < n_items; ++i)
            if (!items[i].params) {
                enec_tune_item t;
                t.in = items[i].in;
                t.n_elems = items[i].n_elems;
                todo.push_back(t);
                who.push_back(i);
            }
        if (!todo.empty()) {
            std::vector<enec_params> found(todo.size());
            int rc = enec_tune_batch(todo.data(), todo.size(), dtype, 1, found.data(), nullptr, workspace, workspace_bytes, s);
            if (rc != ENEC_OK) return rc;
            for (size_t j = 0; j < who.size(); ++j) prep[who[j]].prm = found[j];
        }
    }
    for (size_t i = 0; i < n_items; ++i) {
        const enec_compress_item &it = items[i];
        if (it.params) prep[i].prm = *it.params;
        const enec_params &prm = prep[i].prm;
        if (prm.n < 1 || prm.n > exp_bits(dtype) || prm.m > prm.n || prm.b >= (1u << exp_bits(dtype)) ||
            !group_ok(prm.L) || !group_fits_block(prm.L, prep[i].B))
            return ENEC_E_PARAMS;
        if (it.out_capacity < enec_compress_bound(it.n_elems, dtype, prep[i].B)) return ENEC_E_CAPACITY;
        if (it.out_bytes && !device_accessible(it.out_bytes)) return ENEC_E_ARG;
    }

    // ---- one launch per group of tensors that share (m, n - m, L, block size) ----------------
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    std::vector<char> done(n_items, 0);
    for (size_t i = 0; i < n_items; ++i) {
        if (done[i]) continue;
        if (prep[i].nb == 0) {
            compress_empty_kernel<<<1, 64, 0, s>>>(static_cast<uint8_t *>(items[i].out), items[i].out_bytes,
                                                   prep[i].B, prep[i].prm.b, prep[i].prm.n, prep[i].prm.m,
                                                   (uint32_t)dtype, prep[i].prm.L);
            done[i] = 1;
            continue;
        }
        CompressArgs a;
        a.ws_ctl = reinterpret_cast<uint32_t *>(ws + WS_CTL);
        a.B = prep[i].B;
        a.logB = ilog2(a.B);
        a.n_items = 0;
        a.total = 0;
        size_t word = acc_words, acc = 0;   // scan words handed out to this launch (tags make reuse between launches safe)
        for (size_t j = i; j < n_items && a.n_items < (uint32_t)MAX_BATCH; ++j) {
            if (done[j] || prep[j].nb == 0 || prep[j].B != a.B || prep[j].prm.m != prep[i].prm.m ||
                prep[j].prm.n != prep[i].prm.n || prep[j].prm.L != prep[i].prm.L)
                continue;
            CompressItem &c = a.item[a.n_items++];
            c.in = static_cast<const uint16_t *>(items[j].in);
            c.out = static_cast<uint8_t *>(items[j].out);
            c.out_bytes = items[j].out_bytes;
            c.ws_acc = reinterpret_cast<uint64_t *>(ws + WS_STATE) + acc;
            acc += ws_groups(prep[j].nb);
            c.ws_group = reinterpret_cast<uint64_t *>(ws + WS_STATE) + word;
            word += ws_groups(prep[j].nb);
            c.ws_block = reinterpret_cast<uint64_t *>(ws + WS_STATE) + word;
            word += prep[j].nb;
            c.n_elems = items[j].n_elems;
            c.payload_base = payload_base(items[j].n_elems, a.B, dtype);
            c.tail_base = table_end(items[j].n_elems, a.B);
            c.nb = prep[j].nb;
            c.first = a.total;
            c.b = prep[j].prm.b;
            c.mode = subtract_mode(prep[j].prm.b, prep[j].prm.n, dtype);
            a.total += c.nb;
            done[j] = 1;
        }
        CompressFn fn = pick_compress(prep[i].prm.m, prep[i].prm.n - prep[i].prm.m, dtype, prep[i].prm.L);
        if (!fn) return ENEC_E_PARAMS;
        const unsigned threads = a.B / 64 < 64 ? 64 : a.B / 64;
        const size_t plane_bits = prep[i].prm.n + (dtype == ENEC_FP16 ? 3 : 0);
        // two images of the packed part, and the sign/mantissa bytes of the block that waits to be stored
        const size_t lds = 2 * ((size_t)a.B / (8 * prep[i].prm.L) + plane_bits * a.B / 8) +
                           (compress_sm_in_lds(dtype, prep[i].prm.L == 8 ? 1 : prep[i].prm.L == 16 ? 2 : 4) ? a.B : 0);
        const unsigned resident = resident_workgroups((const void *)fn, threads, lds);
        if (resident == 0) return ENEC_E_HIP;
        const unsigned grid = persistent_grid(a.total, resident);
        a.ncls = grid < 8 ? grid : 8;
        // The next ticket is drawn while the current block is worked on only if there are blocks for
        // two rounds: with fewer, an early workgroup would take the block of one that starts a moment later.
        a.lookahead = a.total >= 2 * grid ? 1u : 0u;
        a.spin_limit = spin_limit();
        hipLaunchKernelGGL(fn, dim3(grid), dim3(threads), lds, s, a);
    }
    return hipGetLastError() == hipSuccess ? ENEC_OK : ENEC_E_HIP;
}

int enec_compress(const void *in, size_t n_elems, int dtype, uint32_t block_size,
                  const enec_params *params, void *out, size_t out_capacity, uint64_t *out_bytes,
                  void *workspace, size_t workspace_bytes, void *stream)
{
    enec_compress_item it;
    it.in = in; it.n_elems = n_elems; it.block_size = block_size; it.params = params;
    it.out = out; it.out_capacity = out_capacity; it.out_bytes = out_bytes;
    return enec_compress_batch(&it, 1, dtype, workspace, workspace_bytes, stream);
}

// ---- enec_compress for callers that cannot allocate: the workspace is the library's own array ----
}  // extern "C"

namespace {

// Scan state, ticket counters and call tags of enec_compress_static: one array per GPU, held until the
// process ends.  In host code the array's name stands for the symbol, not for device memory; the
// address on a device comes from hipGetSymbolAddress with that device current, once per device.
static __device__ __align__(256) uint8_t scratch[ENEC_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
void *scratch_ptr[MAX_DEVICES];       // per device: the array's address there, null until its first call
std::mutex scratch_mu;

// address of `scratch` on the current device; the first call on a device looks it up and enqueues
// the fill kernel that brings the array into the state enec_workspace_init leaves a workspace in
int static_scratch(hipStream_t s, void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) { (void)hipGetLastError(); return ENEC_E_HIP; }
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return ENEC_E_HIP; }
        const int rc = enec_workspace_init(ptr, ENEC_STATIC_SCRATCH_BYTES, s);
        if (rc != ENEC_OK) return rc;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return ENEC_OK;
}

}  // namespace

extern "C" {

int enec_compress_static(const void *in, size_t n_elems, int dtype, uint32_t block_size, const enec_params *params,
                         void *out, size_t out_capacity, uint64_t *out_bytes, void *stream)
{
    if (!params) return ENEC_E_ARG;                       // tuning waits for the stream: not for these callers
    if (!dtype_ok(dtype)) return ENEC_E_DTYPE;
    const uint32_t B = block_size ? block_size : enec_default_block_size(n_elems);
    if (!block_ok(B)) return ENEC_E_BLOCK;
    if (n_elems > MAX_ELEMS) return ENEC_E_ARG;
    if (enec_workspace_bytes(n_elems, B) > ENEC_STATIC_SCRATCH_BYTES) return ENEC_E_CAPACITY;
    void *ws = nullptr;
    const int rc = static_scratch((hipStream_t)stream, &ws);
    if (rc != ENEC_OK) return rc;
    return enec_compress(in, n_elems, dtype, B, params, out, out_capacity, out_bytes, ws, ENEC_STATIC_SCRATCH_BYTES, stream);
}

size_t enec_compress_bound_per_block(size_t n_elems, int dtype, uint32_t block_size)
{
    const size_t bound = enec_compress_bound(n_elems, dtype, block_size);
    if (!bound) return 0;
    const uint32_t B = block_size ? block_size : enec_default_block_size(n_elems);
    return bound + tuple_table_bytes(n_elems, B);
}

int enec_compress_per_block_batch(const enec_per_block_item *items, size_t n_items, int dtype, uint32_t group_length,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    if (!dtype_ok(dtype)) return ENEC_E_DTYPE;
    if ((!items && n_items) || !workspace || !aligned16(workspace)) return ENEC_E_ARG;
    const unsigned L = group_length ? group_length : 16u;
    if (!group_ok(L)) return ENEC_E_PARAMS;
    hipStream_t s = (hipStream_t)stream;
    // every argument is checked before anything is enqueued
    std::vector<uint32_t> Bs(n_items);
    size_t need = PB_TICKET_CLASSES * PB_TICKET_STRIDE / 2;      // the ticket counters, in 8-byte words
    uint64_t blocks = 0;
    for (size_t i = 0; i < n_items; ++i) {
        const enec_per_block_item &it = items[i];
        if (!it.out || (!it.in && it.n_elems) || !aligned16(it.in) || !aligned16(it.out) || it.n_elems > MAX_ELEMS)
            return ENEC_E_ARG;
        const uint32_t B = it.block_size ? it.block_size : enec_default_block_size(it.n_elems);
        if (!block_ok(B)) return ENEC_E_BLOCK;
        if (!group_fits_block(L, B)) return ENEC_E_PARAMS;
        if (it.out_capacity < enec_compress_bound_per_block(it.n_elems, dtype, B)) return ENEC_E_CAPACITY;
        if (it.out_bytes && !device_accessible(it.out_bytes)) return ENEC_E_ARG;
        Bs[i] = B;
        const size_t nb = num_blocks(it.n_elems, B);
        need += nb + (nb & 1);                                   // look-back words, an even number per tensor
        blocks += nb;
    }
    if (blocks > 0xFFFFFFFFull) return ENEC_E_ARG;               // block numbers are 32 bits wide
    // ticket counters and look-back words behind the accumulators, cleared for this call
    size_t first = ws_acc_words(workspace_bytes);
    first += first & 1;                                          // 16-byte aligned for the fill kernel
    if (ws_state_words(workspace_bytes) < first + need) return ENEC_E_CAPACITY;
    PbCompressFn fn = pick_compress_per_block(dtype, L);
    if (!fn) return ENEC_E_DTYPE;
    uint64_t *base = reinterpret_cast<uint64_t *>(static_cast<uint8_t *>(workspace) + WS_STATE) + first;
    const uint64_t nvec = need / 2;
    const unsigned fill_grid = (unsigned)((nvec + 255) / 256 < 1024 ? (nvec + 255) / 256 : 1024);
    fill_zero_kernel<<<fill_grid, 256, 0, s>>>(reinterpret_cast<uint4 *>(base), nvec);
    uint64_t *words = base + PB_TICKET_CLASSES * PB_TICKET_STRIDE / 2;
    uint64_t next_block = 0;        // the data blocks of the call are numbered through, launch after launch
    std::vector<char> done(n_items, 0);
    for (size_t i0 = 0; i0 < n_items; ++i0) {
        if (done[i0]) continue;
        const enec_per_block_item &it0 = items[i0];
        if (it0.n_elems == 0) {     // a header and an empty table
            compress_empty_kernel<<<1, 64, 0, s>>>(static_cast<uint8_t *>(it0.out), it0.out_bytes, Bs[i0], 0, 0, 0,
                                                   (uint32_t)dtype, L | 0x100u);
            done[i0] = 1;
            continue;
        }
        // one launch for up to MAX_BATCH tensors of this block size, in the order given
        const uint32_t B = Bs[i0];
        PbCompressArgs a;
        a.ticket = reinterpret_cast<uint32_t *>(base);
        a.n_items = 0;
        a.first_block = (uint32_t)next_block;
        a.B = B; a.logB = ilog2(B);
        a.spin_limit = spin_limit();
        for (size_t i = i0; i < n_items && a.n_items < (uint32_t)MAX_BATCH; ++i) {
            const enec_per_block_item &it = items[i];
            if (done[i] || Bs[i] != B || it.n_elems == 0) continue;
            const size_t nb = num_blocks(it.n_elems, B);
            PbCompressItem &d = a.item[a.n_items++];
            d.in = it.in;
            d.out = static_cast<uint8_t *>(it.out);
            d.out_bytes = reinterpret_cast<unsigned long long *>(it.out_bytes);
            d.words = words;
            d.n_elems = it.n_elems;
            d.tuples_at = table_end(it.n_elems, B);
            d.tail_base = d.tuples_at + tuple_table_bytes(it.n_elems, B);
            d.payload_base = payload_base(it.n_elems, B, dtype) + tuple_table_bytes(it.n_elems, B);
            d.nb = (uint32_t)nb;
            d.first = (uint32_t)next_block;
            words += nb + (nb & 1);
            next_block += nb;
            done[i] = 1;
        }
        for (uint32_t i = a.n_items; i < (uint32_t)MAX_BATCH; ++i) a.item[i] = a.item[0];
        a.n_blocks = (uint32_t)(next_block - a.first_block);
        // one workgroup per data block, a thread per 64 elements (at least a wave); dynamic LDS: mask | low
        // plane | high records (at most 8 plane bits together), before that the histogram copies; behind
        // it the raw bytes of the rows that do not wait in registers
        const unsigned threads = B / 64 < 64 ? 64 : B / 64;
        const size_t image = (size_t)B / (8 * L) + (size_t)B, hist = (size_t)PB_HIST_COPIES * PB_HIST_STRIDE * 4;
        const size_t lds = (image > hist ? image : hist) + 15 & ~(size_t)15;
        a.park_at = (uint32_t)lds;
        hipLaunchKernelGGL(fn, dim3(a.n_blocks), dim3(threads), lds + (size_t)(8 - PB_SM_REG_ROWS) * threads * 8, s, a);
    }
    return hipGetLastError() == hipSuccess ? ENEC_OK : ENEC_E_HIP;
}

int enec_compress_per_block(const void *in, size_t n_elems, int dtype, uint32_t block_size, uint32_t group_length,
                            void *out, size_t out_capacity, uint64_t *out_bytes, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    enec_per_block_item it;
    it.in = in;
    it.n_elems = n_elems;
    it.block_size = block_size;
    it.out = out;
    it.out_capacity = out_capacity;
    it.out_bytes = out_bytes;
    return enec_compress_per_block_batch(&it, 1, dtype, group_length, workspace, workspace_bytes, stream);
}

int enec_decompress_batch(const enec_decompress_item *items, size_t n_items, void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    if (!items) return ENEC_E_ARG;
    std::vector<Header> hdr(n_items);
    for (size_t i = 0; i < n_items; ++i) {
        const enec_decompress_item &it = items[i];
        if (!it.in || !it.host_header || (!it.out && it.n_elems) || !aligned16(it.in) || !aligned16(it.out) ||
            ((uintptr_t)it.status & 3))
            return ENEC_E_ARG;
        if (it.status && !device_accessible(it.status)) return ENEC_E_ARG;
        Header &h = hdr[i];
        int rc = parse_header(it.host_header, &h);
        if (rc != ENEC_OK) return rc;
        if (h.status != ENEC_OK || h.n_elems != it.n_elems || !block_ok(h.B) || it.n_elems > MAX_ELEMS ||
            h.nb != num_blocks(it.n_elems, h.B) || !group_fits_block(h.prm.L, h.B) || h.total > it.in_bytes)
            return ENEC_E_FORMAT;
        if (h.per_block) {
            if (h.prm.n != 0 || h.prm.m != 0 || h.prm.b != 0 ||
                h.total < payload_base(it.n_elems, h.B, h.dtype) + tuple_table_bytes(it.n_elems, h.B))
                return ENEC_E_FORMAT;
        } else if (h.prm.n < 1 || h.prm.n > exp_bits(h.dtype) || h.prm.m > h.prm.n ||
                   h.prm.b >= (1u << exp_bits(h.dtype)) || h.total < payload_base(it.n_elems, h.B, h.dtype)) {
            return ENEC_E_FORMAT;
        }
    }
    std::vector<char> done(n_items, 0);
    {
        for (size_t i = 0; i < n_items; ++i) {
            if (done[i]) continue;
            if (hdr[i].nb == 0) { done[i] = 1; continue; }
            if (hdr[i].per_block) {
                // streams with one tuple per block: those of one element format, group length and block size
                // share a launch (up to MAX_BATCH each); their tuples are read from the streams
                const Header &h0 = hdr[i];
                PbDecompressArgs a;
                a.n_items = 0;
                a.n_blocks = 0;
                a.B = h0.B; a.logB = ilog2(h0.B);
                for (size_t j = i; j < n_items && a.n_items < (uint32_t)MAX_BATCH; ++j) {
                    const Header &h = hdr[j];
                    if (done[j] || h.nb == 0 || !h.per_block || h.B != h0.B || h.dtype != h0.dtype || h.prm.L != h0.prm.L ||
                        (uint64_t)a.n_blocks + h.nb > 0xFFFFFFFFull)
                        continue;
                    PbDecompressItem &d = a.item[a.n_items++];
                    d.in = static_cast<const uint8_t *>(items[j].in);
                    d.out = items[j].out;
                    d.n_elems = items[j].n_elems;
                    d.tuples_at = table_end(d.n_elems, h.B);
                    d.tail_base = d.tuples_at + tuple_table_bytes(d.n_elems, h.B);
                    d.payload_base = payload_base(d.n_elems, h.B, h.dtype) + tuple_table_bytes(d.n_elems, h.B);
                    d.payload_bytes = h.total - d.payload_base;
                    d.nb = h.nb;
                    d.first = a.n_blocks;
                    d.status = items[j].status;
                    std::memcpy(d.hdr, items[j].host_header, sizeof d.hdr);
                    a.n_blocks += h.nb;
                    done[j] = 1;
                }
                for (uint32_t j = a.n_items; j < (uint32_t)MAX_BATCH; ++j) a.item[j] = a.item[0];
                PbDecompressFn fn = pick_decompress_per_block(h0.dtype, h0.prm.L);
                if (!fn) return ENEC_E_FORMAT;
                const unsigned threads = h0.B / 64 < 64 ? 64 : h0.B / 64;
                const size_t lds = (size_t)h0.B / (8 * h0.prm.L) + h0.B + 16;     // the packed part of the widest block
                hipLaunchKernelGGL(fn, dim3(a.n_blocks), dim3(threads), lds, s, a);
                continue;
            }
            DecompressArgs a;
            a.B = hdr[i].B;
            a.logB = ilog2(a.B);
            a.n_items = 0;
            a.total = 0;
            for (size_t j = i; j < n_items && a.n_items < (uint32_t)MAX_BATCH; ++j) {
                const Header &h = hdr[j];
                if (done[j] || h.nb == 0 || h.per_block || h.B != a.B || h.prm.m != hdr[i].prm.m ||
                    h.prm.n != hdr[i].prm.n || h.dtype != hdr[i].dtype || h.prm.L != hdr[i].prm.L)
                    continue;
                DecompressItem &c = a.item[a.n_items++];
                c.in = static_cast<const uint8_t *>(items[j].in);
                c.out = static_cast<uint16_t *>(items[j].out);
                c.n_elems = items[j].n_elems;
                c.payload_base = payload_base(items[j].n_elems, h.B, h.dtype);
                c.payload_bytes = h.total - c.payload_base;
                c.tail_base = table_end(items[j].n_elems, h.B);
                c.nb = h.nb;
                c.first = a.total;
                c.b = h.prm.b;
                c.mode = subtract_mode(h.prm.b, h.prm.n, h.dtype) == 0 ? 0u : 1u;
                c.status = items[j].status;
                std::memcpy(c.hdr, items[j].host_header, sizeof c.hdr);
                a.total += c.nb;
                done[j] = 1;
            }
            DecompressFn fn = pick_decompress(hdr[i].prm.m, hdr[i].prm.n - hdr[i].prm.m, hdr[i].dtype, hdr[i].prm.L);
            if (!fn) return ENEC_E_FORMAT;
            const unsigned threads = a.B / 64 < 64 ? 64 : a.B / 64;
            const size_t plane_bits = hdr[i].prm.n + (hdr[i].dtype == ENEC_FP16 ? 3 : 0);
            const size_t lds = 2 * ((size_t)a.B / (8 * hdr[i].prm.L) + plane_bits * a.B / 8);   // two images of the packed part
            const unsigned resident = resident_workgroups((const void *)fn, threads, lds);
            if (resident == 0) return ENEC_E_HIP;
            hipLaunchKernelGGL(fn, dim3(persistent_grid(a.total, resident)), dim3(threads), lds, s, a);
        }
    }
    return hipGetLastError() == hipSuccess ? ENEC_OK : ENEC_E_HIP;
}

int enec_decompress_with_header(const void *in, size_t in_bytes, const void *host_header, void *out,
                                size_t n_elems, uint32_t *status, void *stream)
{
    enec_decompress_item it;
    it.in = in; it.in_bytes = in_bytes; it.host_header = host_header; it.out = out; it.n_elems = n_elems;
    it.status = status;
    return enec_decompress_batch(&it, 1, stream);
}

int enec_decompress(const void *in, size_t in_bytes, void *out, size_t n_elems, void *stream)
{
    if (!in || !aligned16(in)) return ENEC_E_ARG;
    if (in_bytes < ENEC_HEADER_BYTES) return ENEC_E_FORMAT;
    uint8_t hdr[ENEC_HEADER_BYTES];
    hipStream_t s = (hipStream_t)stream;
    if (hipMemcpyAsync(hdr, in, sizeof hdr, hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
        (void)hipGetLastError();
        return ENEC_E_HIP;
    }
    return enec_decompress_with_header(in, in_bytes, hdr, out, n_elems, nullptr, stream);
}

int enec_stream_info(const void *host_header, enec_params *params, uint64_t *n_elems,
                     uint32_t *block_size, uint64_t *total_bytes, int *dtype, uint32_t *status)
{
    if (!host_header) return ENEC_E_ARG;
    Header h;
    int rc = parse_header(host_header, &h);
    if (rc != ENEC_OK) return rc;
    if (params) *params = h.prm;
    if (n_elems) *n_elems = h.n_elems;
    if (block_size) *block_size = h.B;
    if (total_bytes) *total_bytes = h.total;
    if (dtype) *dtype = h.dtype;
    if (status) *status = h.status;
    return ENEC_OK;
}

int enec_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || !aligned16(dst) || !aligned16(src) || (bytes & 15)) return ENEC_E_ARG;
    const uint64_t nvec = bytes / 16;
    if (nvec == 0) return ENEC_OK;
    uint64_t want = (nvec + 255) / 256;
    const unsigned grid = (unsigned)(want > 8192 ? 8192 : want);
    copy_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(static_cast<uint4 *>(dst), static_cast<const uint4 *>(src), nvec);
    return hipGetLastError() == hipSuccess ? ENEC_OK : ENEC_E_HIP;
}

}  // extern "C"
