/*
 * libenec -- ENEC lossless codec for bf16 / fp16 / fp32 model weights on AMD MI355X (gfx950).
 *
 * C ABI.  Every entry point takes plain pointers and sizes; the doc of each argument
 * says whether it is a HOST or a DEVICE pointer.  The library allocates no device
 * memory: inputs, outputs and the workspace are the caller's.  All work is enqueued
 * on the HIP stream passed as `stream` (a hipStream_t handed over as void*, NULL =
 * the default stream).  Unless stated otherwise a call returns as soon as its work
 * is enqueued.
 *
 * The codec (paper sections in brackets):
 *   bf16 word -> exponent x (8 bit) and a raw sign+mantissa byte       [Sec. IV-B; Sec. V-A step 1]
 *   fp16 / fp32 are split the same way, only exponents are coded        [Alg. 1 input; Sec. VI-B]
 *   y = (b - x) mod 2^n, the branch-free integer transformation        [Sec. V-C; Eq. 2]
 *   per group of L consecutive elements (16 in the paper): OR of the y; the group is
 *   stored with m bits per element if OR < 2^m, else with n bits       [Sec. V-B]
 *   fixed-length fields are packed with hierarchical halving
 *   bit-packing with byte normalisation                                 [Sec. V-B, Alg. 2]
 *   a prefix sum over per-data-block compressed sizes places each data
 *   block in the output stream                                          [Fig. 4]
 *   decompression: offset lookup, prefix sum over mask bits, unpack,
 *   x = b - sext_n(y), recombine                                        [Sec. IV-B Alg. 1 (decompression); Sec. V-A]
 *   parameters (b, n, m, L) from the exponent histogram                 [Sec. V-E, Eq. 1-4]
 *
 * Stream format, version 1 (all integers little-endian):
 *   0   "ENEC"                 4   u16 version = 1      6  u8 dtype (enec_dtype) 7  u8 L (8, 16, 32)
 *   8   u64 n_elems            16  u32 block_size B     20 u32 n_blocks nb = ceil(n_elems / B)
 *   24  u8 b   25 u8 n   26 u8 m   27 u8 exponent bits (8; fp16: 5)
 *   28  u32 status (ENEC_OK or ENEC_E_RANGE)            32 u64 total_bytes (0 if status != OK)
 *   40  u8 tuple mode: 0 = (b, n, m) above hold for every data block; 1 = one tuple per data block
 *       (then bytes 24..26 are zero and the tuples follow the offset table, see enec_compress_per_block)
 *   41..63 zero
 *   64  (nb + 1) x u64: offset of each data block's payload relative to the payload base,
 *       i.e. the exclusive prefix sums of payload sizes; entry nb is their total
 *   zero bytes up to align16(64 + 8 (nb + 1)) = payload base for bf16 and fp16
 *   tuple mode 1 only: nb x 4 bytes (b, n, m, 0), then zero bytes up to a multiple of 16
 *   fp32 only: the lower 16 bits of every element, element order, then zero bytes up to a
 *       multiple of 16; the payload base follows.  (The upper 16 bits of an fp32 element are a
 *       bf16 word and are coded as such.)
 *   per data block, at payload base + offset[k] (always 16-byte aligned):
 *       B bytes            sign<<7 | first seven mantissa bits of every element, element order
 *       B/(8L) bytes       group mask: group g (elements gL .. gL+L-1) is bit (g mod 8), LSB first,
 *                          of byte (g div 8); 1 = stored with n bits
 *       m*B/8 bytes        Alg. 2 over (y mod 2^m) of all B elements; fp16: (m+3)*B/8 bytes, Alg. 2
 *                          over (y mod 2^m) | (last three mantissa bits) << m
 *       (n-m)L/8 bytes per masked group, in group order: Alg. 2 over (y >> m) of its L elements
 *                          (without the zero byte Alg. 2 appends to an odd byte count)
 *       zero bytes up to a multiple of 16
 *   The last data block is completed with elements that encode as y = 0 and zero sign and
 *   mantissa bits.
 */
#ifndef ENEC_H
#define ENEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ENEC_OK = 0,
    ENEC_E_ARG = 1,       /* null / misaligned pointer, size out of range */
    ENEC_E_DTYPE = 2,     /* not one of enec_dtype */
    ENEC_E_BLOCK = 3,     /* block_size not a power of two in [2048, 32768] */
    ENEC_E_PARAMS = 4,    /* need 1 <= n <= E, 0 <= m <= n, b < 2^E (E = exponent bits: 8, fp16: 5), L in {8, 16, 32}
                             with 128 L <= block_size <= 2048 L */
    ENEC_E_CAPACITY = 5,  /* out_capacity < enec_compress_bound() or workspace too small */
    ENEC_E_RANGE = 6,     /* an exponent lies outside [b - 2^(n-1) + 1, b + 2^(n-1)] while n < E */
    ENEC_E_FORMAT = 7,    /* not an ENEC stream, or header does not match the call */
    ENEC_E_HIP = 8        /* a HIP runtime call failed; as a header status: the scan gave up on a corrupt workspace
                             (every stream of that launch then carries it) */
} enec_status;

/* Element formats [Alg. 1 input line; Table VI]: sign | exponent | mantissa = 1|8|7, 1|5|10, 1|8|23.
 * Tensors are arrays of little-endian 16-bit (bf16, fp16) or 32-bit (fp32) words. */
typedef enum { ENEC_BF16 = 0, ENEC_FP16 = 1, ENEC_FP32 = 2 } enec_dtype;

/* Codec parameters [Sec. V-E; Table VI]: mapping centre b, stored width n, threshold width m,
 * group length L (8, 16 or 32; the tuners return 16 unless asked otherwise). */
typedef struct { uint8_t b, n, m, L; } enec_params;

#define ENEC_HEADER_BYTES 64u
#define ENEC_DEFAULT_BLOCK 16384u

uint32_t enec_version(void);                 /* stream format version this library writes (1) */
const char *enec_strerror(int status);       /* static string, never NULL */

/* Data-block size used when block_size = 0 is passed: 16384 [Sec. VI-D "Data Block Size"], or for
 * tensors shorter than that the largest power of two <= n_elems, but at least 2048. */
uint32_t enec_default_block_size(size_t n_elems);

/* Worst-case stream size in bytes for n_elems elements (every group stored with 8 bits).
 * Returns 0 on invalid dtype / block_size.  block_size = 0 means the default. */
size_t enec_compress_bound(size_t n_elems, int dtype, uint32_t block_size);

/* Size in bytes of the DEVICE workspace enec_compress / enec_tune need for a tensor of n_elems
 * elements (inter-block scan state, ticket counters, histogram), or for a batch of up to 16 tensors
 * with n_elems elements in total.  A workspace sized for a larger tensor serves smaller ones.
 * Returns 0 on invalid block_size. */
size_t enec_workspace_bytes(size_t n_elems, uint32_t block_size);

/* Enqueues a fill kernel that zeroes `bytes` bytes of the DEVICE workspace.  Must run once after
 * the workspace is allocated; after that one workspace serves any number of calls that do not
 * overlap in time (the library keeps its counters and call tags in it).  16-byte aligned.
 * Pass the same workspace_bytes with a workspace on every call: the library places its state by
 * that size.  After a size change, or after a process died in the middle of a call, initialise
 * the workspace again. */
int enec_workspace_init(void *workspace, size_t bytes, void *stream);

/* Compress n_elems values [Sec. V-A compression path; Sec. V-B; Sec. V-C; Fig. 4].
 *   in            DEVICE, n_elems * 2 bytes (fp32: * 4), 16-byte aligned, read only
 *   dtype         an enec_dtype
 *   block_size    data-block size B in elements: power of two in [2048, 32768], 0 = default
 *   params        HOST, read before return.  NULL = tune on the device first (this makes the call
 *                 synchronous: it waits for the histogram, see enec_tune)
 *   out           DEVICE, out_capacity bytes, 16-byte aligned, must not overlap in / workspace
 *   out_capacity  must be >= enec_compress_bound(n_elems, dtype, block_size)
 *   out_bytes     NULL, or a DEVICE-ACCESSIBLE pointer (device memory, or pinned host memory from
 *                 hipHostMalloc), 8-byte aligned: the kernel stores the stream size there
 *                 (0 on ENEC_E_RANGE); valid once the stream has been synchronised.  Pageable
 *                 host memory is rejected with ENEC_E_ARG.
 *   workspace     DEVICE, zeroed by enec_workspace_init; calls sharing one workspace must not
 *                 run concurrently
 *   workspace_bytes  its size; ENEC_E_CAPACITY if < enec_workspace_bytes(n_elems, block_size)
 *   stream        hipStream_t
 * One kernel launch.  The stream written is a pure function of (input bytes, params, block_size).
 * Errors detectable on the host return at once with nothing enqueued.  The data-dependent
 * ENEC_E_RANGE is found by the kernel: header.status = ENEC_E_RANGE, header.total_bytes = 0,
 * *out_bytes = 0, payload undefined.  The same holds for header.status = ENEC_E_HIP, which the kernel
 * writes instead of waiting for ever if the workspace was not in the state the last call left it in. */
int enec_compress(const void *in, size_t n_elems, int dtype, uint32_t block_size,
                  const enec_params *params, void *out, size_t out_capacity,
                  uint64_t *out_bytes, void *workspace, size_t workspace_bytes, void *stream);

/* enec_compress for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scan state, ticket
 * counters and call tags live in an array of ENEC_STATIC_SCRATCH_BYTES bytes inside the library's code
 * object, one per GPU, held until the process ends; the call allocates nothing, on the device or through
 * any library.  Arguments as for enec_compress, without the workspace; params must not be NULL
 * (ENEC_E_ARG: tuning would wait for the stream).  ENEC_E_CAPACITY if the tensor needs more scan state
 * than the array holds, i.e. if enec_workspace_bytes(n_elems, block_size) > ENEC_STATIC_SCRATCH_BYTES
 * (at the default block size about 1.6e9 elements fit, at block size 2048 about 2.0e8).  The first
 * call on a GPU enqueues a fill kernel on `stream` that zeroes the array; after that the array keeps
 * the state the last call left, as a workspace does.  All calls on one GPU share that GPU's array:
 * calls that overlap in time on one GPU (two streams, two host threads) race and must be serialised by
 * the caller.  The stream written is the one enec_compress writes. */
#define ENEC_STATIC_SCRATCH_BYTES (1u << 20)
int enec_compress_static(const void *in, size_t n_elems, int dtype, uint32_t block_size,
                         const enec_params *params, void *out, size_t out_capacity, uint64_t *out_bytes,
                         void *stream);

/* Compress several tensors with as few kernel launches as possible: tensors that share (m, n - m, L,
 * block size) go into one launch (up to 16 tensors each), whose workgroups walk the data blocks of all of them, so that
 * small tensors cost no launch of their own and the device never drains between tensors.
 * Every field of an item means what the argument of the same name means for enec_compress
 * (params == NULL tunes that tensor first, which makes the call synchronous).  The workspace
 * must hold enec_workspace_bytes(sum of the items' n_elems, block size).  Items are independent:
 * a range error in one is reported in that item's header only. */
typedef struct {
    const void *in;             /* DEVICE */
    size_t n_elems;
    uint32_t block_size;        /* 0 = default */
    const enec_params *params;  /* HOST, or NULL */
    void *out;                  /* DEVICE */
    size_t out_capacity;
    uint64_t *out_bytes;        /* device-accessible, or NULL */
} enec_compress_item;
int enec_compress_batch(const enec_compress_item *items, size_t n_items, int dtype, void *workspace,
                        size_t workspace_bytes, void *stream);

/* Decompress [Sec. V-A decompression path; Alg. 1 decompression part].
 *   in        DEVICE, a stream written by enec_compress, 16-byte aligned
 *   in_bytes  size of the buffer behind `in`; ENEC_E_FORMAT if the header's total_bytes exceeds it.
 *             The kernel never reads past the header's total_bytes.
 *   out       DEVICE, n_elems * 2 bytes (4 if the header's dtype is fp32), 16-byte aligned
 *   n_elems   must equal the header's n_elems
 * This variant copies the 64-byte header to the host first (one small synchronous copy on
 * `stream`), validates it (ENEC_E_FORMAT / ENEC_E_DTYPE), then enqueues one kernel. */
int enec_decompress(const void *in, size_t in_bytes, void *out, size_t n_elems, void *stream);

/* Same, fully asynchronous: `host_header` is a HOST copy of the stream's first 64 bytes that the
 * caller already holds (kept from compression, or read from a file).  The kernel compares it with
 * the header in device memory and writes nothing if they differ.
 *   status   NULL, or a DEVICE-ACCESSIBLE pointer (device or pinned host memory, 4-byte aligned) to a
 *            word the caller has set to 0: the kernel stores ENEC_E_FORMAT there if it leaves any data
 *            block undecoded (header in memory differs from host_header, or an offset-table entry is
 *            misaligned, out of order, outside the stream or implies an impossible size).  The blocks it
 *            does decode are exact; a skipped block's part of `out` is not written.  Valid once the
 *            stream has been synchronised.  With NULL such blocks are skipped silently. */
int enec_decompress_with_header(const void *in, size_t in_bytes, const void *host_header, void *out,
                                size_t n_elems, uint32_t *status, void *stream);

/* Decompress several streams with one launch per (dtype, m, n - m, block size); fields as the arguments of
 * enec_decompress_with_header.  Fully asynchronous. */
typedef struct {
    const void *in;             /* DEVICE */
    size_t in_bytes;
    const void *host_header;    /* HOST, 64 bytes */
    void *out;                  /* DEVICE */
    size_t n_elems;
    uint32_t *status;           /* device-accessible word set to 0 by the caller, or NULL */
} enec_decompress_item;
int enec_decompress_batch(const enec_decompress_item *items, size_t n_items, void *stream);

/* Decompression pipelines [Sec. VI, "End-to-End Inference Configurations": weights are decompressed layer
 * by layer, the decompression of layer k+1 overlapping the forward pass of layer k; Sec. VI, "End-to-End
 * Inference Speedup": what is saved is the transfer of weights from the CPU].  A pipeline is a HOST object that orders
 * work on the caller's HIP streams with events; it owns no device memory and launches only what
 * enec_decompress_batch launches.  Layers are decoded into `n_slots` sets of output buffers that the caller
 * owns (two = double buffering): slot s holds layer k while the consumer computes with it and is handed to
 * layer k + n_slots afterwards.
 *   enec_pipeline_prefetch            on the decompression stream: wait until the consumer has released
 *                                     the slot, then decompress `items` (DEVICE streams, as for
 *                                     enec_decompress_batch) into the slot's buffers
 *   enec_pipeline_prefetch_from_host  the same for streams held in pinned HOST memory (hipHostMalloc): each
 *                                     stream is copied into one half of the DEVICE staging buffer on the
 *                                     copy stream and decoded out of it on the decompression stream, so that
 *                                     the copy of stream i + 1 overlaps the decoding of stream i.  The header
 *                                     is read from the host copy.  ENEC_E_CAPACITY if a stream is larger than
 *                                     half the staging buffer.
 *   enec_pipeline_acquire             the consumer's stream waits until the slot's prefetch has finished
 *   enec_pipeline_release             marks, on the consumer's stream, the point after which the slot's
 *                                     buffers may be overwritten
 * All four return at once (nothing waits on the host).  Calls on one pipeline must come from one host
 * thread at a time.  Streams are hipStream_t handles and stay the caller's; keep them at the default
 * priority.  Items (also the host headers they point to) are read before the call returns.
 *   n_slots            1..64
 *   decompress_stream  where the decompression kernels run (a side stream, so that they overlap the consumer)
 *   copy_stream        NULL, or a third stream for the host-to-device copies (needed for ..._from_host)
 *   staging            NULL, or DEVICE, 16-byte aligned, staging_bytes bytes, used in two halves
 *   trace              non-zero: record timing events around every copy and every decompression;
 *                      enec_pipeline_trace then waits for them and returns, per step in call order, four
 *                      times in milliseconds since the first event: copy start, copy end, decompression
 *                      start, decompression end (-1 for the copy of a step that had none), and forgets them
 * enec_pipeline_destroy frees the host object and its events; work already enqueued is not affected. */
typedef struct enec_pipeline enec_pipeline;
typedef struct {
    const void *host_stream;    /* HOST, pinned: a whole ENEC stream */
    size_t stream_bytes;
    void *out;                  /* DEVICE, 16-byte aligned */
    size_t n_elems;
    uint32_t *status;           /* as in enec_decompress_item, or NULL */
} enec_offload_item;
int enec_pipeline_create(enec_pipeline **pipeline, uint32_t n_slots, void *decompress_stream, void *copy_stream,
                         void *staging, size_t staging_bytes, int trace);
void enec_pipeline_destroy(enec_pipeline *pipeline);
int enec_pipeline_prefetch(enec_pipeline *pipeline, uint32_t slot, const enec_decompress_item *items, size_t n_items);
int enec_pipeline_prefetch_from_host(enec_pipeline *pipeline, uint32_t slot, const enec_offload_item *items,
                                     size_t n_items);
int enec_pipeline_acquire(enec_pipeline *pipeline, uint32_t slot, void *consumer_stream);
int enec_pipeline_release(enec_pipeline *pipeline, uint32_t slot, void *consumer_stream);
int enec_pipeline_trace(enec_pipeline *pipeline, float *ms, size_t max_steps, size_t *n_steps);

/* Parameter tuning [Sec. V-E phases 1-3]: exponent histogram on the device (one read of the
 * tensor), then the search for (b, n) by Eq. 1-3 and for m by Eq. 4 (L = 16) on the host.
 *   in         DEVICE, n_elems * 2 bytes (fp32: * 4), 16-byte aligned
 *   params     HOST, written before return
 *   histogram  NULL, or HOST array of 256 u64 that receives the exponent counts
 *   workspace  DEVICE, as for enec_compress (workspace_bytes: its size)
 * Synchronous: returns after the histogram has been copied back. */
int enec_tune(const void *in, size_t n_elems, int dtype, enec_params *params,
              uint64_t *histogram, void *workspace, size_t workspace_bytes, void *stream);

/* Many tensors at once: the histograms of up to sixteen tensors are counted into sixteen slots of the
 * workspace, copied back together, and the stream is waited for once per sixteen tensors (tuning a
 * layer's tensors one by one spends most of its time in those waits).
 *   items       HOST array; in = DEVICE, 16-byte aligned
 *   every       1 = all exponents, k = every k-th chunk of 4096 elements (see enec_tune_sampled)
 *   params      HOST array of n_items tuples, written before return
 *   histograms  NULL, or HOST array of n_items * 256 u64
 * enec_compress and enec_compress_batch tune the tensors they are given without a tuple this way. */
typedef struct {
    const void *in;
    size_t n_elems;
} enec_tune_item;
int enec_tune_batch(const enec_tune_item *items, size_t n_items, int dtype, uint32_t every, enec_params *params,
                    uint64_t *histograms, void *workspace, size_t workspace_bytes, void *stream);

/* The tuner on a sample [Sec. V-E phase 1 counts exponents; a sample keeps the counting cheap]: only
 * the elements whose index e has (e / 4096) % every == 0 are counted, i.e. every `every`-th chunk
 * of 4096 elements, the first one included; every = 1 is enec_tune.  An exponent that the sample
 * misses can fall outside the window of the tuple found: enec_compress then reports ENEC_E_RANGE in
 * the header.  ENEC_E_ARG if every == 0; otherwise as enec_tune. */
int enec_tune_sampled(const void *in, size_t n_elems, int dtype, uint32_t every, enec_params *params,
                      uint64_t *histogram, void *workspace, size_t workspace_bytes, void *stream);

/* enec_tune_sampled, then enec_compress with the tuple found; if the kernel reports ENEC_E_RANGE the
 * tensor is compressed once more with n widened to the exponent field's width, for which the
 * transform is a bijection and no exponent is out of range [Sec. V-C]; b, m and L stay.
 *   params_used  HOST, may be NULL: the tuple of the stream that `out` holds on return
 * Other arguments as for enec_compress.  Synchronous (the header's status is read back after each
 * pass).  Returns ENEC_OK, or what enec_tune_sampled / enec_compress return, or the header's status
 * if it is neither ENEC_OK nor ENEC_E_RANGE. */
int enec_compress_sampled(const void *in, size_t n_elems, int dtype, uint32_t block_size, uint32_t every,
                          enec_params *params_used, void *out, size_t out_capacity, void *workspace,
                          size_t workspace_bytes, void *stream);

/* One tuple per data block.  The paper tunes one (b, n, m) per tensor [Sec. V-E] and reports that
 * tensors differ [Table VI]; here the same search (Eq. 1-4) runs inside the compress kernel
 * on the exponents of each data block's own elements, and the block is coded with what it finds, so
 * no exponent is ever out of range and a tensor whose blocks differ in kind or scale is coded as
 * well as its parts would be.  Stream layout: as described at the top, with
 *   header byte 40 = 1, header (b, n, m) = (0, 0, 0) (n = 0 occurs in no other stream),
 *   the tuples, 4 bytes per block (b, n, m, 0), zero-padded to a multiple of 16, between the offset
 *   table and the fp32 region / the payloads.
 * enec_decompress, enec_decompress_with_header and enec_decompress_batch read such streams as any
 * other (in a batch, such streams of one element format, group length and block size share a launch).  Arguments as for enec_compress, without params;
 * group_length = 8, 16, 32 or 0 (= 16) is the group length the blocks are coded with (ENEC_E_PARAMS if
 * the block size does not admit it; the search evaluates Eq. 4, 1/L + n + (m - n) p(m)^L, with that length);
 * out_capacity >= enec_compress_bound_per_block(n_elems, dtype, block_size) (0 for an invalid dtype
 * or block size).  The workspace is used as by enec_compress and must not be shared with a call
 * that is still running.  Asynchronous. */
size_t enec_compress_bound_per_block(size_t n_elems, int dtype, uint32_t block_size);
int enec_compress_per_block(const void *in, size_t n_elems, int dtype, uint32_t block_size, uint32_t group_length,
                            void *out, size_t out_capacity, uint64_t *out_bytes, void *workspace,
                            size_t workspace_bytes, void *stream);

/* enec_compress_per_block for several tensors at once [Sec. V-E, per data block]: tensors of one block
 * size share a launch (up to 16 tensors each, in the order given), whose workgroups take the data
 * blocks of all of them, so that small tensors cost no launch of their own and the device does not
 * drain between tensors.  Every field of an item means what the argument of the same name means for
 * enec_compress_per_block; dtype and group_length hold for all items.  The streams written are the
 * ones enec_compress_per_block writes.  The workspace must hold enec_workspace_bytes(sum of the
 * items' n_elems, smallest block size among them) (ENEC_E_CAPACITY otherwise); ENEC_E_ARG also if
 * the tensors have more than 2^32 - 1 data blocks together.  Every argument is checked before
 * anything is enqueued.  Asynchronous. */
typedef struct {
    const void *in;             /* DEVICE */
    size_t n_elems;
    uint32_t block_size;        /* 0 = default */
    void *out;                  /* DEVICE */
    size_t out_capacity;
    uint64_t *out_bytes;        /* device-accessible, or NULL */
} enec_per_block_item;
int enec_compress_per_block_batch(const enec_per_block_item *items, size_t n_items, int dtype, uint32_t group_length,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* Host-only search of Sec. V-E phases 2-3 on a given 256-bin exponent histogram (HOST); dtype
 * fixes the cap of Eq. 1's width (the exponent field: 8 bits, fp16: 5). */
int enec_tune_histogram(const uint64_t *histogram, int dtype, enec_params *params);

/* The same search with the group length L chosen together with m, as Eq. 4 states it [Sec. V-E phase 3]:
 * group_lengths is the OR of the candidate lengths (8, 16, 32).  The paper's hardware forces L >= 16 and
 * finds 16 optimal throughout [Sec. VI-D], which is what enec_tune and enec_tune_histogram return;
 * without that rule shorter groups often win.  block_size (0 = 16384) is the data-block size the tensor
 * will be compressed with: a length it does not admit (128 L <= block_size <= 2048 L, i.e. L = 32 needs
 * block_size >= 4096 and L = 8 block_size <= 16384) is left out of the search, and 16, which every block
 * size admits, stands in if none is left.  ENEC_E_PARAMS if group_lengths names no or other lengths,
 * ENEC_E_BLOCK for an invalid block size. */
int enec_tune_histogram_groups(const uint64_t *histogram, int dtype, uint32_t group_lengths, uint32_t block_size,
                               enec_params *params);

/* Parse a HOST copy of a stream's first 64 bytes.  Any output pointer may be NULL.
 * Returns ENEC_E_FORMAT if it is not a version-1 ENEC header. */
int enec_stream_info(const void *host_header, enec_params *params, uint64_t *n_elems,
                     uint32_t *block_size, uint64_t *total_bytes, int *dtype, uint32_t *status);

/* Measurement aid: a plain 128-bit grid-stride copy of `bytes` bytes (multiple of 16) between two
 * 16-byte aligned DEVICE buffers.  Its achieved bandwidth is the practical ceiling the codec
 * kernels are compared with, and the scale for the HBM traffic counters. */
int enec_copy(void *dst, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ENEC_H */
