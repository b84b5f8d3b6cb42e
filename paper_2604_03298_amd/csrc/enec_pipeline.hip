// Host side of libenec's decompression pipelines: event choreography on the caller's HIP streams around
// enec_decompress_batch.  No kernel lives here and nothing is allocated on the device.
// See include/enec.h for the contract of every entry point.
#include "enec.h"

#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

struct enec_pipeline {
    uint32_t n_slots = 0;
    hipStream_t dec = nullptr, copy = nullptr;
    uint8_t *staging = nullptr;
    size_t half_bytes = 0;
    bool trace = false;
    std::vector<hipEvent_t> ready, released;        // per slot
    std::vector<char> released_once;                // a slot that was never released is free
    hipEvent_t staged[2] = {nullptr, nullptr};      // per half of the staging buffer: copy into it finished
    hipEvent_t drained[2] = {nullptr, nullptr};     //                                 decompression out of it finished
    bool half_used[2] = {false, false};
    uint64_t copies = 0;
    // trace: four timing events per recorded step (copy start / end, decompression start / end); a step
    // without a copy leaves the first two null
    std::vector<hipEvent_t> tr;
};

namespace {

bool ok(hipError_t e)
{
    if (e == hipSuccess) return true;
    (void)hipGetLastError();
    return false;
}

hipEvent_t new_event(bool timing)
{
    hipEvent_t e = nullptr;
    if (!ok(hipEventCreateWithFlags(&e, timing ? hipEventDefault : hipEventDisableTiming))) return nullptr;
    return e;
}

void drop_trace(enec_pipeline *p)
{
    for (hipEvent_t e : p->tr)
        if (e) (void)hipEventDestroy(e);
    p->tr.clear();
}

// timing event recorded on `s` now, kept in the trace; false if the runtime refuses
bool mark(enec_pipeline *p, hipStream_t s)
{
    hipEvent_t e = new_event(true);
    if (!e) return false;
    p->tr.push_back(e);
    return ok(hipEventRecord(e, s));
}

}  // namespace

extern "C" {

int enec_pipeline_create(enec_pipeline **out, uint32_t n_slots, void *decompress_stream, void *copy_stream,
                         void *staging, size_t staging_bytes, int trace)
{
    if (!out || n_slots == 0 || n_slots > 64 || ((uintptr_t)staging & 15)) return ENEC_E_ARG;
    if (copy_stream && copy_stream == decompress_stream) return ENEC_E_ARG;       // nothing could overlap
    enec_pipeline *p = new (std::nothrow) enec_pipeline;
    if (!p) return ENEC_E_ARG;
    p->n_slots = n_slots;
    p->dec = (hipStream_t)decompress_stream;
    p->copy = (hipStream_t)copy_stream;
    p->staging = static_cast<uint8_t *>(staging);
    p->half_bytes = (staging_bytes / 2) & ~(size_t)15;
    p->trace = trace != 0;
    p->ready.assign(n_slots, nullptr);
    p->released.assign(n_slots, nullptr);
    p->released_once.assign(n_slots, 0);
    bool good = true;
    for (uint32_t i = 0; i < n_slots; ++i) {
        good &= (p->ready[i] = new_event(false)) != nullptr;
        good &= (p->released[i] = new_event(false)) != nullptr;
    }
    for (int h = 0; h < 2; ++h) {
        good &= (p->staged[h] = new_event(false)) != nullptr;
        good &= (p->drained[h] = new_event(false)) != nullptr;
    }
    if (!good) {
        enec_pipeline_destroy(p);
        return ENEC_E_HIP;
    }
    *out = p;
    return ENEC_OK;
}

void enec_pipeline_destroy(enec_pipeline *p)
{
    if (!p) return;
    for (hipEvent_t e : p->ready) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : p->released) if (e) (void)hipEventDestroy(e);
    for (int h = 0; h < 2; ++h) {
        if (p->staged[h]) (void)hipEventDestroy(p->staged[h]);
        if (p->drained[h]) (void)hipEventDestroy(p->drained[h]);
    }
    drop_trace(p);
    delete p;
}

int enec_pipeline_prefetch(enec_pipeline *p, uint32_t slot, const enec_decompress_item *items, size_t n_items)
{
    if (!p || slot >= p->n_slots || (!items && n_items)) return ENEC_E_ARG;
    // the slot's buffers may still be read by the consumer of the layer that held them before
    if (p->released_once[slot] && !ok(hipStreamWaitEvent(p->dec, p->released[slot], 0))) return ENEC_E_HIP;
    if (p->trace) {
        p->tr.push_back(nullptr);
        p->tr.push_back(nullptr);
        if (!mark(p, p->dec)) return ENEC_E_HIP;
    }
    const int rc = enec_decompress_batch(items, n_items, p->dec);
    if (rc != ENEC_OK) return rc;
    if (p->trace && !mark(p, p->dec)) return ENEC_E_HIP;
    return ok(hipEventRecord(p->ready[slot], p->dec)) ? ENEC_OK : ENEC_E_HIP;
}

int enec_pipeline_prefetch_from_host(enec_pipeline *p, uint32_t slot, const enec_offload_item *items, size_t n_items)
{
    if (!p || slot >= p->n_slots || (!items && n_items)) return ENEC_E_ARG;
    if (!p->copy || !p->staging) return ENEC_E_ARG;
    for (size_t i = 0; i < n_items; ++i) {
        if (!items[i].host_stream || items[i].stream_bytes < ENEC_HEADER_BYTES) return ENEC_E_FORMAT;
        if (items[i].stream_bytes > p->half_bytes) return ENEC_E_CAPACITY;
    }
    if (p->released_once[slot] && !ok(hipStreamWaitEvent(p->dec, p->released[slot], 0))) return ENEC_E_HIP;
    for (size_t i = 0; i < n_items; ++i) {
        const int h = (int)(p->copies & 1u);
        uint8_t *half = p->staging + (size_t)h * p->half_bytes;
        // copy stream: the half must have been drained by the decompression that last read it
        if (p->half_used[h] && !ok(hipStreamWaitEvent(p->copy, p->drained[h], 0))) return ENEC_E_HIP;
        if (p->trace && !mark(p, p->copy)) return ENEC_E_HIP;
        if (!ok(hipMemcpyAsync(half, items[i].host_stream, items[i].stream_bytes, hipMemcpyHostToDevice, p->copy)))
            return ENEC_E_HIP;
        if (p->trace && !mark(p, p->copy)) return ENEC_E_HIP;
        if (!ok(hipEventRecord(p->staged[h], p->copy))) return ENEC_E_HIP;
        // decompression stream: wait for the copy, decode out of the half, hand the half back
        if (!ok(hipStreamWaitEvent(p->dec, p->staged[h], 0))) return ENEC_E_HIP;
        if (p->trace && !mark(p, p->dec)) return ENEC_E_HIP;
        enec_decompress_item d;
        d.in = half;
        d.in_bytes = items[i].stream_bytes;
        d.host_header = items[i].host_stream;           // the stream's first 64 bytes, read here on the host
        d.out = items[i].out;
        d.n_elems = items[i].n_elems;
        d.status = items[i].status;
        const int rc = enec_decompress_batch(&d, 1, p->dec);
        if (p->trace && !mark(p, p->dec)) return ENEC_E_HIP;
        // also after a refused stream: the half is free again as far as this pipeline is concerned
        if (!ok(hipEventRecord(p->drained[h], p->dec))) return ENEC_E_HIP;
        p->half_used[h] = true;
        ++p->copies;
        if (rc != ENEC_OK) return rc;
    }
    return ok(hipEventRecord(p->ready[slot], p->dec)) ? ENEC_OK : ENEC_E_HIP;
}

int enec_pipeline_acquire(enec_pipeline *p, uint32_t slot, void *consumer_stream)
{
    if (!p || slot >= p->n_slots) return ENEC_E_ARG;
    return ok(hipStreamWaitEvent((hipStream_t)consumer_stream, p->ready[slot], 0)) ? ENEC_OK : ENEC_E_HIP;
}

int enec_pipeline_release(enec_pipeline *p, uint32_t slot, void *consumer_stream)
{
    if (!p || slot >= p->n_slots) return ENEC_E_ARG;
    if (!ok(hipEventRecord(p->released[slot], (hipStream_t)consumer_stream))) return ENEC_E_HIP;
    p->released_once[slot] = 1;
    return ENEC_OK;
}

int enec_pipeline_trace(enec_pipeline *p, float *ms, size_t max_steps, size_t *n_steps)
{
    if (!p || !n_steps || (!ms && max_steps)) return ENEC_E_ARG;
    const size_t steps = p->tr.size() / 4;
    *n_steps = steps;
    if (!p->trace) return ENEC_E_ARG;
    hipEvent_t origin = nullptr;
    for (hipEvent_t e : p->tr)
        if (e) { origin = e; break; }
    int rc = ENEC_OK;
    for (size_t i = 0; i < 4 * steps && rc == ENEC_OK; ++i) {
        hipEvent_t e = p->tr[i];
        if (e && !ok(hipEventSynchronize(e))) rc = ENEC_E_HIP;
        if (i / 4 >= max_steps) continue;
        float t = -1.0f;
        if (e && rc == ENEC_OK && !ok(hipEventElapsedTime(&t, origin, e))) rc = ENEC_E_HIP;
        ms[i] = t;
    }
    drop_trace(p);
    return rc;
}

}  // extern "C"
