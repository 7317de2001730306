// Just-in-time layer decode (paper Section 3.3): compressed layers stay resident, a layer's
// weights are decoded into a shared, pre-allocated buffer right before they are used, and the
// buffer is reused by a later layer.  This file is the stream-ordered bookkeeping around
// ecf8_decode_batched: one decode stream owned by the manager, one "ready" event per layer,
// one "released" event per buffer.  With two or more buffers the decode of layer l+1 runs
// while layer l computes.  Host code only; the manager owns no device memory.
#include <hip/hip_runtime.h>
#include <cstring>
#include <new>
#include <vector>

#include "ecf8.h"
#include "ecfw.h"

struct ecf8_jit {
    enum State { FREE, READY, ACQUIRED };
    struct Layer {
        const void *d_items = nullptr;    // ecf8_batch_item[] or, for a layer of wider elements, ecfw_batch_item[]
        uint32_t n_tensors = 0;
        bool wide = false;
        ecf8_batch_info info{};
        ecfw_batch_info winfo{};
        bool prepared = false;
        hipEvent_t ready = nullptr;
    };
    struct Buffer {
        void *base = nullptr;
        State state = FREE;
        uint32_t layer = 0;
        bool released_recorded = false;   // `released` has been recorded at least once
        hipEvent_t released = nullptr;
    };
    std::vector<Layer> layers;
    std::vector<Buffer> buffers;
    uint64_t buffer_bytes = 0;
    uint32_t max_workgroups = 0;
    hipStream_t decode_stream = nullptr;
};

namespace {
constexpr uint64_t ALIGN = 256;
uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }
}

extern "C" {

int ecf8_jit_create(uint32_t n_layers, uint32_t n_buffers, void *const *d_buffers, uint64_t buffer_bytes,
                    ecf8_jit **out)
{
    if (!out || !d_buffers || n_layers == 0 || n_buffers == 0 || buffer_bytes == 0) return ECF8_E_ARG;
    for (uint32_t b = 0; b < n_buffers; b++) {
        if (!d_buffers[b]) return ECF8_E_ARG;
        if ((uintptr_t)d_buffers[b] & 15) return ECF8_E_ALIGN;
    }
    ecf8_jit *j = new (std::nothrow) ecf8_jit;
    if (!j) return ECF8_E_NOMEM;
    try {
        j->layers.resize(n_layers);
        j->buffers.resize(n_buffers);
    } catch (...) {
        delete j;
        return ECF8_E_NOMEM;
    }
    j->buffer_bytes = buffer_bytes;
    bool ok = hipStreamCreateWithFlags(&j->decode_stream, hipStreamNonBlocking) == hipSuccess;
    for (uint32_t b = 0; ok && b < n_buffers; b++) {
        j->buffers[b].base = d_buffers[b];
        ok = hipEventCreateWithFlags(&j->buffers[b].released, hipEventDisableTiming) == hipSuccess;
    }
    for (uint32_t l = 0; ok && l < n_layers; l++)
        ok = hipEventCreateWithFlags(&j->layers[l].ready, hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        ecf8_jit_destroy(j);
        return ECF8_E_HIP;
    }
    *out = j;
    return ECF8_OK;
}

void ecf8_jit_destroy(ecf8_jit *j)
{
    if (!j) return;
    if (j->decode_stream) {
        (void)hipStreamSynchronize(j->decode_stream);
        (void)hipStreamDestroy(j->decode_stream);
    }
    for (auto &b : j->buffers)
        if (b.released) (void)hipEventDestroy(b.released);
    for (auto &l : j->layers)
        if (l.ready) (void)hipEventDestroy(l.ready);
    delete j;
}

int ecf8_jit_layer_prepare(ecf8_jit *j, uint32_t layer, const ecf8_header *hdrs, const void *const *d_blobs,
                           uint32_t n_tensors, ecf8_batch_item *items_host, uint64_t *offsets)
{
    if (!j || !hdrs || !d_blobs || !items_host || !offsets || n_tensors == 0) return ECF8_E_ARG;
    if (layer >= j->layers.size()) return ECF8_E_ARG;
    const ecf8_jit::Buffer &buf = j->buffers[layer % j->buffers.size()];
    std::vector<void *> outs;
    std::vector<uint64_t> caps;
    try {
        outs.resize(n_tensors);
        caps.resize(n_tensors);
    } catch (...) {
        return ECF8_E_NOMEM;
    }
    uint64_t at = 0;
    for (uint32_t i = 0; i < n_tensors; i++) {
        if (hdrs[i].n_elem == 0 || hdrs[i].n_elem > j->buffer_bytes) return ECF8_E_CAPACITY;
        offsets[i] = at;
        caps[i] = hdrs[i].n_elem;
        at = round_up(at + hdrs[i].n_elem, ALIGN);
        if (offsets[i] + hdrs[i].n_elem > j->buffer_bytes) return ECF8_E_CAPACITY;
        outs[i] = (uint8_t *)buf.base + offsets[i];
    }
    ecf8_batch_info info;
    int rc = ecf8_batch_prepare(hdrs, d_blobs, outs.data(), caps.data(), n_tensors, items_host, &info);
    if (rc) return rc;
    ecf8_jit::Layer &L = j->layers[layer];
    L.info = info;
    L.n_tensors = n_tensors;
    L.d_items = nullptr;
    L.wide = false;
    L.prepared = true;
    return ECF8_OK;
}

int ecf8_jit_layer_commit(ecf8_jit *j, uint32_t layer, const ecf8_batch_item *d_items)
{
    if (!j || !d_items || layer >= j->layers.size() || !j->layers[layer].prepared || j->layers[layer].wide) return ECF8_E_ARG;
    if ((uintptr_t)d_items & 15) return ECF8_E_ALIGN;
    j->layers[layer].d_items = d_items;
    return ECF8_OK;
}

// The same two steps for a layer held in the wide-alphabet container (E5M2, BF16): a manager can
// mix such layers with FP8 ones; everything else (prefetch, acquire, release) is format-blind.
int ecfw_jit_layer_prepare(ecf8_jit *j, uint32_t layer, const ecfw_header *hdrs, const void *const *d_blobs,
                           uint32_t n_tensors, ecfw_batch_item *items_host, uint64_t *offsets)
{
    if (!j || !hdrs || !d_blobs || !items_host || !offsets || n_tensors == 0) return ECF8_E_ARG;
    if (layer >= j->layers.size()) return ECF8_E_ARG;
    const ecf8_jit::Buffer &buf = j->buffers[layer % j->buffers.size()];
    std::vector<void *> outs;
    std::vector<uint64_t> caps;
    try {
        outs.resize(n_tensors);
        caps.resize(n_tensors);
    } catch (...) {
        return ECF8_E_NOMEM;
    }
    uint64_t at = 0;
    for (uint32_t i = 0; i < n_tensors; i++) {
        const uint64_t elem = hdrs[i].fmt == ECFW_FMT_BF16 ? 2 : 1;
        if (hdrs[i].n_elem == 0 || hdrs[i].n_elem > j->buffer_bytes / elem) return ECF8_E_CAPACITY;
        const uint64_t bytes = hdrs[i].n_elem * elem;
        offsets[i] = at;
        caps[i] = bytes;
        at = round_up(at + bytes, ALIGN);
        if (offsets[i] + bytes > j->buffer_bytes) return ECF8_E_CAPACITY;
        outs[i] = (uint8_t *)buf.base + offsets[i];
    }
    ecfw_batch_info info;
    int rc = ecfw_batch_prepare(hdrs, d_blobs, outs.data(), caps.data(), n_tensors, items_host, &info);
    if (rc) return rc;
    ecf8_jit::Layer &L = j->layers[layer];
    L.winfo = info;
    L.n_tensors = n_tensors;
    L.d_items = nullptr;
    L.wide = true;
    L.prepared = true;
    return ECF8_OK;
}

int ecfw_jit_layer_commit(ecf8_jit *j, uint32_t layer, const ecfw_batch_item *d_items)
{
    if (!j || !d_items || layer >= j->layers.size() || !j->layers[layer].prepared || !j->layers[layer].wide) return ECF8_E_ARG;
    if ((uintptr_t)d_items & 15) return ECF8_E_ALIGN;
    j->layers[layer].d_items = d_items;
    return ECF8_OK;
}

int ecf8_jit_set_decode_workgroups(ecf8_jit *j, uint32_t max_workgroups)
{
    if (!j) return ECF8_E_ARG;
    j->max_workgroups = max_workgroups;
    return ECF8_OK;
}

int ecf8_jit_prefetch(ecf8_jit *j, uint32_t layer)
{
    if (!j || layer >= j->layers.size()) return ECF8_E_ARG;
    ecf8_jit::Layer &L = j->layers[layer];
    ecf8_jit::Buffer &B = j->buffers[layer % j->buffers.size()];
    if (!L.d_items || B.state != ecf8_jit::FREE) return ECF8_E_ARG;   // not committed, or the buffer is still in use
    // the previous user of the buffer must be done with it before the decode overwrites it
    if (B.released_recorded && hipStreamWaitEvent(j->decode_stream, B.released, 0) != hipSuccess) return ECF8_E_HIP;
    int rc;
    if (L.wide) {
        L.winfo.max_workgroups = j->max_workgroups;
        rc = ecfw_decode_batched(L.d_items, L.n_tensors, &L.winfo, j->decode_stream);
    } else {
        L.info.max_workgroups = j->max_workgroups;
        rc = ecf8_decode_batched((const ecf8_batch_item *)L.d_items, L.n_tensors, &L.info, j->decode_stream);
    }
    if (rc) return rc;
    if (hipEventRecord(L.ready, j->decode_stream) != hipSuccess) return ECF8_E_HIP;
    B.state = ecf8_jit::READY;
    B.layer = layer;
    return ECF8_OK;
}

int ecf8_jit_acquire(ecf8_jit *j, uint32_t layer, void *stream, void **d_base)
{
    if (!j || layer >= j->layers.size()) return ECF8_E_ARG;
    ecf8_jit::Buffer &B = j->buffers[layer % j->buffers.size()];
    if (B.state != ecf8_jit::READY || B.layer != layer) return ECF8_E_ARG;   // prefetch(layer) first
    if (hipStreamWaitEvent((hipStream_t)stream, j->layers[layer].ready, 0) != hipSuccess) return ECF8_E_HIP;
    B.state = ecf8_jit::ACQUIRED;
    if (d_base) *d_base = B.base;
    return ECF8_OK;
}

int ecf8_jit_release(ecf8_jit *j, uint32_t layer, void *stream)
{
    if (!j || layer >= j->layers.size()) return ECF8_E_ARG;
    ecf8_jit::Buffer &B = j->buffers[layer % j->buffers.size()];
    if (B.state != ecf8_jit::ACQUIRED || B.layer != layer) return ECF8_E_ARG;
    if (hipEventRecord(B.released, (hipStream_t)stream) != hipSuccess) return ECF8_E_HIP;
    B.released_recorded = true;
    B.state = ecf8_jit::FREE;
    return ECF8_OK;
}

} // extern "C"
