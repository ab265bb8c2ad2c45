// Host-memory tier for the previous messages: pinned host rows, a few windows of
// rows in HBM, prefetch and write-back on a copy stream ordered against the
// compute stream with events (Section 3.3 of the paper).  Host code only: the
// codec kernels run unchanged on a window, with window row numbers as sample ids.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "aqsgd.h"

struct aqsgd_tier {
    char* host_rows;
    char* dev_rows;
    int64_t* dev_row_ids;
    int64_t n_samples, row_bytes;
    int32_t slots, batch;
    std::vector<int64_t> held;          // [slots * batch] sample id of each window row, -1 = empty
    std::vector<hipEvent_t> ready;      // per window: rows have arrived (recorded on the copy stream)
    std::vector<hipEvent_t> updated;    // per window: codec work is queued/done (compute stream)
    hipEvent_t all_copies;              // last copy issued
    bool copies_pending;
};

namespace {
bool ok(hipError_t e) { return e == hipSuccess; }
}

extern "C" {

int aqsgd_tier_create(aqsgd_tier** out, void* host_rows, void* dev_rows, int64_t* dev_row_ids,
                      int64_t n_samples, int64_t row_bytes, int32_t slots, int32_t batch) {
    if (!out || !host_rows || !dev_rows || !dev_row_ids) return AQSGD_ERR_NULL;
    if (n_samples <= 0 || row_bytes <= 0 || slots <= 0 || batch <= 0) return AQSGD_ERR_SHAPE;
    aqsgd_tier* t = new (std::nothrow) aqsgd_tier;
    if (!t) return AQSGD_ERR_LAUNCH;
    t->host_rows = static_cast<char*>(host_rows);
    t->dev_rows = static_cast<char*>(dev_rows);
    t->dev_row_ids = dev_row_ids;
    t->n_samples = n_samples; t->row_bytes = row_bytes; t->slots = slots; t->batch = batch;
    t->held.assign(static_cast<size_t>(slots) * batch, -1);
    t->copies_pending = false;
    std::vector<int64_t> ids(static_cast<size_t>(slots) * batch);
    for (size_t i = 0; i < ids.size(); ++i) ids[i] = static_cast<int64_t>(i);
    bool good = ok(hipMemcpy(dev_row_ids, ids.data(), ids.size() * sizeof(int64_t), hipMemcpyHostToDevice));
    t->ready.resize(slots); t->updated.resize(slots);
    for (int s = 0; s < slots && good; ++s)
        good = ok(hipEventCreateWithFlags(&t->ready[s], hipEventDisableTiming)) &&
               ok(hipEventCreateWithFlags(&t->updated[s], hipEventDisableTiming));
    good = good && ok(hipEventCreateWithFlags(&t->all_copies, hipEventDisableTiming));
    if (!good) { delete t; return AQSGD_ERR_LAUNCH; }
    *out = t;
    return AQSGD_OK;
}

int aqsgd_tier_prefetch(aqsgd_tier* t, int32_t slot, const int64_t* host_ids, void* copy_stream) {
    if (!t || !host_ids) return AQSGD_ERR_NULL;
    if (slot < 0 || slot >= t->slots) return AQSGD_ERR_SHAPE;
    for (int i = 0; i < t->batch; ++i) {
        if (host_ids[i] < 0 || host_ids[i] >= t->n_samples) return AQSGD_ERR_SHAPE;
        if (t->held[static_cast<size_t>(slot) * t->batch + i] != -1) return AQSGD_ERR_SHAPE;   // not released
        // a sample that sits in a window (this call's or an unreleased one) has a newer row
        // there than in host memory: loading it again would fork it
        for (int64_t h : t->held)
            if (h == host_ids[i]) return AQSGD_ERR_SHAPE;
        for (int j = 0; j < i; ++j)
            if (host_ids[j] == host_ids[i]) return AQSGD_ERR_SHAPE;
    }
    hipStream_t cs = static_cast<hipStream_t>(copy_stream);
    for (int i = 0; i < t->batch; ++i) {
        const size_t row = static_cast<size_t>(slot) * t->batch + i;
        if (!ok(hipMemcpyAsync(t->dev_rows + row * t->row_bytes, t->host_rows + host_ids[i] * t->row_bytes,
                               static_cast<size_t>(t->row_bytes), hipMemcpyHostToDevice, cs)))
            return AQSGD_ERR_LAUNCH;
        t->held[row] = host_ids[i];
    }
    if (!ok(hipEventRecord(t->ready[slot], cs)) || !ok(hipEventRecord(t->all_copies, cs)))
        return AQSGD_ERR_LAUNCH;
    t->copies_pending = true;
    return AQSGD_OK;
}

int aqsgd_tier_acquire(aqsgd_tier* t, int32_t slot, void* compute_stream, const int64_t** sample_ids) {
    if (!t || !sample_ids) return AQSGD_ERR_NULL;
    if (slot < 0 || slot >= t->slots) return AQSGD_ERR_SHAPE;
    if (t->held[static_cast<size_t>(slot) * t->batch] == -1) return AQSGD_ERR_SHAPE;          // nothing prefetched
    if (!ok(hipStreamWaitEvent(static_cast<hipStream_t>(compute_stream), t->ready[slot], 0)))
        return AQSGD_ERR_LAUNCH;
    *sample_ids = t->dev_row_ids + static_cast<size_t>(slot) * t->batch;
    return AQSGD_OK;
}

int aqsgd_tier_release(aqsgd_tier* t, int32_t slot, void* compute_stream, void* copy_stream) {
    if (!t) return AQSGD_ERR_NULL;
    if (slot < 0 || slot >= t->slots) return AQSGD_ERR_SHAPE;
    if (t->held[static_cast<size_t>(slot) * t->batch] == -1) return AQSGD_ERR_SHAPE;
    hipStream_t cs = static_cast<hipStream_t>(copy_stream);
    if (!ok(hipEventRecord(t->updated[slot], static_cast<hipStream_t>(compute_stream))) ||
        !ok(hipStreamWaitEvent(cs, t->updated[slot], 0)))
        return AQSGD_ERR_LAUNCH;
    for (int i = 0; i < t->batch; ++i) {
        const size_t row = static_cast<size_t>(slot) * t->batch + i;
        if (!ok(hipMemcpyAsync(t->host_rows + t->held[row] * t->row_bytes, t->dev_rows + row * t->row_bytes,
                               static_cast<size_t>(t->row_bytes), hipMemcpyDeviceToHost, cs)))
            return AQSGD_ERR_LAUNCH;
        t->held[row] = -1;
    }
    if (!ok(hipEventRecord(t->all_copies, cs))) return AQSGD_ERR_LAUNCH;
    t->copies_pending = true;
    return AQSGD_OK;
}

int aqsgd_tier_drain(aqsgd_tier* t) {
    if (!t) return AQSGD_ERR_NULL;
    if (t->copies_pending && !ok(hipEventSynchronize(t->all_copies))) return AQSGD_ERR_LAUNCH;
    t->copies_pending = false;
    return AQSGD_OK;
}

void aqsgd_tier_destroy(aqsgd_tier* t) {
    if (!t) return;
    aqsgd_tier_drain(t);
    for (hipEvent_t e : t->ready) (void)hipEventDestroy(e);
    for (hipEvent_t e : t->updated) (void)hipEventDestroy(e);
    (void)hipEventDestroy(t->all_copies);
    delete t;
}

}  // extern "C"
