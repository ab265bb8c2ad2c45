// Tiers below HBM for the previous messages (Section 3.3 and Appendix G of the paper:
// m(xi) lives in host memory or on an SSD, is brought to the GPU before the forward
// pass of its sample and goes back after the update, both behind the computation of
// other samples).  Host code only: the codec kernels run unchanged on a window of
// rows in HBM, with window row numbers as sample ids.
//
//   host tier   all rows in pinned host memory; a window is filled and written back by
//               asynchronous copies on a copy stream, ordered against the compute
//               stream with events.
//   file tier   all rows in a file; pinned host memory holds only one staging row per
//               window row.  A worker thread reads a window's rows from the file into
//               the staging rows and then issues the copy to the device (read-ahead,
//               as far ahead as there are windows), and writes rows back to the file
//               once their copy from the device has finished (write-behind).  The
//               worker takes its tasks in the order they were issued, which is what
//               orders a write-back before a later read of the same sample or window.
#include <hip/hip_runtime.h>

#include <fcntl.h>
#include <sys/stat.h>
#include <unistd.h>

#include <cstdlib>
#include <cstring>

#include <condition_variable>
#include <deque>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "aqsgd.h"

namespace {

bool ok(hipError_t e) { return e == hipSuccess; }

struct Task {
    bool read;                          // read-ahead of a window, else write-behind
    int32_t slot;
    std::vector<int64_t> ids;           // the window's samples
};

}  // namespace

struct aqsgd_tier {
    char* host_rows;                    // host tier: [n_samples, row_bytes]; file tier: [slots*batch, row_bytes]
    char* dev_rows;
    int64_t* dev_row_ids;
    int64_t n_samples, row_bytes;
    int32_t slots, batch;
    std::vector<int64_t> held;          // [slots * batch] sample id of each window row, -1 = empty
    std::vector<hipEvent_t> ready;      // per window: rows have arrived (recorded on the copy stream)
    std::vector<hipEvent_t> updated;    // per window: codec work is queued/done (compute stream)
    std::vector<hipEvent_t> staged;     // file tier, per window: rows are back in the staging rows
    hipEvent_t all_copies;              // last copy issued
    bool all_copies_made;
    bool copies_pending;
    bool copy_stream_known;
    hipStream_t copy_stream;            // the one copy stream of this tier (fixed by its first use)

    // file tier
    int fd;                             // -1: host tier
    int device;
    std::thread worker;
    std::mutex mu;
    std::condition_variable cv;
    std::deque<Task> tasks;
    std::vector<int> issued;            // per window: its read-ahead has issued the copy and the event
    bool busy, stop;
    int failed;                         // sticky status of the worker (AQSGD_OK or an error)
    char* bounce;                       // unbuffered file: one window of 4 KiB-aligned ordinary memory (the
                                        // kernel cannot do direct I/O into pinned GPU-visible pages), else null
};

namespace {

void destroy_events(aqsgd_tier* t) {
    for (hipEvent_t e : t->ready) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : t->updated) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : t->staged) if (e) (void)hipEventDestroy(e);
    if (t->all_copies_made) (void)hipEventDestroy(t->all_copies);
}

bool full_io(bool write, int fd, char* buf, int64_t bytes, int64_t offset) {
    while (bytes > 0) {
        const ssize_t n = write ? pwrite(fd, buf, static_cast<size_t>(bytes), offset)
                                : pread(fd, buf, static_cast<size_t>(bytes), offset);
        if (n <= 0) return false;
        buf += n; offset += n; bytes -= n;
    }
    return true;
}

void worker_loop(aqsgd_tier* t) {
    (void)hipSetDevice(t->device);
    for (;;) {
        Task task;
        {
            std::unique_lock<std::mutex> lock(t->mu);
            t->cv.wait(lock, [t] { return t->stop || !t->tasks.empty(); });
            if (t->tasks.empty()) return;                // stop, and nothing left to do
            task = std::move(t->tasks.front());
            t->tasks.pop_front();
            t->busy = true;
        }
        int status = AQSGD_OK;
        char* window = t->host_rows + static_cast<int64_t>(task.slot) * t->batch * t->row_bytes;
        char* io = t->bounce ? t->bounce : window;       // where the file transfers land / start
        const size_t window_bytes = static_cast<size_t>(t->batch) * t->row_bytes;
        if (task.read) {
            for (int i = 0; i < t->batch && status == AQSGD_OK; ++i)
                if (!full_io(false, t->fd, io + i * t->row_bytes, t->row_bytes, task.ids[i] * t->row_bytes))
                    status = AQSGD_ERR_IO;
            if (status == AQSGD_OK && t->bounce) memcpy(window, t->bounce, window_bytes);
            // staging rows and window rows are both contiguous: one copy fills the window
            if (status == AQSGD_OK &&
                (!ok(hipMemcpyAsync(t->dev_rows + static_cast<int64_t>(task.slot) * t->batch * t->row_bytes, window,
                                    static_cast<size_t>(t->batch) * t->row_bytes, hipMemcpyHostToDevice,
                                    t->copy_stream)) ||
                 !ok(hipEventRecord(t->ready[task.slot], t->copy_stream))))
                status = AQSGD_ERR_LAUNCH;
        } else {
            if (!ok(hipEventSynchronize(t->staged[task.slot]))) status = AQSGD_ERR_LAUNCH;
            if (status == AQSGD_OK && t->bounce) memcpy(t->bounce, window, window_bytes);
            for (int i = 0; i < t->batch && status == AQSGD_OK; ++i)
                if (!full_io(true, t->fd, io + i * t->row_bytes, t->row_bytes, task.ids[i] * t->row_bytes))
                    status = AQSGD_ERR_IO;
        }
        {
            std::lock_guard<std::mutex> lock(t->mu);
            if (status != AQSGD_OK && t->failed == AQSGD_OK) t->failed = status;
            if (task.read) t->issued[task.slot] = 1;
            t->busy = false;
        }
        t->cv.notify_all();
    }
}

int check_ids_for_prefetch(const aqsgd_tier* t, int32_t slot, const int64_t* host_ids) {
    for (int i = 0; i < t->batch; ++i) {
        if (host_ids[i] < 0 || host_ids[i] >= t->n_samples) return AQSGD_ERR_SHAPE;
        if (t->held[static_cast<size_t>(slot) * t->batch + i] != -1) return AQSGD_ERR_SHAPE;   // not released
        // a sample that sits in an unreleased window has a newer row there than below:
        // loading it again would fork it
        for (int64_t h : t->held)
            if (h == host_ids[i]) return AQSGD_ERR_SHAPE;
        for (int j = 0; j < i; ++j)
            if (host_ids[j] == host_ids[i]) return AQSGD_ERR_SHAPE;
    }
    return AQSGD_OK;
}

// Every call of one tier names the same copy stream: the order of its copies is what
// keeps a write-back ahead of a later prefetch of the same window or sample.
int fix_copy_stream(aqsgd_tier* t, void* copy_stream) {
    hipStream_t cs = static_cast<hipStream_t>(copy_stream);
    if (!t->copy_stream_known) {
        t->copy_stream = cs;
        t->copy_stream_known = true;
    }
    return t->copy_stream == cs ? AQSGD_OK : AQSGD_ERR_SHAPE;
}

int create_common(aqsgd_tier** out, void* host_rows, void* dev_rows, int64_t* dev_row_ids, int64_t n_samples,
                  int64_t row_bytes, int32_t slots, int32_t batch, int fd, bool direct_io) {
    aqsgd_tier* t = new (std::nothrow) aqsgd_tier;
    if (!t) return AQSGD_ERR_LAUNCH;
    t->bounce = nullptr;
    if (direct_io) {
        void* p = nullptr;
        if (posix_memalign(&p, 4096, static_cast<size_t>(batch) * row_bytes) != 0) { delete t; return AQSGD_ERR_IO; }
        t->bounce = static_cast<char*>(p);
    }
    t->host_rows = static_cast<char*>(host_rows);
    t->dev_rows = static_cast<char*>(dev_rows);
    t->dev_row_ids = dev_row_ids;
    t->n_samples = n_samples; t->row_bytes = row_bytes; t->slots = slots; t->batch = batch;
    t->held.assign(static_cast<size_t>(slots) * batch, -1);
    t->copies_pending = false; t->all_copies_made = false; t->copy_stream_known = false;
    t->copy_stream = nullptr;
    t->fd = fd; t->busy = false; t->stop = false; t->failed = AQSGD_OK;
    t->issued.assign(slots, 0);
    std::vector<int64_t> ids(static_cast<size_t>(slots) * batch);
    for (size_t i = 0; i < ids.size(); ++i) ids[i] = static_cast<int64_t>(i);
    bool good = ok(hipGetDevice(&t->device)) &&
                ok(hipMemcpy(dev_row_ids, ids.data(), ids.size() * sizeof(int64_t), hipMemcpyHostToDevice));
    t->ready.assign(slots, nullptr); t->updated.assign(slots, nullptr);
    t->staged.assign(fd >= 0 ? slots : 0, nullptr);
    for (int s = 0; s < slots && good; ++s) {
        good = ok(hipEventCreateWithFlags(&t->ready[s], hipEventDisableTiming)) &&
               ok(hipEventCreateWithFlags(&t->updated[s], hipEventDisableTiming));
        if (good && fd >= 0) good = ok(hipEventCreateWithFlags(&t->staged[s], hipEventDisableTiming));
    }
    if (good) {
        good = ok(hipEventCreateWithFlags(&t->all_copies, hipEventDisableTiming));
        t->all_copies_made = good;
    }
    if (!good) {
        destroy_events(t);
        free(t->bounce);
        delete t;
        return AQSGD_ERR_LAUNCH;
    }
    if (fd >= 0) t->worker = std::thread(worker_loop, t);
    *out = t;
    return AQSGD_OK;
}

}  // namespace

extern "C" {

int aqsgd_tier_create(aqsgd_tier** out, void* host_rows, void* dev_rows, int64_t* dev_row_ids,
                      int64_t n_samples, int64_t row_bytes, int32_t slots, int32_t batch) {
    if (!out || !host_rows || !dev_rows || !dev_row_ids) return AQSGD_ERR_NULL;
    if (n_samples <= 0 || row_bytes <= 0 || slots <= 0 || batch <= 0) return AQSGD_ERR_SHAPE;
    return create_common(out, host_rows, dev_rows, dev_row_ids, n_samples, row_bytes, slots, batch, -1, false);
}

int aqsgd_tier_create_file(aqsgd_tier** out, const char* path, int32_t direct_io, void* staging_rows,
                           void* dev_rows, int64_t* dev_row_ids, int64_t n_samples, int64_t row_bytes,
                           int32_t slots, int32_t batch) {
    if (!out || !path || !staging_rows || !dev_rows || !dev_row_ids) return AQSGD_ERR_NULL;
    if (n_samples <= 0 || row_bytes <= 0 || slots <= 0 || batch <= 0) return AQSGD_ERR_SHAPE;
    int flags = O_RDWR | O_CREAT;
    if (direct_io) {                                     // unbuffered: rows must be whole 4 KiB blocks
        if (row_bytes % 4096 != 0) return AQSGD_ERR_ALIGN;
        flags |= O_DIRECT;
    }
    const int fd = open(path, flags, 0600);
    if (fd < 0) return AQSGD_ERR_IO;
    // rows never written read as zeros: Algorithm 1's initial m
    if (ftruncate(fd, static_cast<off_t>(n_samples * row_bytes)) != 0) { close(fd); return AQSGD_ERR_IO; }
    const int rc = create_common(out, staging_rows, dev_rows, dev_row_ids, n_samples, row_bytes, slots, batch, fd,
                                 direct_io != 0);
    if (rc != AQSGD_OK) close(fd);
    return rc;
}

int aqsgd_tier_prefetch(aqsgd_tier* t, int32_t slot, const int64_t* host_ids, void* copy_stream) {
    if (!t || !host_ids) return AQSGD_ERR_NULL;
    if (slot < 0 || slot >= t->slots) return AQSGD_ERR_SHAPE;
    int rc = check_ids_for_prefetch(t, slot, host_ids);
    if (rc == AQSGD_OK) rc = fix_copy_stream(t, copy_stream);
    if (rc != AQSGD_OK) return rc;
    const size_t row0 = static_cast<size_t>(slot) * t->batch;
    if (t->fd >= 0) {
        Task task;
        task.read = true; task.slot = slot; task.ids.assign(host_ids, host_ids + t->batch);
        {
            std::lock_guard<std::mutex> lock(t->mu);
            if (t->failed != AQSGD_OK) return t->failed;
            t->issued[slot] = 0;
            t->tasks.push_back(std::move(task));
        }
        t->cv.notify_all();
        for (int i = 0; i < t->batch; ++i) t->held[row0 + i] = host_ids[i];
        t->copies_pending = true;
        return AQSGD_OK;
    }
    hipStream_t cs = t->copy_stream;
    for (int i = 0; i < t->batch; ++i) {
        if (!ok(hipMemcpyAsync(t->dev_rows + (row0 + i) * t->row_bytes, t->host_rows + host_ids[i] * t->row_bytes,
                               static_cast<size_t>(t->row_bytes), hipMemcpyHostToDevice, cs))) {
            for (int j = 0; j < i; ++j) t->held[row0 + j] = -1;      // the window stays empty
            return AQSGD_ERR_LAUNCH;
        }
        t->held[row0 + i] = host_ids[i];
    }
    if (!ok(hipEventRecord(t->ready[slot], cs)) || !ok(hipEventRecord(t->all_copies, cs))) {
        for (int i = 0; i < t->batch; ++i) t->held[row0 + i] = -1;
        return AQSGD_ERR_LAUNCH;
    }
    t->copies_pending = true;
    return AQSGD_OK;
}

int aqsgd_tier_acquire(aqsgd_tier* t, int32_t slot, void* compute_stream, const int64_t** sample_ids) {
    if (!t || !sample_ids) return AQSGD_ERR_NULL;
    if (slot < 0 || slot >= t->slots) return AQSGD_ERR_SHAPE;
    if (t->held[static_cast<size_t>(slot) * t->batch] == -1) return AQSGD_ERR_SHAPE;          // nothing prefetched
    if (t->fd >= 0) {       // the event exists once the worker has read the rows and issued their copy
        std::unique_lock<std::mutex> lock(t->mu);
        t->cv.wait(lock, [t, slot] { return t->issued[slot] != 0 || t->failed != AQSGD_OK; });
        if (t->failed != AQSGD_OK) return t->failed;
    }
    if (!ok(hipStreamWaitEvent(static_cast<hipStream_t>(compute_stream), t->ready[slot], 0)))
        return AQSGD_ERR_LAUNCH;
    *sample_ids = t->dev_row_ids + static_cast<size_t>(slot) * t->batch;
    return AQSGD_OK;
}

int aqsgd_tier_release(aqsgd_tier* t, int32_t slot, void* compute_stream, void* copy_stream) {
    if (!t) return AQSGD_ERR_NULL;
    if (slot < 0 || slot >= t->slots) return AQSGD_ERR_SHAPE;
    const size_t row0 = static_cast<size_t>(slot) * t->batch;
    if (t->held[row0] == -1) return AQSGD_ERR_SHAPE;
    const int rc = fix_copy_stream(t, copy_stream);
    if (rc != AQSGD_OK) return rc;
    hipStream_t cs = t->copy_stream;
    if (t->fd >= 0) {       // the read-ahead must have issued its copy before the write-back is queued behind it
        std::unique_lock<std::mutex> lock(t->mu);
        t->cv.wait(lock, [t, slot] { return t->issued[slot] != 0 || t->failed != AQSGD_OK; });
        if (t->failed != AQSGD_OK) return t->failed;
    }
    if (!ok(hipEventRecord(t->updated[slot], static_cast<hipStream_t>(compute_stream))) ||
        !ok(hipStreamWaitEvent(cs, t->updated[slot], 0)))
        return AQSGD_ERR_LAUNCH;
    if (t->fd >= 0) {
        char* window = t->host_rows + row0 * t->row_bytes;
        if (!ok(hipMemcpyAsync(window, t->dev_rows + row0 * t->row_bytes, static_cast<size_t>(t->batch) * t->row_bytes,
                               hipMemcpyDeviceToHost, cs)) ||
            !ok(hipEventRecord(t->staged[slot], cs)))
            return AQSGD_ERR_LAUNCH;
        Task task;
        task.read = false; task.slot = slot;
        task.ids.assign(t->held.begin() + static_cast<int64_t>(row0), t->held.begin() + static_cast<int64_t>(row0) + t->batch);
        {
            std::lock_guard<std::mutex> lock(t->mu);
            t->tasks.push_back(std::move(task));
        }
        t->cv.notify_all();
        for (int i = 0; i < t->batch; ++i) t->held[row0 + i] = -1;
        t->copies_pending = true;
        return AQSGD_OK;
    }
    for (int i = 0; i < t->batch; ++i) {
        if (!ok(hipMemcpyAsync(t->host_rows + t->held[row0 + i] * t->row_bytes, t->dev_rows + (row0 + i) * t->row_bytes,
                               static_cast<size_t>(t->row_bytes), hipMemcpyDeviceToHost, cs)))
            return AQSGD_ERR_LAUNCH;                     // rows not yet copied stay held: release again
        t->held[row0 + i] = -1;
    }
    if (!ok(hipEventRecord(t->all_copies, cs))) return AQSGD_ERR_LAUNCH;
    t->copies_pending = true;
    return AQSGD_OK;
}

int aqsgd_tier_drain(aqsgd_tier* t) {
    if (!t) return AQSGD_ERR_NULL;
    if (t->fd >= 0) {
        std::unique_lock<std::mutex> lock(t->mu);
        t->cv.wait(lock, [t] { return (t->tasks.empty() && !t->busy) || t->failed != AQSGD_OK; });
        if (t->failed != AQSGD_OK) return t->failed;
        lock.unlock();
        // the last window copies to the device may still be in flight
        if (t->copy_stream_known && !ok(hipStreamSynchronize(t->copy_stream))) return AQSGD_ERR_LAUNCH;
        t->copies_pending = false;
        return AQSGD_OK;
    }
    if (t->copies_pending && !ok(hipEventSynchronize(t->all_copies))) return AQSGD_ERR_LAUNCH;
    t->copies_pending = false;
    return AQSGD_OK;
}

void aqsgd_tier_destroy(aqsgd_tier* t) {
    if (!t) return;
    (void)aqsgd_tier_drain(t);
    if (t->fd >= 0) {
        {
            std::lock_guard<std::mutex> lock(t->mu);
            t->stop = true;
            if (t->failed != AQSGD_OK) t->tasks.clear();
        }
        t->cv.notify_all();
        if (t->worker.joinable()) t->worker.join();
        (void)fsync(t->fd);
        close(t->fd);
    }
    destroy_events(t);
    free(t->bounce);
    delete t;
}

}  // extern "C"
