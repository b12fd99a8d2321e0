// bmgd_reader: the first of the two transfers of Section 2.1, storage -> host memory, as a host thread that keeps a
// ring of pinned buffers filled from a pair of flat files, so that the second transfer (host -> device, the "buffering
// step" of Algorithm 1) always finds its next buffer in memory.  Host code only; no kernel lives here.
#include "../../include/bmgd.h"
#include "bmgd_internal.h"

#include <hip/hip_runtime.h>

#include <errno.h>
#include <fcntl.h>
#include <string.h>
#include <sys/stat.h>
#include <unistd.h>

#include <chrono>
#include <condition_variable>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

namespace {

enum SlotState { kFree = 0, kFilling = 1, kReady = 2, kHandedOut = 3 };

struct RingSlot {
    void* x = nullptr;
    void* y = nullptr;
    int64_t rows = 0;
    int state = kFree;
    hipEvent_t copied = nullptr;        // completes when the last host -> device copy out of this slot has
    bool wait_copy = false;             // whether `copied` has been recorded since the slot was handed out
};

thread_local std::string g_open_error;

}  // namespace

struct bmgd_reader {
    int fd_x = -1, fd_y = -1;
    int device = 0;
    int64_t p = 0, n_rows = 0, buffer_n = 0, n_buffers = 0;
    size_t x_item = 4;
    bool loop = false;
    std::vector<RingSlot> ring;
    std::thread worker;
    std::mutex mu;
    std::condition_variable cv;
    size_t fill = 0, take = 0, give = 0;    // next slot to fill / to hand out / to take back (all in ring order)
    int64_t next_buffer = 0;                // file position of the next fill, in buffers
    bool eof = false, stop = false, failed = false;
    std::string err, err_out;              // err_out: the copy bmgd_reader_last_error hands out
    int64_t bytes_read = 0;
    double read_seconds = 0.0;
};

namespace {

int open_fail(const std::string& msg)
{
    g_open_error = msg;
    return BMGD_EINVAL;
}

// pread until `bytes` bytes have arrived; false on error or a short file.
bool read_fully(int fd, void* dst, size_t bytes, off_t offset, std::string* why)
{
    char* out = static_cast<char*>(dst);
    while (bytes > 0) {
        const ssize_t got = pread(fd, out, bytes, offset);
        if (got < 0) {
            if (errno == EINTR) continue;
            *why = std::string("pread: ") + strerror(errno);
            return false;
        }
        if (got == 0) {
            *why = "file is shorter than n_rows rows";
            return false;
        }
        out += got;
        offset += got;
        bytes -= (size_t)got;
    }
    return true;
}

void worker_main(bmgd_reader* r)
{
    (void)hipSetDevice(r->device);
    for (;;) {
        RingSlot* slot = nullptr;
        int64_t k = 0;
        {
            std::unique_lock<std::mutex> lk(r->mu);
            r->cv.wait(lk, [&] { return r->stop || r->ring[r->fill].state == kFree; });
            if (r->stop) return;
            if (!r->loop && r->next_buffer >= r->n_buffers) {
                r->eof = true;
                r->cv.notify_all();
                return;
            }
            slot = &r->ring[r->fill];
            slot->state = kFilling;
            k = r->next_buffer % r->n_buffers;
            r->next_buffer += 1;
        }
        // the copy that last read this slot must have finished before the slot is overwritten
        if (slot->wait_copy) {
            (void)hipEventSynchronize(slot->copied);
            slot->wait_copy = false;
        }
        const int64_t row0 = k * r->buffer_n;
        const int64_t rows = std::min<int64_t>(r->buffer_n, r->n_rows - row0);
        const size_t xb = (size_t)rows * (size_t)r->p * r->x_item, yb = (size_t)rows * 4;
        std::string why;
        const auto t0 = std::chrono::steady_clock::now();
        const bool ok = read_fully(r->fd_x, slot->x, xb, (off_t)((size_t)row0 * (size_t)r->p * r->x_item), &why) &&
                        read_fully(r->fd_y, slot->y, yb, (off_t)((size_t)row0 * 4), &why);
        const double dt = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
        {
            std::lock_guard<std::mutex> lk(r->mu);
            if (!ok) {
                r->failed = true;
                r->err = why;
                r->cv.notify_all();
                return;
            }
            slot->rows = rows;
            slot->state = kReady;
            r->fill = (r->fill + 1) % r->ring.size();
            r->bytes_read += (int64_t)(xb + yb);
            r->read_seconds += dt;
        }
        r->cv.notify_all();
    }
}

void destroy_reader(bmgd_reader* r)
{
    if (!r) return;
    {
        std::lock_guard<std::mutex> lk(r->mu);
        r->stop = true;
    }
    r->cv.notify_all();
    if (r->worker.joinable()) r->worker.join();
    (void)hipSetDevice(r->device);
    for (RingSlot& s : r->ring) {
        if (s.wait_copy) (void)hipEventSynchronize(s.copied);
        if (s.copied) (void)hipEventDestroy(s.copied);
        if (s.x) (void)hipHostFree(s.x);
        if (s.y) (void)hipHostFree(s.y);
    }
    if (r->fd_x >= 0) close(r->fd_x);
    if (r->fd_y >= 0) close(r->fd_y);
    delete r;
}

}  // namespace

int reader_take(bmgd_reader* r, bool block, const void** x, const void** y, int64_t* rows, int* end)
{
    *x = *y = nullptr;
    *rows = 0;
    *end = 0;
    std::unique_lock<std::mutex> lk(r->mu);
    if (r->ring[r->take].state == kHandedOut) {
        r->err = "every slot of the ring is handed out: release one first";
        return BMGD_ESTATE;
    }
    auto settled = [&] { return r->failed || r->ring[r->take].state == kReady || (r->eof && r->ring[r->take].state == kFree); };
    if (block) r->cv.wait(lk, settled);
    else if (!settled()) return BMGD_OK;                  // still reading
    if (r->ring[r->take].state != kReady) {
        if (r->failed) return BMGD_EINVAL;                // message in r->err
        *end = 1;
        return BMGD_OK;
    }
    RingSlot& s = r->ring[r->take];
    s.state = kHandedOut;
    r->take = (r->take + 1) % r->ring.size();
    *x = s.x;
    *y = s.y;
    *rows = s.rows;
    return BMGD_OK;
}

#define BMGD_API __attribute__((visibility("default")))

extern "C" {

BMGD_API int bmgd_reader_open(const char* x_path, const char* y_path, int64_t p, int32_t x_dtype, int64_t n_rows, int64_t buffer_n,
                              int32_t ring_slots, int32_t loop, bmgd_reader** out)
{
    if (!out) return open_fail("out must not be NULL");
    *out = nullptr;
    if (!x_path || !y_path) return open_fail("x_path and y_path must not be NULL");
    if (p < 1 || n_rows < 1 || buffer_n < 1 || buffer_n >= (int64_t(1) << 30)) return open_fail("p, n_rows, buffer_n must be positive (buffer_n < 2^30)");
    if (x_dtype != BMGD_F32 && x_dtype != BMGD_BF16) return open_fail("x_dtype must be BMGD_F32 or BMGD_BF16");
    if (ring_slots < 2 || ring_slots > 64) return open_fail("ring_slots must be in [2, 64]");
    bmgd_reader* r = new (std::nothrow) bmgd_reader();
    if (!r) {
        g_open_error = "out of host memory";
        return BMGD_ENOMEM;
    }
    r->p = p; r->n_rows = n_rows; r->buffer_n = std::min(buffer_n, n_rows);
    r->n_buffers = (n_rows + r->buffer_n - 1) / r->buffer_n;
    r->x_item = x_dtype == BMGD_BF16 ? 2 : 4;
    r->loop = loop != 0;
    r->fd_x = open(x_path, O_RDONLY | O_CLOEXEC);
    r->fd_y = open(y_path, O_RDONLY | O_CLOEXEC);
    if (r->fd_x < 0 || r->fd_y < 0) {
        const std::string msg = std::string("cannot open ") + (r->fd_x < 0 ? x_path : y_path) + ": " + strerror(errno);
        destroy_reader(r);
        return open_fail(msg);
    }
    struct stat sx, sy;
    if (fstat(r->fd_x, &sx) != 0 || fstat(r->fd_y, &sy) != 0 || (uint64_t)sx.st_size < (uint64_t)n_rows * (uint64_t)p * r->x_item ||
        (uint64_t)sy.st_size < (uint64_t)n_rows * 4) {
        destroy_reader(r);
        return open_fail("a file is shorter than n_rows rows");
    }
    if (hipGetDevice(&r->device) != hipSuccess) {
        (void)hipGetLastError();
        destroy_reader(r);
        g_open_error = "no usable GPU (pinned memory comes from the HIP runtime)";
        return BMGD_EHIP;
    }
    r->ring.resize((size_t)ring_slots);
    for (RingSlot& s : r->ring) {
        const hipError_t e1 = hipHostMalloc(&s.x, (size_t)r->buffer_n * (size_t)p * r->x_item, hipHostMallocDefault);
        const hipError_t e2 = e1 == hipSuccess ? hipHostMalloc(&s.y, (size_t)r->buffer_n * 4, hipHostMallocDefault) : e1;
        const hipError_t e3 = e2 == hipSuccess ? hipEventCreateWithFlags(&s.copied, hipEventDisableTiming) : e2;
        if (e3 != hipSuccess) {
            (void)hipGetLastError();
            g_open_error = std::string("pinned ring: ") + hipGetErrorString(e3);
            destroy_reader(r);
            return e3 == hipErrorOutOfMemory ? BMGD_ENOMEM : BMGD_EHIP;
        }
    }
    r->worker = std::thread(worker_main, r);
    *out = r;
    return BMGD_OK;
}

BMGD_API int bmgd_reader_acquire(bmgd_reader* r, const void** host_x, const void** host_y, int64_t* rows)
{
    if (!r || !host_x || !host_y || !rows) return BMGD_EINVAL;
    int end = 0;
    return reader_take(r, true, host_x, host_y, rows, &end);
}

BMGD_API int bmgd_reader_release(bmgd_reader* r, void* copy_stream, int32_t after_stream)
{
    if (!r) return BMGD_EINVAL;
    RingSlot* s = nullptr;
    {
        std::lock_guard<std::mutex> lk(r->mu);
        if (r->ring[r->give].state != kHandedOut) {
            r->err = "no slot is handed out";
            return BMGD_ESTATE;
        }
        s = &r->ring[r->give];
    }
    if (after_stream) {
        // the slot may be refilled once everything enqueued on copy_stream so far has completed
        if (hipSetDevice(r->device) != hipSuccess || hipEventRecord(s->copied, static_cast<hipStream_t>(copy_stream)) != hipSuccess) {
            (void)hipGetLastError();
            std::lock_guard<std::mutex> lk(r->mu);
            r->err = "hipEventRecord failed";
            return BMGD_EHIP;
        }
    }
    {
        std::lock_guard<std::mutex> lk(r->mu);
        s->wait_copy = after_stream != 0;
        s->state = kFree;
        r->give = (r->give + 1) % r->ring.size();
    }
    r->cv.notify_all();
    return BMGD_OK;
}

BMGD_API int bmgd_load_from_reader(bmgd_ctx* ctx, bmgd_reader* r, void* copy_stream, int64_t* rows_out)
{
    if (!ctx || !r || !rows_out) return BMGD_EINVAL;
    const void *x = nullptr, *y = nullptr;
    int64_t rows = 0;
    int rc = bmgd_reader_acquire(r, &x, &y, &rows);
    *rows_out = rows;
    if (rc != BMGD_OK || rows == 0) return rc;
    rc = bmgd_load_buffer_async(ctx, x, y, rows, copy_stream);
    // handed back either way; after a successful load the refill waits for the copy
    const int rc2 = bmgd_reader_release(r, copy_stream, rc == BMGD_OK);
    return rc != BMGD_OK ? rc : rc2;
}

BMGD_API int bmgd_reader_stats(bmgd_reader* r, int64_t* bytes_read, double* read_seconds)
{
    if (!r) return BMGD_EINVAL;
    std::lock_guard<std::mutex> lk(r->mu);
    if (bytes_read) *bytes_read = r->bytes_read;
    if (read_seconds) *read_seconds = r->read_seconds;
    return BMGD_OK;
}

BMGD_API const char* bmgd_reader_last_error(bmgd_reader* r)
{
    if (!r) return g_open_error.c_str();
    std::lock_guard<std::mutex> lk(r->mu);
    r->err_out = r->err;
    return r->err_out.c_str();
}

BMGD_API void bmgd_reader_close(bmgd_reader* r) { destroy_reader(r); }

}  // extern "C"
