// History tables kept in a file (the paper's "Conclusion and Future Work" names histories read from disk storage as
// the way past the host-memory limit; its Section 5 "PyGAS" describes the transfer scheme this follows: a worker
// gathers rows into pinned buffers, copies run beside the computation, and a layer waits only for its own rows).
//
// A gas_disk_table is a raw row-major file of n_rows x F elements plus
//   * I/O threads (one pool for all tables of the process; a table uses as many of them as it was opened with, one
//     table's burst at a time) that move rows between the file and a buffer: through a shared mapping of the file (plain
//     copies into and out of the page cache: no system call and no file lock per row, which scattered 1 KiB rows
//     need), or, on request, with pread / pwrite, runs of consecutive rows in one call (errors then come back as
//     status codes instead of signals),
//   * two pinned staging buffers, so that the file I/O of one piece overlaps with the DMA copy of the piece before,
//   * one worker thread that takes the table's jobs in the order they were queued (a pull queued after a push to the
//     same table therefore sees the pushed rows, as Algorithm 1 needs) and a copy stream at the default priority.
// Host code only: the rows cross the host link as plain asynchronous copies, no kernel is launched here.
#include <errno.h>
#include <fcntl.h>
#include <string.h>
#include <sys/mman.h>
#include <sys/stat.h>
#include <sys/types.h>
#include <unistd.h>

#include <algorithm>
#include <condition_variable>
#include <deque>
#include <functional>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "common.h"

namespace {

// n_threads workers that run one range function at a time over [0, n) in `parts` equal parts (the caller takes part 0).
class IoPool {
public:
    explicit IoPool(int n_threads) : n_(std::max(1, n_threads)) {
        for (int t = 1; t < n_; ++t) threads_.emplace_back([this, t] { loop(t); });
    }
    ~IoPool() {
        {
            std::lock_guard<std::mutex> g(m_);
            stop_ = true;
            ++epoch_;
        }
        cv_.notify_all();
        for (auto& t : threads_) t.join();
    }
    int size() const { return n_; }
    // fn(part, begin, end) for each part; returns when all parts are done.  One caller at a time.
    void run(int64_t n, int parts, const std::function<void(int, int64_t, int64_t)>& fn) {
        if (n <= 0) return;
        {
            std::lock_guard<std::mutex> g(m_);
            fn_ = &fn;
            total_ = n;
            parts_ = std::max(1, std::min(parts, n_));
            pending_ = n_ - 1;
            ++epoch_;
        }
        cv_.notify_all();
        part(0);
        std::unique_lock<std::mutex> g(m_);
        done_.wait(g, [this] { return pending_ == 0; });
        fn_ = nullptr;
    }

private:
    void part(int t) {
        if (t >= parts_) return;
        const int64_t per = (total_ + parts_ - 1) / parts_;
        const int64_t b = std::min<int64_t>(total_, per * t), e = std::min<int64_t>(total_, b + per);
        if (b < e) (*fn_)(t, b, e);
    }
    void loop(int t) {
        uint64_t seen = 0;
        for (;;) {
            {
                std::unique_lock<std::mutex> g(m_);
                cv_.wait(g, [&] { return epoch_ != seen; });
                seen = epoch_;
                if (stop_) return;
            }
            part(t);
            {
                std::lock_guard<std::mutex> g(m_);
                --pending_;
            }
            done_.notify_one();
        }
    }
    const int n_;
    std::vector<std::thread> threads_;
    std::mutex m_;
    std::condition_variable cv_, done_;
    const std::function<void(int, int64_t, int64_t)>* fn_ = nullptr;
    int64_t total_ = 0;
    int parts_ = 1;
    int pending_ = 0;
    uint64_t epoch_ = 0;
    bool stop_ = false;
};

struct Job {
    bool push = false;
    bool has_idx = false;
    std::vector<int32_t> idx;
    int64_t base = 0, n = 0;
    char* dev = nullptr;          // device rows: destination of a pull, source of a push
    int64_t pitch = 0;            // bytes
    hipEvent_t after = nullptr;   // work of the caller's stream that must finish first
    int64_t ticket = 0;
};

}  // namespace

struct gas_disk_table {
    int fd = -1;
    char* map = nullptr;          // the file, mapped shared; null: read / write calls
    int64_t map_bytes = 0;
    int64_t n_rows = 0;
    int32_t F = 0;
    gas_dtype dt = GAS_F32;
    int64_t row_bytes = 0;
    int64_t staging_rows = 0;
    int io_threads = 8;
    // device side, set up by the worker at the first transfer
    int device = -1;
    bool device_ready = false;
    void* stage[2] = {nullptr, nullptr};
    hipEvent_t copied[2] = {nullptr, nullptr};
    hipStream_t copy_stream = nullptr;
    // jobs
    std::thread worker;
    std::mutex m;
    std::condition_variable cv_job, cv_done;
    std::deque<Job> queue;
    int64_t issued = 0, finished = 0;
    bool stop = false;
    gas_status status = GAS_OK;   // first failure of a job; later jobs are dropped
    std::string error;
};

namespace {

using gas::fail;

// The process's I/O threads, started at the first transfer of any table and never stopped (they sleep between
// bursts).  One burst at a time: tables take turns for the file copies and overlap them with each other's DMA.
constexpr int kPoolThreads = 16;
std::mutex pool_mutex;
IoPool* shared_pool() {
    static IoPool* pool = new IoPool(kPoolThreads);
    return pool;
}

// Rows [b, e) of the list (idx or base + i) between the file and `buf` (row i of the list at buf + (i - origin) *
// row_bytes).  Runs of consecutive file rows take one call.  Returns 0 or errno.
int io_rows(const gas_disk_table* t, bool write, const int32_t* idx, int64_t base, int64_t origin, int64_t b, int64_t e,
            char* buf) {
    int64_t i = b;
    while (i < e) {
        const int64_t first = idx ? (int64_t)idx[i] : base + i;
        int64_t j = i + 1;
        if (idx)
            while (j < e && (int64_t)idx[j] == first + (j - i)) ++j;
        else
            j = e;
        char* p = buf + (i - origin) * t->row_bytes;
        int64_t left = (j - i) * t->row_bytes;
        off_t off = (off_t)(first * t->row_bytes);
        if (t->map) {
            if (write)
                memcpy(t->map + off, p, (size_t)left);
            else
                memcpy(p, t->map + off, (size_t)left);
            left = 0;
        }
        while (left > 0) {
            const ssize_t r = write ? pwrite(t->fd, p, (size_t)left, off) : pread(t->fd, p, (size_t)left, off);
            if (r < 0) {
                if (errno == EINTR) continue;
                return errno;
            }
            if (r == 0) return EIO;     // the file is shorter than its table
            p += r;
            off += r;
            left -= r;
        }
        i = j;
    }
    return 0;
}

int io_parallel(gas_disk_table* t, bool write, const int32_t* idx, int64_t base, int64_t origin, int64_t b, int64_t e,
                char* buf) {
    std::vector<int> err((size_t)kPoolThreads, 0);
    std::lock_guard<std::mutex> g(pool_mutex);
    shared_pool()->run(e - b, t->io_threads, [&](int part, int64_t pb, int64_t pe) {
        err[(size_t)part] = io_rows(t, write, idx, base, origin, b + pb, b + pe, buf);
    });
    for (int v : err)
        if (v) return v;
    return 0;
}

gas_status job_fail(gas_disk_table* t, gas_status st, const char* what, const char* detail) {
    std::lock_guard<std::mutex> g(t->m);
    if (t->status == GAS_OK) {
        t->status = st;
        t->error = std::string(what) + ": " + detail;
    }
    return st;
}

#define JOB_HIP(expr)                                                               \
    do {                                                                            \
        hipError_t e_ = (expr);                                                     \
        if (e_ != hipSuccess) return job_fail(t, GAS_ERR_HIP, #expr, hipGetErrorString(e_)); \
    } while (0)

gas_status ensure_device(gas_disk_table* t) {
    if (t->device_ready) return GAS_OK;
    JOB_HIP(hipSetDevice(t->device));
    JOB_HIP(hipStreamCreateWithFlags(&t->copy_stream, hipStreamNonBlocking));
    for (int b = 0; b < 2; ++b) {
        JOB_HIP(hipHostMalloc(&t->stage[b], (size_t)(t->staging_rows * t->row_bytes), hipHostMallocDefault));
        JOB_HIP(hipEventCreateWithFlags(&t->copied[b], hipEventDisableTiming));
    }
    t->device_ready = true;
    return GAS_OK;
}

gas_status copy_piece(gas_disk_table* t, bool to_device, char* dev, int64_t pitch, void* host, int64_t rows) {
    const size_t w = (size_t)t->row_bytes;
    if (pitch == t->row_bytes) {
        JOB_HIP(hipMemcpyAsync(to_device ? (void*)dev : host, to_device ? host : (void*)dev, w * (size_t)rows,
                               to_device ? hipMemcpyHostToDevice : hipMemcpyDeviceToHost, t->copy_stream));
    } else if (to_device) {
        JOB_HIP(hipMemcpy2DAsync(dev, (size_t)pitch, host, w, w, (size_t)rows, hipMemcpyHostToDevice, t->copy_stream));
    } else {
        JOB_HIP(hipMemcpy2DAsync(host, w, dev, (size_t)pitch, w, (size_t)rows, hipMemcpyDeviceToHost, t->copy_stream));
    }
    return GAS_OK;
}

// Pull: piece c is read from the file into staging buffer c & 1 while the copy of piece c - 1 runs; the buffer is
// reused once the copy of piece c - 2 has finished.  Push: piece c is copied from the device while piece c - 1 is
// written to the file.  Either way the job ends with everything in place: the rows in device memory (pull) or
// handed to the file system (push).
gas_status run_job(gas_disk_table* t, Job& job) {
    if (job.n == 0) return GAS_OK;
    if (gas_status st = ensure_device(t)) return st;
    if (job.after) {
        JOB_HIP(hipEventSynchronize(job.after));
        JOB_HIP(hipEventDestroy(job.after));
        job.after = nullptr;
    }
    const int32_t* idx = job.has_idx ? job.idx.data() : nullptr;
    const int64_t S = t->staging_rows;
    const int64_t pieces = (job.n + S - 1) / S;
    for (int64_t c = 0; c < pieces; ++c) {
        const int b = (int)(c & 1);
        const int64_t r0 = c * S, r1 = std::min(job.n, r0 + S);
        char* dev = job.dev + r0 * job.pitch;
        if (!job.push) {
            if (c >= 2) JOB_HIP(hipEventSynchronize(t->copied[b]));
            if (int e = io_parallel(t, false, idx, job.base, r0, r0, r1, (char*)t->stage[b]))
                return job_fail(t, GAS_ERR_IO, "reading history rows", strerror(e));
            if (gas_status st = copy_piece(t, true, dev, job.pitch, t->stage[b], r1 - r0)) return st;
            JOB_HIP(hipEventRecord(t->copied[b], t->copy_stream));
        } else {
            if (gas_status st = copy_piece(t, false, dev, job.pitch, t->stage[b], r1 - r0)) return st;
            JOB_HIP(hipEventRecord(t->copied[b], t->copy_stream));
            if (c >= 1) {
                JOB_HIP(hipEventSynchronize(t->copied[b ^ 1]));
                if (int e = io_parallel(t, true, idx, job.base, r0 - S, r0 - S, r0, (char*)t->stage[b ^ 1]))
                    return job_fail(t, GAS_ERR_IO, "writing history rows", strerror(e));
            }
        }
    }
    if (job.push && pieces > 0) {
        const int64_t c = pieces - 1, r0 = c * S;
        JOB_HIP(hipEventSynchronize(t->copied[c & 1]));
        if (int e = io_parallel(t, true, idx, job.base, r0, r0, job.n, (char*)t->stage[c & 1]))
            return job_fail(t, GAS_ERR_IO, "writing history rows", strerror(e));
    }
    JOB_HIP(hipStreamSynchronize(t->copy_stream));
    return GAS_OK;
}

void worker_loop(gas_disk_table* t) {
    for (;;) {
        Job job;
        {
            std::unique_lock<std::mutex> g(t->m);
            t->cv_job.wait(g, [t] { return t->stop || !t->queue.empty(); });
            if (t->queue.empty()) return;     // stop, and nothing left to do
            job = std::move(t->queue.front());
            t->queue.pop_front();
        }
        bool failed;
        {
            std::lock_guard<std::mutex> g(t->m);
            failed = t->status != GAS_OK;
        }
        if (!failed)
            run_job(t, job);
        else if (job.after)
            (void)hipEventDestroy(job.after);
        {
            std::lock_guard<std::mutex> g(t->m);
            t->finished = job.ticket;
        }
        t->cv_done.notify_all();
    }
}

gas_status wait_ticket(gas_disk_table* t, int64_t ticket) {
    std::unique_lock<std::mutex> g(t->m);
    if (ticket > t->issued) return fail(GAS_ERR_ARG, "gas_disk_wait: ticket %lld was never issued", (long long)ticket);
    t->cv_done.wait(g, [&] { return t->finished >= ticket; });
    if (t->status != GAS_OK) return fail(t->status, "gas_disk: a transfer failed: %s", t->error.c_str());
    return GAS_OK;
}

gas_status check_rows(const gas_disk_table* t, const char* who, const int32_t* idx, int64_t base, int64_t n,
                      const void* rows, int64_t ld) {
    GAS_REQUIRE(t != nullptr, "%s: null table", who);
    GAS_REQUIRE(n >= 0, "%s: n=%lld", who, (long long)n);
    if (n == 0) return GAS_OK;
    GAS_REQUIRE(rows != nullptr, "%s: null row pointer", who);
    GAS_REQUIRE(ld >= t->F, "%s: row stride %lld below F=%d", who, (long long)ld, t->F);
    if (idx) {
        for (int64_t i = 0; i < n; ++i)
            if (idx[i] < 0 || idx[i] >= t->n_rows)
                return fail(GAS_ERR_RANGE, "%s: idx[%lld] = %d outside the table's %lld rows", who, (long long)i, idx[i],
                            (long long)t->n_rows);
    } else if (base < 0 || base + n > t->n_rows) {
        return fail(GAS_ERR_RANGE, "%s: rows [%lld, %lld) outside the table's %lld rows", who, (long long)base,
                    (long long)(base + n), (long long)t->n_rows);
    }
    return GAS_OK;
}

gas_status submit(gas_disk_table* t, bool push, const char* who, const int32_t* idx, int64_t base, int64_t n, void* dev,
                  int64_t ld, void* stream, int64_t* ticket) {
    if (gas_status st = check_rows(t, who, idx, base, n, dev, ld)) return st;
    GAS_REQUIRE(ticket != nullptr, "%s: null ticket", who);
    {
        std::lock_guard<std::mutex> g(t->m);
        if (t->status != GAS_OK) return fail(t->status, "%s: an earlier transfer failed: %s", who, t->error.c_str());
    }
    Job job;
    job.push = push;
    job.has_idx = idx != nullptr;
    if (idx) job.idx.assign(idx, idx + n);
    job.base = base;
    job.n = n;
    job.dev = (char*)dev;
    job.pitch = ld * gas::elem_bytes(t->dt);
    if (n > 0) {
        int device = 0;
        GAS_CHECK_HIP(hipGetDevice(&device));
        if (t->device < 0) t->device = device;
        GAS_REQUIRE(t->device == device, "%s: the table was first used on device %d, now %d", who, t->device, device);
        GAS_CHECK_HIP(hipEventCreateWithFlags(&job.after, hipEventDisableTiming));
        const hipError_t e = hipEventRecord(job.after, (hipStream_t)stream);
        if (e != hipSuccess) {
            (void)hipEventDestroy(job.after);
            return fail(GAS_ERR_HIP, "%s: hipEventRecord failed: %s", who, hipGetErrorString(e));
        }
    }
    {
        std::lock_guard<std::mutex> g(t->m);
        job.ticket = *ticket = ++t->issued;
        t->queue.push_back(std::move(job));
    }
    t->cv_job.notify_one();
    return GAS_OK;
}

gas_status host_rows(gas_disk_table* t, bool write, const char* who, const int32_t* idx, int64_t base, int64_t n,
                     void* rows, int64_t ld) {
    if (gas_status st = check_rows(t, who, idx, base, n, rows, ld)) return st;
    int64_t last;
    {
        std::lock_guard<std::mutex> g(t->m);
        last = t->issued;
    }
    if (gas_status st = wait_ticket(t, last)) return st;
    if (n == 0) return GAS_OK;
    const int64_t pitch = ld * gas::elem_bytes(t->dt);
    int e = 0;
    if (pitch == t->row_bytes) {
        e = io_parallel(t, write, idx, base, 0, 0, n, (char*)rows);
    } else {                       // strided host rows: one row per call
        std::vector<int> err((size_t)kPoolThreads, 0);
        std::lock_guard<std::mutex> g(pool_mutex);
        shared_pool()->run(n, t->io_threads, [&](int part, int64_t b, int64_t e2) {
            for (int64_t i = b; i < e2 && !err[(size_t)part]; ++i)
                err[(size_t)part] = io_rows(t, write, idx, base, i, i, i + 1, (char*)rows + i * pitch);
        });
        for (int v : err)
            if (v) e = v;
    }
    if (e) return fail(GAS_ERR_IO, "%s: %s", who, strerror(e));
    return GAS_OK;
}

}  // namespace

extern "C" {

gas_status gas_disk_open(const char* path, int64_t n_rows, int32_t F, gas_dtype dt, int32_t flags, int32_t io_threads,
                         int64_t staging_bytes, gas_disk_table** out) {
    GAS_REQUIRE(path && out, "gas_disk_open: null pointer");
    GAS_REQUIRE((flags & ~(GAS_DISK_CREATE | GAS_DISK_CALLS)) == 0, "gas_disk_open: unknown flags %d", flags);
    const bool create = flags & GAS_DISK_CREATE;
    if (!gas::valid_dtype(dt)) return fail(GAS_ERR_DTYPE, "gas_disk_open: unknown dtype %d", (int)dt);
    GAS_REQUIRE(n_rows >= 0 && F > 0, "gas_disk_open: n_rows=%lld F=%d", (long long)n_rows, F);
    GAS_REQUIRE(io_threads >= 0 && io_threads <= kPoolThreads, "gas_disk_open: io_threads=%d not in [0, %d]", io_threads,
                kPoolThreads);
    GAS_REQUIRE(staging_bytes >= 0 && staging_bytes <= (1ll << 32), "gas_disk_open: staging_bytes=%lld not in [0, 4 GiB]",
                (long long)staging_bytes);
    const int64_t row_bytes = (int64_t)F * gas::elem_bytes(dt);
    const int64_t bytes = n_rows * row_bytes;
    const int fd = open(path, create ? (O_RDWR | O_CREAT | O_CLOEXEC) : (O_RDWR | O_CLOEXEC), 0644);
    if (fd < 0) return fail(GAS_ERR_IO, "gas_disk_open: %s: %s", path, strerror(errno));
    struct stat sb;
    if (fstat(fd, &sb) != 0 || !S_ISREG(sb.st_mode)) {
        close(fd);
        return fail(GAS_ERR_IO, "gas_disk_open: %s is not a regular file", path);
    }
    if (create) {
        // rows never written read as zeros: the initial history
        if (ftruncate(fd, 0) != 0 || ftruncate(fd, (off_t)bytes) != 0) {
            const int e = errno;
            close(fd);
            return fail(GAS_ERR_IO, "gas_disk_open: cannot size %s to %lld bytes: %s", path, (long long)bytes, strerror(e));
        }
    } else if ((int64_t)sb.st_size != bytes) {
        close(fd);
        return fail(GAS_ERR_ARG, "gas_disk_open: %s holds %lld bytes, a table of %lld x %d needs %lld", path,
                    (long long)sb.st_size, (long long)n_rows, F, (long long)bytes);
    }
    (void)posix_fadvise(fd, 0, 0, POSIX_FADV_RANDOM);
    char* map = nullptr;
    if (!(flags & GAS_DISK_CALLS) && bytes > 0) {
        void* m = mmap(nullptr, (size_t)bytes, PROT_READ | PROT_WRITE, MAP_SHARED, fd, 0);
        if (m == MAP_FAILED) {
            const int e = errno;
            close(fd);
            return fail(GAS_ERR_IO, "gas_disk_open: cannot map %s (%lld bytes): %s", path, (long long)bytes, strerror(e));
        }
        (void)madvise(m, (size_t)bytes, MADV_RANDOM);
        map = (char*)m;
    }
    gas_disk_table* t = new gas_disk_table();
    t->fd = fd;
    t->map = map;
    t->map_bytes = bytes;
    t->n_rows = n_rows;
    t->F = F;
    t->dt = dt;
    t->row_bytes = row_bytes;
    const int64_t sb_bytes = staging_bytes > 0 ? staging_bytes : (32ll << 20);
    t->staging_rows = std::max<int64_t>(1, sb_bytes / row_bytes);
    t->io_threads = io_threads > 0 ? io_threads : 8;
    t->worker = std::thread(worker_loop, t);
    *out = t;
    return GAS_OK;
}

gas_status gas_disk_close(gas_disk_table* t) {
    if (!t) return GAS_OK;
    {
        std::lock_guard<std::mutex> g(t->m);
        t->stop = true;
    }
    t->cv_job.notify_all();
    t->worker.join();                 // finishes the queued jobs first
    gas_status st = GAS_OK;
    if (t->status != GAS_OK) st = fail(t->status, "gas_disk_close: a transfer had failed: %s", t->error.c_str());
    if (t->device_ready) {
        (void)hipSetDevice(t->device);
        for (int b = 0; b < 2; ++b) {
            (void)hipHostFree(t->stage[b]);
            (void)hipEventDestroy(t->copied[b]);
        }
        (void)hipStreamDestroy(t->copy_stream);
    }
    if (t->map) (void)munmap(t->map, (size_t)t->map_bytes);
    if (close(t->fd) != 0 && st == GAS_OK) st = fail(GAS_ERR_IO, "gas_disk_close: %s", strerror(errno));
    delete t;
    return st;
}

gas_status gas_disk_pull(gas_disk_table* t, const int32_t* idx, int64_t base, int64_t n, void* dst, int64_t ld_dst,
                         void* stream, int64_t* ticket) {
    return submit(t, false, "gas_disk_pull", idx, base, n, dst, ld_dst, stream, ticket);
}

gas_status gas_disk_push(gas_disk_table* t, const int32_t* idx, int64_t base, int64_t n, const void* src, int64_t ld_src,
                         void* stream, int64_t* ticket) {
    return submit(t, true, "gas_disk_push", idx, base, n, const_cast<void*>(src), ld_src, stream, ticket);
}

gas_status gas_disk_wait(gas_disk_table* t, int64_t ticket) {
    GAS_REQUIRE(t != nullptr, "gas_disk_wait: null table");
    if (ticket <= 0) {
        std::lock_guard<std::mutex> g(t->m);
        ticket = t->issued;
    }
    return wait_ticket(t, ticket);
}

gas_status gas_disk_read_rows(gas_disk_table* t, const int32_t* idx, int64_t base, int64_t n, void* dst, int64_t ld_dst) {
    return host_rows(t, false, "gas_disk_read_rows", idx, base, n, dst, ld_dst);
}

gas_status gas_disk_write_rows(gas_disk_table* t, const int32_t* idx, int64_t base, int64_t n, const void* src,
                               int64_t ld_src) {
    return host_rows(t, true, "gas_disk_write_rows", idx, base, n, const_cast<void*>(src), ld_src);
}

gas_status gas_disk_sync(gas_disk_table* t) {
    GAS_REQUIRE(t != nullptr, "gas_disk_sync: null table");
    int64_t last;
    {
        std::lock_guard<std::mutex> g(t->m);
        last = t->issued;
    }
    if (gas_status st = wait_ticket(t, last)) return st;
    if (t->map && msync(t->map, (size_t)t->map_bytes, MS_SYNC) != 0)
        return fail(GAS_ERR_IO, "gas_disk_sync: msync: %s", strerror(errno));
    if (fdatasync(t->fd) != 0) return fail(GAS_ERR_IO, "gas_disk_sync: %s", strerror(errno));
    return GAS_OK;
}

}  // extern "C"
