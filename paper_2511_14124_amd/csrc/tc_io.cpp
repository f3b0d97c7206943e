// File tier of libtc.so: worker threads that read and write tensor extents
// behind the hook thread, chunked requests, striping over several files.
#include "tc_ctx.h"

#include <errno.h>
#include <stdlib.h>
#include <string.h>
#include <unistd.h>

#include <algorithm>
#include <chrono>

// pwrite until everything is out; no context state is touched (writer threads use it)
static bool pwrite_all(int fd, const uint8_t *src, uint64_t bytes, uint64_t off, std::string &err)
{
    while (bytes) {
        ssize_t w = pwrite(fd, src, bytes, (off_t)off);
        if (w < 0 && errno == EINTR) continue;
        if (w <= 0) { err = std::string("pwrite: ") + strerror(errno); return false; }
        src += w; off += (uint64_t)w; bytes -= (uint64_t)w;
    }
    return true;
}

static bool pread_all(int fd, uint8_t *dst, uint64_t bytes, uint64_t want, uint64_t off, std::string &err)
{
    // `bytes` are requested (rounded for O_DIRECT); at least `want` must arrive: a file
    // whose last extent ends at the tensor's last byte is not a short read
    uint64_t got = 0;
    while (got < bytes) {
        ssize_t r = pread(fd, dst + got, bytes - got, (off_t)(off + got));
        if (r < 0 && errno == EINTR) continue;
        if (r < 0) { err = std::string("pread: ") + strerror(errno); return false; }
        if (r == 0) break;
        got += (uint64_t)r;
    }
    if (got < want) { err = "pread: short file"; return false; }
    return true;
}

// block until the writes of `after` have finished (called by workers: a dependency was always
// queued before the job that names it, and workers take their jobs in order, so this ends)
static void io_wait_writes(tc_ctx *c, const JobSet &after)
{
    if (!after.any) return;
    const auto &pool = c->io[IO_WRITERS];
    for (size_t wi = 0; wi < pool.size(); ++wi) {
        if (!after.seq[wi] || pool[wi]->done.load() >= after.seq[wi]) continue;
        IoWorker &w = *pool[wi];
        std::unique_lock<std::mutex> lk(w.mu);
        w.cv_done.wait(lk, [&] { return w.done.load() >= after.seq[wi]; });
    }
}

// one job, by a worker thread (w) or by the calling thread (w == nullptr).
// O_DIRECT cannot target memory the GPU driver has mapped (pread into a pinned
// region fails with EFAULT on this kernel), so in that mode every request goes
// through a bounce block, ordinary page-aligned memory of the library's own.
static void io_run_job(tc_ctx *c, IoWorker *w, const IoJob &j)
{
    std::string err;
    io_wait_writes(c, j.after);
    if (j.ev) {
        hipError_t e = hipEventSynchronize(j.ev);
        if (e != hipSuccess) err = std::string("hipEventSynchronize (file tier): ") + hipGetErrorString(e);
    }
    if (err.empty()) {
        const auto t0 = std::chrono::steady_clock::now();
        uint8_t *blk = w ? w->bounce : c->io_bounce;
        const uint64_t len = io_len(c, j.bytes);
        if (j.read) {
            if (c->file_direct) {
                if (pread_all(j.fd, blk, len, j.bytes, j.off, err)) memcpy(j.mem, blk, j.bytes);
            } else {
                pread_all(j.fd, j.mem, j.bytes, j.bytes, j.off, err);
            }
        } else if (c->file_direct) {
            memcpy(blk, j.mem, j.bytes);
            memset(blk + j.bytes, 0, len - j.bytes);
            pwrite_all(j.fd, blk, len, j.off, err);
        } else {
            pwrite_all(j.fd, j.mem, j.bytes, j.off, err);
        }
        (j.read ? c->rd_ns : c->wr_ns) += (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
                                              std::chrono::steady_clock::now() - t0).count();
    }
    if (!err.empty()) {
        std::lock_guard<std::mutex> g(c->io_mu);
        if (!c->io_failed.load()) { c->io_err = err; c->io_failed.store(true); }
    }
}

static void io_worker_main(tc_ctx *c, IoWorker *w)
{
    (void)hipSetDevice(c->device);
    for (;;) {
        IoJob j;
        {
            std::unique_lock<std::mutex> lk(w->mu);
            w->cv_job.wait(lk, [&] { return w->quit || !w->q.empty(); });
            if (w->q.empty()) return;                  // quit, and nothing left to do
            j = w->q.front();
            w->q.pop_front();
        }
        io_run_job(c, w, j);
        {
            std::lock_guard<std::mutex> g(w->mu);
            w->done.store(j.seq);
        }
        w->cv_done.notify_all();
    }
}

// a worker's failure surfaces at the next call that waits for or queues a job
int io_check(tc_ctx *c)
{
    if (!c->io_failed.load()) return TC_OK;
    std::lock_guard<std::mutex> g(c->io_mu);
    return fail(c, TC_E_IO, c->io_err);
}

bool io_done(tc_ctx *c, const JobSet &r)
{
    if (!r.any) return true;
    const auto &pool = c->io[r.pool];
    for (size_t w = 0; w < pool.size(); ++w)
        if (r.seq[w] && pool[w]->done.load() < r.seq[w]) return false;
    return true;
}

int io_wait(tc_ctx *c, JobSet &r)
{
    if (r.any) {
        const auto &pool = c->io[r.pool];
        for (size_t wi = 0; wi < pool.size(); ++wi) {
            if (!r.seq[wi] || pool[wi]->done.load() >= r.seq[wi]) continue;
            IoWorker &w = *pool[wi];
            std::unique_lock<std::mutex> lk(w.mu);
            w.cv_done.wait(lk, [&] { return w.done.load() >= r.seq[wi]; });
        }
        r = JobSet{};
    }
    return io_check(c);
}

int io_wait_all(tc_ctx *c)
{
    for (int pool = 0; pool < 2; ++pool)
        for (auto &pw : c->io[pool]) {
            IoWorker &w = *pw;
            {
                std::unique_lock<std::mutex> lk(w.mu);
                w.cv_done.wait(lk, [&] { return w.done.load() >= w.issued; });
            }
        }
    for (auto &e : c->ev_busy) c->ev_free.push_back(e.first);
    c->ev_busy.clear();
    return io_check(c);
}

void io_stop(tc_ctx *c)
{
    (void)io_wait_all(c);
    for (int pool = 0; pool < 2; ++pool) {
        for (auto &pw : c->io[pool]) {
            {
                std::lock_guard<std::mutex> g(pw->mu);
                pw->quit = true;
            }
            pw->cv_job.notify_all();
            if (pw->th.joinable()) pw->th.join();
            if (pw->bounce) free(pw->bounce);
        }
        c->io[pool].clear();
    }
    for (JobSet &r : c->tensor_job) r = JobSet{};
    for (JobSet &r : c->cpu_job) r = JobSet{};
    for (JobSet &r : c->fast_read) r = JobSet{};
    for (JobSet &r : c->fast_write) r = JobSet{};
    for (StBlock &b : c->st_q) b.job = JobSet{};
    for (PUnit &p : c->deferred) p.read_job = JobSet{};
}

int io_start(tc_ctx *c)
{
    for (int pool = 0; pool < 2; ++pool)
        for (uint32_t i = 0; i < c->n_io[pool]; ++i) {
            std::unique_ptr<IoWorker> w(new (std::nothrow) IoWorker());
            if (!w) return fail(c, TC_E_CAPACITY, "no memory for an I/O worker");
            if (c->file_direct) {
                void *blk = nullptr;
                if (posix_memalign(&blk, 4096, c->io_bounce_bytes) != 0)
                    return fail(c, TC_E_CAPACITY, "no memory for an I/O worker's bounce block");
                w->bounce = (uint8_t *)blk;
            }
            try {
                w->th = std::thread(io_worker_main, c, w.get());
            } catch (...) {
                if (w->bounce) free(w->bounce);
                return fail(c, TC_E_CAPACITY, "could not start an I/O worker thread");
            }
            c->io[pool].push_back(std::move(w));
        }
    return TC_OK;
}

// Queue (or, without worker threads of that kind, perform) the transfer of
// tensor t's extent: a write from `mem` or a read into it.  op != 0: the bytes
// to write are being produced by copy operation `op`, issued on stream S a
// moment ago.  `set` names the queued jobs.
int io_submit(tc_ctx *c, uint32_t t, uint8_t *mem, bool read, uint64_t op, int S, JobSet *set, const JobSet *after)
{
    if (op && c->io[read ? IO_READERS : IO_WRITERS].empty()) {
        int rc = tc_wait_op(c, op);
        if (rc != TC_OK) return rc;
        op = 0;
    }
    return io_submit_behind(c, t, mem, read, op != 0, c->streams[S], set, after);
}

// The same with the stream named: behind != 0 makes the jobs wait for everything
// queued on `stream` so far (work that still produces the bytes to write, or
// still uses the memory to read into).
int io_submit_behind(tc_ctx *c, uint32_t t, uint8_t *mem, bool read, bool behind, hipStream_t stream, JobSet *set,
                     const JobSet *after)
{
    *set = JobSet{};
    set->pool = read ? IO_READERS : IO_WRITERS;
    if (c->n_files == 0) return fail(c, TC_E_IO, "an op needs the file tier but no file is bound");
    int rc = io_check(c);
    if (rc != TC_OK) return rc;
    // what has to be in the file or out of the buffer first: a queued write of this very
    // extent (for a read), and whatever the caller names
    JobSet dep;
    if (read && c->tensor_job[t].any && !io_done(c, c->tensor_job[t])) dep = c->tensor_job[t];
    if (after && after->any && after->pool == IO_WRITERS && !io_done(c, *after)) {
        dep.any = true;
        for (uint32_t w = 0; w < IO_MAX_THREADS; ++w) dep.seq[w] = std::max(dep.seq[w], after->seq[w]);
    }
    c->io_begun = true;
    auto &pool = c->io[set->pool];
    if (behind && pool.empty()) {
        HIP_TRY(c, hipStreamSynchronize(stream));
        behind = false;
    }
    const uint64_t n = c->prof.bytes[t], base = c->place.file_off[t];
    hipEvent_t ev = nullptr;
    if (behind) {
        // one event for the whole request, recorded right behind the copy
        while (!c->ev_busy.empty() && io_done(c, c->ev_busy.front().second)) {
            c->ev_free.push_back(c->ev_busy.front().first);
            c->ev_busy.pop_front();
        }
        if (c->ev_free.empty()) {
            HIP_TRY(c, hipEventCreateWithFlags(&ev, hipEventDisableTiming | hipEventBlockingSync));
        } else {
            ev = c->ev_free.back();
            c->ev_free.pop_back();
        }
        hipError_t e = hipEventRecord(ev, stream);
        if (e != hipSuccess) {
            c->ev_free.push_back(ev);
            return fail(c, TC_E_HIP, std::string("hipEventRecord (file tier): ") + hipGetErrorString(e));
        }
    }
    uint64_t lane = t;
    for (uint64_t o = 0; o < n; o += c->io_chunk, ++lane) {
        IoJob j{0, ev, mem + o, std::min(c->io_chunk, n - o), base + o, c->fds[lane % c->n_files], read, dep};
        if (pool.empty()) {
            io_run_job(c, nullptr, j);
            continue;
        }
        const size_t wi = lane % pool.size();
        IoWorker &w = *pool[wi];
        j.seq = ++w.issued;
        {
            std::lock_guard<std::mutex> g(w.mu);
            w.q.push_back(j);
        }
        w.cv_job.notify_one();
        set->any = true;
        set->seq[wi] = j.seq;
    }
    if (ev) c->ev_busy.push_back({ev, *set});
    if (pool.empty()) return io_check(c);
    if (!read) c->tensor_job[t] = *set;
    return TC_OK;
}

// the same, finished before it returns (loads, read-backs, restores)
int io_transfer(tc_ctx *c, uint32_t t, uint8_t *mem, bool read)
{
    JobSet set;
    int rc = io_submit(c, t, mem, read, 0, 0, &set);
    if (rc != TC_OK) return rc;
    return io_wait(c, set);
}

extern "C" int tc_set_io_threads(tc_ctx *c, uint32_t writers, uint32_t readers)
{
    if (!c) return TC_E_ARG;
    if (writers > IO_MAX_THREADS || readers > IO_MAX_THREADS) return fail(c, TC_E_ARG, "at most 8 writer and 8 reader threads");
    c->n_io[IO_WRITERS] = writers;
    c->n_io[IO_READERS] = readers;
    c->io_threads_set = true;
    if (c->stage != 4 || c->n_files == 0 || c->null_mover) return TC_OK;
    int rc = tc_synchronize(c);
    if (rc != TC_OK) return rc;
    io_stop(c);
    return io_start(c);
}

extern "C" int tc_set_io_chunk(tc_ctx *c, uint64_t bytes)
{
    if (!c) return TC_E_ARG;
    if (bytes < 65536 || bytes % 4096) return fail(c, TC_E_ARG, "chunk must be a multiple of 4096, at least 64 KiB");
    if (c->stage == 4 && c->io_begun) return fail(c, TC_E_STATE, "the file tier is already in use");
    c->io_chunk = bytes;
    c->io_chunk_set = true;
    if (c->stage != 4 || c->n_files == 0 || c->null_mover || !c->file_direct) return TC_OK;
    // O_DIRECT bounce blocks are one chunk each: make them anew
    io_stop(c);
    uint64_t largest = 0;
    for (uint32_t t = 0; t < c->prof.n_tensors; ++t) largest = std::max(largest, c->prof.bytes[t]);
    c->io_bounce_bytes = std::min<uint64_t>(c->io_chunk, (largest + 4095) & ~4095ull);
    free(c->io_bounce);
    void *blk = nullptr;
    if (posix_memalign(&blk, 4096, c->io_bounce_bytes) != 0) { c->io_bounce = nullptr; return fail(c, TC_E_CAPACITY, "no memory for the I/O bounce block"); }
    c->io_bounce = (uint8_t *)blk;
    return io_start(c);
}

extern "C" int tc_add_stripe(tc_ctx *c, int fd)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4 || c->null_mover) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    if (fd < 0) return fail(c, TC_E_ARG, "not a file descriptor");
    if (c->n_files == 0) return fail(c, TC_E_STATE, "tc_bind_memory was given no file to add stripes to");
    if (c->io_begun) return fail(c, TC_E_STATE, "the file tier is already in use");
    if (c->n_files >= IO_MAX_FILES) return fail(c, TC_E_CAPACITY, "at most 8 files");
    c->fds[c->n_files++] = fd;
    return TC_OK;
}

