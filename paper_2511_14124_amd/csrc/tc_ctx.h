// The context of libtc.so and what its source files share: the types of the
// dispatch and of the file tier, the context itself, and the functions one file
// offers the others.  Nothing here is part of the public ABI (see include/tc.h).
#pragma once

#include "tc_internal.h"

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <memory>
#include <mutex>
#include <string>
#include <thread>
#include <vector>


// Streams the copies run on.  K: the caller's migration stream, used by the
// migration kernel (small tensors, staging copies inside HBM).  H and D: two
// streams of the library's own, one per direction, that carry the large
// tensors as DMA-engine copies (hipMemcpyAsync).
enum { S_K = 0, S_H = 1, S_D = 2, N_STREAMS = 3 };

const uint32_t OP_RING = 1024;          // events kept for the most recent copy operations

// File I/O runs behind the hook thread on worker threads.  A tensor's extent
// is cut into chunks of io_chunk bytes; chunk i of tensor t belongs to lane
// t + i, and the lane picks the file (if the tier is striped over several), the
// writer and the reader.  One request therefore spreads over the workers, while
// every chunk always goes to the same writer, and a worker works in order: two
// writes of one extent land in the order they were issued.  A read of an extent
// names the write queued for it and starts once that has finished (the reader
// waits, not the hook thread).  A write job may carry an event to wait for
// (bytes a copy is still producing).
const uint32_t IO_MAX_THREADS = 8, IO_MAX_FILES = 8;

enum { IO_WRITERS = 0, IO_READERS = 1 };

struct JobSet {             // the jobs of one request: per worker the newest of them (0: none)
    uint8_t pool = IO_WRITERS;
    bool any = false;
    uint64_t seq[IO_MAX_THREADS] = {};
};

struct IoJob {
    uint64_t seq;
    hipEvent_t ev;          // write: nullptr = the bytes are ready
    uint8_t *mem;           // write: source, read: destination
    uint64_t bytes, off;
    int fd;
    bool read;
    JobSet after;           // writes (writer pool) that must have finished before this job starts
};

struct IoWorker {
    std::thread th;
    std::mutex mu;
    std::condition_variable cv_job, cv_done;
    std::deque<IoJob> q;
    uint64_t issued = 0;                // hook thread only
    std::atomic<uint64_t> done{0};      // stored under mu, polled without
    bool quit = false;                  // under mu
    uint8_t *bounce = nullptr;          // O_DIRECT: page-aligned block of its own
};

struct StBlock {            // live piece of the staging ring
    uint64_t id, off, size;
    uint64_t ops[2];        // copies that read or write it
    JobSet job;             // write that reads it
    bool issued;            // its unit has been launched (ops and job are final)
};

struct BounceBlock {        // live piece of the HBM bounce ring
    uint64_t off, size, op; // op: the copy that reads it last (0 = not issued yet)
};

struct PUnit {              // one exchange unit being prepared
    TcUnit u{};
    int64_t gpu_y = -1;     // flat index of the GPU buffer
    int64_t cpu_out = -1;   // flat index of the host buffer the outgoing tensor goes to
    int64_t cpu_in = -1;    // flat index of the host buffer the incoming tensor comes from
    bool out_staging = false, in_staging = false;
    uint32_t out_tensor = 0;
    uint32_t sig = 0;       // signal the call that prepared it queued on its compute stream (0: none)
    uint64_t st_id = 0;     // its block of the staging ring (0: none)
    JobSet read_job;        // file read that fills in_src (in_staging)
};

// Decisions made ahead for hook calls that follow the profile (tc_migrate_step):
// a window of the profiled steps decided by one launch, consumed call by call.
struct SpecWin {
    bool valid = false, ready = false;  // ready: the host has seen its launch finish
    uint32_t first = 0;                 // first step
    uint32_t n_calls = 0, used = 0;     // hook calls decided / handed out
    uint32_t ops_used = 0;              // op records handed out
    int blk = 0;                        // result block and snapshot it uses
};

struct Timed {              // event pair around one timed operation
    hipEvent_t t0, t1;
    int kind;               // S_K kernel launch, S_H / S_D copy, K_DECIDE decision launch
    uint64_t bytes;         // bytes moved; hook calls decided for K_DECIDE
};
enum { K_DECIDE = 3, N_KINDS = 4 };


struct tc_ctx {
    int stage = 0;          // 0 created, 1 profiled, 2 pools, 3 placed, 4 bound
    std::string err;
    TcProfile prof;
    tc_budget budget{};
    TcPools pools;
    TcPlacement place;

    // bound memory
    uint8_t *hbm = nullptr, *pinned = nullptr, *staging = nullptr;
    uint64_t hbm_bytes = 0, pinned_bytes = 0, staging_bytes = 0;
    int fds[IO_MAX_FILES];              // the file tier: one file, or several that stripe it by lane
    uint32_t n_files = 0;
    bool io_begun = false;              // a file request has been made: files and chunk size are final
    uint64_t io_chunk = 8ull << 20;     // bytes per chunk of an extent
    bool file_direct = false;           // the file was opened with O_DIRECT: 4 KiB aligned memory, offsets and lengths
    uint8_t *io_bounce = nullptr;       // 4 KiB aligned host block (one chunk) for file I/O done by the calling thread in that mode
    uint64_t io_bounce_bytes = 0;
    hipStream_t streams[N_STREAMS]{};   // [S_K] is the caller's migration stream
    hipStream_t dstream = nullptr;      // decision stream (ours)
    bool null_mover = false;
    bool in_use = false;                // a tensor has been loaded or a hook call made: the regions hold data

    // device tables
    uint32_t *dev_block = nullptr;      // one allocation holding every table
    TcDevTables T{};
    TcDecideOut *dout = nullptr;        // pinned: one record per hook call of a window, then the op records
    TcOpRec *dops = nullptr;            // (inside the same pinned block)
    TcDecideOut *dout2 = nullptr;       // second block: a window is decided while the one before is dispatched
    TcOpRec *dops2 = nullptr;
    uint32_t dout_cap = 0;              // op records a block holds
    uint32_t *d_step_ptr = nullptr;     // device copy of a replayed iteration's lists (tc_replay_iteration)
    uint32_t *d_ids = nullptr;
    uint8_t *d_rw = nullptr;
    uint32_t replay_window = 64;        // steps decided per launch by tc_replay_iteration
    // tc_migrate_step decides ahead along the profile: win[0] is being handed out, win[1]
    // was launched behind it; snap[b] holds the mutable tables from before the window in block b
    uint32_t ahead_steps = 16;          // steps per window (0: every call has its own launch)
    SpecWin win[2];
    uint32_t *snap[2] = {nullptr, nullptr};
    hipEvent_t win_ev[2] = {nullptr, nullptr};
    uint8_t *d_prof_rw = nullptr;       // device: R/W flags of the profiled rows
    size_t mut_off = 0, mut_words = 0;  // the mutable tables inside dev_block
    uint32_t ahead_pause = 0;           // calls to sit out after a call left the profile

    // dispatch state
    uint32_t mover_wgs = 12, chunk_bytes = 16384;
    uint32_t *tickets = nullptr;            // device: the migration kernel's two ticket counters
    uint64_t k_launches = 0;                // migration-kernel launches so far (their parity picks the counter)
    uint32_t mover_xcc = 0, mover_xcds = 1; // where the migration kernel's workgroups work (tc_mover_topology)
    uint64_t sdma_threshold = 0;            // tensors at least this large go through the DMA engines (0: none)
    bool dma_when_behind = false;           // ... but only while the compute stream has a backlog to hide them behind
    // the last few times units were issued: where the compute stream was (an event) and the
    // newest copy operation issued then
    struct IssuePoint { hipEvent_t ev = nullptr; uint64_t op = 0; bool used = false; };
    IssuePoint issue_ring[8];
    uint32_t issue_next = 0;
    uint64_t op_id = 0;                 // copy operations issued (kernel launches and DMA copies)
    uint64_t op_done[N_STREAMS]{};      // per stream: operations known complete
    hipEvent_t op_ev[OP_RING]{};
    uint8_t op_stream[OP_RING]{};
    hipEvent_t ev_compute = nullptr;
    bool compute_recorded = false;      // this hook call: ev_compute recorded
    bool stream_waited[N_STREAMS]{};    // this hook call: stream already waits for ev_compute
    std::vector<uint64_t> gpu_ticket, cpu_ticket;   // last operation that touched the buffer
    std::deque<StBlock> st_q;           // staging ring, oldest block first
    uint64_t st_head = 0, st_next_id = 1;
    uint8_t *bounce = nullptr;          // HBM ring: outgoing large tensors wait here for their DMA copy
    uint64_t bounce_bytes = 0, bounce_head = 0;
    std::deque<BounceBlock> bounce_q;
    // file tier behind the hook thread
    int device = 0;
    uint32_t n_io[2] = {4, 4};          // writer and reader threads; 0: that kind of I/O runs in the calling thread
    bool io_threads_set = false, io_chunk_set = false;   // the caller chose them (else a direct file gets defaults of its own)
    std::vector<std::unique_ptr<IoWorker>> io[2];
    std::vector<hipEvent_t> ev_free;
    std::deque<std::pair<hipEvent_t, JobSet>> ev_busy;  // events the queued jobs of a request wait for
    std::vector<JobSet> tensor_job;     // per tensor: newest queued write of its extent
    std::vector<uint8_t> wb_pending;    // per tensor: a prepared unit, not issued yet, will write it back to its extent
    std::vector<JobSet> cpu_job;        // per host buffer: queued write that reads it
    bool host_tier = false;             // two-tier mode: the fast tier is host memory, filled and drained by file I/O
    std::vector<JobSet> fast_read;      // two-tier mode, per fast-tier buffer: the read that fills it
    std::vector<JobSet> fast_write;     // ... and the write that drains it
    std::atomic<uint64_t> wr_ns{0}, rd_ns{0};   // time the workers spent in pwrite / pread
    std::mutex io_mu;
    std::string io_err;                 // first failure of a writer (under io_mu)
    std::atomic<bool> io_failed{false};
    // units prepared but not issued yet: hook calls are merged into larger launches
    std::vector<PUnit> deferred;
    uint64_t deferred_bytes = 0;
    uint64_t merge_bytes = 256ull << 20;
    std::vector<uint8_t> gpu_pending, cpu_pending;  // buffer is touched by a deferred unit
    hipStream_t last_compute = nullptr;
    uint64_t last_k_op = 0;             // newest operation issued on the migration stream
    // Dependencies resolved on the GPU (tc_set_gpu_dependencies): a hook call that prepares units queues a
    // one-lane kernel on its compute stream that raises the word `progress` to the call's number; the launch
    // that carries the units is queued at once and its workgroups wait for that number themselves.  Every
    // launch raises the word `done` to its own number when its last workgroup leaves, and a module that
    // needs what a launch brings is preceded on its stream by a one-lane kernel that waits for that number.
    // No event crosses between the two hardware queues (a wait across queues takes about 17 us here).
    bool gpu_deps = false;
    uint64_t spin_ticks = 500000000ull; // bound of every such wait, in ticks of the 100 MHz clock (5 s)
    uint32_t *fault = nullptr;          // pinned: a waiter that gave up writes here
    uint32_t sig_seq = 0;               // signals queued so far
    bool sig_sent = false;              // this hook call has queued its signal
    hipStream_t sig_stream = nullptr;   // the compute stream the signals were queued on
    uint32_t launch_seq = 0;            // launches that raise `done`
    uint32_t op_lseq[OP_RING]{};        // per copy operation: its launch number (0: not such a launch)
    uint32_t waited_lseq = 0;           // the newest launch number waited_stream has been made to wait for
    // per compute stream: the newest operation of each copy stream it has been made to wait for
    // (a stream is in order, so an older operation of the same copy stream needs no wait of its own)
    hipStream_t waited_stream = nullptr;
    uint64_t waited_op[N_STREAMS] = {};
    bool measure_stall = false;         // pre-hook calls time the wait for their copies on the host
    std::vector<uint64_t> stall_by_step; // ... and add the time each call waited to its step's entry
    // last PRE call, for tc_emulate_compute
    TcStampArgs last_pre{};
    uint32_t iteration = 0;

    // timing of migration launches and DMA copies
    bool timing = false;
    std::vector<Timed> timed;

    std::vector<tc_op> log;
    bool logging = true;
    tc_stats stats{};
};

static inline int fail(tc_ctx *c, int code, const std::string &msg)
{
    if (c) c->err = msg;
    return code;
}

// adds the time until it goes out of scope to one of tc_stats.host_blocked_ns
struct Blocked {
    tc_ctx *c;
    int k;
    std::chrono::steady_clock::time_point t0;
    Blocked(tc_ctx *c_, int k_) : c(c_), k(k_), t0(std::chrono::steady_clock::now()) {}
    ~Blocked()
    {
        c->stats.host_blocked_ns[k] += (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
                                           std::chrono::steady_clock::now() - t0).count();
    }
};
enum { BLK_FILE_READ = 0, BLK_FILE_WRITE = 1, BLK_STAGING = 2, BLK_COPY = 3 };

#define HIP_TRY(c, expr)                                                                          \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess)                                                                     \
            return fail((c), TC_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));        \
    } while (0)

// ---- copy operations (tc_dispatch.cpp) ----
int tc_wait_op(tc_ctx *c, uint64_t id);        // block the host until copy operation `id` has completed

// ---- file tier (tc_io.cpp) ----
static inline uint64_t io_align(const tc_ctx *c) { return c->file_direct ? 4096 : 256; }
static inline uint64_t io_len(const tc_ctx *c, uint64_t n) { return c->file_direct ? (n + 4095) & ~4095ull : n; }
int io_start(tc_ctx *c);                       // start the worker threads (n_io of each kind)
void io_stop(tc_ctx *c);                       // finish everything queued, end the threads
int io_check(tc_ctx *c);                       // a worker's failure, as TC_E_IO
bool io_done(tc_ctx *c, const JobSet &r);
int io_wait(tc_ctx *c, JobSet &r);             // wait for the jobs of one request, then forget them
int io_wait_all(tc_ctx *c);
// ---- addresses of pool buffers ------------------------------------------------
static inline uint8_t *gpu_addr(const tc_ctx *c, uint32_t s, uint32_t k)
{
    return c->hbm + c->pools.hbm_off[s] + (uint64_t)k * c->pools.stride[s];
}
static inline uint8_t *cpu_addr(const tc_ctx *c, uint32_t s, uint32_t k)
{
    return c->pinned + c->pools.host_off[s] + (uint64_t)k * c->pools.stride[s];
}

// Every kernel launch and every DMA copy is one operation with an id and an event in
// a ring.  An id older than the ring has completed by construction.
static inline bool op_complete(const tc_ctx *c, uint64_t id)
{
    if (id == 0 || c->op_id - id >= OP_RING) return true;
    return id <= c->op_done[c->op_stream[id % OP_RING]];
}

// tc_dispatch.cpp
int wait_op(tc_ctx *c, uint64_t id);                 // block the host until operation `id` has completed
int timed_begin(tc_ctx *c, int kind, hipEvent_t *t0);
int timed_end(tc_ctx *c, int kind, hipEvent_t t0, uint64_t bytes);
int flush_deferred(tc_ctx *c, hipStream_t compute);  // issue whatever units are prepared
int flush_for_buffers(tc_ctx *c, const int64_t *ys, uint32_t n, hipStream_t compute);   // ... that fill these GPU buffers, and the ready ones
int dispatch(tc_ctx *c, const TcDecideOut *o, const TcOpRec *ops, uint32_t step, int phase, hipStream_t compute);

// after: writes that must have finished before the request starts (may be nullptr)
int io_submit(tc_ctx *c, uint32_t t, uint8_t *mem, bool read, uint64_t op, int S, JobSet *set,
              const JobSet *after = nullptr);
int io_submit_behind(tc_ctx *c, uint32_t t, uint8_t *mem, bool read, bool behind, hipStream_t stream, JobSet *set,
                     const JobSet *after = nullptr);
int io_transfer(tc_ctx *c, uint32_t t, uint8_t *mem, bool read);
