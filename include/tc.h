/*
 * tc.h - C ABI of the MI355X tensor-cache migration library (libtc.so).
 *
 * The library implements the migration hot path of 10Cache (arXiv 2511.14124):
 * a profiled tensor-access order (Sec. 3.2) drives size-class buffer pools in
 * HBM and pinned host memory (Sec. 3.3.1, Alg. 1-2), an execution-order tensor
 * placement over GPU / CPU / NVMe (Sec. 3.3.2), and a hook-driven
 * prefetch-eviction scheduler (Sec. 3.4, Alg. 3-4) whose decisions run in a
 * GPU kernel and whose copies run in a batched GPU migration kernel.
 *
 * Conventions
 *   - Every call returns TC_OK (0) or a negative TC_E_* code.  Nothing throws
 *     or aborts across this boundary.  tc_strerror() names a code;
 *     tc_last_error() gives the detail text of the context's last failure.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP
 *     device memory; "pinned" pointers are page-locked host memory mapped into
 *     the GPU (hipHostMalloc, or a pin_memory tensor).
 *   - Inputs are caller-owned and copied during the call.  Outputs are
 *     caller-allocated plain structs.  The HBM region, the pinned region, the
 *     staging region, the file descriptor and the streams are caller-owned and
 *     must outlive the context.
 *   - A context serves one GPU and is not thread-safe; calls on one context
 *     must not overlap.
 *   - Call order: tc_create, tc_profile_order, tc_plan_pools,
 *     tc_plan_schedule, tc_bind_memory, then tc_load_tensor / tc_fill_payload,
 *     then per step tc_migrate_step(PRE), (the module's kernels),
 *     tc_migrate_step(POST), and tc_end_iteration after the last step.  A call
 *     made out of order returns TC_E_STATE.
 */
#ifndef TC_H
#define TC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- return codes ---- */
#define TC_OK          0
#define TC_E_ARG      (-1)   /* bad argument (null pointer, id out of range, unordered events, ...) */
#define TC_E_STATE    (-2)   /* call made out of order */
#define TC_E_CAPACITY (-3)   /* a budget, region or limit is too small */
#define TC_E_IO       (-4)   /* file-tier read/write failed or was short */
#define TC_E_HIP      (-5)   /* a HIP runtime call failed */

/* ---- tiers, phases, op codes (values are part of the ABI) ---- */
#define TC_GPU  0
#define TC_CPU  1
#define TC_NVME 2

#define TC_PRE      0   /* pre-hook: residency check + demand fetch */
#define TC_POST     1   /* post-hook: Alg. 3 over the tensors that finished */
#define TC_END      2   /* end of iteration, first two calls: GPU-final tensors return, from host buffers and then from the file tier */
#define TC_END_CPU  3   /* end of iteration, third call: CPU-final tensors return from the file tier */

#define TC_OP_DEMAND    0   /* miss: tensor fetched into a GPU buffer by the pre-hook */
#define TC_OP_PREFETCH  1   /* tensor fetched ahead of use (Alg. 3), or returned home at iteration end */
#define TC_OP_EVICT     2   /* GPU buffer -> CPU buffer (Alg. 4) */
#define TC_OP_RELEASE   3   /* NVMe-final tensor, clean: GPU buffer freed, no bytes move */
#define TC_OP_WRITEBACK 4   /* GPU buffer -> file extent */
#define TC_OP_SPILL     5   /* CPU buffer -> file extent, to make room (Alg. 4) */
#define TC_OP_RESTORE   6   /* file extent -> CPU buffer at iteration end */
#define TC_OP_FAIL      7   /* access that could not be given a GPU buffer */
#define TC_OP_ALLOC     8   /* TC_ALLOC_WRITE_ONLY: a tensor about to be written whole is given its GPU buffer, no bytes move */

#define TC_R 1
#define TC_W 2

#define TC_NONE 0xFFFFFFFFu          /* "no slot" / "never" */
#define TC_MAX_STEP_TENSORS 64       /* most tensors one hook call may name (the lanes of the wavefront that decides it) */
#define TC_MAX_STEPS (1u << 28)      /* step indices of a profile are below this (tables are sized by the last one) */

/* tc_budget.flags */
#define TC_LITERAL_ALG2 1u           /* Alg. 2 exactly as printed: no per-step working-set floor */
#define TC_NO_PREFETCH  2u           /* the paper's base variant (Sec. 4.1.4, the one that does not prefetch): post-hook
                                        calls move nothing, tensors arrive by the pre-hook's demand fetch alone */

#define TC_SMALLEST_FIRST 4u         /* not the paper's allocator but the placement it argues against (Sec. 3.1, Sec. 3.3.2:
                                        tensors placed by size, the large ones below the GPU wherever they stand in the
                                        execution order), as an ablation of tc_plan_pools: beyond the working-set floor, GPU
                                        memory goes to the size classes in ascending size, each taking as many buffers
                                        as it has tensors and the memory left allows */

#define TC_ALLOC_WRITE_ONLY 8u       /* a refinement the paper does not have: an access that only writes (TC_W without
                                        TC_R: a gradient in the backward pass, a checkpoint in the forward pass, the
                                        16-bit parameter in the optimizer sweep) is declared a whole-tensor write, so
                                        what the tensor held is dead.  Where Alg. 3 would prefetch such a tensor (its
                                        profiled row only writes) or the pre-hook would fetch it on demand, it is given
                                        its GPU buffer and no bytes are copied (TC_OP_ALLOC); every decision is what it
                                        is without the flag.  The caller's kernels must then really write the whole
                                        tensor: until they do its bytes are unspecified, and on a replay that leaves
                                        the profile the write may never come (tc_stats.undefined_reads counts reads of
                                        such tensors).  tc_emulate_compute fills a tensor written this way with the
                                        counter pattern of seed 0x10000000 + 4096 * iteration + step. */

/* tc_bind_memory flags */
#define TC_BIND_NULL_MOVER 1u        /* decide and log only; no region needed, no byte moves */
#define TC_BIND_FILE_DIRECT 2u       /* file_fd was opened with O_DIRECT: all file I/O is 4 KiB aligned */
#define TC_BIND_HOST_TIER 4u         /* two tiers, host memory over the file: see tc_bind_memory */

typedef struct tc_ctx tc_ctx;        /* opaque, library-owned */

/* One tensor.  group: 0 = 16-bit (parameter, gradient, checkpoint), 1 = fp32
 * optimizer state; it selects the host budget and separates size classes
 * (Sec. 3.3.1 Step 2 sizes the two kinds in separate runs).  kind is carried
 * through untouched. */
typedef struct {
    uint64_t bytes;                  /* >= 16 */
    uint8_t  group;
    uint8_t  kind;
    uint8_t  pad_[6];
} tc_tensor_desc;

/* One access of the profiled iteration (Sec. 3.2.1: execution order and
 * activation time recorded by the module hooks). */
typedef struct {
    uint32_t step;                   /* non-decreasing over the array */
    uint32_t tensor;
    uint64_t compute_ns;             /* modelled compute time of the step (kept, not used by decisions) */
    uint8_t  rw;                     /* TC_R, TC_W or both */
    uint8_t  pad_[7];
} tc_event;

typedef struct {
    uint64_t hbm_bytes;              /* GPU cache budget ("gpu_avl_mem" of Alg. 2) */
    uint64_t host_bytes[2];          /* pinned-host budget per group ("cpu_avl_mem") */
    uint32_t align;                  /* buffer stride granularity, power of two, >= 16 (default 256 if 0) */
    uint32_t flags;
} tc_budget;

/* One size class of the pool plan (Alg. 2 + Step 3 of Sec. 3.3.1). */
typedef struct {
    uint64_t bytes;                  /* tensor size of the class */
    uint64_t stride;                 /* buffer size: bytes rounded up to align */
    uint64_t hbm_off;                /* offset of buffer 0 in the HBM region */
    uint64_t host_off;               /* offset of buffer 0 in the pinned region */
    uint32_t group;
    uint32_t count;                  /* tensors of the class (c_s) */
    uint32_t used;                   /* tensors of the class seen by the profiled iteration */
    uint32_t step_max;               /* most tensors of the class one step uses */
    uint32_t gpu_count;              /* GPU_BUFFER_COUNT */
    uint32_t cpu_count;              /* CPU_BUFFER_COUNT */
} tc_pool_class;

typedef struct {
    uint32_t n_classes;
    uint32_t n_rows;                 /* rows of the prefetch table */
    uint32_t n_steps;
    uint32_t pad_;
    uint64_t hbm_total;              /* bytes of the HBM region the plan needs */
    uint64_t host_total;             /* bytes of the pinned region the plan needs */
    uint64_t file_total;             /* bytes of the file tier (every tensor owns an extent) */
} tc_pool_plan;

typedef struct {
    uint64_t file_off;               /* tensor's extent in the file tier, 4 KiB aligned */
    uint32_t cls;                    /* size class index (classes ascending by bytes, then group) */
    uint32_t slot;                   /* buffer index within the class on its final tier, TC_NONE for NVMe */
    uint32_t first_use;              /* first row using the tensor, TC_NONE if never used */
    uint8_t  final_tier;             /* TC_GPU / TC_CPU / TC_NVME: the "final location" of Sec. 3.2.1 */
    uint8_t  pad_[3];
} tc_placement;

/* One record of the op log: the schedule, in decision order. */
typedef struct {
    uint32_t iteration;
    uint32_t step;                   /* n_steps for the end-of-iteration calls */
    uint32_t tensor;
    uint32_t src_slot;               /* buffer index within the class, TC_NONE for the file tier */
    uint32_t dst_slot;
    uint8_t  phase;                  /* TC_PRE .. TC_END_CPU */
    uint8_t  op;                     /* TC_OP_* */
    uint8_t  src_tier;
    uint8_t  dst_tier;
    uint64_t bytes;                  /* bytes moved (0 for RELEASE and FAIL) */
} tc_op;

typedef struct {
    uint64_t hits, misses, fails;    /* GPU cache hit / miss counts of pre-hook accesses (Sec. 4.3) */
    uint64_t n_ops[8];               /* per TC_OP_* */
    uint64_t bytes_h2d;              /* bytes copied into HBM (from pinned buffers or file staging) */
    uint64_t bytes_d2h;              /* bytes copied HBM -> pinned buffers */
    uint64_t bytes_file_read, bytes_file_write;
    uint64_t file_read_ns, file_write_ns;     /* host time inside file-tier reads / writes */
    uint64_t mover_launches;         /* migration-kernel launches */
    uint64_t mover_units;            /* exchange units those launches carried */
    uint64_t dma_copies;             /* DMA-engine copies (large tensors) */
    uint64_t decide_launches;        /* decision-kernel launches */
    uint64_t hbm_budget, hbm_pool_bytes;      /* GPU memory offered to / taken by the buffer pools (utilisation, Sec. 4.5) */
    uint64_t host_budget, host_pool_bytes;    /* the same for pinned host memory, both groups together */
    uint64_t stall_ns;               /* time modules waited for their tensors (tc_set_stall_measurement) */
    uint64_t waits_under_30us, waits_total;   /* tensors that waited < 0.03 ms / tensors measured (Sec. 4.2.2) */
    uint64_t waits_under_10us, waits_under_100us;   /* the other two thresholds of Sec. 4.2.2 (0.01 ms, 0.1 ms) */
    uint32_t cursor;                 /* prefetch-table cursor */
    uint32_t iteration;
    uint64_t n_alloc;                /* TC_OP_ALLOC records: fetches left out because the tensor was about to be overwritten */
    uint64_t bytes_not_fetched;      /* ... and the bytes they would have copied into HBM */
    uint64_t undefined_reads;        /* accesses with TC_R to a tensor allocated without fetch and not yet written */
    /* time the calling thread spent blocked inside hook calls, by what it waited for: [0] a file read that
     * had not finished when the copy of its bytes was due, [1] a queued file write that still read the host
     * buffer a copy was about to overwrite, [2] room in the staging ring (its oldest block's copies and
     * write), [3] a copy operation (a buffer a spill or a restore needs, a bounce block, an event to reuse) */
    uint64_t host_blocked_ns[4];
} tc_stats;

const char *tc_strerror(int code);
const char *tc_last_error(const tc_ctx *ctx);

int tc_create(tc_ctx **out);
int tc_destroy(tc_ctx *ctx);

/* Sec. 3.2 (tensor characteristic analyzer).  Builds the prefetch table from
 * one profiled iteration: rows in execution order (a tensor named twice by one
 * step is one row), per-tensor use lists, the size->count dictionary TC and the
 * per-class per-step maximum.  t, ev: host arrays.  TC_E_ARG for events not
 * ordered by step, a step index of TC_MAX_STEPS or more, an unknown tensor, a
 * tensor under 16 bytes, a group other than 0 or 1, rw outside TC_R|TC_W;
 * TC_E_CAPACITY if the host has no memory for the tables. */
int tc_profile_order(tc_ctx *ctx, const tc_tensor_desc *t, uint32_t n_tensors,
                     const tc_event *ev, uint64_t n_events);

/* Sec. 3.3.1 (cache allocator): Alg. 1 (size distribution), Alg. 2 (buffer
 * counts, exact integer arithmetic, rounded down) and Step 3 (one contiguous
 * region per tier cut into per-class chunks, classes ascending).  Unless
 * TC_LITERAL_ALG2 is set every class first gets step_max buffers and Alg. 2
 * divides the rest.  TC_E_CAPACITY if that floor exceeds hbm_bytes.
 * classes_out: host array of at least the number of distinct (bytes, group)
 * pairs (n_classes_cap entries; TC_E_CAPACITY if too few), may be NULL. */
int tc_plan_pools(tc_ctx *ctx, const tc_budget *b, tc_pool_plan *plan_out,
                  tc_pool_class *classes_out, uint32_t n_classes_cap);

/* Sec. 3.3.2 (tensor allocator): in execution order every tensor takes the
 * fastest tier with a free buffer of its class, GPU then CPU then NVMe, lowest
 * buffer first.  out: host array of n_tensors entries, may be NULL. */
int tc_plan_schedule(tc_ctx *ctx, tc_placement *out);

/* Hands the library its memory and builds the device-side tables.
 *   hbm_region     device, >= plan.hbm_total bytes, 256-byte aligned
 *   pinned_region  pinned, >= plan.host_total bytes, 256-byte aligned
 *   staging        pinned bounce buffer for the file tier (may be NULL with
 *                  staging_bytes 0 if no tensor ever touches the file tier;
 *                  otherwise at least twice the largest tensor).  It is used
 *                  as a ring: the deeper it is, the more file reads, copies
 *                  and file writes of successive hook calls overlap (eight
 *                  times the largest tensor is a good size).
 *   file_fd        open read/write file of >= plan.file_total bytes, or -1.
 *                  With TC_BIND_FILE_DIRECT (a file opened with O_DIRECT, to
 *                  bypass the page cache) every request is 4 KiB aligned in
 *                  memory, offset and length and goes through a page-aligned
 *                  bounce block of the library's own (direct I/O cannot
 *                  target GPU-mapped pinned memory); staging must then be
 *                  4 KiB aligned and sized.  Unless tc_set_io_threads /
 *                  tc_set_io_chunk were called before, a direct file is served
 *                  by two threads per direction with one request per tensor
 *                  (few large sequential requests suit a device; many small
 *                  ones suit the page cache).  File reads and writes are
 *                  queued to worker threads of the library's own
 *                  (tc_set_io_threads); writes have reached the file when
 *                  tc_synchronize returns.  A failed request is reported
 *                  (TC_E_IO) by the next call that queues or waits for one.
 *   migrate_stream hipStream_t the copies are issued on (default priority)
 * With TC_BIND_NULL_MOVER no bytes move and the regions may be NULL: the
 * decision kernel still runs and the op log, stats and state are exact.
 *
 * With TC_BIND_HOST_TIER the cache is the one the paper keeps for optimizer
 * states (Sec. 3.4.2, optimizer states scheduling policy): the fast tier is
 * host memory, the slow tier the file, and the same scheduler evicts an
 * updated state and prefetches the next one behind the CPU's update.  The plan
 * must have been made with both host budgets 0 (the budget called hbm_bytes is
 * then the host cache's); hbm_region must be pinned HOST memory of
 * plan.hbm_total bytes; pinned_region and staging are not used (staging only
 * by tc_fill_payload).  Tensors move between the region and the file directly,
 * by the I/O worker threads: no copy kernel runs.  A write-back waits for what
 * the compute stream holds at the POST call, a fetch for what it holds when
 * the fetch is decided; a PRE call returns host pointers once the tensors'
 * bytes have arrived, and the time it had to block is the stall that
 * tc_cache_stats reports (bytes_h2d counts the bytes fetched into the host
 * cache).  Decisions, op log and state are those of the three-tier mode with
 * no host buffers. */
int tc_bind_memory(tc_ctx *ctx, void *hbm_region, uint64_t hbm_bytes,
                   void *pinned_region, uint64_t pinned_bytes,
                   void *staging, uint64_t staging_bytes,
                   int file_fd, void *migrate_stream, uint32_t flags);

/* Copies a tensor's initial bytes (host pointer, tensor's size) into its
 * final location.  Synchronous. */
int tc_load_tensor(tc_ctx *ctx, uint32_t tensor, const void *src);

/* Fills every tensor, where it lives, with the counter pattern
 * word(i) = h(i*0x9E3779B1 + tensor*0x85EBCA77 + seed*0xC2B2AE3D mod 2^32),
 * h = x^=x>>16; x*=0x7FEB352D; x^=x>>15; x*=0x846CA68B; x^=x>>16 (32-bit
 * words, little endian), using a fill kernel.  Synchronous. */
int tc_fill_payload(tc_ctx *ctx, uint32_t seed);

/* Copies a tensor's current bytes, from whichever tier holds it, to dst
 * (host pointer).  Waits for outstanding copies first. */
int tc_read_tensor(tc_ctx *ctx, uint32_t tensor, void *dst);

/* One hook call (Sec. 3.2.1, Sec. 3.4).
 *   TC_PRE : every listed tensor must be in a GPU buffer before the module
 *            runs.  Resident -> hit.  Otherwise a miss: demand fetch.
 *            dev_ptrs_out (host array of n pointers, may be NULL) receives the
 *            device address of each tensor's GPU buffer (NULL for a failed
 *            access), valid until the same step's POST.  compute_stream is
 *            made to wait for the copies that fill those buffers.
 *   TC_POST: Alg. 3 over the listed (finished) tensors: per tensor at most one
 *            eviction (Alg. 4) paired with one prefetch of the next row of the
 *            prefetch table that is not resident.  The copies wait for the
 *            work already enqueued on compute_stream.
 * ids, rw: host arrays of n <= TC_MAX_STEP_TENSORS entries (rw may be NULL
 * for POST).  step indexes the profiled iteration, which ends with its last
 * step that used a tensor (a call with n = 0 may name a later step: a module
 * without tensors; it moves nothing).  Decisions are made by a
 * GPU kernel; the call returns once they are known and the copies are
 * enqueued, not when the copies finish. */
int tc_migrate_step(tc_ctx *ctx, uint32_t step, int phase,
                    const uint32_t *ids, const uint8_t *rw, uint32_t n,
                    void *compute_stream, void **dev_ptrs_out);

/* End of an iteration (Sec. 3.2.1): every tensor goes back to its final location,
 * the cursor returns to row 0.  Every displaced tensor moves exactly once and no
 * other tensor moves: GPU-final tensors return from host buffers first (swapping
 * places with the guests in their class), then GPU-final tensors return from the
 * file tier, then CPU-final tensors return from the file tier; nothing is
 * spilled on the way. */
int tc_end_iteration(tc_ctx *ctx, void *compute_stream);

/* Stand-in for the module's kernels in a replay: on compute_stream, XORs the
 * 16-byte stamp (words 0x10CAC4E5, iteration, step, tensor; little endian)
 * into the first and the last 16 bytes of every tensor the last PRE call
 * listed with TC_W, then spins for busy_ns nanoseconds.  With
 * TC_ALLOC_WRITE_ONLY a tensor listed with TC_W alone is instead overwritten
 * whole with the counter pattern of tc_fill_payload, seed
 * 0x10000000 + 4096 * iteration + step. */
int tc_emulate_compute(tc_ctx *ctx, void *compute_stream, uint64_t busy_ns);

/* Wait-time measurement (Sec. 4.2.2).  While enabled, a PRE call drains
 * compute_stream, then waits on the host for the copy that fills each listed
 * tensor's buffer and records how long that took: stall_ns grows by the
 * longest wait of the call, waits_total by one per tensor, waits_under_30us
 * by one per tensor that waited less than 0.03 ms.  Decisions are unchanged;
 * the calls no longer overlap with the compute stream. */
int tc_set_stall_measurement(tc_ctx *ctx, int enable);

/* Where the wait time of Sec. 4.2.2 falls within the iteration: the stall each
 * profiled step's PRE calls have added to stall_ns since the context was bound
 * or the counts were last cleared, so that forward, backward and optimizer
 * steps can be told apart.  ns_out: host array of at least n_steps entries
 * (cap says how many it holds; TC_E_CAPACITY if fewer), may be NULL; clear:
 * reset the counts after copying them. */
int tc_stall_by_step(tc_ctx *ctx, uint64_t *ns_out, uint32_t cap, int clear);

/* Replays one whole iteration whose accesses are known up front: for every
 * step the pre-hook call, tc_emulate_compute, the post-hook call, then
 * tc_end_iteration.  step_ptr: n_steps+1 offsets into ids/rw, starting at 0
 * (host arrays); busy_ns: per-step modelled compute or NULL; measure_stall: enable
 * tc_set_stall_measurement for the duration of the call.  Decisions, op
 * log, statistics and bytes are those of the same sequence of
 * tc_migrate_step calls; the difference is that the decision kernel takes a
 * window of steps per launch (tc_set_replay_window) instead of one hook call,
 * which the scheduler allows because its decisions depend on the access
 * order and the tables only, never on when a copy finishes.  After an error
 * the context must be destroyed (the device tables may be ahead of the
 * copies issued). */
int tc_replay_iteration(tc_ctx *ctx, const uint32_t *step_ptr, const uint32_t *ids, const uint8_t *rw,
                        uint32_t n_steps, void *compute_stream, const uint64_t *busy_ns, int measure_stall);

/* Waits for every copy issued so far. */
int tc_synchronize(tc_ctx *ctx);

int tc_cache_stats(const tc_ctx *ctx, tc_stats *out);

/* Copies the op log from record `first` on: at most cap records into buf;
 * *n_total receives the log's length.  The log is kept on the host. */
int tc_dump_oplog(const tc_ctx *ctx, uint64_t first, tc_op *buf, uint64_t cap, uint64_t *n_total);

/* The op log grows by one 32-byte record per decision for as long as it is
 * enabled (it is at creation): a long run switches it off or clears it between
 * iterations.  enable: keep recording or not; clear: drop what is recorded. */
int tc_set_oplog(tc_ctx *ctx, int enable, int clear);

/* Current tier and buffer of every tensor (host arrays of n_tensors entries;
 * any may be NULL).  Reads the device tables; synchronises the decision stream. */
int tc_dump_state(tc_ctx *ctx, uint8_t *tier, uint32_t *gpu_slot, uint32_t *cpu_slot);

/* Migration-kernel tuning.  workgroups: how many workgroups of 256 lanes move
 * data (0 = default 12, at most 8192); they all run on one XCD, the launch
 * itself has as many times more as the GPU has XCDs (probed once per device)
 * and those dealt to other XCDs exit at once.
 * chunk_bytes: the piece of work a workgroup takes from the launch's ticket
 * counter at a time (0 = default 16 KiB; a multiple of 4096). */
int tc_set_mover(tc_ctx *ctx, uint32_t workgroups, uint32_t chunk_bytes);

/* Measures the number of working workgroups instead of assuming it: a few
 * exchange launches of up to 64 MiB between the bound HBM and pinned regions
 * for each of 8..24 workgroups (about 30 ms in all), the fastest becomes the
 * setting and is returned in *workgroups_out (may be NULL).  The optimum sits
 * at a knee that depends on the host (too few workgroups leave the link idle,
 * too many crowd each other out).  Only between tc_bind_memory and the first
 * tensor loaded or hook call made, while the regions hold nothing: their
 * contents are overwritten (TC_E_STATE afterwards).  Regions under 4 MiB are
 * left alone and the current setting is returned. */
int tc_tune_mover(tc_ctx *ctx, uint32_t *workgroups_out);

/* File-tier I/O runs behind the calling thread.  Writes (Sec. 3.4.2: dirty
 * tensors leaving for NVMe; Alg. 4: a host buffer spilled to make room) go to
 * `writers` threads, reads into staging (a fetch from the file tier) to
 * `readers` threads (0..8 each; default 4 and 4).  An extent is cut into
 * chunks (tc_set_io_chunk); chunk i of tensor t belongs to lane t + i, and the lane picks the
 * worker, so one large request spreads over the threads while a given chunk
 * always goes to the same writer: writes of one extent keep their order.  A
 * read of an extent names the write queued for it, and its reader starts only
 * once that write has finished (the calling thread does not wait for it).
 * A copy whose bytes are still on their way from the file is launched by the
 * first later call that finds the read finished, at the latest by the call
 * that needs one of its buffers (which then waits).  0 = that kind of I/O runs
 * in the calling thread.  On a bound context the call first waits for
 * everything in flight. */
int tc_set_io_threads(tc_ctx *ctx, uint32_t writers, uint32_t readers);

/* Bytes per chunk of an extent (a multiple of 4096, at least 64 KiB; default
 * 8 MiB): the size of one request to the file system and the unit of striping.
 * Only before the first request to the file tier (TC_E_STATE afterwards). */
int tc_set_io_chunk(tc_ctx *ctx, uint64_t bytes);

/* Stripes the file tier over one more file (at most 8 in all, the first being
 * tc_bind_memory's file_fd): with n files the chunk of lane l lives in file
 * l mod n, at the offset it would have in a single file, so every file must
 * allow offsets up to plan.file_total (files may be sparse) and be opened the
 * way file_fd was (O_DIRECT or not).  Several files let buffered writes, which
 * a file system serialises per file, and several devices work in parallel.
 * Only before the first request to the file tier (TC_E_STATE afterwards); the
 * descriptor stays the caller's. */
int tc_add_stripe(tc_ctx *ctx, int fd);

/* tc_migrate_step decides ahead: a training loop repeats the profiled iteration
 * (Sec. 3.2.1), so instead of one decision launch and one wait per hook call the
 * library decides windows of `steps` profiled steps per launch (the next window
 * while the current one is handed out) and a call that is the profile's next one
 * just takes its result.  A call that is not (another step, other tensors, other
 * R/W flags) is still decided exactly: the tables return to their state before
 * the window, the calls already handed out are decided again, and the call gets
 * a launch of its own; results never depend on this setting.  0 = one launch per
 * call; default 16; at most 256. */
int tc_set_decide_ahead(tc_ctx *ctx, uint32_t steps);

/* While a migration launch is still running, the copies of further hook calls
 * are held back and merged into one launch, until `bytes` bytes are prepared,
 * a prepared buffer is needed, or the file tier is involved; when the
 * migration stream is idle they are issued at once.  0 = one launch per hook
 * call.  Default 256 MiB. */
int tc_set_merge_bytes(tc_ctx *ctx, uint64_t bytes);

/* Steps decided per decision-kernel launch by tc_replay_iteration, 1 .. 256
 * (default 64).  Each launch the host waits for interrupts a running
 * migration launch for some microseconds. */
int tc_set_replay_window(tc_ctx *ctx, uint32_t steps);

/* Tensors of at least `bytes` bytes move as DMA-engine copies (hipMemcpyAsync
 * on two side streams, one per direction), smaller ones in the migration
 * kernel's batched launch.  0 (default) = everything in the kernel; setting 0
 * after another value waits for the copies in flight and gives the side
 * streams and the bounce block back. */
int tc_set_dma_threshold(tc_ctx *ctx, uint64_t bytes);

/* Dependencies between module kernels and migration launches resolved on the
 * GPU instead of by events between the two streams (a wait across hardware
 * queues takes about 17 us on this hardware, twice per launch where launches
 * and modules alternate).  enable != 0: a hook call that prepares copies
 * queues a one-lane kernel on its compute stream that raises a sequence word
 * behind the modules queued so far; the migration launch is queued at once and
 * its workgroups wait for that word themselves; a one-lane kernel queued
 * behind every launch on the migration stream raises a second word to the
 * launch's number, and a module that needs what a launch brings is preceded
 * on its stream by a one-lane kernel that waits for that number.
 * Every such wait is bounded by timeout_ms (0 = 5000): a waiter that gives up
 * moves nothing, and the next hook call or tc_synchronize returns TC_E_HIP; the
 * bytes are then not to be trusted and the context should be destroyed.  Use
 * it where every module's kernels finish well within the timeout and the
 * compute stream and the migration stream run on different hardware queues
 * (two streams of one process normally do).  With the modules on the migration
 * stream itself nothing changes (that stream is in order).  A launch that
 * waits on the GPU has at most 32 working workgroups whatever tc_set_mover
 * says: workgroups that wait hold their places on the XCD they run on, and
 * must leave room there for the one-workgroup kernel that ends their wait.
 * Not for modules that compute for milliseconds: a launch that waits keeps
 * its dozen workgroups resident (and polling) on one XCD for as long as the
 * modules before it run, which slows those modules (measured on a training
 * step of 87 ms: 164 ms through the cache with this setting against 133
 * without).  Decisions and bytes never depend on the setting.  The call waits
 * for the copies in flight.  Default: off. */
int tc_set_gpu_dependencies(tc_ctx *ctx, int enable, uint32_t timeout_ms);

/* When the tensors above the DMA threshold take the DMA engines: always
 * (when_behind = 0, the default), or only while there is compute to hide them
 * behind (when_behind = 1): the compute stream has not yet reached one of the
 * last few points at which copies were issued, and no copies issued at a point
 * it has passed are still unfinished (that would mean the step waits for the
 * link).  The kernel is faster on the link, but its reads of host memory slow
 * compute that runs beside it, which DMA copies hardly do.  Decisions and
 * bytes never depend on the path taken. */
int tc_set_dma_policy(tc_ctx *ctx, int when_behind);

/* Time spent inside migration work since the last call, measured with HIP
 * events on the stream each piece ran on.  Only work issued while timing is
 * enabled is counted. */
typedef struct {
    double   kernel_ns;              /* sum of migration-kernel launch durations */
    uint64_t kernel_launches;
    uint64_t kernel_bytes;           /* bytes those launches moved (both directions, incl. HBM staging copies) */
    double   h2d_ns;                 /* sum of host->HBM DMA copy durations */
    uint64_t h2d_copies;
    uint64_t h2d_bytes;
    double   d2h_ns;                 /* sum of HBM->host DMA copy durations */
    uint64_t d2h_copies;
    uint64_t d2h_bytes;
    double   decide_ns;              /* sum of decision-kernel launch durations */
    uint64_t decide_launches;
    uint64_t decide_calls;           /* hook calls those launches decided */
} tc_timing;
int tc_mover_timing(tc_ctx *ctx, int enable, tc_timing *out);

/* ---- stand-alone kernels ---- */

/* One segment of a pack / unpack / copy batch. */
typedef struct {
    const void *src;
    void       *dst;
    uint64_t    bytes;
} tc_segment;

/* Batched copy: one launch per 48 segments moves them all (device or pinned
 * pointers, 16-byte aligned, any size).  segs: host array, copied.
 * Asynchronous on stream; the kernel's ticket counters come from and go back
 * to the stream-ordered allocator (hipMallocAsync / hipFreeAsync).
 * workgroups, chunk_bytes: as for tc_set_mover. */
int tc_copy_batch(const tc_segment *segs, uint32_t n, void *stream,
                  uint32_t workgroups, uint32_t chunk_bytes);

/* Batched exchange: unit i copies out[i] and in[i] (same byte count, either
 * may have bytes == 0 to leave that half out) with the ordering guarantee of
 * the migration kernel: every 16-byte piece of both sources is read before
 * either destination piece is written, so out[i].src may equal in[i].dst (a
 * tensor leaves a buffer while another arrives) and out[i].dst may equal
 * in[i].src (a swap).  Pointers 16-byte aligned.  Asynchronous on stream. */
int tc_exchange_batch(const tc_segment *out, const tc_segment *in, uint32_t n, void *stream,
                      uint32_t workgroups, uint32_t chunk_bytes);

/* Pack: gathers n small tensors (device pointers, any alignment, any size)
 * into one contiguous device slab, segment i at slab_off[i]; unpack is the
 * reverse.  Segments must be sorted by slab_off and must not overlap; bytes of
 * the slab (pack) or of a tensor (unpack) that no segment covers are not
 * written.  The slab is processed in 16 KiB tiles, one workgroup each.  A tile
 * that at most 256 segments reach into moves register to register, 128 bits
 * per request with all its loads in flight at once: aligned on the slab side,
 * at whatever address the tensor has on the other (bytes at segment edges that
 * fill no whole 16-byte vector of the slab move bytewise).  A tile of more,
 * tinier segments is staged in LDS so that the slab side still moves 128 bits
 * per request.
 *   slab        device, 16-byte aligned, total_bytes long
 *   ptrs, bytes, slab_off   device arrays of n entries
 *   tile_first  device array of tc_pack_tiles(total_bytes) entries written by
 *               tc_pack_index for this slab_off / total_bytes, or NULL (each
 *               workgroup then bisects slab_off itself: correct but slower).
 *               A layout that repeats every iteration is indexed once.
 * All three calls are asynchronous on stream and allocate nothing. */
uint64_t tc_pack_tiles(uint64_t total_bytes);
int tc_pack_index(const uint64_t *slab_off, uint32_t n, uint64_t total_bytes, uint32_t *tile_first, void *stream);
int tc_pack(void *slab, const void *const *ptrs, const uint64_t *bytes,
            const uint64_t *slab_off, uint32_t n, uint64_t total_bytes, const uint32_t *tile_first, void *stream);
int tc_unpack(const void *slab, void *const *ptrs, const uint64_t *bytes,
              const uint64_t *slab_off, uint32_t n, uint64_t total_bytes, const uint32_t *tile_first, void *stream);

/* Pack (unpack = 0) or unpack (unpack != 0) for callers that cannot allocate
 * and have no workspace to bring: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same kernels as tc_pack /
 * tc_unpack with an index, but the tile index is rebuilt by every call in a
 * device array of the library's own (1 MiB per GPU, held until the process
 * ends), so the call takes no tile_first and calls no allocator of any kind.
 * The array bounds the slab: total_bytes above TC_PACK_STATIC_MAX_BYTES is
 * refused with TC_E_CAPACITY and nothing is launched.  All arguments as for
 * tc_pack.  Asynchronous on stream.  Every call on a GPU uses that GPU's one
 * array: calls that may overlap on one GPU (different streams or threads)
 * race on it and must be ordered by the caller. */
#define TC_PACK_STATIC_MAX_BYTES (4ull << 30)
int tc_pack_static(void *slab, const void *const *ptrs, const uint64_t *bytes, const uint64_t *slab_off,
                   uint32_t n, uint64_t total_bytes, int unpack, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TC_H */
