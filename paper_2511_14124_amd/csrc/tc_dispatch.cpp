// Dispatch of libtc.so: copy operations (ids, events, dependencies between the
// streams), the bounce and staging rings, and the per-hook dispatch that turns
// the decision kernel's op records into migration-kernel launches, DMA copies
// and file-tier I/O.
#include "tc_ctx.h"

#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <chrono>

// ---- copy operations: ids, events, dependencies -----------------------------
// Every kernel launch and every DMA copy is one operation with an id and an
// event in a ring.  A stream is in order, so per stream it is enough to know the
// newest operation seen complete.  An id older than the ring has completed by
// construction: begin_op waits for the operation whose event it recycles.

// block the host until operation `id` has completed
int wait_op(tc_ctx *c, uint64_t id)
{
    if (op_complete(c, id)) return TC_OK;
    const uint32_t st = c->op_stream[id % OP_RING];
    HIP_TRY(c, hipEventSynchronize(c->op_ev[id % OP_RING]));
    c->op_done[st] = std::max(c->op_done[st], id);
    return TC_OK;
}

int tc_wait_op(tc_ctx *c, uint64_t id) { return wait_op(c, id); }

// has operation `id` completed?  (asks the runtime, without blocking)
static bool poll_op(tc_ctx *c, uint64_t id)
{
    if (op_complete(c, id)) return true;
    if (hipEventQuery(c->op_ev[id % OP_RING]) != hipSuccess) return false;
    const uint32_t st = c->op_stream[id % OP_RING];
    c->op_done[st] = std::max(c->op_done[st], id);
    return true;
}

// make stream S wait for operation `id` (nothing to do if it ran on S or is done)
static int dep(tc_ctx *c, int S, uint64_t id)
{
    if (op_complete(c, id) || c->op_stream[id % OP_RING] == S) return TC_OK;
    HIP_TRY(c, hipStreamWaitEvent(c->streams[S], c->op_ev[id % OP_RING], 0));
    return TC_OK;
}

// start an operation on stream S: the first one of a hook call on that stream
// makes the stream wait for the work already queued on the compute stream
// (wait_compute false: the operation waits for the modules it depends on by itself)
static int begin_op(tc_ctx *c, int S, hipStream_t compute, uint64_t *id, bool wait_compute = true)
{
    const uint64_t n = c->op_id + 1;
    if (n > OP_RING) {
        Blocked b(c, BLK_COPY);
        int rc = wait_op(c, n - OP_RING);              // the event about to be reused
        if (rc != TC_OK) return rc;
    }
    c->op_lseq[n % OP_RING] = 0;
    if (c->streams[S] == compute) c->stream_waited[S] = true;    // one queue, in order: nothing to wait for
    if (wait_compute && !c->stream_waited[S]) {
        if (!c->compute_recorded) {
            HIP_TRY(c, hipEventRecord(c->ev_compute, compute));
            c->compute_recorded = true;
        }
        HIP_TRY(c, hipStreamWaitEvent(c->streams[S], c->ev_compute, 0));
        c->stream_waited[S] = true;
    }
    *id = n;
    return TC_OK;
}

static int end_op(tc_ctx *c, int S, uint64_t id)
{
    c->op_stream[id % OP_RING] = (uint8_t)S;
    c->op_id = id;
    HIP_TRY(c, hipEventRecord(c->op_ev[id % OP_RING], c->streams[S]));
    return TC_OK;
}

static inline hipStream_t kind_stream(tc_ctx *c, int kind) { return kind == K_DECIDE ? c->dstream : c->streams[kind]; }

int timed_begin(tc_ctx *c, int kind, hipEvent_t *t0)
{
    *t0 = nullptr;
    if (!c->timing) return TC_OK;
    HIP_TRY(c, hipEventCreate(t0));
    HIP_TRY(c, hipEventRecord(*t0, kind_stream(c, kind)));
    return TC_OK;
}

int timed_end(tc_ctx *c, int kind, hipEvent_t t0, uint64_t bytes)
{
    if (!t0) return TC_OK;
    hipEvent_t t1;
    HIP_TRY(c, hipEventCreate(&t1));
    HIP_TRY(c, hipEventRecord(t1, kind_stream(c, kind)));
    c->timed.push_back(Timed{t0, t1, kind, bytes});
    return TC_OK;
}

// File-tier I/O.  With an O_DIRECT file every request must be 4 KiB aligned in
// memory, offset and length: extents are 4 KiB aligned and sized, so a length
// rounded up stays inside the tensor's own extent, and the memory side is the
// bounce block.


// ---------------------------------------------------------------------------
// dispatch: op records -> migration-kernel launches, DMA copies and file I/O
//
// A hook call's records are grouped into exchange units (an optional outgoing
// copy that leaves a GPU buffer and the incoming copy that fills it).  By
// default every unit, whatever its size, goes into a migration-kernel launch on
// stream K: per-copy overhead would dominate the small ones, the kernel's
// load-load-store-store order lets a unit swap two buffers in place, and with
// both directions loaded the kernel carries the large ones as fast as two DMA
// engines do (49.7 against 48.6 GB/s per direction) without the bounce copy and
// the waits between three streams a swap by DMA copies needs.  What the
// DMA engines are good for is compute running beside the copies, which the
// kernel's host accesses slow down and DMA copies do not: with a DMA threshold
// set (tc_set_dma_threshold, tc_set_dma_policy) units at least that large take
// them, always or only while the compute stream has a backlog to hide them
// behind.  Such a unit's outgoing tensor is first copied inside HBM to a bounce
// block (a device-to-device copy on stream K), then the incoming tensor is
// copied into the GPU buffer on stream H and the outgoing one leaves the bounce
// block on stream D.  Ordering between streams comes from per-buffer tickets:
// each buffer remembers the last operation that touched it, and an operation
// waits for the tickets of the buffers it touches.
// ---------------------------------------------------------------------------
// a block of the HBM bounce ring, or nullptr if none can be had without
// waiting for a copy of the batch being prepared
static int bounce_alloc(tc_ctx *c, uint64_t bytes, uint8_t **out)
{
    *out = nullptr;
    const uint64_t need = (bytes + 255) & ~255ull;
    if (!c->bounce || need > c->bounce_bytes) return TC_OK;
    for (;;) {
        while (!c->bounce_q.empty() && c->bounce_q.front().op && op_complete(c, c->bounce_q.front().op))
            c->bounce_q.pop_front();
        if (c->bounce_q.empty()) c->bounce_head = 0;
        const uint64_t tail = c->bounce_q.empty() ? 0 : c->bounce_q.front().off;
        uint64_t at = UINT64_MAX;
        if (c->bounce_q.empty() || c->bounce_head > tail) {        // free: [head, end) and [0, tail)
            if (c->bounce_head + need <= c->bounce_bytes) at = c->bounce_head;
            else if (need <= tail && !c->bounce_q.empty()) at = 0;
        } else if (c->bounce_head < tail) {                        // free: [head, tail)
            if (c->bounce_head + need <= tail) at = c->bounce_head;
        }
        if (at != UINT64_MAX) {
            c->bounce_q.push_back(BounceBlock{at, need, 0});
            c->bounce_head = at + need;
            *out = c->bounce + at;
            return TC_OK;
        }
        if (c->bounce_q.front().op == 0) return TC_OK;             // held by this very batch: give up
        Blocked b(c, BLK_COPY);
        int rc = wait_op(c, c->bounce_q.front().op);               // oldest reader must finish first
        if (rc != TC_OK) return rc;
    }
}

static StBlock *st_find(tc_ctx *c, uint64_t id)
{
    for (StBlock &b : c->st_q)
        if (b.id == id) return &b;
    return nullptr;
}

// issue the prepared units of a hook call
static int issue_units(tc_ctx *c, std::vector<PUnit> &units, hipStream_t compute)
{
    if (units.empty()) return TC_OK;
    // a host buffer some unit is about to overwrite may still be the source of a queued
    // spill, and bytes coming from the file tier may still be on their way into staging
    for (PUnit &p : units) {
        int rc = TC_OK;
        if (p.cpu_out >= 0 && !io_done(c, c->cpu_job[(size_t)p.cpu_out])) {
            Blocked b(c, BLK_FILE_WRITE);
            rc = io_wait(c, c->cpu_job[(size_t)p.cpu_out]);
        }
        if (rc == TC_OK && !io_done(c, p.read_job)) {
            Blocked b(c, BLK_FILE_READ);
            rc = io_wait(c, p.read_job);
        }
        if (rc != TC_OK) return rc;
    }
    // DMA copies are slower on the link than the kernel but hardly slow compute that runs beside
    // them; the kernel's host reads do.  With the policy "when behind" the large units take the
    // DMA engines only while the compute stream still has not reached the point it was at when
    // units were last issued (a backlog to hide the copies behind), and the kernel otherwise
    // (nothing to hide behind: the step is the link's).
    bool dma_now = c->sdma_threshold != 0;
    tc_ctx::IssuePoint *point = nullptr;
    if (dma_now && c->dma_when_behind) {
        // Of the last few issue points: one the compute stream has passed while its copies are
        // still not done means the copies lag (the step is the link's: take the kernel); one the
        // compute stream has not reached yet means there is a backlog to hide DMA copies behind.
        bool copies_lag = false, compute_behind = false;
        for (auto &pt : c->issue_ring) {
            if (!pt.used) continue;
            const bool reached = hipEventQuery(pt.ev) == hipSuccess;
            (void)hipGetLastError();                        // "not ready" is an answer, not an error
            if (!reached) { compute_behind = true; continue; }
            if (poll_op(c, pt.op)) pt.used = false;         // both sides are past it
            else copies_lag = true;
        }
        dma_now = compute_behind && !copies_lag;
        point = &c->issue_ring[c->issue_next++ % 8];
        if (!point->ev) HIP_TRY(c, hipEventCreateWithFlags(&point->ev, hipEventDisableTiming));
        HIP_TRY(c, hipEventRecord(point->ev, compute));
        point->used = false;                                // until its newest copy is known (below)
    }
    struct Large { size_t unit; uint8_t *bounce; uint64_t kop; };
    std::vector<Large> large;
    std::vector<size_t> small;
    for (size_t i = 0; i < units.size(); ++i) {
        PUnit &p = units[i];
        bool dma = dma_now && p.u.bytes >= c->sdma_threshold && p.u.in_src;
        Large L{i, nullptr, 0};
        if (dma && p.u.out_src) {
            int rc = bounce_alloc(c, p.u.bytes, &L.bounce);
            if (rc != TC_OK) return rc;
            if (!L.bounce) dma = false;                            // no room: the kernel swaps it in place
        }
        if (dma) large.push_back(L); else small.push_back(i);
    }
    // ---- stream K: small units and the staging copies of large ones, at most TC_MOVER_MAX_UNITS per launch
    std::vector<std::pair<TcUnit, int64_t>> kunits;                // unit, index into `large` or -1-small
    for (size_t i : small) kunits.push_back({units[i].u, -1 - (int64_t)i});
    // the outgoing halves of the large units go to their bounce blocks as device-to-device
    // copies of the runtime, one operation for all of them: beside running compute these cost a
    // tenth of what the same copies cost as units of the migration kernel, whose dozen
    // workgroups stream HBM for milliseconds
    {
        bool any = false;
        for (const Large &L : large) any = any || L.bounce;
        if (any) {
            uint64_t id;
            int rc = begin_op(c, S_K, compute, &id);
            if (rc != TC_OK) return rc;
            for (Large &L : large) {
                if (!L.bounce) continue;
                const PUnit &p = units[L.unit];
                if ((rc = dep(c, S_K, c->gpu_ticket[(size_t)p.gpu_y])) != TC_OK) return rc;
                HIP_TRY(c, hipMemcpyAsync(L.bounce, p.u.out_src, p.u.bytes, hipMemcpyDeviceToDevice, c->streams[S_K]));
                L.kop = id;
            }
            if ((rc = end_op(c, S_K, id)) != TC_OK) return rc;
            for (Large &L : large)
                if (L.bounce) c->gpu_ticket[(size_t)units[L.unit].gpu_y] = id;
            c->last_k_op = id;
        }
    }
    for (size_t at = 0; at < kunits.size(); at += TC_MOVER_MAX_UNITS) {
        const size_t end = std::min(kunits.size(), at + (size_t)TC_MOVER_MAX_UNITS);
        TcMoverArgs args{};
        args.chunk_bytes = c->chunk_bytes;
        args.tickets = c->tickets;                          // (every launch of this context is on stream K, in order)
        args.xcc = c->mover_xcc;
        args.n_xcd = c->mover_xcds;
        uint64_t id, bytes = 0;
        // Dependencies resolved on the GPU: the launch is not made to wait for the compute stream; its
        // workgroups wait for the newest of the signals the calls that prepared its units have queued
        // there.  (Not with the modules on the migration stream itself, which is in order anyway, nor
        // for a unit without a signal or with one queued on another stream than this call's.)
        bool gate = c->gpu_deps && compute != c->streams[S_K] && c->sig_stream == compute;
        uint32_t need_sig = 0;
        for (size_t k = at; k < end && gate; ++k) {
            const PUnit &p = units[(size_t)(-1 - kunits[k].second)];
            if (p.sig == 0 || (int32_t)(c->sig_seq - p.sig) < 0) gate = false;
            else if (need_sig == 0 || (int32_t)(p.sig - need_sig) > 0) need_sig = p.sig;
        }
        int rc = begin_op(c, S_K, compute, &id, !gate);
        if (rc != TC_OK) return rc;
        uint32_t done_seq = 0;
        if (c->gpu_deps) {
            done_seq = ++c->launch_seq;
            if (gate) {
                args.fault = c->fault;
                args.gave_up = c->tickets + 35;
                args.spin_ticks = c->spin_ticks;
                args.progress = c->tickets + 32;
                args.need_seq = need_sig;
            }
        }
        for (size_t k = at; k < end; ++k) {
            TcUnit u = kunits[k].first;
            u.chunk0 = args.n_chunks;
            args.n_chunks += (u.bytes + c->chunk_bytes - 1) / c->chunk_bytes;
            args.u[args.n_units++] = u;
            bytes += u.bytes * ((u.out_src ? 1 : 0) + (u.in_src ? 1 : 0));
            const PUnit &p = kunits[k].second < 0 ? units[(size_t)(-1 - kunits[k].second)] : units[large[(size_t)kunits[k].second].unit];
            if ((rc = dep(c, S_K, c->gpu_ticket[(size_t)p.gpu_y])) != TC_OK) return rc;
            if (kunits[k].second < 0) {
                if (p.cpu_out >= 0 && (rc = dep(c, S_K, c->cpu_ticket[(size_t)p.cpu_out])) != TC_OK) return rc;
                if (p.cpu_in >= 0 && (rc = dep(c, S_K, c->cpu_ticket[(size_t)p.cpu_in])) != TC_OK) return rc;
            }
        }
        hipEvent_t t0;
        if ((rc = timed_begin(c, S_K, &t0)) != TC_OK) return rc;
        // Workgroups that wait on the GPU hold their places on the XCD they run on while they wait.  If
        // they took all of them, a one-workgroup kernel of the compute stream that the dispatcher deals
        // to that XCD (the signal they wait for among them) would find no place: the wait would end only
        // by its bound.  A gated launch therefore has at most one working workgroup per compute unit of
        // an XCD (the measured optimum is a dozen).
        const uint32_t wgs = gate ? std::min<uint32_t>(c->mover_wgs, 32) : c->mover_wgs;
        HIP_TRY(c, tc_launch_mover(args, wgs, c->streams[S_K], &c->k_launches));
        if ((rc = timed_end(c, S_K, t0, bytes)) != TC_OK) return rc;
        // the launch's number goes into the done word by a one-lane kernel right behind it on this stream
        if (c->gpu_deps) HIP_TRY(c, tc_launch_signal(c->tickets + 33, done_seq, c->streams[S_K]));
        if ((rc = end_op(c, S_K, id)) != TC_OK) return rc;
        if (c->gpu_deps) c->op_lseq[id % OP_RING] = done_seq;
        c->last_k_op = id;
        c->stats.mover_launches++;
        c->stats.mover_units += args.n_units;
        for (size_t k = at; k < end; ++k) {
            if (kunits[k].second < 0) {
                const PUnit &p = units[(size_t)(-1 - kunits[k].second)];
                c->gpu_ticket[(size_t)p.gpu_y] = id;
                if (p.cpu_out >= 0) c->cpu_ticket[(size_t)p.cpu_out] = id;
                if (p.cpu_in >= 0) c->cpu_ticket[(size_t)p.cpu_in] = id;
                if (StBlock *b = p.st_id ? st_find(c, p.st_id) : nullptr) {
                    b->issued = true;
                    b->ops[0] = id;
                    if (p.out_staging && (rc = io_submit(c, p.out_tensor, p.u.out_dst, false, id, S_K, &b->job)) != TC_OK) return rc;
                }
            } else {
                Large &L = large[(size_t)kunits[k].second];
                L.kop = id;
                c->gpu_ticket[(size_t)units[L.unit].gpu_y] = id;
            }
        }
    }
    // ---- streams H and D: the large units, one DMA copy per direction
    for (Large &L : large) {
        const PUnit &p = units[L.unit];
        uint64_t idh, idd;
        int rc = begin_op(c, S_H, compute, &idh);
        if (rc != TC_OK) return rc;
        if ((rc = dep(c, S_H, c->gpu_ticket[(size_t)p.gpu_y])) != TC_OK) return rc;   // staging copy, earlier users
        if (p.cpu_in >= 0 && (rc = dep(c, S_H, c->cpu_ticket[(size_t)p.cpu_in])) != TC_OK) return rc;
        hipEvent_t t0;
        if ((rc = timed_begin(c, S_H, &t0)) != TC_OK) return rc;
        HIP_TRY(c, hipMemcpyAsync(p.u.in_dst, p.u.in_src, p.u.bytes, hipMemcpyHostToDevice, c->streams[S_H]));
        if ((rc = timed_end(c, S_H, t0, p.u.bytes)) != TC_OK) return rc;
        if ((rc = end_op(c, S_H, idh)) != TC_OK) return rc;
        c->gpu_ticket[(size_t)p.gpu_y] = idh;
        if (p.cpu_in >= 0) c->cpu_ticket[(size_t)p.cpu_in] = idh;
        StBlock *blk = p.st_id ? st_find(c, p.st_id) : nullptr;
        if (blk) {
            blk->issued = true;
            if (p.in_staging) blk->ops[0] = idh;
        }
        c->stats.dma_copies++;
        if (!L.bounce) continue;
        if ((rc = begin_op(c, S_D, compute, &idd)) != TC_OK) return rc;
        // the outgoing bytes sit in the bounce block once the staging launch is done;
        // in a swap the host buffer they go to must first have been read by the copy above
        if ((rc = dep(c, S_D, L.kop)) != TC_OK) return rc;
        if (p.cpu_out >= 0 && p.cpu_out == p.cpu_in && (rc = dep(c, S_D, idh)) != TC_OK) return rc;
        if (p.cpu_out >= 0 && (rc = dep(c, S_D, c->cpu_ticket[(size_t)p.cpu_out])) != TC_OK) return rc;
        if ((rc = timed_begin(c, S_D, &t0)) != TC_OK) return rc;
        HIP_TRY(c, hipMemcpyAsync(p.u.out_dst, L.bounce, p.u.bytes, hipMemcpyDeviceToHost, c->streams[S_D]));
        if ((rc = timed_end(c, S_D, t0, p.u.bytes)) != TC_OK) return rc;
        if ((rc = end_op(c, S_D, idd)) != TC_OK) return rc;
        if (p.cpu_out >= 0) c->cpu_ticket[(size_t)p.cpu_out] = idd;
        for (BounceBlock &bb : c->bounce_q)
            if (c->bounce + bb.off == L.bounce) bb.op = idd;
        c->stats.dma_copies++;
        if (p.out_staging && blk) {
            blk->ops[1] = idd;
            if ((rc = io_submit(c, p.out_tensor, p.u.out_dst, false, idd, S_D, &blk->job)) != TC_OK) return rc;
        }
    }
    for (const PUnit &p : units) {
        c->gpu_pending[(size_t)p.gpu_y] = 0;
        if (p.cpu_out >= 0) c->cpu_pending[(size_t)p.cpu_out] = 0;
        if (p.cpu_in >= 0) c->cpu_pending[(size_t)p.cpu_in] = 0;
        if (p.out_staging) c->wb_pending[p.out_tensor] = 0;
    }
    if (point) {
        point->op = c->op_id;
        point->used = true;
    }
    units.clear();
    c->deferred_bytes = 0;
    return TC_OK;
}

// issue whatever earlier hook calls left prepared
int flush_deferred(tc_ctx *c, hipStream_t compute)
{
    if (c->deferred.empty()) return TC_OK;
    c->compute_recorded = false;
    for (int i = 0; i < N_STREAMS; ++i) c->stream_waited[i] = false;
    return issue_units(c, c->deferred, compute);
}

// Issue those prepared units that are ready (their file reads have arrived and no queued write still
// reads the host buffer they overwrite) and those `must` names, ready or not (issue_units waits for their
// file I/O); the rest stay prepared.  Prepared units touch disjoint buffers and disjoint extents (a unit
// that touches a buffer of a prepared one, or reads an extent a prepared one writes, issues those first),
// so any of them may go ahead of the others.  Staging blocks free in the order taken: a block issued ahead
// of an older one is simply held until that one is done.
template <class Must>
static int issue_some(tc_ctx *c, std::vector<PUnit> &units, hipStream_t compute, Must must)
{
    std::vector<PUnit> go, stay;
    for (const PUnit &p : units) {
        const bool ready = io_done(c, p.read_job) && (p.cpu_out < 0 || io_done(c, c->cpu_job[(size_t)p.cpu_out]));
        (ready || must(p) ? go : stay).push_back(p);
    }
    if (go.empty()) return TC_OK;
    if (stay.empty()) return issue_units(c, units, compute);
    units.swap(stay);
    const int rc = issue_units(c, go, compute);
    c->deferred_bytes = 0;
    for (const PUnit &p : units) c->deferred_bytes += p.u.bytes * ((p.u.out_src ? 1 : 0) + (p.u.in_src ? 1 : 0));
    return rc;
}

static int issue_ready(tc_ctx *c, std::vector<PUnit> &units, hipStream_t compute)
{
    return issue_some(c, units, compute, [](const PUnit &) { return false; });
}

// what a module is about to use: the prepared units that fill these GPU buffers have to be on their way,
// and whatever else is ready goes with them
int flush_for_buffers(tc_ctx *c, const int64_t *ys, uint32_t n, hipStream_t compute)
{
    if (c->deferred.empty()) return TC_OK;
    c->compute_recorded = false;
    for (int i = 0; i < N_STREAMS; ++i) c->stream_waited[i] = false;
    return issue_some(c, c->deferred, compute, [&](const PUnit &p) {
        for (uint32_t i = 0; i < n; ++i)
            if (p.gpu_y == ys[i]) return true;
        return false;
    });
}

// The staging region is a ring: a block is taken when a record needs bounce
// space for the file tier and is free again once the copies that touch it have
// completed and, for an outgoing tensor, its write has reached the file.  Blocks
// free in the order they were taken, so file reads, copies and writes of
// successive hook calls overlap as far as the ring is deep.
static int staging_alloc(tc_ctx *c, std::vector<PUnit> &units, uint64_t bytes, hipStream_t compute, uint8_t **out,
                         uint64_t *id)
{
    const uint64_t need = (bytes + io_align(c) - 1) & ~(io_align(c) - 1);
    if (need > c->staging_bytes) return fail(c, TC_E_CAPACITY, "staging region smaller than a tensor that needs the file tier");
    for (;;) {
        while (!c->st_q.empty()) {
            const StBlock &f = c->st_q.front();
            if (!(f.issued && poll_op(c, f.ops[0]) && poll_op(c, f.ops[1]) && io_done(c, f.job))) break;
            c->st_q.pop_front();
        }
        if (c->st_q.empty()) c->st_head = 0;
        const uint64_t tail = c->st_q.empty() ? 0 : c->st_q.front().off;
        uint64_t at = UINT64_MAX;
        if (c->st_q.empty() || c->st_head > tail) {                // free: [head, end) and [0, tail)
            if (c->st_head + need <= c->staging_bytes) at = c->st_head;
            else if (!c->st_q.empty() && need <= tail) at = 0;
        } else if (c->st_head < tail) {                            // free: [head, tail)
            if (c->st_head + need <= tail) at = c->st_head;
        }
        if (at != UINT64_MAX) {
            StBlock b{};
            b.id = c->st_next_id++;
            b.off = at;
            b.size = need;
            c->st_q.push_back(b);
            c->st_head = at + need;
            *out = c->staging + at;
            *id = b.id;
            return TC_OK;
        }
        // no room: the oldest block has to go first.  While this thread waits for it, the units
        // whose bytes have arrived should be moving: issue them now (a unit prepared but not issued
        // keeps the link idle and its staging block taken).
        {
            int rc = issue_ready(c, units, compute);
            if (rc != TC_OK) return rc;
        }
        if (!c->st_q.front().issued) {
            const uint64_t front = c->st_q.front().id;             // its unit goes now, ready or not
            int rc = issue_some(c, units, compute, [front](const PUnit &p) { return p.st_id == front; });
            if (rc != TC_OK) return rc;
            if (!c->st_q.front().issued) return fail(c, TC_E_STATE, "staging ring holds a block no prepared unit owns");
        }
        StBlock &f = c->st_q.front();
        Blocked b(c, BLK_STAGING);
        int rc = wait_op(c, f.ops[0]);
        if (rc == TC_OK) rc = wait_op(c, f.ops[1]);
        if (rc == TC_OK) rc = io_wait(c, f.job);
        if (rc != TC_OK) return rc;
        c->st_q.pop_front();
    }
}

// Two-tier mode (Sec. 3.4.2, optimizer states): the fast tier is host memory and a
// tensor moves between its buffer and its file extent directly, by the I/O workers:
// no copy kernel, no staging, nothing deferred.
static int dispatch_host_tier(tc_ctx *c, const TcOpRec &r, uint32_t t, uint32_t s, hipStream_t compute)
{
    switch (r.op) {
    case TC_OP_WRITEBACK: {
        const uint32_t y = c->pools.gpu_base[s] + r.src_slot;
        // a tensor is written back only after a module has used it, so the read that filled
        // the buffer has long finished; the wait guards the order all the same
        int rc = io_wait(c, c->fast_read[y]);
        if (rc != TC_OK) return rc;
        // the update may still be running on the compute stream: the writer waits for it
        return io_submit_behind(c, t, gpu_addr(c, s, r.src_slot), false, true, compute, &c->fast_write[y]);
    }
    case TC_OP_DEMAND:
    case TC_OP_PREFETCH: {
        if (r.src_tier != TC_NVME) return fail(c, TC_E_HIP, "two-tier mode: a fetch from a host buffer");
        const uint32_t y = c->pools.gpu_base[s] + r.dst_slot;
        // an earlier read into the same buffer (of a tensor dropped before its use)
        int rc = io_wait(c, c->fast_read[y]);
        if (rc != TC_OK) return rc;
        // the reader starts once the buffer's last tensor is in the file and the compute
        // stream is done with whatever it held
        return io_submit_behind(c, t, gpu_addr(c, s, r.dst_slot), true, true, compute, &c->fast_read[y],
                                &c->fast_write[y]);
    }
    case TC_OP_ALLOC: {
        // nothing to read: the update may write the buffer once its last tensor has reached the
        // file, so the PRE call's wait for "the read that fills the buffer" becomes a wait for that write
        const uint32_t y = c->pools.gpu_base[s] + r.dst_slot;
        int rc = io_wait(c, c->fast_read[y]);
        if (rc != TC_OK) return rc;
        c->fast_read[y] = c->fast_write[y];
        return TC_OK;
    }
    case TC_OP_RELEASE:
    case TC_OP_FAIL:
        return TC_OK;
    default:
        return fail(c, TC_E_HIP, "two-tier mode: an op that needs host buffers");
    }
}

// the signal the units of this hook call wait for, on its compute stream: queued when a call prepares a unit
// and no signal queued behind the last module is at hand
static int call_signal(tc_ctx *c, hipStream_t compute, uint32_t *sig)
{
    *sig = 0;
    if (!c->gpu_deps || compute == c->streams[S_K]) return TC_OK;
    if (!c->sig_sent) {
        uint32_t n = c->sig_seq + 1;
        if (n == 0) n = 1;                              // 0 means "none"
        HIP_TRY(c, tc_launch_signal(c->tickets + 32, n, compute));
        c->sig_seq = n;
        c->sig_stream = compute;
        c->sig_sent = true;
    }
    *sig = c->sig_seq;
    return TC_OK;
}

int dispatch(tc_ctx *c, const TcDecideOut *o, const TcOpRec *ops, uint32_t step, int phase,
                    hipStream_t compute)
{
    if (o->overflow) return fail(c, TC_E_CAPACITY, "decision log overflow");
    // Units are not issued per hook call: a launch that moves tens of MiB spends a
    // visible share of its time ramping the link up in both directions, so calls
    // are merged until merge_bytes are prepared, a prepared buffer is needed
    // (by a module, by a later unit or by the host), or the file tier is involved.
    std::vector<PUnit> &units = c->deferred;
    c->last_compute = compute;
    PUnit pend{};                   // outgoing half waiting for its incoming partner
    bool have_out = false;
    uint8_t *reserved_in = nullptr; // bounce space kept for the partner of a write-back
    c->compute_recorded = false;
    // A signal stands for "the modules queued so far": it stays good for the units of later calls until a
    // module may have been queued behind it, i.e. until a PRE call has returned (cache buffers are used only
    // between a step's PRE and POST).  So a POST or end-of-iteration call starts without one, a PRE call
    // keeps the one the call before it queued.
    if (phase != TC_PRE || c->sig_stream != compute) c->sig_sent = false;
    for (int i = 0; i < N_STREAMS; ++i) c->stream_waited[i] = false;
    for (uint32_t i = 0; i < o->n_ops; ++i) {
        const TcOpRec &r = ops[i];
        const uint32_t t = r.tensor;
        // never turn a record into an address before it is known to be in range
        if (t >= c->prof.n_tensors || r.op > TC_OP_ALLOC)
            return fail(c, TC_E_HIP, "decision record out of range (tensor/op)");
        const uint32_t s = c->prof.class_of[t];
        {
            const bool src_ok = r.src_tier == TC_GPU ? r.src_slot < c->pools.gpu_count[s]
                              : r.src_tier == TC_CPU ? r.src_slot < c->pools.cpu_count[s] : r.src_slot == TC_NONE;
            const bool dst_ok = r.dst_tier == TC_GPU ? r.dst_slot < c->pools.gpu_count[s]
                              : r.dst_tier == TC_CPU ? r.dst_slot < c->pools.cpu_count[s] : r.dst_slot == TC_NONE;
            if (r.op != TC_OP_FAIL && !(src_ok && dst_ok))
                return fail(c, TC_E_HIP, "decision record out of range (slot)");
        }
        const uint64_t n = c->prof.bytes[t];
        tc_op rec;
        rec.iteration = c->iteration; rec.step = step; rec.tensor = t;
        rec.src_slot = r.src_slot; rec.dst_slot = r.dst_slot;
        rec.phase = r.phase; rec.op = r.op; rec.src_tier = r.src_tier; rec.dst_tier = r.dst_tier;
        rec.bytes = (r.op == TC_OP_RELEASE || r.op == TC_OP_FAIL || r.op == TC_OP_ALLOC) ? 0 : n;
        if (c->logging) c->log.push_back(rec);
        if (r.op == TC_OP_ALLOC) { c->stats.n_alloc++; c->stats.bytes_not_fetched += n; }
        else c->stats.n_ops[r.op]++;
        switch (r.op) {
        case TC_OP_EVICT: c->stats.bytes_d2h += n; break;
        case TC_OP_WRITEBACK: case TC_OP_SPILL: c->stats.bytes_file_write += n; break;
        case TC_OP_RESTORE: c->stats.bytes_file_read += n; break;
        case TC_OP_DEMAND: case TC_OP_PREFETCH:
            c->stats.bytes_h2d += n;
            if (r.src_tier == TC_NVME) c->stats.bytes_file_read += n;
            break;
        default: break;
        }
        if (c->null_mover) continue;
        if (c->host_tier) {
            int rc = dispatch_host_tier(c, r, t, s, compute);
            if (rc != TC_OK) return rc;
            continue;
        }
        switch (r.op) {
        case TC_OP_SPILL: {
            // host buffer -> file extent, now: the buffer is about to be reused
            const uint32_t flat = c->pools.cpu_base[s] + r.src_slot;
            int rc = c->cpu_pending[flat] ? issue_units(c, units, compute) : TC_OK;
            if (rc != TC_OK) return rc;
            // the copy that last touched the buffer may still run: the writers wait for it, not this thread
            const uint64_t tk = c->cpu_ticket[flat];
            const bool running = !poll_op(c, tk);
            rc = io_submit(c, t, cpu_addr(c, s, r.src_slot), false, running ? tk : 0,
                           running ? c->op_stream[tk % OP_RING] : 0, &c->cpu_job[flat]);
            if (rc != TC_OK) return rc;
            break;
        }
        case TC_OP_EVICT: {
            pend = PUnit{};
            pend.u.out_src = gpu_addr(c, s, r.src_slot);
            pend.u.out_dst = cpu_addr(c, s, r.dst_slot);
            pend.u.bytes = n;
            pend.gpu_y = c->pools.gpu_base[s] + r.src_slot;
            pend.cpu_out = c->pools.cpu_base[s] + r.dst_slot;
            have_out = true;
            break;
        }
        case TC_OP_WRITEBACK: {
            // room for the outgoing bytes and, right behind them, for an
            // incoming tensor of the same class should it come from the file tier
            uint8_t *st = nullptr;
            const uint64_t half = (n + io_align(c) - 1) & ~(io_align(c) - 1);
            uint64_t st_id = 0;
            int rc = staging_alloc(c, units, 2 * half, compute, &st, &st_id);
            if (rc != TC_OK) return rc;
            reserved_in = st + half;
            pend = PUnit{};
            pend.st_id = st_id;
            pend.u.out_src = gpu_addr(c, s, r.src_slot);
            pend.u.out_dst = st;
            pend.u.bytes = n;
            pend.gpu_y = c->pools.gpu_base[s] + r.src_slot;
            pend.out_staging = true;
            pend.out_tensor = t;
            have_out = true;
            break;
        }
        case TC_OP_DEMAND:
        case TC_OP_PREFETCH: {
            PUnit p = have_out ? pend : PUnit{};
            p.u.bytes = n;
            p.u.in_dst = gpu_addr(c, s, r.dst_slot);
            p.gpu_y = c->pools.gpu_base[s] + r.dst_slot;
            if (r.src_tier == TC_CPU) {
                p.u.in_src = cpu_addr(c, s, r.src_slot);
                p.cpu_in = c->pools.cpu_base[s] + r.src_slot;
            } else {
                uint8_t *st = nullptr;
                int rc = TC_OK;
                // the tensor's write-back may still sit in a prepared unit (it left the GPU a call
                // or two ago and its unit waits for a read): that write has to be queued before
                // this read of the same extent, which then names it
                if (c->wb_pending[t] && (rc = issue_units(c, units, compute)) != TC_OK) return rc;
                if (have_out && p.out_staging) st = reserved_in;
                else rc = staging_alloc(c, units, n, compute, &st, &p.st_id);
                if (rc != TC_OK) return rc;
                rc = io_submit(c, t, st, true, 0, 0, &p.read_job);
                if (rc != TC_OK) return rc;
                p.u.in_src = st;
                p.in_staging = true;
            }
            // a buffer that a prepared unit already touches: issue those first
            if (c->gpu_pending[(size_t)p.gpu_y] || (p.cpu_out >= 0 && c->cpu_pending[(size_t)p.cpu_out]) ||
                (p.cpu_in >= 0 && c->cpu_pending[(size_t)p.cpu_in])) {
                int rc = issue_units(c, units, compute);
                if (rc != TC_OK) return rc;
            }
            c->gpu_pending[(size_t)p.gpu_y] = 1;
            if (p.cpu_out >= 0) c->cpu_pending[(size_t)p.cpu_out] = 1;
            if (p.cpu_in >= 0) c->cpu_pending[(size_t)p.cpu_in] = 1;
            c->deferred_bytes += n * ((p.u.out_src ? 1 : 0) + 1);
            if (p.out_staging) c->wb_pending[p.out_tensor] = 1;
            {
                int rc = call_signal(c, compute, &p.sig);
                if (rc != TC_OK) return rc;
            }
            units.push_back(p);
            have_out = false;
            break;
        }
        case TC_OP_ALLOC: {
            // the tensor is about to be written whole: its GPU buffer changes hands and nothing is
            // copied in.  If a tensor leaves that buffer (the eviction recorded just before), its
            // copy is a unit without an incoming half; the module's kernels wait for it through the
            // buffer's ticket, like for any copy.
            if (!have_out) break;
            PUnit p = pend;
            if (p.gpu_y != (int64_t)(c->pools.gpu_base[s] + r.dst_slot))
                return fail(c, TC_E_HIP, "decision records: an allocation that does not follow its eviction");
            if (c->gpu_pending[(size_t)p.gpu_y] || (p.cpu_out >= 0 && c->cpu_pending[(size_t)p.cpu_out])) {
                int rc = issue_units(c, units, compute);
                if (rc != TC_OK) return rc;
            }
            c->gpu_pending[(size_t)p.gpu_y] = 1;
            if (p.cpu_out >= 0) c->cpu_pending[(size_t)p.cpu_out] = 1;
            c->deferred_bytes += n;
            if (p.out_staging) c->wb_pending[p.out_tensor] = 1;
            {
                int rc = call_signal(c, compute, &p.sig);
                if (rc != TC_OK) return rc;
            }
            units.push_back(p);
            have_out = false;
            break;
        }
        case TC_OP_RESTORE: {
            // file extent -> host buffer, by the host; earlier copies that read
            // or wrote the buffer must have finished
            int rc = issue_units(c, units, compute);
            if (rc != TC_OK) return rc;
            // the same end-of-iteration call may have written this very tensor back to
            // its extent a moment ago: that write has to reach the file first
            const uint32_t flat = c->pools.cpu_base[s] + r.dst_slot;
            {
                Blocked b(c, BLK_FILE_WRITE);
                rc = io_wait(c, c->tensor_job[t]);
                if (rc == TC_OK) rc = io_wait(c, c->cpu_job[flat]);
            }
            if (rc != TC_OK) return rc;
            {
                Blocked b(c, BLK_COPY);
                rc = wait_op(c, c->cpu_ticket[flat]);
            }
            if (rc != TC_OK) return rc;
            Blocked b(c, BLK_FILE_READ);
            rc = io_transfer(c, t, cpu_addr(c, s, r.dst_slot), true);
            if (rc != TC_OK) return rc;
            break;
        }
        default: break;                               // RELEASE, FAIL: nothing moves
        }
    }
    if (c->null_mover) return TC_OK;
    if (have_out) return fail(c, TC_E_HIP, "decision records end with an eviction that has no incoming tensor");
    if (phase < TC_END) {
        // Units whose bytes are still being read from the file, or whose host buffer a
        // queued spill still reads, stay prepared: a later hook call issues them, at the
        // latest the one that needs a buffer they touch.
        bool staged = false, waiting = false;
        for (const PUnit &p : units) {
            waiting = waiting || !io_done(c, p.read_job) || (p.cpu_out >= 0 && !io_done(c, c->cpu_job[(size_t)p.cpu_out]));
            staged = staged || p.st_id != 0;
        }
        if (waiting) return issue_ready(c, units, compute);     // those in front that can go, go
        // the link is busy: keep them for a larger launch (file-tier units go at once,
        // their staging blocks and their writes should not wait).  Keeping a second launch queued
        // behind the running one instead was measured and changes nothing: with the host ahead of
        // the GPU it is the module that needs a prepared buffer that decides when units are issued.
        if (!staged && c->deferred_bytes < c->merge_bytes && units.size() < 4 * TC_MOVER_MAX_UNITS &&
            !poll_op(c, c->last_k_op))
            return TC_OK;
    }
    return issue_units(c, units, compute);
}

