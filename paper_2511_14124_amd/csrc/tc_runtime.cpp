// Runtime of libtc.so: the context, memory binding, the hook calls (deciding,
// deciding ahead, replay in windows), statistics, and the C ABI of include/tc.h.
// The dispatch of the decided ops is in tc_dispatch.cpp, the file tier in tc_io.cpp.
#include "tc_ctx.h"

#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <exception>

extern "C" const char *tc_strerror(int code)
{
    switch (code) {
    case TC_OK: return "ok";
    case TC_E_ARG: return "bad argument";
    case TC_E_STATE: return "call out of order";
    case TC_E_CAPACITY: return "capacity exceeded";
    case TC_E_IO: return "file-tier I/O failed";
    case TC_E_HIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

extern "C" const char *tc_last_error(const tc_ctx *c) { return c ? c->err.c_str() : ""; }

extern "C" int tc_create(tc_ctx **out)
{
    if (!out) return TC_E_ARG;
    *out = new (std::nothrow) tc_ctx();
    return *out ? TC_OK : TC_E_CAPACITY;
}

static void release_device(tc_ctx *c)
{
    io_stop(c);
    for (hipEvent_t e : c->ev_free) (void)hipEventDestroy(e);
    c->ev_free.clear();
    if (c->dstream) { (void)hipStreamSynchronize(c->dstream); }
    for (int i = 0; i < N_STREAMS; ++i)
        if (c->streams[i] || (i == S_K && c->stage >= 4)) { (void)hipStreamSynchronize(c->streams[i]); }
    for (auto &p : c->timed) { (void)hipEventDestroy(p.t0); (void)hipEventDestroy(p.t1); }
    c->timed.clear();
    for (uint32_t i = 0; i < OP_RING; ++i)
        if (c->op_ev[i]) { (void)hipEventDestroy(c->op_ev[i]); c->op_ev[i] = nullptr; }
    if (c->ev_compute) { (void)hipEventDestroy(c->ev_compute); c->ev_compute = nullptr; }
    for (auto &pt : c->issue_ring) {
        if (pt.ev) (void)hipEventDestroy(pt.ev);
        pt = tc_ctx::IssuePoint{};
    }
    c->issue_next = 0;
    if (c->dstream) { (void)hipStreamDestroy(c->dstream); c->dstream = nullptr; }
    for (int i = S_H; i < N_STREAMS; ++i)
        if (c->streams[i]) { (void)hipStreamDestroy(c->streams[i]); c->streams[i] = nullptr; }
    if (c->dev_block) { (void)hipFree(c->dev_block); c->dev_block = nullptr; }
    if (c->d_step_ptr) { (void)hipFree(c->d_step_ptr); c->d_step_ptr = nullptr; }
    if (c->d_ids) { (void)hipFree(c->d_ids); c->d_ids = nullptr; }
    if (c->d_rw) { (void)hipFree(c->d_rw); c->d_rw = nullptr; }
    if (c->bounce) { (void)hipFree(c->bounce); c->bounce = nullptr; }
    if (c->tickets) { (void)hipFree(c->tickets); c->tickets = nullptr; }
    if (c->fault) { (void)hipHostFree(c->fault); c->fault = nullptr; }
    for (int b = 0; b < 2; ++b) {
        if (c->snap[b]) { (void)hipFree(c->snap[b]); c->snap[b] = nullptr; }
        if (c->win_ev[b]) { (void)hipEventDestroy(c->win_ev[b]); c->win_ev[b] = nullptr; }
        c->win[b] = SpecWin{};
    }
    if (c->d_prof_rw) { (void)hipFree(c->d_prof_rw); c->d_prof_rw = nullptr; }
    if (c->dout) { (void)hipHostFree(c->dout); c->dout = nullptr; }
    if (c->io_bounce) { free(c->io_bounce); c->io_bounce = nullptr; }
}

extern "C" int tc_destroy(tc_ctx *c)
{
    if (!c) return TC_E_ARG;
    if (c->stage >= 4) release_device(c);
    delete c;
    return TC_OK;
}

extern "C" int tc_profile_order(tc_ctx *c, const tc_tensor_desc *t, uint32_t n_t, const tc_event *ev,
                                uint64_t n_ev)
{
    if (!c || !t || (!ev && n_ev) || n_t == 0) return fail(c, TC_E_ARG, "null or empty input");
    if (c->stage >= 4) return fail(c, TC_E_STATE, "context is already bound");
    std::string err;
    TcProfile p;
    int rc;
    try {
        rc = tc_build_profile(p, t, n_t, ev, n_ev, err);
    } catch (const std::exception &) {                  // bad_alloc, length_error: nothing may cross the C boundary
        return fail(c, TC_E_CAPACITY, "out of host memory while building the prefetch table");
    }
    if (rc != TC_OK) return fail(c, rc, err);
    c->prof = std::move(p);
    c->stage = 1;
    return TC_OK;
}

extern "C" int tc_plan_pools(tc_ctx *c, const tc_budget *b, tc_pool_plan *plan_out,
                             tc_pool_class *classes_out, uint32_t cap)
{
    if (!c || !b) return fail(c, TC_E_ARG, "null argument");
    if (c->stage < 1 || c->stage >= 4) return fail(c, TC_E_STATE, "tc_profile_order must come first");
    const uint32_t n_c = (uint32_t)c->prof.count.size();
    if (classes_out && cap < n_c) return fail(c, TC_E_CAPACITY, "classes_out too small");
    std::string err;
    TcPools pools;
    int rc;
    try {
        rc = tc_build_pools(c->prof, *b, pools, err);
    } catch (const std::exception &) {
        return fail(c, TC_E_CAPACITY, "out of host memory while planning the pools");
    }
    if (rc != TC_OK) return fail(c, rc, err);
    c->pools = std::move(pools);
    c->budget = *b;
    // the file tier's size is known already: every tensor owns a 4 KiB aligned extent
    uint64_t file_total = 0;
    for (uint32_t t = 0; t < c->prof.n_tensors; ++t) file_total += (c->prof.bytes[t] + 4095) / 4096 * 4096;
    if (plan_out) {
        plan_out->n_classes = n_c;
        plan_out->n_rows = (uint32_t)c->prof.rows_tensor.size();
        plan_out->n_steps = c->prof.n_steps;
        plan_out->pad_ = 0;
        plan_out->hbm_total = c->pools.hbm_total;
        plan_out->host_total = c->pools.host_total;
        plan_out->file_total = file_total;
    }
    if (classes_out)
        for (uint32_t s = 0; s < n_c; ++s) {
            tc_pool_class &k = classes_out[s];
            k.bytes = c->prof.class_bytes[s];
            k.stride = c->pools.stride[s];
            k.hbm_off = c->pools.hbm_off[s];
            k.host_off = c->pools.host_off[s];
            k.group = c->prof.class_group[s];
            k.count = c->prof.count[s];
            k.used = c->prof.used[s];
            k.step_max = c->prof.step_max[s];
            k.gpu_count = c->pools.gpu_count[s];
            k.cpu_count = c->pools.cpu_count[s];
        }
    c->stage = 2;
    return TC_OK;
}

extern "C" int tc_plan_schedule(tc_ctx *c, tc_placement *out)
{
    if (!c) return TC_E_ARG;
    if (c->stage < 2 || c->stage >= 4) return fail(c, TC_E_STATE, "tc_plan_pools must come first");
    try {
        tc_build_placement(c->prof, c->pools, c->place);
    } catch (const std::exception &) {
        return fail(c, TC_E_CAPACITY, "out of host memory while placing the tensors");
    }
    if (out)
        for (uint32_t t = 0; t < c->prof.n_tensors; ++t) {
            out[t].file_off = c->place.file_off[t];
            out[t].cls = c->prof.class_of[t];
            out[t].slot = c->place.slot[t];
            out[t].first_use = c->prof.first_use[t];
            out[t].final_tier = c->place.final_tier[t];
            out[t].pad_[0] = out[t].pad_[1] = out[t].pad_[2] = 0;
        }
    c->stage = 3;
    return TC_OK;
}

// ---------------------------------------------------------------------------
// binding: device tables
// ---------------------------------------------------------------------------
extern "C" int tc_bind_memory(tc_ctx *c, void *hbm, uint64_t hbm_bytes, void *pinned, uint64_t pinned_bytes,
                              void *staging, uint64_t staging_bytes, int fd, void *mstream, uint32_t flags)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 3) return fail(c, TC_E_STATE, "tc_plan_schedule must come first (and bind only once)");
    const bool null_mover = (flags & TC_BIND_NULL_MOVER) != 0;
    const bool direct = (flags & TC_BIND_FILE_DIRECT) != 0 && fd >= 0 && !null_mover;
    if (direct && ((((uintptr_t)staging) & 4095) || (staging_bytes & 4095)))
        return fail(c, TC_E_ARG, "with TC_BIND_FILE_DIRECT the staging region must be 4 KiB aligned and sized");
    const bool host_tier = (flags & TC_BIND_HOST_TIER) != 0;
    if (host_tier) {
        if (c->pools.host_total || c->pools.cpu_slots)
            return fail(c, TC_E_ARG, "TC_BIND_HOST_TIER needs a plan made with both host budgets 0");
        if (!null_mover && hbm) {
            hipPointerAttribute_t at{};
            if (hipPointerGetAttributes(&at, hbm) != hipSuccess || at.type != hipMemoryTypeHost) {
                (void)hipGetLastError();
                return fail(c, TC_E_ARG, "TC_BIND_HOST_TIER: the fast-tier region must be pinned host memory");
            }
        }
    }
    if (!null_mover) {
        if (c->pools.hbm_total && (!hbm || hbm_bytes < c->pools.hbm_total))
            return fail(c, TC_E_CAPACITY, "HBM region smaller than the plan");
        if (c->pools.host_total && (!pinned || pinned_bytes < c->pools.host_total))
            return fail(c, TC_E_CAPACITY, "pinned region smaller than the plan");
        if (((uintptr_t)hbm | (uintptr_t)pinned | (uintptr_t)staging) & 255)
            return fail(c, TC_E_ARG, "regions must be 256-byte aligned");
    }
    const TcProfile &p = c->prof;
    const TcPools &pl = c->pools;
    const uint32_t n_t = p.n_tensors, n_c = (uint32_t)p.count.size();
    const uint32_t n_rows = (uint32_t)p.rows_tensor.size();

    // one device allocation for every table (set-up time, not the hot path)
    std::vector<uint32_t> img;
    auto put = [&](const std::vector<uint32_t> &v) {
        size_t off = img.size();
        img.insert(img.end(), v.begin(), v.end());
        if (v.empty()) img.push_back(0);
        return off;
    };
    std::vector<uint32_t> final32(c->place.final_tier.begin(), c->place.final_tier.end());
    std::vector<uint32_t> cur(final32), gslot(n_t, TC_NONE), cslot(n_t, TC_NONE), zeros_t(n_t, 0);
    std::vector<uint32_t> gpu_owner(pl.gpu_slots, TC_NONE), cpu_owner(pl.cpu_slots, TC_NONE);
    for (uint32_t t = 0; t < n_t; ++t) {
        uint32_t s = p.class_of[t];
        if (c->place.final_tier[t] == TC_GPU) { gslot[t] = c->place.slot[t]; gpu_owner[pl.gpu_base[s] + gslot[t]] = t; }
        if (c->place.final_tier[t] == TC_CPU) { cslot[t] = c->place.slot[t]; cpu_owner[pl.cpu_base[s] + cslot[t]] = t; }
    }
    size_t o_rows = put(p.rows_tensor), o_rb = put(p.row_begin), o_op = put(p.occ_ptr), o_or = put(p.occ_rows);
    size_t o_cls = put(p.class_of), o_fin = put(final32);
    size_t o_gc = put(pl.gpu_count), o_cc = put(pl.cpu_count), o_gb = put(pl.gpu_base), o_cb = put(pl.cpu_base);
    size_t o_mp = put(c->place.member_ptr), o_mem = put(c->place.members);
    size_t o_cur = put(cur), o_gs = put(gslot), o_cs = put(cslot), o_dirty = put(zeros_t), o_moved = put(zeros_t);
    size_t o_undef = put(zeros_t);
    size_t o_go = put(gpu_owner), o_gf = put(std::vector<uint32_t>(pl.gpu_slots, 0));
    size_t o_co = put(cpu_owner), o_cf = put(std::vector<uint32_t>(pl.cpu_slots, 0));
    size_t o_des = put(std::vector<uint32_t>(pl.cpu_slots, 0));
    size_t o_sc = put(std::vector<uint32_t>(4, 0));

    HIP_TRY(c, hipMalloc((void **)&c->dev_block, img.size() * sizeof(uint32_t)));
    hipError_t e = hipMemcpy(c->dev_block, img.data(), img.size() * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    uint32_t *d = c->dev_block;
    TcDevTables &T = c->T;
    T.rows_tensor = d + o_rows; T.row_begin = d + o_rb; T.occ_ptr = d + o_op; T.occ_rows = d + o_or;
    T.class_of = d + o_cls; T.final_tier = d + o_fin;
    T.gpu_count = d + o_gc; T.cpu_count = d + o_cc; T.gpu_base = d + o_gb; T.cpu_base = d + o_cb;
    T.member_ptr = d + o_mp; T.members = d + o_mem;
    T.n_rows = n_rows; T.n_steps = p.n_steps; T.n_tensors = n_t; T.n_classes = n_c;
    T.flags = c->budget.flags;
    T.cur = d + o_cur; T.gslot = d + o_gs; T.cslot = d + o_cs; T.dirty = d + o_dirty; T.moved = d + o_moved;
    T.undefined = d + o_undef;
    T.gpu_owner = d + o_go; T.gpu_freed = d + o_gf; T.cpu_owner = d + o_co; T.cpu_freed = d + o_cf;
    T.designated = d + o_des; T.scalars = d + o_sc;

    // result block: room for the end-of-iteration call (every tensor may move, with
    // a spill and an eviction each) and for a full window of hook calls (per listed
    // tensor at most a spill, an eviction and a fetch)
    c->dout_cap = std::max<uint32_t>(3 * n_t + 64, TC_WINDOW_MAX * 2 * 3 * TC_MAX_STEP_TENSORS);
    const size_t rec_bytes = (size_t)2 * TC_WINDOW_MAX * sizeof(TcDecideOut);
    const size_t blk_bytes = (rec_bytes + (size_t)c->dout_cap * sizeof(TcOpRec) + 255) & ~(size_t)255;
    e = hipHostMalloc((void **)&c->dout, 2 * blk_bytes, hipHostMallocDefault);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    memset(c->dout, 0, 2 * blk_bytes);
    c->dops = (TcOpRec *)((uint8_t *)c->dout + rec_bytes);
    c->dout2 = (TcDecideOut *)((uint8_t *)c->dout + blk_bytes);
    c->dops2 = (TcOpRec *)((uint8_t *)c->dout2 + rec_bytes);
    e = hipMalloc((void **)&c->d_step_ptr, ((size_t)p.n_steps + 1) * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_ids, std::max<size_t>(1, (size_t)p.n_steps * TC_MAX_STEP_TENSORS) * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_rw, std::max<size_t>(1, (size_t)p.n_steps * TC_MAX_STEP_TENSORS));
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    e = hipStreamCreateWithFlags(&c->dstream, hipStreamNonBlocking);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    c->mut_off = o_cur;
    c->mut_words = img.size() - o_cur;
    for (int b = 0; b < 2 && e == hipSuccess; ++b) {
        e = hipMalloc((void **)&c->snap[b], c->mut_words * sizeof(uint32_t));
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->win_ev[b], hipEventDisableTiming);
        c->win[b] = SpecWin{};
    }
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_prof_rw, std::max<size_t>(1, p.rows_rw.size()));
    if (e == hipSuccess && !p.rows_rw.empty())
        e = hipMemcpy(c->d_prof_rw, p.rows_rw.data(), p.rows_rw.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    c->T.rows_rw = c->d_prof_rw;
    c->ahead_pause = 0;
    e = hipMalloc((void **)&c->tickets, 256);
    if (e == hipSuccess) e = hipMemset(c->tickets, 0, 256);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    c->k_launches = 0;
    e = hipHostMalloc((void **)&c->fault, 64, hipHostMallocDefault);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    *c->fault = 0;
    c->sig_seq = c->launch_seq = c->waited_lseq = 0;
    e = tc_mover_topology(&c->mover_xcc, &c->mover_xcds);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    for (uint32_t i = 0; i < OP_RING; ++i) {
        e = hipEventCreateWithFlags(&c->op_ev[i], hipEventDisableTiming);
        if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    }
    e = hipEventCreateWithFlags(&c->ev_compute, hipEventDisableTiming);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    c->hbm = (uint8_t *)hbm; c->hbm_bytes = hbm_bytes;
    c->pinned = (uint8_t *)pinned; c->pinned_bytes = pinned_bytes;
    c->staging = (uint8_t *)staging; c->staging_bytes = staging_bytes;
    c->n_files = 0;
    if (fd >= 0) c->fds[c->n_files++] = fd;
    c->io_begun = false;
    c->file_direct = direct;
    if (direct) {
        uint64_t largest = 0;
        for (uint32_t t = 0; t < n_t; ++t) largest = std::max(largest, p.bytes[t]);
        // A device read and written directly wants few, large, sequential requests (measured on a virtual
        // disk: one request per tensor and two threads per direction 7.0 GB/s host->HBM, four threads each
        // with 64 MiB chunks 6.3, eight each with 16 MiB chunks 5.4, four each with 8 MiB chunks 3.4): unless
        // the caller has chosen, a direct file gets one request per tensor and two threads each way.
        if (!c->io_chunk_set) c->io_chunk = std::max<uint64_t>(c->io_chunk, (largest + (1ull << 20) - 1) >> 20 << 20);
        if (!c->io_threads_set) c->n_io[IO_WRITERS] = c->n_io[IO_READERS] = 2;
        c->io_bounce_bytes = std::min<uint64_t>(c->io_chunk, (largest + 4095) & ~4095ull);
        void *blk = nullptr;
        if (posix_memalign(&blk, 4096, c->io_bounce_bytes) != 0) { release_device(c); return fail(c, TC_E_CAPACITY, "no memory for the I/O bounce block"); }
        c->io_bounce = (uint8_t *)blk;
    }
    c->streams[S_K] = (hipStream_t)mstream;
    c->null_mover = null_mover;
    c->in_use = false;
    c->stats.hbm_budget = c->budget.hbm_bytes;
    c->stats.hbm_pool_bytes = pl.hbm_total;
    c->stats.host_budget = c->budget.host_bytes[0] + c->budget.host_bytes[1];
    c->stats.host_pool_bytes = pl.host_total;
    c->gpu_ticket.assign(pl.gpu_slots, 0);
    c->cpu_ticket.assign(pl.cpu_slots, 0);
    c->gpu_pending.assign(pl.gpu_slots, 0);
    c->cpu_pending.assign(pl.cpu_slots, 0);
    c->stall_by_step.assign(p.n_steps, 0);
    c->tensor_job.assign(n_t, JobSet{});
    c->wb_pending.assign(n_t, 0);
    c->cpu_job.assign(pl.cpu_slots, JobSet{});
    c->host_tier = host_tier;
    c->fast_read.assign(host_tier ? pl.gpu_slots : 0, JobSet{});
    c->fast_write.assign(host_tier ? pl.gpu_slots : 0, JobSet{});
    e = hipGetDevice(&c->device);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    if (fd >= 0 && !null_mover) {
        int rc = io_start(c);
        if (rc != TC_OK) { release_device(c); return rc; }
    }
    c->stage = 4;
    return TC_OK;
}

static int run_decide(tc_ctx *c, const TcStepArgs &a)
{
    hipEvent_t t0;
    int rc = timed_begin(c, K_DECIDE, &t0);
    if (rc != TC_OK) return rc;
    HIP_TRY(c, tc_launch_decide(c->T, a, c->dout, c->dops, c->dstream));
    if ((rc = timed_end(c, K_DECIDE, t0, 1)) != TC_OK) return rc;
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    c->stats.decide_launches++;
    c->stats.cursor = c->dout->cursor;
    return TC_OK;
}

// ---- deciding ahead along the profile ---------------------------------------
// A training loop repeats the profiled iteration, so tc_migrate_step need not pay a
// launch and a wait per hook call: it decides a window of the profiled steps in one
// launch (and the window after it behind that one) and hands the results out as the
// calls arrive.  A call that is not the profile's next one (another step, other
// tensors, other R/W flags) ends this: the tables go back to what they were before
// the window being handed out, the calls already handed out are decided again, and
// the odd call gets a launch of its own.  Decisions depend on the tables and the
// calls only, never on when a copy finishes, so deciding early changes no result.
static bool call_follows_profile(const tc_ctx *c, uint32_t step, int phase, const uint32_t *ids, const uint8_t *rw,
                                 uint32_t n)
{
    const TcProfile &p = c->prof;
    if (step >= p.n_steps) return false;                  // a module without tensors behind the profile's last step
    const uint32_t b = p.row_begin[step];
    if (p.row_begin[step + 1] - b != n) return false;
    for (uint32_t i = 0; i < n; ++i) {
        if (p.rows_tensor[b + i] != ids[i]) return false;
        if (phase == TC_PRE && p.rows_rw[b + i] != rw[i]) return false;   // (the post-hook decisions ignore the flags)
    }
    return true;
}

static int launch_window_ahead(tc_ctx *c, SpecWin &w, uint32_t first, int blk, uint32_t n_calls)
{
    TcWindowArgs a{};
    a.step_ptr = c->T.row_begin; a.ids = c->T.rows_tensor; a.rw = c->d_prof_rw;
    a.first = first;
    a.count = std::min(c->ahead_steps, c->prof.n_steps - first);
    a.cap = c->dout_cap;
    a.n_calls = n_calls ? n_calls : 2 * a.count;
    a.count = (a.n_calls + 1) / 2;
    hipEvent_t t0;
    int rc = timed_begin(c, K_DECIDE, &t0);
    if (rc != TC_OK) return rc;
    HIP_TRY(c, tc_launch_decide_window(c->T, a, blk ? c->dout2 : c->dout, blk ? c->dops2 : c->dops, c->dstream));
    if ((rc = timed_end(c, K_DECIDE, t0, a.n_calls)) != TC_OK) return rc;
    HIP_TRY(c, hipEventRecord(c->win_ev[blk], c->dstream));
    c->stats.decide_launches++;
    w = SpecWin{};
    w.valid = true; w.first = first; w.n_calls = a.n_calls; w.blk = blk;
    return TC_OK;
}

// start a window at `first`: the tables as they are now go into the block's snapshot
static int start_window_ahead(tc_ctx *c, SpecWin &w, uint32_t first, int blk)
{
    HIP_TRY(c, hipMemcpyAsync(c->snap[blk], c->dev_block + c->mut_off, c->mut_words * sizeof(uint32_t),
                              hipMemcpyDeviceToDevice, c->dstream));
    return launch_window_ahead(c, w, first, blk, 0);
}

// Bring the tables back in step with the calls made so far: needed before anything
// else decides or reads them (a call off the profile, the end of the iteration, a
// replay, a state dump).
static int settle_ahead(tc_ctx *c)
{
    if (!c->win[0].valid) return TC_OK;
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    const SpecWin w = c->win[0];
    c->win[0] = SpecWin{};
    c->win[1] = SpecWin{};
    HIP_TRY(c, hipMemcpyAsync(c->dev_block + c->mut_off, c->snap[w.blk], c->mut_words * sizeof(uint32_t),
                              hipMemcpyDeviceToDevice, c->dstream));
    if (w.used) {
        SpecWin again;
        int rc = launch_window_ahead(c, again, w.first, w.blk, w.used);
        if (rc != TC_OK) return rc;
    }
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    return TC_OK;
}

// the decision of this call if it is the profile's next one (*o == nullptr otherwise)
static int take_ahead(tc_ctx *c, uint32_t step, int phase, const uint32_t *ids, const uint8_t *rw, uint32_t n,
                      const TcDecideOut **o, const TcOpRec **ops)
{
    *o = nullptr;
    if (!c->ahead_steps) return TC_OK;
    const bool follows = call_follows_profile(c, step, phase, ids, rw, n);
    SpecWin &w = c->win[0];
    if (w.valid && !(follows && step == w.first + w.used / 2 && (uint32_t)phase == (w.used & 1u))) {
        c->ahead_pause = 8;                               // the loop has left the profile: sit a few calls out
        return settle_ahead(c);
    }
    if (!w.valid) {
        if (c->ahead_pause) { c->ahead_pause--; return TC_OK; }
        if (!follows || phase != TC_PRE) return TC_OK;
        int rc = start_window_ahead(c, c->win[0], step, 0);
        if (rc != TC_OK) return rc;
        const uint32_t next = step + c->win[0].n_calls / 2;
        if (next < c->prof.n_steps && (rc = start_window_ahead(c, c->win[1], next, 1)) != TC_OK) return rc;
    }
    if (!w.ready) {
        HIP_TRY(c, hipEventSynchronize(c->win_ev[w.blk]));
        w.ready = true;
    }
    *o = (w.blk ? c->dout2 : c->dout) + w.used;
    *ops = (w.blk ? c->dops2 : c->dops) + w.ops_used;
    return TC_OK;
}

// the call's decision has been dispatched and its results are no longer needed
static int advance_ahead(tc_ctx *c, const TcDecideOut *o)
{
    SpecWin &w = c->win[0];
    w.ops_used += o->n_ops;
    w.used++;
    c->stats.cursor = o->cursor;
    if (w.used < w.n_calls) return TC_OK;
    // the window is used up: the one decided behind it takes its place, and its block
    // and snapshot serve the window after that
    const int freed = w.blk;
    c->win[0] = c->win[1];
    c->win[1] = SpecWin{};
    if (!c->win[0].valid) return TC_OK;
    const uint32_t next = c->win[0].first + c->win[0].n_calls / 2;
    if (next < c->prof.n_steps) return start_window_ahead(c, c->win[1], next, freed);
    return TC_OK;
}

// what a pre-hook call does once its decisions are dispatched: counters, the
// buffers' addresses, the waits of the compute stream, the stamp list
static int finish_pre(tc_ctx *c, const TcDecideOut *o, uint32_t step, const uint32_t *ids, const uint8_t *rw,
                      uint32_t n, hipStream_t compute, void **dev_ptrs_out)
{
    c->stats.hits += o->hits;
    c->stats.misses += o->misses;
    c->stats.fails += o->fails;
    c->stats.undefined_reads += o->undefined_reads;
    TcStampArgs &sa = c->last_pre;
    sa = TcStampArgs{};
    sa.iteration = c->iteration;
    sa.step = step;
    {
        // copies that fill the module's buffers have to be on their way before the module runs
        int64_t ys[TC_MAX_STEP_TENSORS];
        uint32_t n_y = 0;
        for (uint32_t i = 0; i < n && !c->null_mover; ++i) {
            if (o->slots[i] == TC_NONE) continue;
            const int64_t y = (int64_t)c->pools.gpu_base[c->prof.class_of[ids[i]]] + o->slots[i];
            if ((size_t)y < c->gpu_pending.size() && c->gpu_pending[(size_t)y]) ys[n_y++] = y;
        }
        if (n_y) {
            int rc = flush_for_buffers(c, ys, n_y, compute);
            if (rc != TC_OK) return rc;
        }
    }
    std::chrono::steady_clock::time_point t0;
    uint64_t waited_ns = 0;
    if (c->host_tier && !c->null_mover) {
        t0 = std::chrono::steady_clock::now();             // the host blocks for every fetch: always timed
    } else if (c->measure_stall && !c->null_mover) {
        // wait time as the paper measures it (Sec. 4.2.2): once the modules queued so
        // far have finished, how long until each tensor of this one is in its buffer
        HIP_TRY(c, hipStreamSynchronize(compute));
        t0 = std::chrono::steady_clock::now();
    }
    for (uint32_t i = 0; i < n; ++i) {
        const uint32_t t = ids[i], s = c->prof.class_of[t];
        uint8_t *ptr = nullptr;
        if (o->slots[i] != TC_NONE) {
            if (o->slots[i] >= c->pools.gpu_count[s]) return fail(c, TC_E_HIP, "decision record out of range (buffer)");
            if (!c->null_mover) {
                ptr = gpu_addr(c, s, o->slots[i]);
                // the module's kernels wait only for the copies that fill ITS buffers
                const uint64_t ticket = c->gpu_ticket[c->pools.gpu_base[s] + o->slots[i]];
                if (c->host_tier || c->measure_stall) {
                    int rc = c->host_tier ? io_wait(c, c->fast_read[c->pools.gpu_base[s] + o->slots[i]])
                                          : wait_op(c, ticket);
                    if (rc != TC_OK) return rc;
                    const uint64_t ns = (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
                                            std::chrono::steady_clock::now() - t0).count();
                    waited_ns = std::max(waited_ns, ns);
                    c->stats.waits_total++;
                    if (ns < 10000) c->stats.waits_under_10us++;
                    if (ns < 30000) c->stats.waits_under_30us++;
                    if (ns < 100000) c->stats.waits_under_100us++;
                } else if (!op_complete(c, ticket)) {
                    // one wait per copy operation and compute stream: what the stream already waits
                    // for covers every older operation of the same copy stream
                    const uint32_t st = c->op_stream[ticket % OP_RING];
                    if (c->waited_stream != compute) {
                        c->waited_stream = compute;
                        c->waited_lseq = 0;
                        for (int k = 0; k < N_STREAMS; ++k) c->waited_op[k] = 0;
                    }
                    if (ticket > c->waited_op[st]) {
                        // (a module queued on the very stream the copy runs on is behind it anyway)
                        const uint32_t lseq = c->op_lseq[ticket % OP_RING];
                        if (c->streams[st] == compute) {
                        } else if (c->gpu_deps && lseq) {
                            // a launch that says on the GPU when it is done: a one-lane kernel in front of
                            // the module waits for its number (launches of the stream end in order)
                            if ((int32_t)(lseq - c->waited_lseq) > 0 || c->waited_lseq == 0) {
                                HIP_TRY(c, tc_launch_wait(c->tickets + 33, lseq, c->spin_ticks, c->fault, c->tickets + 35, compute));
                                c->waited_lseq = lseq;
                            }
                        } else {
                            HIP_TRY(c, hipStreamWaitEvent(compute, c->op_ev[ticket % OP_RING], 0));
                        }
                        c->waited_op[st] = ticket;
                    }
                }
            }
        }
        if (dev_ptrs_out) dev_ptrs_out[i] = ptr;
        if ((rw[i] & TC_W) && ptr) {
            sa.ptr[sa.n] = ptr;
            sa.bytes[sa.n] = c->prof.bytes[t];
            sa.tensor[sa.n] = t;
            sa.whole[sa.n] = (rw[i] == TC_W && (c->budget.flags & TC_ALLOC_WRITE_ONLY)) ? 1 : 0;
            sa.n++;
        }
    }
    c->stats.stall_ns += waited_ns;
    if (waited_ns && step < c->stall_by_step.size()) c->stall_by_step[step] += waited_ns;
    return TC_OK;
}

// a bounded wait on the GPU ran out (tc_set_gpu_dependencies): a launch moved nothing or a module ran
// without its tensors; the bytes are not to be trusted from here on
static int gpu_wait_gave_up(tc_ctx *c)
{
    return fail(c, TC_E_HIP, *(volatile uint32_t *)c->fault == 1
                                 ? "a migration launch gave up waiting for the modules before it (do the compute stream "
                                   "and the migration stream share a hardware queue, or does a module run longer than the timeout?)"
                                 : "a module's wait for its migration launch ran out");
}

extern "C" int tc_migrate_step(tc_ctx *c, uint32_t step, int phase, const uint32_t *ids, const uint8_t *rw,
                               uint32_t n, void *compute_stream, void **dev_ptrs_out)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    if (phase != TC_PRE && phase != TC_POST) return fail(c, TC_E_ARG, "phase must be TC_PRE or TC_POST");
    if (c->fault && *(volatile uint32_t *)c->fault) return gpu_wait_gave_up(c);
    if (n > TC_MAX_STEP_TENSORS || (n && !ids)) return fail(c, TC_E_ARG, "too many tensors or null ids");
    // the profile ends with its last step that used a tensor: a module without tensors may follow
    if (step >= c->prof.n_steps && n) return fail(c, TC_E_ARG, "step outside the profiled iteration");
    if (phase == TC_PRE && n && !rw) return fail(c, TC_E_ARG, "PRE needs rw flags");
    TcStepArgs a{};
    for (uint32_t i = 0; i < n; ++i) {
        if (ids[i] >= c->prof.n_tensors) return fail(c, TC_E_ARG, "unknown tensor id");
        a.ids[i] = ids[i];
        a.rw[i] = rw ? rw[i] : (uint8_t)TC_R;
    }
    a.n = n; a.step = step; a.phase = (uint32_t)phase; a.cap = c->dout_cap;
    c->in_use = true;
    hipStream_t compute = (hipStream_t)compute_stream;
    const TcDecideOut *o = nullptr;
    const TcOpRec *ops = nullptr;
    int rc = take_ahead(c, step, phase, a.ids, a.rw, n, &o, &ops);
    if (rc != TC_OK) return rc;
    const bool ahead = o != nullptr;
    if (!ahead) {
        if ((rc = run_decide(c, a)) != TC_OK) return rc;
        o = c->dout;
        ops = c->dops;
    }
    rc = dispatch(c, o, ops, step, phase, compute);
    if (rc == TC_OK && phase == TC_PRE) rc = finish_pre(c, o, step, ids, a.rw, n, compute, dev_ptrs_out);
    if (rc != TC_OK) return rc;
    return ahead ? advance_ahead(c, o) : TC_OK;
}

extern "C" int tc_end_iteration(tc_ctx *c, void *compute_stream)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    TcStepArgs a{};
    a.n = 0; a.step = c->prof.n_steps; a.phase = TC_END; a.cap = c->dout_cap;
    c->in_use = true;
    int rc = settle_ahead(c);
    if (rc != TC_OK) return rc;
    rc = run_decide(c, a);
    if (rc != TC_OK) return rc;
    rc = dispatch(c, c->dout, c->dops, c->prof.n_steps, TC_END, (hipStream_t)compute_stream);
    if (rc != TC_OK) return rc;
    c->iteration = c->dout->iteration;
    c->stats.iteration = c->iteration;
    return TC_OK;
}

extern "C" int tc_emulate_compute(tc_ctx *c, void *compute_stream, uint64_t busy_ns)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    // Tensors written whole are filled, the others listed with TC_W are stamped.  A list may name a
    // tensor more than once: the writes apply in list order, so only the last whole write of a tensor
    // counts and only the stamps listed behind it survive.  The fills are launched ahead of the stamp
    // kernel on the same stream.
    const TcStampArgs &lp = c->last_pre;
    TcStampArgs sa{};
    sa.iteration = lp.iteration;
    sa.step = lp.step;
    sa.busy_ns = busy_ns;
    for (uint32_t i = 0; i < lp.n; ++i) {
        bool whole_later = false;                           // a whole write of the same tensor further down the list
        for (uint32_t k = i + 1; k < lp.n; ++k) whole_later = whole_later || (lp.whole[k] && lp.ptr[k] == lp.ptr[i]);
        if (whole_later) continue;
        if (lp.whole[i]) {
            const uint32_t seed = 0x10000000u + 4096u * lp.iteration + lp.step;
            HIP_TRY(c, tc_launch_fill(lp.ptr[i], lp.bytes[i], lp.tensor[i], seed, (hipStream_t)compute_stream));
        } else {
            sa.ptr[sa.n] = lp.ptr[i];
            sa.bytes[sa.n] = lp.bytes[i];
            sa.tensor[sa.n] = lp.tensor[i];
            sa.n++;
        }
    }
    if (sa.n || busy_ns) HIP_TRY(c, tc_launch_stamp(sa, (hipStream_t)compute_stream));
    return TC_OK;
}

extern "C" int tc_set_stall_measurement(tc_ctx *c, int enable)
{
    if (!c) return TC_E_ARG;
    c->measure_stall = enable != 0;
    return TC_OK;
}

extern "C" int tc_stall_by_step(tc_ctx *c, uint64_t *ns_out, uint32_t cap, int clear)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    if (ns_out) {
        if (cap < c->stall_by_step.size()) return fail(c, TC_E_CAPACITY, "ns_out holds fewer entries than the profile has steps");
        for (size_t k = 0; k < c->stall_by_step.size(); ++k) ns_out[k] = c->stall_by_step[k];
    }
    if (clear) std::fill(c->stall_by_step.begin(), c->stall_by_step.end(), 0);
    return TC_OK;
}

static int replay_windows(tc_ctx *c, const uint32_t *step_ptr, const uint32_t *ids, const uint8_t *rw,
                          uint32_t n_steps, void *compute_stream, const uint64_t *busy_ns);

extern "C" int tc_replay_iteration(tc_ctx *c, const uint32_t *step_ptr, const uint32_t *ids, const uint8_t *rw,
                                   uint32_t n_steps, void *compute_stream, const uint64_t *busy_ns, int measure_stall)
{
    if (!c || !step_ptr || !ids || !rw) return fail(c, TC_E_ARG, "null argument");
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    if (step_ptr[0] != 0) return fail(c, TC_E_ARG, "step_ptr must start at 0");
    // modules without tensors behind the profile's last step decide nothing and move nothing
    while (n_steps > c->prof.n_steps && step_ptr[n_steps] == step_ptr[n_steps - 1]) --n_steps;
    if (n_steps > c->prof.n_steps) return fail(c, TC_E_ARG, "more steps than the profiled iteration");
    for (uint32_t k = 0; k < n_steps; ++k) {
        if (step_ptr[k + 1] < step_ptr[k]) return fail(c, TC_E_ARG, "step_ptr must not decrease");
        if (step_ptr[k + 1] - step_ptr[k] > TC_MAX_STEP_TENSORS) return fail(c, TC_E_ARG, "too many tensors in a step");
    }
    const uint32_t n_ids = step_ptr[n_steps];
    for (uint32_t i = 0; i < n_ids; ++i) {
        if (ids[i] >= c->prof.n_tensors) return fail(c, TC_E_ARG, "unknown tensor id");
        if (rw[i] < 1 || rw[i] > 3) return fail(c, TC_E_ARG, "rw must be TC_R, TC_W or both");
    }
    const bool saved = c->measure_stall;
    c->measure_stall = saved || measure_stall != 0;
    c->in_use = true;
    int rc = settle_ahead(c);
    if (rc == TC_OK) rc = replay_windows(c, step_ptr, ids, rw, n_steps, compute_stream, busy_ns);
    c->measure_stall = saved;
    if (rc != TC_OK) return rc;
    return tc_end_iteration(c, compute_stream);
}

static int replay_windows(tc_ctx *c, const uint32_t *step_ptr, const uint32_t *ids, const uint8_t *rw,
                          uint32_t n_steps, void *compute_stream, const uint64_t *busy_ns)
{
    hipStream_t compute = (hipStream_t)compute_stream;
    const uint32_t n_ids = step_ptr[n_steps];
    // The lists go to the device once; the decision kernel then takes a window of
    // steps per launch.  Every launch the host waits for costs a running migration
    // launch some link time, so a replay that knows its trace decides in windows,
    // and window i+1 is decided (into the second result block) while window i is
    // dispatched.
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    HIP_TRY(c, hipMemcpy(c->d_step_ptr, step_ptr, ((size_t)n_steps + 1) * sizeof(uint32_t), hipMemcpyHostToDevice));
    if (n_ids) {
        HIP_TRY(c, hipMemcpy(c->d_ids, ids, (size_t)n_ids * sizeof(uint32_t), hipMemcpyHostToDevice));
        HIP_TRY(c, hipMemcpy(c->d_rw, rw, (size_t)n_ids, hipMemcpyHostToDevice));
    }
    auto launch = [&](uint32_t k0, uint32_t blk) -> int {
        TcWindowArgs w{};
        w.step_ptr = c->d_step_ptr; w.ids = c->d_ids; w.rw = c->d_rw;
        w.first = k0;
        w.count = std::min(c->replay_window, n_steps - k0);
        w.cap = c->dout_cap;
        w.n_calls = 2 * w.count;
        hipEvent_t t0;
        int rc = timed_begin(c, K_DECIDE, &t0);
        if (rc != TC_OK) return rc;
        HIP_TRY(c, tc_launch_decide_window(c->T, w, blk ? c->dout2 : c->dout, blk ? c->dops2 : c->dops, c->dstream));
        if ((rc = timed_end(c, K_DECIDE, t0, 2ull * w.count)) != TC_OK) return rc;
        c->stats.decide_launches++;
        return TC_OK;
    };
    uint32_t blk = 0;
    if (n_steps) {
        int rc = launch(0, 0);
        if (rc != TC_OK) return rc;
    }
    for (uint32_t k0 = 0; k0 < n_steps; k0 += c->replay_window, blk ^= 1) {
        const uint32_t count = std::min(c->replay_window, n_steps - k0);
        HIP_TRY(c, hipStreamSynchronize(c->dstream));
        if (c->fault && *(volatile uint32_t *)c->fault) return gpu_wait_gave_up(c);
        if (k0 + count < n_steps) {
            int rc = launch(k0 + count, blk ^ 1);
            if (rc != TC_OK) return rc;
        }
        const TcDecideOut *recs = blk ? c->dout2 : c->dout;
        const TcOpRec *ops = blk ? c->dops2 : c->dops;
        for (uint32_t k = k0; k < k0 + count; ++k) {
            const uint32_t n = step_ptr[k + 1] - step_ptr[k];
            const uint32_t *id = ids + step_ptr[k];
            const uint8_t *a = rw + step_ptr[k];
            const TcDecideOut *pre = recs + 2 * (k - k0), *post = pre + 1;
            int rc = dispatch(c, pre, ops, k, TC_PRE, compute);
            if (rc != TC_OK) return rc;
            ops += pre->n_ops;
            rc = finish_pre(c, pre, k, id, a, n, compute, nullptr);
            if (rc != TC_OK) return rc;
            rc = tc_emulate_compute(c, compute_stream, busy_ns ? busy_ns[k] : 0);
            if (rc != TC_OK) return rc;
            rc = dispatch(c, post, ops, k, TC_POST, compute);
            if (rc != TC_OK) return rc;
            ops += post->n_ops;
            c->stats.cursor = post->cursor;
        }
    }
    return TC_OK;
}

extern "C" int tc_synchronize(tc_ctx *c)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    if (!c->null_mover) {
        int rc = flush_deferred(c, c->last_compute);
        if (rc != TC_OK) return rc;
        for (int i = 0; i < N_STREAMS; ++i) {
            if (i == S_K || c->streams[i]) HIP_TRY(c, hipStreamSynchronize(c->streams[i]));
            c->op_done[i] = c->op_id;
        }
        rc = io_wait_all(c);                           // queued file I/O
        if (rc != TC_OK) return rc;
        c->st_q.clear();
        if (c->fault && *(volatile uint32_t *)c->fault) return gpu_wait_gave_up(c);
    }
    return TC_OK;
}

extern "C" int tc_cache_stats(const tc_ctx *c, tc_stats *out)
{
    if (!c || !out) return TC_E_ARG;
    *out = c->stats;
    out->file_write_ns += c->wr_ns.load();
    out->file_read_ns += c->rd_ns.load();
    return TC_OK;
}

extern "C" int tc_dump_oplog(const tc_ctx *c, uint64_t first, tc_op *buf, uint64_t cap, uint64_t *n_total)
{
    if (!c) return TC_E_ARG;
    if (n_total) *n_total = c->log.size();
    if (buf)
        for (uint64_t i = first, k = 0; i < c->log.size() && k < cap; ++i, ++k) buf[k] = c->log[i];
    return TC_OK;
}

extern "C" int tc_set_oplog(tc_ctx *c, int enable, int clear)
{
    if (!c) return TC_E_ARG;
    c->logging = enable != 0;
    if (clear) { c->log.clear(); c->log.shrink_to_fit(); }
    return TC_OK;
}

extern "C" int tc_dump_state(tc_ctx *c, uint8_t *tier, uint32_t *gpu_slot, uint32_t *cpu_slot)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    const uint32_t n_t = c->prof.n_tensors;
    int rcs = settle_ahead(c);
    if (rcs != TC_OK) return rcs;
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    std::vector<uint32_t> tmp(n_t);
    if (tier) {
        HIP_TRY(c, hipMemcpy(tmp.data(), c->T.cur, n_t * 4, hipMemcpyDeviceToHost));
        for (uint32_t t = 0; t < n_t; ++t) tier[t] = (uint8_t)tmp[t];
    }
    if (gpu_slot) HIP_TRY(c, hipMemcpy(gpu_slot, c->T.gslot, n_t * 4, hipMemcpyDeviceToHost));
    if (cpu_slot) HIP_TRY(c, hipMemcpy(cpu_slot, c->T.cslot, n_t * 4, hipMemcpyDeviceToHost));
    return TC_OK;
}

// where tensor t lives right now (reads three words of the device tables)
static int locate(tc_ctx *c, uint32_t t, uint32_t *tier, uint32_t *gs, uint32_t *cs)
{
    int rc = settle_ahead(c);
    if (rc != TC_OK) return rc;
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    HIP_TRY(c, hipMemcpy(tier, c->T.cur + t, 4, hipMemcpyDeviceToHost));
    HIP_TRY(c, hipMemcpy(gs, c->T.gslot + t, 4, hipMemcpyDeviceToHost));
    HIP_TRY(c, hipMemcpy(cs, c->T.cslot + t, 4, hipMemcpyDeviceToHost));
    return TC_OK;
}

extern "C" int tc_load_tensor(tc_ctx *c, uint32_t t, const void *src)
{
    if (!c || !src) return TC_E_ARG;
    if (c->stage != 4 || c->null_mover) return fail(c, TC_E_STATE, "needs bound memory");
    if (t >= c->prof.n_tensors) return fail(c, TC_E_ARG, "unknown tensor id");
    c->in_use = true;
    int rc = tc_synchronize(c);
    if (rc != TC_OK) return rc;
    uint32_t tier, gs, cs;
    rc = locate(c, t, &tier, &gs, &cs);
    if (rc != TC_OK) return rc;
    const uint32_t s = c->prof.class_of[t];
    const uint64_t n = c->prof.bytes[t];
    if (tier == TC_GPU && c->host_tier) memcpy(gpu_addr(c, s, gs), src, n);
    else if (tier == TC_GPU) HIP_TRY(c, hipMemcpy(gpu_addr(c, s, gs), src, n, hipMemcpyHostToDevice));
    else if (tier == TC_CPU) memcpy(cpu_addr(c, s, cs), src, n);
    else return io_transfer(c, t, const_cast<uint8_t *>((const uint8_t *)src), false);
    return TC_OK;
}

extern "C" int tc_read_tensor(tc_ctx *c, uint32_t t, void *dst)
{
    if (!c || !dst) return TC_E_ARG;
    if (c->stage != 4 || c->null_mover) return fail(c, TC_E_STATE, "needs bound memory");
    if (t >= c->prof.n_tensors) return fail(c, TC_E_ARG, "unknown tensor id");
    int rc = tc_synchronize(c);
    if (rc != TC_OK) return rc;
    HIP_TRY(c, hipDeviceSynchronize());
    uint32_t tier, gs, cs;
    rc = locate(c, t, &tier, &gs, &cs);
    if (rc != TC_OK) return rc;
    const uint32_t s = c->prof.class_of[t];
    const uint64_t n = c->prof.bytes[t];
    if (tier == TC_GPU && c->host_tier) memcpy(dst, gpu_addr(c, s, gs), n);
    else if (tier == TC_GPU) HIP_TRY(c, hipMemcpy(dst, gpu_addr(c, s, gs), n, hipMemcpyDeviceToHost));
    else if (tier == TC_CPU) memcpy(dst, cpu_addr(c, s, cs), n);
    else return io_transfer(c, t, (uint8_t *)dst, true);
    return TC_OK;
}

extern "C" int tc_fill_payload(tc_ctx *c, uint32_t seed)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4 || c->null_mover) return fail(c, TC_E_STATE, "needs bound memory");
    c->in_use = true;
    int rc = tc_synchronize(c);
    if (rc != TC_OK) return rc;
    const uint32_t n_t = c->prof.n_tensors;
    std::vector<uint8_t> tier(n_t);
    std::vector<uint32_t> gs(n_t), cs(n_t);
    rc = tc_dump_state(c, tier.data(), gs.data(), cs.data());
    if (rc != TC_OK) return rc;
    for (uint32_t t = 0; t < n_t; ++t) {
        const uint32_t s = c->prof.class_of[t];
        const uint64_t n = c->prof.bytes[t];
        if (tier[t] == TC_GPU) HIP_TRY(c, tc_launch_fill(gpu_addr(c, s, gs[t]), n, t, seed, c->streams[S_K]));
        else if (tier[t] == TC_CPU) HIP_TRY(c, tc_launch_fill(cpu_addr(c, s, cs[t]), n, t, seed, c->streams[S_K]));
        else {
            if (io_len(c, n) > c->staging_bytes) return fail(c, TC_E_CAPACITY, "staging region smaller than a file-tier tensor");
            HIP_TRY(c, tc_launch_fill(c->staging, n, t, seed, c->streams[S_K]));
            HIP_TRY(c, hipStreamSynchronize(c->streams[S_K]));
            rc = io_transfer(c, t, c->staging, false);
            if (rc != TC_OK) return rc;
        }
    }
    HIP_TRY(c, hipStreamSynchronize(c->streams[S_K]));
    return TC_OK;
}

extern "C" int tc_set_mover(tc_ctx *c, uint32_t workgroups, uint32_t chunk_bytes)
{
    if (!c) return TC_E_ARG;
    if (chunk_bytes && (chunk_bytes % 4096)) return fail(c, TC_E_ARG, "chunk_bytes must be a multiple of 4096");
    if (workgroups > 8192) return fail(c, TC_E_ARG, "too many workgroups");
    c->mover_wgs = workgroups ? workgroups : 12;
    c->chunk_bytes = chunk_bytes ? chunk_bytes : 16384;
    return TC_OK;
}

// The best number of working workgroups sits at a knee (too few leave the link idle, too
// many crowd each other) whose place depends on the host: measure it.  The regions hold
// nothing yet when this may be called, so exchanges between them can be timed freely.
extern "C" int tc_tune_mover(tc_ctx *c, uint32_t *workgroups_out)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4 || c->null_mover) return fail(c, TC_E_STATE, "needs bound memory");
    if (c->in_use) return fail(c, TC_E_STATE, "the regions already hold tensors");
    if (c->host_tier) {                                     // no copy kernel runs in the two-tier mode
        if (workgroups_out) *workgroups_out = c->mover_wgs;
        return TC_OK;
    }
    uint64_t bytes = std::min<uint64_t>(64ull << 20, std::min(c->hbm_bytes, c->pinned_bytes / 2));
    bytes &= ~(uint64_t)65535;
    if (workgroups_out) *workgroups_out = c->mover_wgs;
    if (bytes < (4ull << 20)) return TC_OK;                // too small to tell anything: keep the setting
    hipEvent_t e0, e1;
    HIP_TRY(c, hipEventCreate(&e0));
    HIP_TRY(c, hipEventCreate(&e1));
    const uint32_t candidates[] = {8, 10, 12, 14, 16, 20, 24};
    float best_ms = 1e30f;
    uint32_t best = c->mover_wgs;
    int rc = TC_OK;
    for (uint32_t wg : candidates) {
        float ms_min = 1e30f;
        for (int rep = 0; rep < 3 && rc == TC_OK; ++rep) {   // the first is a warm-up
            TcMoverArgs a{};
            a.chunk_bytes = c->chunk_bytes;
            a.tickets = c->tickets;
            a.xcc = c->mover_xcc;
            a.n_xcd = c->mover_xcds;
            const uint64_t per = (bytes / 4) & ~(uint64_t)4095;
            for (uint32_t u = 0; u < 4; ++u) {              // out: HBM -> pinned; in: the pinned half behind it -> HBM
                TcUnit &U = a.u[a.n_units++];
                U.out_src = c->hbm + u * per;
                U.out_dst = c->pinned + u * per;
                U.in_src = c->pinned + bytes + u * per;
                U.in_dst = c->hbm + u * per;
                U.bytes = per;
                U.chunk0 = a.n_chunks;
                a.n_chunks += (per + a.chunk_bytes - 1) / a.chunk_bytes;
            }
            hipError_t e = hipEventRecord(e0, c->streams[S_K]);
            if (e == hipSuccess) e = tc_launch_mover(a, wg, c->streams[S_K], &c->k_launches);
            if (e == hipSuccess) e = hipEventRecord(e1, c->streams[S_K]);
            if (e == hipSuccess) e = hipEventSynchronize(e1);
            float ms = 0;
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
            if (e != hipSuccess) { rc = fail(c, TC_E_HIP, hipGetErrorString(e)); break; }
            if (rep > 0) ms_min = std::min(ms_min, ms);
        }
        if (rc != TC_OK) break;
        if (ms_min < best_ms) { best_ms = ms_min; best = wg; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != TC_OK) return rc;
    c->mover_wgs = best;
    if (workgroups_out) *workgroups_out = best;
    return TC_OK;
}

static int collect_timing(tc_ctx *c, double busy_ns[N_KINDS], uint64_t count[N_KINDS], uint64_t bytes[N_KINDS])
{
    for (int i = 0; i < N_KINDS; ++i) { busy_ns[i] = 0; count[i] = 0; bytes[i] = 0; }
    int rcf = flush_deferred(c, c->last_compute);
    if (rcf != TC_OK) return rcf;
    if (c->timed.empty()) return TC_OK;
    for (int i = 0; i < N_STREAMS; ++i)
        if (i == S_K || c->streams[i]) HIP_TRY(c, hipStreamSynchronize(c->streams[i]));
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    for (auto &p : c->timed) {
        float ms = 0;
        if (hipEventElapsedTime(&ms, p.t0, p.t1) == hipSuccess) {
            busy_ns[p.kind] += (double)ms * 1e6;
            count[p.kind]++;
            bytes[p.kind] += p.bytes;
        }
        (void)hipEventDestroy(p.t0);
        (void)hipEventDestroy(p.t1);
    }
    c->timed.clear();
    return TC_OK;
}

extern "C" int tc_mover_timing(tc_ctx *c, int enable, tc_timing *out)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    double busy[N_KINDS];
    uint64_t cnt[N_KINDS], bytes[N_KINDS];
    int rc = collect_timing(c, busy, cnt, bytes);
    if (rc != TC_OK) return rc;
    if (out) {
        out->kernel_ns = busy[S_K]; out->kernel_launches = cnt[S_K]; out->kernel_bytes = bytes[S_K];
        out->h2d_ns = busy[S_H]; out->h2d_copies = cnt[S_H]; out->h2d_bytes = bytes[S_H];
        out->d2h_ns = busy[S_D]; out->d2h_copies = cnt[S_D]; out->d2h_bytes = bytes[S_D];
        out->decide_ns = busy[K_DECIDE]; out->decide_launches = cnt[K_DECIDE]; out->decide_calls = bytes[K_DECIDE];
    }
    c->timing = enable != 0;
    return TC_OK;
}

extern "C" int tc_set_merge_bytes(tc_ctx *c, uint64_t bytes)
{
    if (!c) return TC_E_ARG;
    c->merge_bytes = bytes;
    return TC_OK;
}

extern "C" int tc_set_gpu_dependencies(tc_ctx *c, int enable, uint32_t timeout_ms)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    if (enable && timeout_ms == 0) timeout_ms = 5000;
    if (timeout_ms > 600000) return fail(c, TC_E_ARG, "timeout above ten minutes");
    if (c->null_mover || c->host_tier) return TC_OK;        // no copy kernel runs
    // everything queued under the old setting finishes first: the two kinds of waiting do not mix
    int rc = tc_synchronize(c);
    if (rc != TC_OK) return rc;
    c->gpu_deps = enable != 0;
    c->sig_sent = false;
    if (enable) c->spin_ticks = (uint64_t)timeout_ms * 100000ull;      // the clock runs at 100 MHz
    return TC_OK;
}

extern "C" int tc_set_dma_policy(tc_ctx *c, int when_behind)
{
    if (!c) return TC_E_ARG;
    c->dma_when_behind = when_behind != 0;
    return TC_OK;
}

extern "C" int tc_set_decide_ahead(tc_ctx *c, uint32_t steps)
{
    if (!c) return TC_E_ARG;
    if (steps > TC_WINDOW_MAX) return fail(c, TC_E_ARG, "window out of range");
    if (c->stage == 4) {
        int rc = settle_ahead(c);
        if (rc != TC_OK) return rc;
    }
    c->ahead_steps = steps;
    return TC_OK;
}

extern "C" int tc_set_replay_window(tc_ctx *c, uint32_t steps)
{
    if (!c) return TC_E_ARG;
    if (steps == 0 || steps > TC_WINDOW_MAX) return fail(c, TC_E_ARG, "window must be 1 .. 256 steps");
    c->replay_window = steps;
    return TC_OK;
}

extern "C" int tc_set_dma_threshold(tc_ctx *c, uint64_t bytes)
{
    if (!c) return TC_E_ARG;
    if (bytes && c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    if (bytes && c->null_mover) return fail(c, TC_E_STATE, "no copies are made in this context");
    if (bytes && !c->bounce) {
        // The side streams and the bounce ring exist only once this path is asked
        // for: every stream a process holds is mapped onto a few hardware queues,
        // and an idle stream of ours could push the caller's compute stream onto
        // the queue the migration launches run on.
        for (int i = S_H; i < N_STREAMS; ++i)
            if (!c->streams[i]) HIP_TRY(c, hipStreamCreateWithFlags(&c->streams[i], hipStreamNonBlocking));
        // bounce ring in HBM: room for four of the largest tensors, 64 MiB .. 2 GiB
        uint64_t largest = 0;
        for (uint64_t st : c->pools.stride) largest = std::max(largest, st);
        c->bounce_bytes = std::min<uint64_t>(std::max<uint64_t>(4 * largest, 64ull << 20), 2048ull << 20);
        HIP_TRY(c, hipMalloc((void **)&c->bounce, c->bounce_bytes));
        // The runtime picks a stream's DMA engine at the stream's FIRST copy, among the engines idle at
        // that moment, and keeps it.  Two streams whose first copies do not overlap end up on one engine,
        // and copies in the two directions then run one after the other for good (measured: 28.6 GB/s per
        // direction instead of 48.6).  So the two side streams make their first copies here, at once: host
        // to HBM on one and, while that runs, HBM to host on the other, between the bounce block and a
        // pinned block that exists for this only.
        {
            const uint64_t w = 16ull << 20;
            void *tmp = nullptr;
            HIP_TRY(c, hipHostMalloc(&tmp, 2 * w, hipHostMallocDefault));
            hipError_t e = hipMemcpyAsync(c->bounce, tmp, w, hipMemcpyHostToDevice, c->streams[S_H]);
            if (e == hipSuccess)
                e = hipMemcpyAsync((uint8_t *)tmp + w, c->bounce + w, w, hipMemcpyDeviceToHost, c->streams[S_D]);
            if (e == hipSuccess) e = hipStreamSynchronize(c->streams[S_H]);
            if (e == hipSuccess) e = hipStreamSynchronize(c->streams[S_D]);
            (void)hipHostFree(tmp);
            if (e != hipSuccess) return fail(c, TC_E_HIP, std::string("first copies of the DMA streams: ") + hipGetErrorString(e));
        }
    }
    if (!bytes && c->bounce) {
        // back to the kernel alone: the side streams and the bounce ring go again (an idle
        // stream of ours is not harmless, see above)
        int rc = tc_synchronize(c);
        if (rc != TC_OK) return rc;
        for (int i = S_H; i < N_STREAMS; ++i)
            if (c->streams[i]) { HIP_TRY(c, hipStreamDestroy(c->streams[i])); c->streams[i] = nullptr; }
        HIP_TRY(c, hipFree(c->bounce));
        c->bounce = nullptr;
        c->bounce_bytes = 0;
        c->bounce_q.clear();
        c->bounce_head = 0;
    }
    c->sdma_threshold = bytes;
    return TC_OK;
}