// Runtime of libtc.so: the context, memory binding, the per-hook dispatch that
// turns the decision kernel's op records into migration-kernel launches and
// file-tier I/O, statistics, and the C ABI of include/tc.h.
#include "tc_internal.h"

#include <errno.h>
#include <string.h>
#include <unistd.h>

#include <algorithm>
#include <chrono>

namespace {

const uint32_t EVENT_RING = 256;

struct Pending {            // file write that must wait for a migration launch
    uint64_t launch;
    const uint8_t *src;
    uint64_t bytes, file_off;
};

} // namespace

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
    int fd = -1;
    hipStream_t mstream = nullptr;      // migration stream (caller's)
    hipStream_t dstream = nullptr;      // decision stream (ours)
    bool null_mover = false;

    // device tables
    uint32_t *dev_block = nullptr;      // one allocation holding every table
    TcDevTables T{};
    TcDecideOut *dout = nullptr;        // pinned result block of the decision kernel
    uint32_t dout_cap = 0;

    // dispatch state
    uint32_t mover_wgs = 512, chunk_bytes = 65536;
    uint64_t launch_id = 0;             // migration launches issued
    uint64_t launch_done = 0;           // launches known complete
    hipEvent_t ring[EVENT_RING]{};
    hipEvent_t ev_compute = nullptr;
    std::vector<uint64_t> gpu_ticket, cpu_ticket;   // last launch that touched the buffer
    uint64_t staging_ticket = 0;
    uint64_t staging_used = 0;
    std::vector<Pending> pending;
    // last PRE call, for tc_emulate_compute
    TcStampArgs last_pre{};
    uint64_t last_pre_ticket = 0;
    uint32_t iteration = 0;

    // mover timing
    bool timing = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> timed;

    std::vector<tc_op> log;
    tc_stats stats{};
};

static int fail(tc_ctx *c, int code, const std::string &msg)
{
    if (c) c->err = msg;
    return code;
}

#define HIP_TRY(c, expr)                                                                          \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess)                                                                     \
            return fail((c), TC_E_HIP, std::string(#expr) + ": " + hipGetErrorString(e_));        \
    } while (0)

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
    if (c->dstream) { (void)hipStreamSynchronize(c->dstream); }
    if (c->mstream || c->stage >= 4) { (void)hipStreamSynchronize(c->mstream); }
    for (auto &p : c->timed) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
    c->timed.clear();
    for (uint32_t i = 0; i < EVENT_RING; ++i)
        if (c->ring[i]) { (void)hipEventDestroy(c->ring[i]); c->ring[i] = nullptr; }
    if (c->ev_compute) { (void)hipEventDestroy(c->ev_compute); c->ev_compute = nullptr; }
    if (c->dstream) { (void)hipStreamDestroy(c->dstream); c->dstream = nullptr; }
    if (c->dev_block) { (void)hipFree(c->dev_block); c->dev_block = nullptr; }
    if (c->dout) { (void)hipHostFree(c->dout); c->dout = nullptr; }
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
    int rc = tc_build_profile(p, t, n_t, ev, n_ev, err);
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
    int rc = tc_build_pools(c->prof, *b, pools, err);
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
    tc_build_placement(c->prof, c->pools, c->place);
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
    T.cur = d + o_cur; T.gslot = d + o_gs; T.cslot = d + o_cs; T.dirty = d + o_dirty; T.moved = d + o_moved;
    T.gpu_owner = d + o_go; T.gpu_freed = d + o_gf; T.cpu_owner = d + o_co; T.cpu_freed = d + o_cf;
    T.designated = d + o_des; T.scalars = d + o_sc;

    c->dout_cap = 3 * n_t + 64;
    e = hipHostMalloc((void **)&c->dout, sizeof(TcDecideOut) + (size_t)c->dout_cap * sizeof(TcOpRec), hipHostMallocDefault);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    memset(c->dout, 0, sizeof(TcDecideOut));
    e = hipStreamCreateWithFlags(&c->dstream, hipStreamNonBlocking);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    for (uint32_t i = 0; i < EVENT_RING; ++i) {
        e = hipEventCreateWithFlags(&c->ring[i], hipEventDisableTiming);
        if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }
    }
    e = hipEventCreateWithFlags(&c->ev_compute, hipEventDisableTiming);
    if (e != hipSuccess) { release_device(c); return fail(c, TC_E_HIP, hipGetErrorString(e)); }

    c->hbm = (uint8_t *)hbm; c->hbm_bytes = hbm_bytes;
    c->pinned = (uint8_t *)pinned; c->pinned_bytes = pinned_bytes;
    c->staging = (uint8_t *)staging; c->staging_bytes = staging_bytes;
    c->fd = fd;
    c->mstream = (hipStream_t)mstream;
    c->null_mover = null_mover;
    c->gpu_ticket.assign(pl.gpu_slots, 0);
    c->cpu_ticket.assign(pl.cpu_slots, 0);
    c->stage = 4;
    return TC_OK;
}

// ---------------------------------------------------------------------------
// addresses and waits
// ---------------------------------------------------------------------------
static inline uint8_t *gpu_addr(const tc_ctx *c, uint32_t s, uint32_t k)
{
    return c->hbm + c->pools.hbm_off[s] + (uint64_t)k * c->pools.stride[s];
}
static inline uint8_t *cpu_addr(const tc_ctx *c, uint32_t s, uint32_t k)
{
    return c->pinned + c->pools.host_off[s] + (uint64_t)k * c->pools.stride[s];
}

// block the host until migration launch `id` has completed
static int wait_launch(tc_ctx *c, uint64_t id)
{
    if (id <= c->launch_done) return TC_OK;
    if (c->launch_id - id >= EVENT_RING) {           // its event was recycled: the stream is in order
        HIP_TRY(c, hipStreamSynchronize(c->mstream));
        c->launch_done = c->launch_id;
        return TC_OK;
    }
    HIP_TRY(c, hipEventSynchronize(c->ring[id % EVENT_RING]));
    c->launch_done = std::max(c->launch_done, id);
    return TC_OK;
}

static int file_write(tc_ctx *c, const uint8_t *src, uint64_t bytes, uint64_t off)
{
    if (c->fd < 0) return fail(c, TC_E_IO, "an op needs the file tier but no file is bound");
    while (bytes) {
        ssize_t w = pwrite(c->fd, src, bytes, (off_t)off);
        if (w < 0 && errno == EINTR) continue;
        if (w <= 0) return fail(c, TC_E_IO, std::string("pwrite: ") + strerror(errno));
        src += w; off += (uint64_t)w; bytes -= (uint64_t)w;
    }
    return TC_OK;
}

static int file_read(tc_ctx *c, uint8_t *dst, uint64_t bytes, uint64_t off)
{
    if (c->fd < 0) return fail(c, TC_E_IO, "an op needs the file tier but no file is bound");
    while (bytes) {
        ssize_t r = pread(c->fd, dst, bytes, (off_t)off);
        if (r < 0 && errno == EINTR) continue;
        if (r <= 0) return fail(c, TC_E_IO, r == 0 ? std::string("pread: short file") : std::string("pread: ") + strerror(errno));
        dst += r; off += (uint64_t)r; bytes -= (uint64_t)r;
    }
    return TC_OK;
}

// ---------------------------------------------------------------------------
// dispatch: op records -> migration launches + file I/O
// ---------------------------------------------------------------------------
namespace {
struct Batch {
    TcMoverArgs args{};                                      // zeroed: counts start at 0
    std::vector<std::pair<uint32_t, uint32_t>> gpu_touched;  // flat buffer indices
    std::vector<uint32_t> cpu_touched;
    bool uses_staging = false;
};
}

static int flush_batch(tc_ctx *c, Batch &b, bool wait_compute, hipStream_t compute)
{
    if (b.args.n_units == 0) return TC_OK;
    const uint64_t id = c->launch_id + 1;
    hipEvent_t ev = c->ring[id % EVENT_RING];
    if (id > EVENT_RING) {                            // the event's previous user must be done
        int rc = wait_launch(c, id - EVENT_RING);
        if (rc != TC_OK) return rc;
    }
    if (wait_compute) {
        HIP_TRY(c, hipEventRecord(c->ev_compute, compute));
        HIP_TRY(c, hipStreamWaitEvent(c->mstream, c->ev_compute, 0));
    }
    hipEvent_t t0 = nullptr, t1 = nullptr;
    if (c->timing) {
        HIP_TRY(c, hipEventCreate(&t0));
        HIP_TRY(c, hipEventCreate(&t1));
        HIP_TRY(c, hipEventRecord(t0, c->mstream));
    }
    HIP_TRY(c, tc_launch_mover(b.args, c->mover_wgs, c->mstream));
    if (c->timing) {
        HIP_TRY(c, hipEventRecord(t1, c->mstream));
        c->timed.push_back({t0, t1});
    }
    HIP_TRY(c, hipEventRecord(ev, c->mstream));
    c->launch_id = id;
    for (auto &g : b.gpu_touched) c->gpu_ticket[g.first] = id;
    for (uint32_t x : b.cpu_touched) c->cpu_ticket[x] = id;
    if (b.uses_staging) c->staging_ticket = id;
    c->stats.mover_launches++;
    c->stats.mover_units += b.args.n_units;
    b = Batch();
    return TC_OK;
}

// writes that waited for a launch (GPU buffer -> staging -> file)
static int drain_pending(tc_ctx *c)
{
    for (const Pending &p : c->pending) {
        int rc = wait_launch(c, p.launch);
        if (rc != TC_OK) return rc;
        rc = file_write(c, p.src, p.bytes, p.file_off);
        if (rc != TC_OK) return rc;
    }
    c->pending.clear();
    return TC_OK;
}

static int staging_alloc(tc_ctx *c, Batch &b, uint64_t bytes, bool wait_compute, hipStream_t compute, uint8_t **out)
{
    const uint64_t need = (bytes + 255) & ~255ull;
    if (need > c->staging_bytes) return fail(c, TC_E_CAPACITY, "staging region smaller than a tensor that needs the file tier");
    if (c->staging_used + need > c->staging_bytes) {
        // out of bounce space: issue what is batched, let it finish, start over
        int rc = flush_batch(c, b, wait_compute, compute);
        if (rc != TC_OK) return rc;
        rc = drain_pending(c);
        if (rc != TC_OK) return rc;
        rc = wait_launch(c, c->staging_ticket);
        if (rc != TC_OK) return rc;
        c->staging_used = 0;
    }
    if (c->staging_used == 0) {
        int rc = wait_launch(c, c->staging_ticket);   // earlier calls' reads of the bounce space
        if (rc != TC_OK) return rc;
    }
    *out = c->staging + c->staging_used;
    c->staging_used += need;
    b.uses_staging = true;
    return TC_OK;
}

static int dispatch(tc_ctx *c, uint32_t step, hipStream_t compute)
{
    const TcDecideOut *o = c->dout;
    const TcOpRec *ops = (const TcOpRec *)(o + 1);
    if (o->overflow) return fail(c, TC_E_CAPACITY, "decision log overflow");
    Batch b{};
    TcUnit pend{};                  // outgoing half waiting for its incoming partner
    bool have_out = false;
    std::pair<uint32_t, uint32_t> out_gpu{0, 0};
    int64_t out_cpu = -1;
    bool out_staging = false;
    uint32_t out_tensor = 0;
    uint8_t *reserved_in = nullptr;  // bounce space kept for the partner of a write-back
    c->staging_used = 0;
    for (uint32_t i = 0; i < o->n_ops; ++i) {
        const TcOpRec &r = ops[i];
        const uint32_t t = r.tensor;
        // never turn a record into an address before it is known to be in range
        if (t >= c->prof.n_tensors || r.op > TC_OP_FAIL)
            return fail(c, TC_E_HIP, "decision record out of range (tensor/op)");
        {
            const uint32_t sc = c->prof.class_of[t];
            const bool src_ok = r.src_tier == TC_GPU ? r.src_slot < c->pools.gpu_count[sc]
                              : r.src_tier == TC_CPU ? r.src_slot < c->pools.cpu_count[sc] : r.src_slot == TC_NONE;
            const bool dst_ok = r.dst_tier == TC_GPU ? r.dst_slot < c->pools.gpu_count[sc]
                              : r.dst_tier == TC_CPU ? r.dst_slot < c->pools.cpu_count[sc] : r.dst_slot == TC_NONE;
            if (r.op != TC_OP_FAIL && !(src_ok && dst_ok))
                return fail(c, TC_E_HIP, "decision record out of range (slot)");
        }
        const uint32_t s = c->prof.class_of[t];
        const uint64_t n = c->prof.bytes[t];
        tc_op rec;
        rec.iteration = c->iteration; rec.step = step; rec.tensor = t;
        rec.src_slot = r.src_slot; rec.dst_slot = r.dst_slot;
        rec.phase = r.phase; rec.op = r.op; rec.src_tier = r.src_tier; rec.dst_tier = r.dst_tier;
        rec.bytes = (r.op == TC_OP_RELEASE || r.op == TC_OP_FAIL) ? 0 : n;
        c->log.push_back(rec);
        c->stats.n_ops[r.op]++;
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
        const bool wait_compute = true;
        switch (r.op) {
        case TC_OP_SPILL: {
            // host buffer -> file extent, now: the buffer is about to be reused
            const uint32_t flat = c->pools.cpu_base[s] + r.src_slot;
            int rc = wait_launch(c, c->cpu_ticket[flat]);
            if (rc != TC_OK) return rc;
            rc = file_write(c, cpu_addr(c, s, r.src_slot), n, c->place.file_off[t]);
            if (rc != TC_OK) return rc;
            break;
        }
        case TC_OP_EVICT: {
            pend = TcUnit{};
            pend.out_src = gpu_addr(c, s, r.src_slot);
            pend.out_dst = cpu_addr(c, s, r.dst_slot);
            pend.bytes = n;
            have_out = true;
            out_gpu = {c->pools.gpu_base[s] + r.src_slot, 0};
            out_cpu = c->pools.cpu_base[s] + r.dst_slot;
            out_staging = false;
            break;
        }
        case TC_OP_WRITEBACK: {
            // room for the outgoing bytes and, right behind them, for an
            // incoming tensor of the same class should it come from the file tier
            uint8_t *st = nullptr;
            const uint64_t half = (n + 255) & ~255ull;
            int rc = staging_alloc(c, b, 2 * half, wait_compute, compute, &st);
            if (rc != TC_OK) return rc;
            reserved_in = st + half;
            pend = TcUnit{};
            pend.out_src = gpu_addr(c, s, r.src_slot);
            pend.out_dst = st;
            pend.bytes = n;
            have_out = true;
            out_gpu = {c->pools.gpu_base[s] + r.src_slot, 0};
            out_cpu = -1;
            out_staging = true;
            out_tensor = t;
            break;
        }
        case TC_OP_DEMAND:
        case TC_OP_PREFETCH: {
            TcUnit u = have_out ? pend : TcUnit{};
            u.bytes = n;
            u.in_dst = gpu_addr(c, s, r.dst_slot);
            int64_t in_cpu = -1;
            if (r.src_tier == TC_CPU) {
                u.in_src = cpu_addr(c, s, r.src_slot);
                in_cpu = c->pools.cpu_base[s] + r.src_slot;
            } else {
                uint8_t *st = nullptr;
                int rc = TC_OK;
                if (have_out && out_staging) st = reserved_in;
                else rc = staging_alloc(c, b, n, wait_compute, compute, &st);
                if (rc != TC_OK) return rc;
                rc = file_read(c, st, n, c->place.file_off[t]);
                if (rc != TC_OK) return rc;
                u.in_src = st;
            }
            if (b.args.n_units == TC_MOVER_MAX_UNITS) {
                int rc = flush_batch(c, b, wait_compute, compute);
                if (rc != TC_OK) return rc;
            }
            u.chunk0 = b.args.n_chunks;
            b.args.n_chunks += (n + c->chunk_bytes - 1) / c->chunk_bytes;
            b.args.chunk_bytes = c->chunk_bytes;
            b.args.u[b.args.n_units++] = u;
            b.gpu_touched.push_back({c->pools.gpu_base[s] + r.dst_slot, 0});
            if (have_out) b.gpu_touched.push_back(out_gpu);
            if (in_cpu >= 0) b.cpu_touched.push_back((uint32_t)in_cpu);
            if (have_out && out_cpu >= 0) b.cpu_touched.push_back((uint32_t)out_cpu);
            if (r.src_tier != TC_CPU || (have_out && out_staging)) b.uses_staging = true;
            if (have_out && out_staging) {
                Pending p;
                p.launch = c->launch_id + 1;          // the launch this batch becomes
                p.src = u.out_dst;
                p.bytes = c->prof.bytes[out_tensor];
                p.file_off = c->place.file_off[out_tensor];
                c->pending.push_back(p);
            }
            have_out = false;
            break;
        }
        case TC_OP_RESTORE: {
            // file extent -> host buffer, by the host; earlier copies that read
            // or wrote the buffer must have finished
            int rc = flush_batch(c, b, wait_compute, compute);
            if (rc != TC_OK) return rc;
            const uint32_t flat = c->pools.cpu_base[s] + r.dst_slot;
            rc = wait_launch(c, c->cpu_ticket[flat]);
            if (rc != TC_OK) return rc;
            rc = file_read(c, cpu_addr(c, s, r.dst_slot), n, c->place.file_off[t]);
            if (rc != TC_OK) return rc;
            break;
        }
        default: break;                               // RELEASE, FAIL: nothing moves
        }
    }
    if (c->null_mover) return TC_OK;
    int rc = flush_batch(c, b, true, compute);
    if (rc != TC_OK) return rc;
    return drain_pending(c);
}

static int run_decide(tc_ctx *c, const TcStepArgs &a)
{
    HIP_TRY(c, tc_launch_decide(c->T, a, c->dout, c->dstream));
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    c->stats.decide_launches++;
    c->stats.cursor = c->dout->cursor;
    return TC_OK;
}

extern "C" int tc_migrate_step(tc_ctx *c, uint32_t step, int phase, const uint32_t *ids, const uint8_t *rw,
                               uint32_t n, void *compute_stream, void **dev_ptrs_out)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    if (phase != TC_PRE && phase != TC_POST) return fail(c, TC_E_ARG, "phase must be TC_PRE or TC_POST");
    if (n > TC_MAX_STEP_TENSORS || (n && !ids)) return fail(c, TC_E_ARG, "too many tensors or null ids");
    if (step >= c->prof.n_steps) return fail(c, TC_E_ARG, "step outside the profiled iteration");
    if (phase == TC_PRE && n && !rw) return fail(c, TC_E_ARG, "PRE needs rw flags");
    TcStepArgs a{};
    for (uint32_t i = 0; i < n; ++i) {
        if (ids[i] >= c->prof.n_tensors) return fail(c, TC_E_ARG, "unknown tensor id");
        a.ids[i] = ids[i];
        a.rw[i] = rw ? rw[i] : (uint8_t)TC_R;
    }
    a.n = n; a.step = step; a.phase = (uint32_t)phase; a.cap = c->dout_cap;
    int rc = run_decide(c, a);
    if (rc != TC_OK) return rc;
    hipStream_t compute = (hipStream_t)compute_stream;
    rc = dispatch(c, step, compute);
    if (rc != TC_OK) return rc;
    if (phase == TC_PRE) {
        const TcDecideOut *o = c->dout;
        c->stats.hits += o->hits;
        c->stats.misses += o->misses;
        c->stats.fails += o->fails;
        TcStampArgs &sa = c->last_pre;
        sa = TcStampArgs{};
        sa.iteration = c->iteration;
        sa.step = step;
        uint64_t ticket = 0;
        for (uint32_t i = 0; i < n; ++i) {
            const uint32_t t = ids[i], s = c->prof.class_of[t];
            uint8_t *ptr = nullptr;
            if (o->slots[i] != TC_NONE) {
                if (!c->null_mover) ptr = gpu_addr(c, s, o->slots[i]);
                ticket = std::max(ticket, c->gpu_ticket[c->pools.gpu_base[s] + o->slots[i]]);
            }
            if (dev_ptrs_out) dev_ptrs_out[i] = ptr;
            if ((a.rw[i] & TC_W) && ptr) {
                sa.ptr[sa.n] = ptr;
                sa.bytes[sa.n] = c->prof.bytes[t];
                sa.tensor[sa.n] = t;
                sa.n++;
            }
        }
        c->last_pre_ticket = ticket;
        // the module's kernels wait only for the copies that fill ITS buffers
        if (!c->null_mover && ticket > c->launch_done && c->launch_id - ticket < EVENT_RING)
            HIP_TRY(c, hipStreamWaitEvent(compute, c->ring[ticket % EVENT_RING], 0));
        else if (!c->null_mover && ticket > c->launch_done) {
            rc = wait_launch(c, ticket);
            if (rc != TC_OK) return rc;
        }
    }
    return TC_OK;
}

extern "C" int tc_end_iteration(tc_ctx *c, void *compute_stream)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    TcStepArgs a{};
    a.n = 0; a.step = c->prof.n_steps; a.phase = TC_END; a.cap = c->dout_cap;
    int rc = run_decide(c, a);
    if (rc != TC_OK) return rc;
    rc = dispatch(c, c->prof.n_steps, (hipStream_t)compute_stream);
    if (rc != TC_OK) return rc;
    c->iteration = c->dout->iteration;
    c->stats.iteration = c->iteration;
    return TC_OK;
}

extern "C" int tc_emulate_compute(tc_ctx *c, void *compute_stream, uint64_t busy_ns, int measure_stall)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    hipStream_t compute = (hipStream_t)compute_stream;
    TcStampArgs sa = c->last_pre;
    sa.busy_ns = busy_ns;
    if (measure_stall) {
        // stall = how long the copies this step depends on outlast the compute
        // already queued: drain compute, then time the wait for the ticket
        HIP_TRY(c, hipStreamSynchronize(compute));
        auto t0 = std::chrono::steady_clock::now();
        int rc = wait_launch(c, c->last_pre_ticket);
        if (rc != TC_OK) return rc;
        uint64_t ns = (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
                          std::chrono::steady_clock::now() - t0).count();
        c->stats.stall_ns += ns;
        c->stats.waits_total++;
        if (ns < 30000) c->stats.waits_under_30us++;
    }
    if (sa.n || busy_ns) HIP_TRY(c, tc_launch_stamp(sa, compute));
    return TC_OK;
}

extern "C" int tc_replay_iteration(tc_ctx *c, const uint32_t *step_ptr, const uint32_t *ids, const uint8_t *rw,
                                   uint32_t n_steps, void *compute_stream, const uint64_t *busy_ns, int measure_stall)
{
    if (!c || !step_ptr || !ids || !rw) return fail(c, TC_E_ARG, "null argument");
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    if (n_steps > c->prof.n_steps) return fail(c, TC_E_ARG, "more steps than the profiled iteration");
    for (uint32_t k = 0; k < n_steps; ++k) {
        if (step_ptr[k + 1] < step_ptr[k]) return fail(c, TC_E_ARG, "step_ptr must not decrease");
        const uint32_t n = step_ptr[k + 1] - step_ptr[k];
        const uint32_t *id = ids + step_ptr[k];
        const uint8_t *a = rw + step_ptr[k];
        int rc = tc_migrate_step(c, k, TC_PRE, id, a, n, compute_stream, nullptr);
        if (rc != TC_OK) return rc;
        rc = tc_emulate_compute(c, compute_stream, busy_ns ? busy_ns[k] : 0, measure_stall);
        if (rc != TC_OK) return rc;
        rc = tc_migrate_step(c, k, TC_POST, id, a, n, compute_stream, nullptr);
        if (rc != TC_OK) return rc;
    }
    return tc_end_iteration(c, compute_stream);
}

extern "C" int tc_synchronize(tc_ctx *c)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    HIP_TRY(c, hipStreamSynchronize(c->dstream));
    if (!c->null_mover) {
        HIP_TRY(c, hipStreamSynchronize(c->mstream));
        c->launch_done = c->launch_id;
    }
    return TC_OK;
}

extern "C" int tc_cache_stats(const tc_ctx *c, tc_stats *out)
{
    if (!c || !out) return TC_E_ARG;
    *out = c->stats;
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

extern "C" int tc_dump_state(tc_ctx *c, uint8_t *tier, uint32_t *gpu_slot, uint32_t *cpu_slot)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    const uint32_t n_t = c->prof.n_tensors;
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
    int rc = tc_synchronize(c);
    if (rc != TC_OK) return rc;
    uint32_t tier, gs, cs;
    rc = locate(c, t, &tier, &gs, &cs);
    if (rc != TC_OK) return rc;
    const uint32_t s = c->prof.class_of[t];
    const uint64_t n = c->prof.bytes[t];
    if (tier == TC_GPU) HIP_TRY(c, hipMemcpy(gpu_addr(c, s, gs), src, n, hipMemcpyHostToDevice));
    else if (tier == TC_CPU) memcpy(cpu_addr(c, s, cs), src, n);
    else return file_write(c, (const uint8_t *)src, n, c->place.file_off[t]);
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
    if (tier == TC_GPU) HIP_TRY(c, hipMemcpy(dst, gpu_addr(c, s, gs), n, hipMemcpyDeviceToHost));
    else if (tier == TC_CPU) memcpy(dst, cpu_addr(c, s, cs), n);
    else return file_read(c, (uint8_t *)dst, n, c->place.file_off[t]);
    return TC_OK;
}

extern "C" int tc_fill_payload(tc_ctx *c, uint32_t seed)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4 || c->null_mover) return fail(c, TC_E_STATE, "needs bound memory");
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
        if (tier[t] == TC_GPU) HIP_TRY(c, tc_launch_fill(gpu_addr(c, s, gs[t]), n, t, seed, c->mstream));
        else if (tier[t] == TC_CPU) HIP_TRY(c, tc_launch_fill(cpu_addr(c, s, cs[t]), n, t, seed, c->mstream));
        else {
            if (n > c->staging_bytes) return fail(c, TC_E_CAPACITY, "staging region smaller than a file-tier tensor");
            HIP_TRY(c, tc_launch_fill(c->staging, n, t, seed, c->mstream));
            HIP_TRY(c, hipStreamSynchronize(c->mstream));
            rc = file_write(c, c->staging, n, c->place.file_off[t]);
            if (rc != TC_OK) return rc;
        }
    }
    HIP_TRY(c, hipStreamSynchronize(c->mstream));
    return TC_OK;
}

extern "C" int tc_set_mover(tc_ctx *c, uint32_t workgroups, uint32_t chunk_bytes)
{
    if (!c) return TC_E_ARG;
    if (chunk_bytes && (chunk_bytes % 4096)) return fail(c, TC_E_ARG, "chunk_bytes must be a multiple of 4096");
    if (workgroups > 65536) return fail(c, TC_E_ARG, "too many workgroups");
    c->mover_wgs = workgroups ? workgroups : 512;
    c->chunk_bytes = chunk_bytes ? chunk_bytes : 65536;
    return TC_OK;
}

extern "C" int tc_mover_timing(tc_ctx *c, int enable, double *avg_ns, uint64_t *n)
{
    if (!c) return TC_E_ARG;
    if (c->stage != 4) return fail(c, TC_E_STATE, "tc_bind_memory must come first");
    double total = 0;
    uint64_t cnt = 0;
    if (!c->timed.empty()) {
        HIP_TRY(c, hipStreamSynchronize(c->mstream));
        for (auto &p : c->timed) {
            float ms = 0;
            if (hipEventElapsedTime(&ms, p.first, p.second) == hipSuccess) { total += (double)ms * 1e6; cnt++; }
            (void)hipEventDestroy(p.first);
            (void)hipEventDestroy(p.second);
        }
        c->timed.clear();
    }
    if (avg_ns) *avg_ns = cnt ? total / (double)cnt : 0.0;
    if (n) *n = cnt;
    c->timing = enable != 0;
    return TC_OK;
}

// ---------------------------------------------------------------------------
// stand-alone kernels
// ---------------------------------------------------------------------------
extern "C" int tc_copy_batch(const tc_segment *segs, uint32_t n, void *stream, uint32_t workgroups,
                             uint32_t chunk_bytes)
{
    if (!segs && n) return TC_E_ARG;
    if (!workgroups) workgroups = 512;
    if (!chunk_bytes) chunk_bytes = 65536;
    if (chunk_bytes % 4096) return TC_E_ARG;
    uint32_t i = 0;
    while (i < n) {
        TcMoverArgs a{};
        a.chunk_bytes = chunk_bytes;
        for (; i < n && a.n_units < TC_MOVER_MAX_UNITS; ++i) {
            if (!segs[i].bytes) continue;
            if (!segs[i].src || !segs[i].dst) return TC_E_ARG;
            if ((((uintptr_t)segs[i].src) | ((uintptr_t)segs[i].dst)) & 15) return TC_E_ARG;
            TcUnit &u = a.u[a.n_units++];
            u.in_src = (const uint8_t *)segs[i].src;
            u.in_dst = (uint8_t *)segs[i].dst;
            u.bytes = segs[i].bytes;
            u.chunk0 = a.n_chunks;
            a.n_chunks += (segs[i].bytes + chunk_bytes - 1) / chunk_bytes;
        }
        if (tc_launch_mover(a, workgroups, (hipStream_t)stream) != hipSuccess) return TC_E_HIP;
    }
    return TC_OK;
}

extern "C" int tc_pack(void *slab, const void *const *ptrs, const uint64_t *bytes, const uint64_t *slab_off,
                       uint32_t n, uint64_t total, void *stream)
{
    if ((!slab || !ptrs || !bytes || !slab_off) && n) return TC_E_ARG;
    if ((uintptr_t)slab & 15) return TC_E_ARG;
    return tc_launch_pack(slab, ptrs, bytes, slab_off, n, total, 0, (hipStream_t)stream) == hipSuccess ? TC_OK : TC_E_HIP;
}

extern "C" int tc_unpack(const void *slab, void *const *ptrs, const uint64_t *bytes, const uint64_t *slab_off,
                         uint32_t n, uint64_t total, void *stream)
{
    if ((!slab || !ptrs || !bytes || !slab_off) && n) return TC_E_ARG;
    if ((uintptr_t)slab & 15) return TC_E_ARG;
    return tc_launch_pack((void *)slab, (const void *const *)ptrs, bytes, slab_off, n, total, 1,
                          (hipStream_t)stream) == hipSuccess ? TC_OK : TC_E_HIP;
}
