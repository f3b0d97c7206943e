// HIP kernels for gfx950 (MI355X): the scheduler's decision kernel, the batched
// migration kernel, the stamp/spin stand-in for module compute, the payload
// fill kernel and the pack/unpack kernel.
#include "tc_internal.h"

#include <mutex>

#define NONE 0xFFFFFFFFu
#define WAVE 64

// ===========================================================================
// Decision kernel: the prefetch-eviction scheduler of Sec. 3.4 (Alg. 3 and
// Alg. 4) as ONE wavefront.
//
// The scheduler is a sequential state machine (each decision moves the
// cursor and the owner tables the next one reads), so the sequence of
// decisions stays in one wave.  What the wave parallelises is each decision's
// table search: residency of the rows ahead of the cursor and lowest free
// buffer by ballot + find-first-set, farthest-next-use victim by a 64-lane
// max-reduction.  All control flow is wave-uniform.  Every lane performs every
// state store itself (same address, same value), so a lane's later loads see
// the table as updated without any cross-lane memory ordering.
// ===========================================================================

struct DecideCtx {
    TcDevTables T;
    TcDecideOut *out;
    TcOpRec *ops;
    uint32_t cap, n_ops;
    uint32_t call, bound, step, phase;
    uint32_t lane;
};

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        uint32_t lo = __shfl_xor((uint32_t)v, off, WAVE);
        uint32_t hi = __shfl_xor((uint32_t)(v >> 32), off, WAVE);
        uint64_t o = ((uint64_t)hi << 32) | lo;
        v = o > v ? o : v;
    }
    return v;
}

// first row >= bound that uses tensor t, NONE if there is none
__device__ __forceinline__ uint32_t next_use(const TcDevTables &T, uint32_t t, uint32_t bound)
{
    uint32_t b = T.occ_ptr[t], e = T.occ_ptr[t + 1];
    const uint32_t end = e;
    while (b < e) {
        uint32_t m = (b + e) >> 1;
        if (T.occ_rows[m] < bound) b = m + 1; else e = m;
    }
    return b < end ? T.occ_rows[b] : NONE;
}

__device__ __forceinline__ void emit(DecideCtx &c, uint32_t op, uint32_t t, uint32_t st, uint32_t ss,
                                     uint32_t dt, uint32_t ds)
{
    if (c.n_ops < c.cap) {
        if (c.lane == 0) {
            TcOpRec r;
            r.tensor = t; r.src_slot = ss; r.dst_slot = ds;
            r.op = (uint8_t)op; r.phase = (uint8_t)c.phase; r.src_tier = (uint8_t)st; r.dst_tier = (uint8_t)dt;
            c.ops[c.n_ops] = r;
        }
    }
    c.n_ops++;
}

// lowest free buffer of a class that was not freed by this hook call
__device__ __forceinline__ uint32_t lowest_free(const DecideCtx &c, const uint32_t *owner,
                                                const uint32_t *freed, uint32_t count)
{
    for (uint32_t base = 0; base < count; base += WAVE) {
        uint32_t k = base + c.lane;
        bool ok = k < count && owner[k] == NONE && freed[k] != c.call;
        uint64_t m = __ballot(ok);
        if (m) return base + (uint32_t)__ffsll((long long)m) - 1;
    }
    return NONE;
}

// key of "used farthest in the future, ties -> lowest id"; larger is better
__device__ __forceinline__ uint64_t far_key(uint32_t nu, uint32_t id)
{
    return ((uint64_t)nu << 32) | (uint64_t)(NONE - id);
}

// Alg. 4's spill victim: an occupied host buffer of the class, GPU-designated
// ones first, whose tensor was not moved by this call and is used farthest in
// the future.
__device__ uint32_t spill_victim(const DecideCtx &c, uint32_t s)
{
    const TcDevTables &T = c.T;
    const uint32_t cb = T.cpu_base[s], cc = T.cpu_count[s];
    uint64_t best_d = 0, best_a = 0;
    for (uint32_t k = c.lane; k < cc; k += WAVE) {
        uint32_t o = T.cpu_owner[cb + k];
        if (o == NONE || T.moved[o] == c.call) continue;
        uint64_t key = far_key(next_use(T, o, c.bound), o);
        if (T.designated[cb + k]) best_d = key > best_d ? key : best_d;
        best_a = key > best_a ? key : best_a;
    }
    best_d = wave_max_u64(best_d);
    best_a = wave_max_u64(best_a);
    uint64_t best = best_d ? best_d : best_a;
    return best ? NONE - (uint32_t)best : NONE;
}

// EvictTensor (Alg. 4).  partner = host buffer of the tensor about to take
// v's GPU buffer (the two swap places), or NONE.
__device__ void evict(DecideCtx &c, uint32_t v, uint32_t partner)
{
    const TcDevTables &T = c.T;
    const uint32_t s = T.class_of[v], y = T.gslot[v];
    const uint32_t gb = T.gpu_base[s], cb = T.cpu_base[s];
    if (T.final_tier[v] == TC_NVME) {
        if (T.dirty[v]) {
            emit(c, TC_OP_WRITEBACK, v, TC_GPU, y, TC_NVME, NONE);
            T.dirty[v] = 0;
        } else {
            emit(c, TC_OP_RELEASE, v, TC_GPU, y, TC_NVME, NONE);
        }
        T.cur[v] = TC_NVME;
    } else {
        uint32_t x = partner;
        if (x == NONE) x = lowest_free(c, T.cpu_owner + cb, T.cpu_freed + cb, T.cpu_count[s]);
        if (x == NONE) {
            uint32_t w = spill_victim(c, s);
            if (w != NONE) {
                x = T.cslot[w];
                emit(c, TC_OP_SPILL, w, TC_CPU, x, TC_NVME, NONE);
                T.cur[w] = TC_NVME;
                T.cslot[w] = NONE;
                T.moved[w] = c.call;
                T.cpu_owner[cb + x] = NONE;
                T.designated[cb + x] = 0;
            }
        }
        if (x == NONE) {            // the class has no host buffer to give: straight to the file tier
            emit(c, TC_OP_WRITEBACK, v, TC_GPU, y, TC_NVME, NONE);
            T.cur[v] = TC_NVME;
        } else {
            T.designated[cb + x] = (T.final_tier[v] == TC_GPU) ? 1u : 0u;
            T.cpu_owner[cb + x] = v;
            T.cslot[v] = x;
            emit(c, TC_OP_EVICT, v, TC_GPU, y, TC_CPU, x);
            T.cur[v] = TC_CPU;
        }
    }
    T.gslot[v] = NONE;
    T.gpu_owner[gb + y] = NONE;
    T.gpu_freed[gb + y] = c.call;
    T.moved[v] = c.call;
}

// evict v (if any) and bring u into GPU buffer y of their common class
__device__ void exchange(DecideCtx &c, uint32_t v, uint32_t u, uint32_t y, uint32_t op_in)
{
    const TcDevTables &T = c.T;
    const uint32_t s = T.class_of[u];
    const uint32_t gb = T.gpu_base[s], cb = T.cpu_base[s];
    const uint32_t src_tier = T.cur[u], src_slot = T.cslot[u];
    if (v != NONE) {
        uint32_t swap = (src_tier == TC_CPU && T.final_tier[v] != TC_NVME) ? src_slot : NONE;
        if (swap != NONE) {
            T.cpu_owner[cb + swap] = NONE;
            T.designated[cb + swap] = 0;
        }
        evict(c, v, swap);
    }
    if (src_tier == TC_CPU && T.cpu_owner[cb + src_slot] == u) {
        T.cpu_owner[cb + src_slot] = NONE;
        T.designated[cb + src_slot] = 0;
        T.cpu_freed[cb + src_slot] = c.call;
    }
    emit(c, op_in, u, src_tier, src_tier == TC_CPU ? src_slot : NONE, TC_GPU, y);
    if (op_in == TC_OP_ALLOC) T.undefined[u] = 1;         // handed over as it is: no copy fills the buffer
    T.cur[u] = TC_GPU;
    T.gslot[u] = y;
    T.cslot[u] = NONE;
    T.gpu_owner[gb + y] = u;
    T.moved[u] = c.call;
}

__device__ __forceinline__ bool in_list(const TcStepArgs &a, uint32_t x)
{
    bool hit = false;
    for (uint32_t i = 0; i < a.n; ++i) hit |= (a.ids[i] == x);
    return hit;
}

// pre-hook: residency of the step's tensors, demand fetch of the missing ones
__device__ void decide_pre(DecideCtx &c, const TcStepArgs &a)
{
    const TcDevTables &T = c.T;
    c.bound = a.step < T.n_steps ? T.row_begin[a.step] : T.n_rows;
    // residency of the whole list in one ballot: an all-hit step (the common
    // case when prefetching keeps up) is resolved without the serial loop
    {
        const bool mine = c.lane < a.n;
        const uint32_t t = a.ids[mine ? c.lane : 0];
        const bool res = mine && T.cur[t] == TC_GPU;
        const uint64_t mk = __ballot(res);
        if ((uint32_t)__popcll(mk) == a.n) {
            // the dirty marks are scheduler state a later call of the same launch reads on every
            // lane: like every other state store, each lane makes all of them itself
            uint32_t ur = 0;
            for (uint32_t i = 0; i < a.n; ++i) {
                if ((a.rw[i] & TC_R) && T.undefined[a.ids[i]]) ur++;
                if (a.rw[i] & TC_W) T.dirty[a.ids[i]] = 1;
                if (a.rw[i] == TC_W && (T.flags & TC_ALLOC_WRITE_ONLY)) T.undefined[a.ids[i]] = 0;
            }
            if (mine) c.out->slots[c.lane] = T.gslot[t];
            if (c.lane == 0) { c.out->hits = a.n; c.out->misses = 0; c.out->fails = 0; c.out->undefined_reads = ur; }
            return;
        }
    }
    uint32_t h = 0, m = 0, f = 0, ur = 0;
    for (uint32_t i = 0; i < a.n; ++i) {
        const uint32_t t = a.ids[i];
        const uint32_t s = T.class_of[t];
        const uint32_t gb = T.gpu_base[s], gc = T.gpu_count[s];
        const bool whole = a.rw[i] == TC_W && (T.flags & TC_ALLOC_WRITE_ONLY);   // the module overwrites all of it
        if (T.cur[t] == TC_GPU) {
            h++;
        } else {
            m++;
            uint32_t y = lowest_free(c, T.gpu_owner + gb, T.gpu_freed + gb, gc);
            uint32_t v = NONE;
            if (y == NONE) {
                uint64_t best = 0;
                for (uint32_t k = c.lane; k < gc; k += WAVE) {
                    uint32_t x = T.gpu_owner[gb + k];
                    if (x == NONE || T.moved[x] == c.call || in_list(a, x)) continue;
                    uint64_t key = far_key(next_use(T, x, c.bound), x);
                    best = key > best ? key : best;
                }
                best = wave_max_u64(best);
                if (best) { v = NONE - (uint32_t)best; y = T.gslot[v]; }
            }
            if (y == NONE) {
                f++;
                emit(c, TC_OP_FAIL, t, T.cur[t], NONE, TC_GPU, NONE);
                if (c.lane == 0) c.out->slots[i] = NONE;
                continue;
            }
            exchange(c, v, t, y, whole ? TC_OP_ALLOC : TC_OP_DEMAND);
        }
        if ((a.rw[i] & TC_R) && T.undefined[t]) ur++;
        if (a.rw[i] & TC_W) T.dirty[t] = 1;
        if (whole) T.undefined[t] = 0;
        if (c.lane == 0) c.out->slots[i] = T.gslot[t];
    }
    if (c.lane == 0) { c.out->hits = h; c.out->misses = m; c.out->fails = f; c.out->undefined_reads = ur; }
}

// post-hook: PrefetchTensor (Alg. 3) over the tensors that finished
__device__ void decide_post(DecideCtx &c, const TcStepArgs &a)
{
    const TcDevTables &T = c.T;
    if (T.flags & TC_NO_PREFETCH) return;                 // base variant: nothing moves after a module
    const uint32_t n_rows = T.n_rows;
    c.bound = a.step < T.n_steps ? T.row_begin[a.step + 1] : n_rows;
    uint32_t cursor = T.scalars[0];
    cursor = cursor > c.bound ? cursor : c.bound;
    for (uint32_t i = 0; i < a.n; ++i) {
        const uint32_t t = a.ids[i];
        if (cursor >= n_rows) break;
        // skip rows already in the active tensor window, 64 rows per ballot
        while (cursor < n_rows) {
            uint32_t r = cursor + c.lane;
            bool stop = false;
            if (r < n_rows) {
                uint32_t x = T.rows_tensor[r];
                stop = !(T.cur[x] == TC_GPU || T.gpu_count[T.class_of[x]] == 0);
            }
            uint64_t mk = __ballot(stop);
            if (mk) { cursor += (uint32_t)__ffsll((long long)mk) - 1; break; }
            cursor = cursor + WAVE < n_rows ? cursor + WAVE : n_rows;
        }
        if (cursor >= n_rows) break;
        const uint32_t u = T.rows_tensor[cursor];
        if (T.moved[u] == c.call) break;                  // in flight
        const uint32_t s = T.class_of[u];
        const uint32_t gb = T.gpu_base[s], gc = T.gpu_count[s];
        uint32_t v = NONE, y = NONE;
        if (T.class_of[t] == s && T.cur[t] == TC_GPU && T.moved[t] != c.call &&
            next_use(T, t, c.bound) > cursor) {
            v = t;                                        // the finished tensor gives up its buffer
            y = T.gslot[t];
        } else {
            y = lowest_free(c, T.gpu_owner + gb, T.gpu_freed + gb, gc);
            if (y == NONE) {
                uint64_t best = 0;
                for (uint32_t k = c.lane; k < gc; k += WAVE) {
                    uint32_t x = T.gpu_owner[gb + k];
                    if (x == NONE || T.moved[x] == c.call) continue;
                    uint32_t nu = next_use(T, x, c.bound);
                    if (nu <= cursor) continue;           // needed before u: stays
                    uint64_t key = far_key(nu, x);
                    best = key > best ? key : best;
                }
                best = wave_max_u64(best);
                if (best) { v = NONE - (uint32_t)best; y = T.gslot[v]; }
            }
        }
        if (y == NONE) continue;                          // halt for this tensor
        // a row that only writes: the tensor's bytes are dead, the buffer alone is handed over
        const bool whole = (T.flags & TC_ALLOC_WRITE_ONLY) && T.rows_rw[cursor] == TC_W;
        exchange(c, v, u, y, whole ? TC_OP_ALLOC : TC_OP_PREFETCH);
        cursor++;
    }
    T.scalars[0] = cursor;
}

// End of iteration: every tensor goes back to its final location (Sec. 3.2.1), each displaced
// tensor in one move and no other tensor at all.  Three hook calls: GPU-final tensors come home
// from host buffers, then GPU-final tensors come home from the file tier (a CPU-final guest they
// displace then finds a free host buffer, since no GPU-final tensor holds one any more), then
// CPU-final tensors return from the file tier.
__device__ void decide_end(DecideCtx &c)
{
    const TcDevTables &T = c.T;
    c.bound = T.n_rows;
    // first and second call: GPU-final tensors come home, class by class, placement order
    for (uint32_t source = TC_CPU; source <= TC_NVME; ++source) {
        if (source == TC_NVME) c.call++;
        for (uint32_t s = 0; s < T.n_classes; ++s) {
            const uint32_t gb = T.gpu_base[s], gc = T.gpu_count[s];
            const uint32_t mb = T.member_ptr[s], me = T.member_ptr[s + 1];
            uint32_t i = mb;
            while (i < me) {
                // next member that is GPU-final and on the tier this call serves, 64 members per ballot
                uint32_t j = i + c.lane;
                bool want = false;
                if (j < me) {
                    uint32_t u = T.members[j];
                    want = T.final_tier[u] == TC_GPU && T.cur[u] == source;
                }
                uint64_t mk = __ballot(want);
                if (!mk) { i += WAVE; continue; }
                i += (uint32_t)__ffsll((long long)mk) - 1;
                const uint32_t u = T.members[i];
                i++;
                uint32_t y = lowest_free(c, T.gpu_owner + gb, T.gpu_freed + gb, gc);
                uint32_t v = NONE;
                if (y == NONE) {
                    uint32_t best = NONE;                      // lowest-id guest
                    for (uint32_t k = c.lane; k < gc; k += WAVE) {
                        uint32_t x = T.gpu_owner[gb + k];
                        if (x == NONE || T.final_tier[x] == TC_GPU || T.moved[x] == c.call) continue;
                        best = x < best ? x : best;
                    }
                    uint64_t r = wave_max_u64((uint64_t)(NONE - best));
                    best = NONE - (uint32_t)r;
                    if (best == NONE) continue;
                    v = best;
                    y = T.gslot[v];
                }
                exchange(c, v, u, y, TC_OP_PREFETCH);
            }
        }
    }
    // third call: CPU-final tensors on the file tier return to host buffers
    c.call++;
    c.phase = TC_END_CPU;
    for (uint32_t s = 0; s < T.n_classes; ++s) {
        const uint32_t cb = T.cpu_base[s], cc = T.cpu_count[s];
        const uint32_t mb = T.member_ptr[s], me = T.member_ptr[s + 1];
        uint32_t i = mb;
        while (i < me) {
            uint32_t j = i + c.lane;
            bool want = false;
            if (j < me) {
                uint32_t u = T.members[j];
                want = T.final_tier[u] == TC_CPU && T.cur[u] == TC_NVME;
            }
            uint64_t mk = __ballot(want);
            if (!mk) { i += WAVE; continue; }
            i += (uint32_t)__ffsll((long long)mk) - 1;
            const uint32_t u = T.members[i];
            i++;
            uint32_t x = lowest_free(c, T.cpu_owner + cb, T.cpu_freed + cb, cc);
            if (x == NONE) continue;
            emit(c, TC_OP_RESTORE, u, TC_NVME, NONE, TC_CPU, x);
            T.cur[u] = TC_CPU;
            T.cslot[u] = x;
            T.cpu_owner[cb + x] = u;
            T.moved[u] = c.call;
        }
        for (uint32_t k = c.lane; k < cc; k += WAVE) T.designated[cb + k] = 0;
    }
    T.scalars[0] = 0;
    T.scalars[2] = T.scalars[2] + 1;
}

// one hook call: the call id advances, the phase's routine runs, the record is filled
__device__ void decide_call(DecideCtx &c, const TcStepArgs &a, TcDecideOut *out, TcOpRec *ops, uint32_t cap)
{
    const TcDevTables &T = c.T;
    c.out = out;
    c.ops = ops;
    c.cap = cap;
    c.n_ops = 0;
    c.step = a.step;
    c.phase = a.phase;
    c.call = T.scalars[1] + 1;
    c.bound = 0;
    if (c.lane == 0) { out->hits = 0; out->misses = 0; out->fails = 0; out->undefined_reads = 0; }
    if (a.phase == TC_PRE) decide_pre(c, a);
    else if (a.phase == TC_POST) decide_post(c, a);
    else decide_end(c);
    T.scalars[1] = c.call;
    if (c.lane == 0) {
        out->cursor = T.scalars[0];
        out->iteration = T.scalars[2];
        out->overflow = c.n_ops > cap ? 1u : 0u;
        out->n_ops = c.n_ops < cap ? c.n_ops : cap;
    }
}

__global__ __launch_bounds__(WAVE) void tc_decide_kernel(TcDevTables T, TcStepArgs a, TcDecideOut *out, TcOpRec *ops)
{
    DecideCtx c;
    c.T = T;
    c.lane = threadIdx.x;
    decide_call(c, a, out, ops, a.cap);
}

// A window of steps in one launch: for each step the pre-hook call, then the
// post-hook call, exactly the sequence the per-hook kernel would run.  The
// decisions depend on the trace and the tables only, never on when a copy
// finishes, so deciding a window ahead of the copies changes nothing but the
// number of launches.  Record 2*i is step first+i's pre-hook call, record
// 2*i+1 its post-hook call; their op records follow each other in `ops`.
__global__ __launch_bounds__(WAVE) void tc_decide_window_kernel(TcDevTables T, TcWindowArgs w, TcDecideOut *out,
                                                                TcOpRec *ops)
{
    DecideCtx c;
    c.T = T;
    c.lane = threadIdx.x;
    uint32_t used = 0;
    for (uint32_t k = 0; k < w.count; ++k) {
        TcStepArgs a;
        const uint32_t b = w.step_ptr[w.first + k];
        uint32_t n = w.step_ptr[w.first + k + 1] - b;
        n = n < TC_MAX_STEP_TENSORS ? n : TC_MAX_STEP_TENSORS;
        for (uint32_t i = 0; i < TC_MAX_STEP_TENSORS; ++i) {
            a.ids[i] = i < n ? w.ids[b + i] : 0;
            a.rw[i] = i < n ? w.rw[b + i] : 0;
        }
        a.n = n;
        a.step = w.first + k;
        for (uint32_t ph = TC_PRE; ph <= TC_POST; ++ph) {
            if (2 * k + ph >= w.n_calls) return;
            a.phase = ph;
            TcDecideOut *rec = out + 2 * k + ph;
            decide_call(c, a, rec, ops + used, w.cap - used);
            used += c.n_ops < w.cap - used ? c.n_ops : w.cap - used;
        }
    }
}

hipError_t tc_launch_decide(const TcDevTables &T, const TcStepArgs &a, TcDecideOut *out, TcOpRec *ops, hipStream_t s)
{
    hipLaunchKernelGGL(tc_decide_kernel, dim3(1), dim3(WAVE), 0, s, T, a, out, ops);
    return hipGetLastError();
}

hipError_t tc_launch_decide_window(const TcDevTables &T, const TcWindowArgs &w, TcDecideOut *out, TcOpRec *ops,
                                   hipStream_t s)
{
    if (w.count == 0 || w.count > TC_WINDOW_MAX || w.n_calls == 0 || w.n_calls > 2 * w.count) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tc_decide_window_kernel, dim3(1), dim3(WAVE), 0, s, T, w, out, ops);
    return hipGetLastError();
}

// ===========================================================================
// Migration kernel: one launch moves every exchange unit of a hook call.
//
// The link to host memory, not HBM and not the ALUs, bounds this kernel, so the
// design goal is enough 128-bit requests in flight to cover the host link's
// latency, on both directions at once, and not more.  Work is cut into chunks
// of chunk_bytes; a workgroup takes the next chunk from a ticket counter, moves
// it in blocks of 16 KiB (each lane 16 bytes per request, a wave's 64 lanes
// cover 1 KiB of consecutive addresses, four requests per lane and direction
// before the first store) and comes back for another.  For a unit with both
// directions each lane holds the outgoing and the incoming 16 bytes of the same
// index before storing either, which is what lets a tensor leave a GPU buffer
// while another arrives in it.
//
// All working workgroups sit on ONE XCD.  With both directions loaded, requests
// from different XCDs are served very unevenly (measured per 16 KiB block under
// load: 10 us on two XCDs, 19 us on three, 40-120 us on the other three), every
// launch ends waiting ~100 us for the workgroups on the starved XCDs, and a
// 16 MiB exchange runs at 39 GB/s per direction instead of 48.  Workgroups are
// dealt to the XCDs in turn, so the grid is n_xcd times the number wanted and a
// workgroup that finds itself on another XCD than `xcc` exits at once (workgroup
// 0 always stays, so that every chunk is moved wherever the dispatcher puts
// things).  A
// dozen workgroups (192 KiB in flight per direction) are the optimum: fewer
// leave the link idle, more crowd each other out.
//
// The ticket counter is one of two words: a launch uses word `slot` and clears
// the other for the launch that follows it on the same stream.
// ===========================================================================

#define MOVER_THREADS 256
#define MOVER_UNROLL 4

// streaming accesses: nothing the mover touches is used again by it (worth 1 % on the duplex rate)
typedef uint32_t mover_v4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16(const uint8_t *p)
{
    mover_v4 v = __builtin_nontemporal_load((const mover_v4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st16(uint8_t *p, uint4 v)
{
    __builtin_nontemporal_store(mover_v4{v.x, v.y, v.z, v.w}, (mover_v4 *)p);
}

// has the word reached seq?  (sequence numbers wrap: compare the difference)
__device__ __forceinline__ bool seq_reached(const uint32_t *word, uint32_t seq)
{
    const uint32_t v = __hip_atomic_load(word, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
    return (int32_t)(v - seq) >= 0;
}

// bounded wait for a sequence word, by one lane; false: gave up, after `ticks` of the 100 MHz clock
// or because a waiter before it did (so that a context whose streams cannot make progress against
// each other drains in one timeout, not one per launch)
__device__ bool seq_wait(const uint32_t *word, uint32_t seq, uint64_t ticks, uint32_t *fault, uint32_t *gave_up, uint32_t code)
{
    if (seq_reached(word, seq)) return true;
    const uint64_t t0 = wall_clock64();
    for (uint32_t n = 0;; ++n) {
        if ((n & 255u) == 0 && __hip_atomic_load(gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
        // a short wait is polled closely (0.1 us), a long one every microsecond or so: polls go to memory, and a
        // dozen waiters polling one word closely for milliseconds slow the kernels that run meanwhile
        if (n < 64) __builtin_amdgcn_s_sleep(4);
        else __builtin_amdgcn_s_sleep(32);
        if (seq_reached(word, seq)) return true;
        if (wall_clock64() - t0 > ticks) break;
    }
    __hip_atomic_store(gave_up, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(fault, code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    return false;
}

__global__ __launch_bounds__(MOVER_THREADS) void tc_mover_kernel(TcMoverArgs a)
{
    uint32_t xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    const uint32_t tid = threadIdx.x;
    if ((xcc & 15u) != a.xcc && blockIdx.x != 0) return;
    __shared__ uint32_t ticket;
    __shared__ uint32_t go;
    if (blockIdx.x == 0 && tid == 0) a.tickets[a.slot ^ 1u] = 0;
    if (a.progress) {
        // the modules this launch has to wait for may still be running: wait for their signal
        if (tid == 0) {
            go = seq_wait(a.progress, a.need_seq, a.spin_ticks, a.fault, a.gave_up, 1u) ? 1u : 0u;
        }
        __syncthreads();
        if (!go) return;                                   // gave up: move nothing
        __threadfence();                                   // what those modules wrote is read from here on
    }
    uint32_t ui = 0;                                       // tickets only grow: the unit search resumes where it stopped
    for (;;) {
        __syncthreads();                                   // everyone has read the ticket before
        if (tid == 0) ticket = atomicAdd(&a.tickets[a.slot], 1u);
        __syncthreads();
        const uint64_t c = ticket;
        if (c >= a.n_chunks) break;
        // unit of this chunk: the last one whose first chunk is <= c
        while (ui + 1 < a.n_units && a.u[ui + 1].chunk0 <= c) ++ui;
        const TcUnit &U = a.u[ui];
        const uint64_t off = (c - U.chunk0) * (uint64_t)a.chunk_bytes;
        const uint64_t left = U.bytes - off;
        const uint32_t len = left < a.chunk_bytes ? (uint32_t)left : a.chunk_bytes;
        const uint32_t n16 = len >> 4;
        const uint8_t *os = U.out_src ? U.out_src + off : nullptr;
        uint8_t *od = U.out_dst ? U.out_dst + off : nullptr;
        const uint8_t *is = U.in_src ? U.in_src + off : nullptr;
        uint8_t *id = U.in_dst ? U.in_dst + off : nullptr;
        uint32_t i = tid;
        if (os && is) {
            for (; i + (MOVER_UNROLL - 1) * MOVER_THREADS < n16; i += MOVER_UNROLL * MOVER_THREADS) {
                uint4 vo[MOVER_UNROLL], vi[MOVER_UNROLL];
#pragma unroll
                for (int k = 0; k < MOVER_UNROLL; ++k) vi[k] = ld16(is + (uint64_t)(i + k * MOVER_THREADS) * 16);
#pragma unroll
                for (int k = 0; k < MOVER_UNROLL; ++k) vo[k] = ld16(os + (uint64_t)(i + k * MOVER_THREADS) * 16);
#pragma unroll
                for (int k = 0; k < MOVER_UNROLL; ++k) st16(od + (uint64_t)(i + k * MOVER_THREADS) * 16, vo[k]);
#pragma unroll
                for (int k = 0; k < MOVER_UNROLL; ++k) st16(id + (uint64_t)(i + k * MOVER_THREADS) * 16, vi[k]);
            }
            for (; i < n16; i += MOVER_THREADS) {
                uint4 vi = ld16(is + (uint64_t)i * 16);
                uint4 vo = ld16(os + (uint64_t)i * 16);
                st16(od + (uint64_t)i * 16, vo);
                st16(id + (uint64_t)i * 16, vi);
            }
            const uint32_t tail = len & 15u;               // only the unit's last chunk has one
            if (tid < tail) {
                uint8_t bo = os[(uint64_t)n16 * 16 + tid], bi = is[(uint64_t)n16 * 16 + tid];
                od[(uint64_t)n16 * 16 + tid] = bo;
                id[(uint64_t)n16 * 16 + tid] = bi;
            }
        } else {
            const uint8_t *s = os ? os : is;
            uint8_t *d = os ? od : id;
            if (!s) continue;
            for (; i + (MOVER_UNROLL - 1) * MOVER_THREADS < n16; i += MOVER_UNROLL * MOVER_THREADS) {
                uint4 v[MOVER_UNROLL];
#pragma unroll
                for (int k = 0; k < MOVER_UNROLL; ++k) v[k] = ld16(s + (uint64_t)(i + k * MOVER_THREADS) * 16);
#pragma unroll
                for (int k = 0; k < MOVER_UNROLL; ++k) st16(d + (uint64_t)(i + k * MOVER_THREADS) * 16, v[k]);
            }
            for (; i < n16; i += MOVER_THREADS) st16(d + (uint64_t)i * 16, ld16(s + (uint64_t)i * 16));
            const uint32_t tail = len & 15u;
            if (tid < tail) d[(uint64_t)n16 * 16 + tid] = s[(uint64_t)n16 * 16 + tid];
        }
    }
}

// The other side of the dependencies resolved on the GPU: one lane raises a sequence word behind what is
// queued so far on its stream (the modules on the compute stream; a launch on the migration stream), one
// lane waits for a word in front of a module (bounded).
__global__ void tc_signal_kernel(uint32_t *word, uint32_t seq)
{
    if (threadIdx.x == 0) {
        // (what the kernels before this one on the stream wrote was released when they ended; the
        // exchange is a release all the same)
        // never lower the word: signals of two compute streams may arrive out of order.  The usual
        // case is the number before this one, so that is the first guess: one trip to memory.
        uint32_t v = seq - 1;
        while ((int32_t)(seq - v) > 0 &&
               !__hip_atomic_compare_exchange_strong(word, &v, seq, __ATOMIC_RELEASE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
        }
    }
}

__global__ void tc_wait_kernel(const uint32_t *word, uint32_t seq, uint64_t ticks, uint32_t *fault, uint32_t *gave_up)
{
    if (threadIdx.x == 0) {
        (void)seq_wait(word, seq, ticks, fault, gave_up, 2u);
        __threadfence();
    }
}

hipError_t tc_launch_signal(uint32_t *word, uint32_t seq, hipStream_t s)
{
    if (!word) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tc_signal_kernel, dim3(1), dim3(64), 0, s, word, seq);
    return hipGetLastError();
}

hipError_t tc_launch_wait(const uint32_t *word, uint32_t seq, uint64_t spin_ticks, uint32_t *fault, uint32_t *gave_up,
                          hipStream_t s)
{
    if (!word || !fault || !gave_up || !spin_ticks) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tc_wait_kernel, dim3(1), dim3(64), 0, s, word, seq, spin_ticks, fault, gave_up);
    return hipGetLastError();
}

// clears the two ticket counters of a stand-alone launch (a kernel, not a memset node: a caller
// may be capturing the stream into a graph)
__global__ void tc_zero_tickets_kernel(uint32_t *p)
{
    if (threadIdx.x < 2) p[threadIdx.x] = 0;
}

hipError_t tc_launch_zero_tickets(uint32_t *tickets, hipStream_t s)
{
    hipLaunchKernelGGL(tc_zero_tickets_kernel, dim3(1), dim3(64), 0, s, tickets);
    return hipGetLastError();
}

// Which XCDs does the dispatcher deal workgroups to?  A probe launch of 64
// workgroups writes down where each one ran: the number of distinct XCDs is the
// factor between the grid and the workgroups that work, and the XCD of workgroup
// 0 is the one they work on (with a single XCD visible, as in a partitioned
// GPU, nothing is filtered).  Once per device and process.
#define XCC_PROBE_WGS 64

__global__ void tc_xcc_probe_kernel(uint32_t *out)
{
    uint32_t xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    if (threadIdx.x == 0) out[blockIdx.x] = xcc & 15u;
}

hipError_t tc_mover_topology(uint32_t *xcc, uint32_t *n_xcd)
{
    static std::mutex mu;
    static struct { bool known; uint32_t xcc, n; } cache[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> g(mu);
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!cache[dev].known) {
        uint32_t *d = nullptr, h[XCC_PROBE_WGS];
        if ((e = hipMalloc((void **)&d, sizeof(h))) != hipSuccess) return e;
        hipLaunchKernelGGL(tc_xcc_probe_kernel, dim3(XCC_PROBE_WGS), dim3(64), 0, nullptr, d);
        e = hipGetLastError();
        if (e == hipSuccess) e = hipMemcpy(h, d, sizeof(h), hipMemcpyDeviceToHost);
        (void)hipFree(d);
        if (e != hipSuccess) return e;
        uint32_t seen = 0;
        for (uint32_t i = 0; i < XCC_PROBE_WGS; ++i) seen |= 1u << h[i];
        cache[dev].xcc = h[0];
        cache[dev].n = (uint32_t)__builtin_popcount(seen);
        cache[dev].known = true;
    }
    *xcc = cache[dev].xcc;
    *n_xcd = cache[dev].n;
    return hipSuccess;
}

hipError_t tc_launch_mover(TcMoverArgs &a, uint32_t workgroups, hipStream_t s, uint64_t *launches)
{
    if (a.n_units == 0 || a.n_chunks == 0) return hipSuccess;
    // the kernel trusts these counts: check them against the units before it runs
    if (a.n_units > TC_MOVER_MAX_UNITS || a.chunk_bytes == 0 || (a.chunk_bytes & 15)) return hipErrorInvalidValue;
    if (!a.tickets || !launches || workgroups == 0 || workgroups > 8192 || a.n_xcd == 0 || a.n_xcd > 16)
        return hipErrorInvalidValue;
    if (a.progress && (!a.fault || !a.gave_up || !a.spin_ticks)) return hipErrorInvalidValue;
    uint64_t chunks = 0;
    for (uint32_t i = 0; i < a.n_units; ++i) {
        const TcUnit &u = a.u[i];
        if (u.chunk0 != chunks || u.bytes == 0) return hipErrorInvalidValue;
        if ((u.out_src == nullptr) != (u.out_dst == nullptr)) return hipErrorInvalidValue;
        if ((u.in_src == nullptr) != (u.in_dst == nullptr)) return hipErrorInvalidValue;
        if (!u.out_src && !u.in_src) return hipErrorInvalidValue;
        chunks += (u.bytes + a.chunk_bytes - 1) / a.chunk_bytes;
    }
    if (chunks != a.n_chunks || chunks >= 0xFFFF0000ull) return hipErrorInvalidValue;   // tickets are 32-bit
    // the counters alternate between the launches that really happen: each clears the other's
    a.slot = (uint32_t)(*launches & 1);
    const uint64_t g = (a.n_chunks < workgroups ? a.n_chunks : workgroups) * a.n_xcd;
    hipLaunchKernelGGL(tc_mover_kernel, dim3((uint32_t)g), dim3(MOVER_THREADS), 0, s, a);
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) ++*launches;
    return e;
}

// ===========================================================================
// Stand-in for a module's kernels in a replay: stamp written tensors, then spin.
// A 32-lane group per list entry (sixteen groups take the entries in turn): lanes
// 0-15 XOR the head bytes, lanes 16-31 the tail bytes.  When head and tail overlap
// (tensors under 32 bytes) lane 0 applies both in order.
// ===========================================================================
#define STAMP_THREADS 512
__global__ __launch_bounds__(STAMP_THREADS) void tc_stamp_kernel(TcStampArgs a)
{
    const uint32_t j = threadIdx.x & 31;
    for (uint32_t i = threadIdx.x >> 5; i < a.n; i += STAMP_THREADS / 32) {
    // a list may name a tensor more than once; its stamps are identical and XOR
    // cancels in pairs, so the first occurrence applies it iff the count is odd
    bool apply = false;
    if (a.ptr[i]) {
        uint32_t same = 0, earlier = 0;
        for (uint32_t k = 0; k < a.n; ++k) {
            same += (a.ptr[k] == a.ptr[i]);
            earlier += (k < i && a.ptr[k] == a.ptr[i]);
        }
        apply = earlier == 0 && (same & 1);
    }
    if (apply) {
        const uint32_t w[4] = {0x10CAC4E5u, a.iteration, a.step, a.tensor[i]};
        uint8_t *p = a.ptr[i];
        const uint64_t n = a.bytes[i];
        if (n >= 32) {
            const uint32_t b = j & 15;
            uint8_t *q = j < 16 ? p + b : p + n - 16 + b;
            *q ^= (uint8_t)(w[b >> 2] >> (8 * (b & 3)));
        } else if (j == 0) {
            for (uint32_t b = 0; b < 16; ++b) p[b] ^= (uint8_t)(w[b >> 2] >> (8 * (b & 3)));
            for (uint32_t b = 0; b < 16; ++b) p[n - 16 + b] ^= (uint8_t)(w[b >> 2] >> (8 * (b & 3)));
        }
    }
    }
    if (a.busy_ns && threadIdx.x == 0) {
        // wall_clock64 counts at 100 MHz; the loop ends once busy_ns have passed
        const uint64_t t0 = wall_clock64();
        const uint64_t ticks = a.busy_ns / 10;
        while (wall_clock64() - t0 < ticks) { __builtin_amdgcn_s_sleep(8); }
    }
}

hipError_t tc_launch_stamp(const TcStampArgs &a, hipStream_t s)
{
    if (a.n > TC_MAX_STEP_TENSORS) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tc_stamp_kernel, dim3(1), dim3(STAMP_THREADS), 0, s, a);
    return hipGetLastError();
}

// ===========================================================================
// Payload fill: word i of tensor t = h(i*0x9E3779B1 + t*0x85EBCA77 + seed*0xC2B2AE3D)
// ===========================================================================
__device__ __forceinline__ uint32_t hash32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
    return x;
}

__global__ __launch_bounds__(256) void tc_fill_kernel(uint8_t *dst, uint64_t bytes, uint32_t base)
{
    const uint64_t n16 = bytes >> 4;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        uint32_t w0 = (uint32_t)(i * 4);
        uint4 v;
        v.x = hash32((w0 + 0) * 0x9E3779B1u + base);
        v.y = hash32((w0 + 1) * 0x9E3779B1u + base);
        v.z = hash32((w0 + 2) * 0x9E3779B1u + base);
        v.w = hash32((w0 + 3) * 0x9E3779B1u + base);
        *(uint4 *)(dst + i * 16) = v;
    }
    if (blockIdx.x == 0 && threadIdx.x < (bytes & 15)) {
        uint64_t b = n16 * 16 + threadIdx.x;
        uint32_t w = hash32((uint32_t)(b >> 2) * 0x9E3779B1u + base);
        dst[b] = (uint8_t)(w >> (8 * (b & 3)));
    }
}

hipError_t tc_launch_fill(void *dst, uint64_t bytes, uint32_t tensor, uint32_t seed, hipStream_t s)
{
    uint32_t base = tensor * 0x85EBCA77u + seed * 0xC2B2AE3Du;
    uint64_t n16 = bytes >> 4;
    uint32_t blocks = (uint32_t)((n16 + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(tc_fill_kernel, dim3(blocks), dim3(256), 0, s, (uint8_t *)dst, bytes, base);
    return hipGetLastError();
}

// ===========================================================================
// Pack / unpack of small tensors: HBM buffers <-> one contiguous HBM slab.
//
// Bound by HBM bandwidth: every payload byte is read once and written once.
// The slab is cut into 16 KiB tiles, one workgroup per tile: many short-lived
// workgroups keep more requests in flight than a few long-lived ones (measured:
// a plain copy written either way differs by about 8 %).  A workgroup must know
// which segments reach into its tile.  That is one bisection of the offset
// table per tile, done ahead of time by the index kernel (the layout of a
// slab repeats every training iteration, so the index is computed once); without
// an index the workgroup bisects for itself and pays that latency on every
// launch.
//
// Register path (a tile that at most 32 pieces reach into): the first 33 lanes
// of each wave fetch consecutive table entries in one round trip, the pieces go
// into a small per-wave table in LDS, and each lane then moves four 128-bit
// vectors, looking up the piece of each vector in that table: all loads of the
// tile are in flight before the first store.  The slab side of a vector is
// always 16-byte aligned.  The tensor side is aligned too in the normal case
// (pool buffers are 256-byte aligned; slab offsets that are multiples of 16);
// where it is not, the access simply goes to the odd address: 128-bit global
// loads at any byte address run at 95-97 % of the aligned rate and stores at
// 91-92 % (measured on a plain tile copy), which beats realigning the tile
// through LDS (the earlier table-driven LDS path reached 63 % of the HBM peak
// for a 4-byte shift and 50 % for an odd one).  Vectors that a piece covers only
// partly (a piece that does not begin or end on a 16-byte boundary of the slab)
// move bytewise afterwards, 32 byte-tasks per piece.
//
// Wide-table path (33 to 256 pieces in one 16 KiB tile, i.e. pieces of 64 to 500
// bytes): the register path again, with one table entry per lane of the workgroup
// and a bisection per vector instead of a scan.
//
// Many-piece path (more pieces than that): pieces are taken one after the other
// and the tile is staged in LDS as the slab sees it, so that however small the
// pieces, the slab side moves as 128-bit requests; a piece whose two addresses
// agree modulo 16 goes register to register.
//
// Bytes of the slab (pack) or of a tensor (unpack) that no piece covers are
// never written.  Segments must be sorted by slab offset and must not overlap.
// ===========================================================================
#define PACK_TILE 16384
#define PACK_THREADS 256
#define PACK_CAND 32
typedef uint32_t pack_v4 __attribute__((ext_vector_type(4)));
struct __attribute__((packed, aligned(1))) pack_u16 { pack_v4 v; };   // 16 bytes at any address
struct __attribute__((packed, aligned(1))) pack_u4 { uint32_t v; };   // 4 bytes at any address

// A tensor at an odd address (pack).  A 128-bit load at an address that is a multiple of 4
// runs at nearly the aligned rate, one at an odd address does not.  So an interior vector of
// such a piece (the 16 bytes before it and the 16 behind it belong to the same tensor) is read
// as the 16 bytes at g - r, r = g mod 4, and the four bytes behind those come from the lane
// that holds the next vector of the same piece (a cross-lane move once the loads are back);
// only where there is no such lane (the last lane of a wave, the vector before an edge one)
// they are loaded.  pack_join shifts the five dwords into place.
__device__ __forceinline__ pack_v4 pack_join(pack_v4 lo, uint32_t hi, uint32_t r)
{
    // v_alignbyte_b32: the low dword of {first, second} >> 8 r; r = 0 returns lo unchanged
    return pack_v4{__builtin_amdgcn_alignbyte(lo.y, lo.x, r), __builtin_amdgcn_alignbyte(lo.z, lo.y, r),
                   __builtin_amdgcn_alignbyte(lo.w, lo.z, r), __builtin_amdgcn_alignbyte(hi, lo.w, r)};
}

// The same for stores (unpack).  An interior vector of a piece whose tensor lies at an odd
// address is written as the 16 bytes at g - r: the last r bytes of the slab vector before it
// (held by the lane before this one; loaded by the first lane of a wave) and the first 16 - r
// of its own.  Its last r bytes are the first of the next interior vector's store; behind the
// last interior vector comes the piece's last whole vector, written where it lies, and that
// lane also writes the dword before it.  Bytes written twice get the same value both times.
// pack_join_before returns bytes 4 - r .. 20 - r of {before, v}; r = 1 .. 3.
__device__ __forceinline__ pack_v4 pack_join_before(uint32_t before, pack_v4 v, uint32_t r)
{
    const uint32_t q = 4 - r;
    return pack_v4{__builtin_amdgcn_alignbyte(v.x, before, q), __builtin_amdgcn_alignbyte(v.y, v.x, q),
                   __builtin_amdgcn_alignbyte(v.z, v.y, q), __builtin_amdgcn_alignbyte(v.w, v.z, q)};
}

// dst and src agree modulo 16; any address space mix (global/LDS); len <= PACK_TILE,
// so a lane has at most four vectors and all of them are loaded before the first store
__device__ __forceinline__ void pack_copy_aligned(uint8_t *dst, const uint8_t *src, uint32_t len, uint32_t tid)
{
    uint32_t head = (uint32_t)((16 - ((uintptr_t)dst & 15)) & 15);
    head = head < len ? head : len;
    if (tid < head) dst[tid] = src[tid];
    const uint32_t body = (len - head) & ~15u;
    const uint8_t *s = src + head;
    uint8_t *d = dst + head;
    const uint32_t i0 = tid * 16, i1 = i0 + PACK_THREADS * 16, i2 = i1 + PACK_THREADS * 16, i3 = i2 + PACK_THREADS * 16;
    uint4 v0 = {}, v1 = {}, v2 = {}, v3 = {};
    if (i0 < body) v0 = *(const uint4 *)(s + i0);
    if (i1 < body) v1 = *(const uint4 *)(s + i1);
    if (i2 < body) v2 = *(const uint4 *)(s + i2);
    if (i3 < body) v3 = *(const uint4 *)(s + i3);
    if (i0 < body) *(uint4 *)(d + i0) = v0;
    if (i1 < body) *(uint4 *)(d + i1) = v1;
    if (i2 < body) *(uint4 *)(d + i2) = v2;
    if (i3 < body) *(uint4 *)(d + i3) = v3;
    for (uint32_t j = head + body + tid; j < len; j += PACK_THREADS) dst[j] = src[j];
}

// src is 128-bit aligned after `head` bytes; dst (LDS) may sit at any shift
__device__ __forceinline__ void pack_global_to_lds(uint8_t *l, const uint8_t *g, uint32_t len, uint32_t tid)
{
    uint32_t head = (uint32_t)((16 - ((uintptr_t)g & 15)) & 15);
    head = head < len ? head : len;
    if (tid < head) l[tid] = g[tid];
    const uint32_t body = (len - head) & ~15u;
    const uint32_t shift = (uint32_t)((uintptr_t)(l + head) & 15);     // the same for every lane
    for (uint32_t i = tid * 16; i < body; i += PACK_THREADS * 16) {
        const uint4 v = *(const uint4 *)(g + head + i);
        uint8_t *q = l + head + i;
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        if ((shift & 3) == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) ((uint32_t *)q)[k] = w[k];
        } else if ((shift & 1) == 0) {
#pragma unroll
            for (int k = 0; k < 8; ++k) ((uint16_t *)q)[k] = (uint16_t)(w[k >> 1] >> (16 * (k & 1)));
        } else {
#pragma unroll
            for (int k = 0; k < 16; ++k) q[k] = (uint8_t)(w[k >> 2] >> (8 * (k & 3)));
        }
    }
    for (uint32_t j = head + body + tid; j < len; j += PACK_THREADS) l[j] = g[j];
}

// dst is 128-bit aligned after `head` bytes; src (LDS) may sit at any shift
__device__ __forceinline__ void pack_lds_to_global(uint8_t *g, const uint8_t *l, uint32_t len, uint32_t tid)
{
    uint32_t head = (uint32_t)((16 - ((uintptr_t)g & 15)) & 15);
    head = head < len ? head : len;
    if (tid < head) g[tid] = l[tid];
    const uint32_t body = (len - head) & ~15u;
    const uint32_t shift = (uint32_t)((uintptr_t)(l + head) & 15);     // the same for every lane
    for (uint32_t i = tid * 16; i < body; i += PACK_THREADS * 16) {
        const uint8_t *q = l + head + i;
        uint32_t w[4] = {0, 0, 0, 0};
        if ((shift & 3) == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) w[k] = ((const uint32_t *)q)[k];
        } else if ((shift & 1) == 0) {
#pragma unroll
            for (int k = 0; k < 8; ++k) w[k >> 1] |= (uint32_t)((const uint16_t *)q)[k] << (16 * (k & 1));
        } else {
#pragma unroll
            for (int k = 0; k < 16; ++k) w[k >> 2] |= (uint32_t)q[k] << (8 * (k & 3));
        }
        *(uint4 *)(g + head + i) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    for (uint32_t j = head + body + tid; j < len; j += PACK_THREADS) g[j] = l[j];
}

// last i with slab_off[i] <= t0 (0 if there is none)
__device__ __forceinline__ uint32_t pack_bisect(const uint64_t *slab_off, uint32_t n, uint64_t t0)
{
    uint32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const uint32_t m = (lo + hi) >> 1;
        if (slab_off[m] <= t0) lo = m; else hi = m;
    }
    return lo;
}

__global__ __launch_bounds__(256) void tc_pack_index_kernel(const uint64_t *slab_off, uint32_t n, uint64_t n_tiles,
                                                            uint32_t tile_bytes, uint32_t *tile_first)
{
    const uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (t < n_tiles) tile_first[t] = pack_bisect(slab_off, n, t * tile_bytes);
}

// one tile, piece after piece, any alignment
__device__ void pack_tile_general(uint8_t *tile, uint8_t *slab, uint8_t *const *ptrs, const uint64_t *bytes,
                                  const uint64_t *slab_off, uint32_t n, uint32_t seg, uint64_t t0, uint64_t t1,
                                  int unpack, uint32_t tid)
{
    while (seg < n && slab_off[seg] + bytes[seg] <= t0) ++seg;
    bool staged = false;
    for (uint32_t sg = seg; sg < n && slab_off[sg] < t1; ++sg) {
        const uint64_t so = slab_off[sg], sb = bytes[sg];
        const uint64_t b = so > t0 ? so : t0;               // overlap of segment and tile, slab coordinates
        const uint64_t e = so + sb < t1 ? so + sb : t1;
        if (e <= b) continue;
        uint8_t *g = ptrs[sg] + (b - so);
        uint8_t *s = slab + b;
        const uint32_t len = (uint32_t)(e - b);
        if ((((uintptr_t)g ^ (uintptr_t)s) & 15) == 0) {
            if (unpack) pack_copy_aligned(g, s, len, tid); else pack_copy_aligned(s, g, len, tid);
        } else {
            staged = true;
            uint8_t *l = tile + (b - t0);                   // s and l agree modulo 16
            if (unpack) pack_copy_aligned(l, s, len, tid); else pack_global_to_lds(l, g, len, tid);
        }
    }
    if (staged) {                                           // the same for every lane of the workgroup
        __syncthreads();
        for (uint32_t sg = seg; sg < n && slab_off[sg] < t1; ++sg) {
            const uint64_t so = slab_off[sg], sb = bytes[sg];
            const uint64_t b = so > t0 ? so : t0;
            const uint64_t e = so + sb < t1 ? so + sb : t1;
            if (e <= b) continue;
            uint8_t *g = ptrs[sg] + (b - so);
            uint8_t *s = slab + b;
            if ((((uintptr_t)g ^ (uintptr_t)s) & 15) == 0) continue;
            const uint32_t len = (uint32_t)(e - b);
            const uint8_t *l = tile + (b - t0);
            if (unpack) pack_lds_to_global(g, l, len, tid); else pack_copy_aligned(s, l, len, tid);
        }
    }
}

// One tile that up to PACK_WIDE pieces reach into: the register path with one table
// entry per lane of the workgroup (the table lives where the many-piece path stages
// its tile) and a bisection per vector instead of a scan.  Returns false, having moved
// nothing, if the tile has more pieces than that.
#define PACK_WIDE PACK_THREADS
__device__ __noinline__ bool pack_tile_wide(uint8_t *stage, uint8_t *slab, uint8_t *const *ptrs, const uint64_t *bytes,
                                            const uint64_t *slab_off, uint32_t n, uint32_t seg, uint64_t t0,
                                            uint64_t t1, int unpack, uint32_t tid)
{
    constexpr int VEC = PACK_TILE / (PACK_THREADS * 16);
    uint64_t *wb = (uint64_t *)stage, *we = wb + PACK_WIDE;
    uint8_t **wg = (uint8_t **)(we + PACK_WIDE);
    uint32_t *flag = (uint32_t *)(wg + PACK_WIDE);          // [0]: too many pieces, [1]: some piece has ragged edges
    // entry seg + tid; a segment that does not reach into the tile becomes the empty piece [t1, t1),
    // which keeps the begins sorted and is never the answer of a bisection for x < t1
    uint64_t b = t1, e = t1;
    uint8_t *g = nullptr;
    if (seg + tid < n) {
        const uint64_t so = slab_off[seg + tid], se = so + bytes[seg + tid];
        if (so < t1 && se > t0) {
            b = so > t0 ? so : t0;
            e = se < t1 ? se : t1;
            g = ptrs[seg + tid] - so;                       // tensor address of slab offset x is g + x
        }
    }
    if (tid == 0) {
        flag[0] = (seg + PACK_WIDE < n && slab_off[seg + PACK_WIDE] < t1) ? 1u : 0u;
        flag[1] = 0;
    }
    wb[tid] = b;
    we[tid] = e;
    wg[tid] = g;
    __syncthreads();
    if (flag[0]) {
        __syncthreads();                                    // the caller reuses the table's memory
        return false;
    }
    if (((b | e) & 15) != 0) flag[1] = 1;                   // (every writer writes the same value)
    uint8_t *ga[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        const uint64_t x = t0 + ((uint64_t)tid + (uint64_t)k * PACK_THREADS) * 16;
        // the last piece that begins at or before x
        uint32_t lo = 0, hi = PACK_WIDE;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (wb[mid] <= x) lo = mid + 1; else hi = mid;
        }
        ga[k] = (lo > 0 && x + 16 <= we[lo - 1]) ? wg[lo - 1] + x : nullptr;
    }
    pack_v4 v[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        const uint64_t x = t0 + ((uint64_t)tid + (uint64_t)k * PACK_THREADS) * 16;
        v[k] = pack_v4{0, 0, 0, 0};
        if (ga[k]) v[k] = unpack ? __builtin_nontemporal_load((const pack_v4 *)(slab + x))
                                 : __builtin_nontemporal_load(&((const pack_u16 *)ga[k])->v);
    }
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        const uint64_t x = t0 + ((uint64_t)tid + (uint64_t)k * PACK_THREADS) * 16;
        if (ga[k]) {
            if (unpack) __builtin_nontemporal_store(v[k], &((pack_u16 *)ga[k])->v);
            else __builtin_nontemporal_store(v[k], (pack_v4 *)(slab + x));
        }
    }
    __syncthreads();
    if (!flag[1]) return true;
    // the bytes of each piece before its first and behind its last whole vector of the slab
    for (uint32_t task = tid; task < PACK_WIDE * 32; task += PACK_THREADS) {
        const uint32_t r = task >> 5, idx = task & 31;
        const uint64_t pb = wb[r], pe = we[r];
        const uint64_t up = (pb + 15) & ~15ull, dn = pe & ~15ull;
        uint64_t y;
        bool mine;
        if (idx < 16) {
            y = pb + idx;
            mine = y < (pe < up ? pe : up);
        } else {
            y = (up > dn ? up : dn) + (idx - 16);
            mine = y < pe;
        }
        if (mine) {
            uint8_t *gq = wg[r] + y;
            if (unpack) *gq = slab[y]; else slab[y] = *gq;
        }
    }
    return true;
}

// Lanes of one wave exchange data through LDS without a workgroup barrier: the
// hardware executes a wave's LDS instructions in order, but to the compiler every
// lane is a thread of its own, and without this it may place one lane's load ahead
// of another lane's store (it did: a value written under `if (lane == 63)` was read
// by the other lanes first).  The fences are compiler-only at wavefront scope.
__device__ __forceinline__ void pack_wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(PACK_THREADS) __attribute__((amdgpu_waves_per_eu(8, 8))) void tc_pack_kernel(
    uint8_t *slab, uint8_t *const *ptrs, const uint64_t *bytes, const uint64_t *slab_off,
    uint32_t n, uint64_t total, int unpack, const uint32_t *tile_first)
{
    constexpr int VEC = PACK_TILE / (PACK_THREADS * 16);    // 128-bit vectors per lane
    constexpr uint32_t TILE = PACK_TILE;
    __shared__ __attribute__((aligned(16))) uint8_t stage[PACK_TILE];
    __shared__ uint64_t tab_b[PACK_THREADS / WAVE][PACK_CAND], tab_e[PACK_THREADS / WAVE][PACK_CAND];
    __shared__ uint8_t *tab_g[PACK_THREADS / WAVE][PACK_CAND];
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), wave = tid / WAVE;
    const uint64_t t0 = (uint64_t)blockIdx.x * TILE;
    const uint64_t t1 = t0 + TILE < total ? t0 + TILE : total;
    const uint32_t seg = tile_first ? tile_first[blockIdx.x] : pack_bisect(slab_off, n, t0);

    // 33 consecutive table entries in one round trip: 32 candidates and the one after them
    bool valid = false, ok = true, beyond = false;
    uint64_t b = 0, e = 0;
    uint8_t *g = nullptr;
    if (lane <= PACK_CAND && seg + lane < n) {
        const uint64_t so = slab_off[seg + lane];
        if (lane == PACK_CAND) {
            beyond = so < t1;                               // more pieces than the table holds
        } else {
            const uint64_t se = so + bytes[seg + lane];
            valid = so < t1 && se > t0;
            if (valid) {
                b = so > t0 ? so : t0;
                e = se < t1 ? se : t1;
                g = ptrs[seg + lane] + (b - so);
                ok = (((b | e) & 15) == 0) && (((uintptr_t)g & 15) == 0);   // the slab itself is 16-byte aligned
            }
        }
    }
    const uint64_t vmask = __ballot(valid);
    // the same in every wave (all read the same entries): which way this tile goes
    if (__ballot(beyond) != 0) {
        if (!pack_tile_wide(stage, slab, ptrs, bytes, slab_off, n, seg, t0, t1, unpack, tid))
            pack_tile_general(stage, slab, ptrs, bytes, slab_off, n, seg, t0, t1, unpack, tid);
        return;
    }
    const bool ragged = __ballot(valid && !ok) != 0;       // some piece is not whole 16-byte vectors on both sides
    const uint32_t n_p = (uint32_t)__popcll(vmask);
    if (valid) {
        const uint32_t p = (uint32_t)__popcll(vmask & ((1ull << lane) - 1));
        tab_b[wave][p] = b;
        tab_e[wave][p] = e;
        tab_g[wave][p] = g - b;                             // tensor address of slab offset x is tab_g + x
    }
    // each wave reads only what its own lanes wrote: no workgroup barrier, a wave-level one
    pack_wave_lds_sync();
    // Every 128-bit vector of the tile that lies inside one piece moves through registers:
    // address pairs first (table look-ups), then every load, then every store.  The slab
    // side is always 16-byte aligned; the tensor side is wherever the tensor is (the
    // hardware takes 128-bit global accesses at any byte address, at 91-97 % of the
    // aligned rate when the address is a multiple of 4, which beats realigning through
    // LDS; interior vectors at odd addresses are moved as the dwords around them).
    uint8_t *ga[VEC];
    uint32_t shift = 0;                                     // two bits per vector: its r (0: moved where it is)
    uint32_t extra = 0;                                     // unpack: this lane also writes the dword before vector k
    uint32_t p = 0;
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        const uint64_t x = t0 + ((uint64_t)tid + (uint64_t)k * PACK_THREADS) * 16;
        while (p < n_p && tab_e[wave][p] <= x) ++p;
        const bool in = p < n_p && tab_b[wave][p] <= x && x + 16 <= tab_e[wave][p];
        ga[k] = in ? tab_g[wave][p] + x : nullptr;
        if (in) {
            const uint32_t r = (uint32_t)((uintptr_t)ga[k] & 3);
            const bool behind = x + 32 <= tab_e[wave][p];
            if (tab_b[wave][p] + 16 <= x && behind) shift |= r << (2 * k);
            else if (unpack && r && !behind && tab_b[wave][p] + 32 <= x) extra |= 1u << k;   // the vector before is interior
        }
    }
    // does the next lane hold the next vector of the same piece, read the same way?  (its first
    // dword is then the one behind this lane's sixteen bytes)
    uint32_t from_next = 0;
    if (!unpack && __ballot(shift != 0) != 0) {
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const uintptr_t mine = (uintptr_t)ga[k];
            const uint32_t nlo = (uint32_t)__shfl_down((int)(uint32_t)mine, 1, WAVE);
            const uint32_t nhi = (uint32_t)__shfl_down((int)(uint32_t)(mine >> 32), 1, WAVE);
            const uint32_t nsh = (uint32_t)__shfl_down((int)shift, 1, WAVE);
            const uint32_t r = (shift >> (2 * k)) & 3;
            const bool ok_next = lane + 1 < WAVE && r != 0 && (((uintptr_t)nhi << 32) | nlo) == mine + 16 &&
                                 ((nsh >> (2 * k)) & 3) == r;
            from_next |= (ok_next ? 1u : 0u) << k;
        }
    }
    // streaming accesses: nothing moved here is read again by this kernel
    pack_v4 v[VEC];
    uint32_t hi[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        const uint64_t x = t0 + ((uint64_t)tid + (uint64_t)k * PACK_THREADS) * 16;
        const uint32_t r = (shift >> (2 * k)) & 3;
        v[k] = pack_v4{0, 0, 0, 0};
        hi[k] = 0;
        if (ga[k]) {
            if (unpack) {
                v[k] = __builtin_nontemporal_load((const pack_v4 *)(slab + x));
                // x - 16 is a whole vector of the same piece, so x - 4 lies inside this tile
                if (lane == 0 && (r || ((extra >> k) & 1))) hi[k] = __builtin_nontemporal_load((const uint32_t *)(slab + x - 4));
            } else {
                v[k] = __builtin_nontemporal_load(&((const pack_u16 *)(ga[k] - r))->v);
                if (r && !((from_next >> k) & 1)) hi[k] = __builtin_nontemporal_load((const uint32_t *)(ga[k] - r + 16));
            }
        }
    }
    if (unpack) {
        if (__ballot((shift | extra) != 0) != 0) {
            // the lane before this one holds the slab vector before this one (every lane that asks
            // has a whole vector of its piece there); lanes that do not ask never look at hi
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const uint32_t pv = (uint32_t)__shfl_up((int)v[k].w, 1, WAVE);
                if (lane != 0) hi[k] = pv;
            }
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const uint32_t r = (shift >> (2 * k)) & 3;
                if (r) v[k] = pack_join_before(hi[k], v[k], r);
            }
        }
    } else {
        if (__ballot(from_next != 0) != 0) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const uint32_t nx = (uint32_t)__shfl_down((int)v[k].x, 1, WAVE);
                if ((from_next >> k) & 1) hi[k] = nx;
            }
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) v[k] = pack_join(v[k], hi[k], (shift >> (2 * k)) & 3);
    }
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        const uint64_t x = t0 + ((uint64_t)tid + (uint64_t)k * PACK_THREADS) * 16;
        if (ga[k]) {
            if (unpack) {
                __builtin_nontemporal_store(v[k], &((pack_u16 *)(ga[k] - ((shift >> (2 * k)) & 3)))->v);
                if ((extra >> k) & 1) __builtin_nontemporal_store(hi[k], &((pack_u4 *)(ga[k] - 4))->v);
            } else {
                __builtin_nontemporal_store(v[k], (pack_v4 *)(slab + x));
            }
        }
    }
    if (!ragged) return;
    // the bytes of each piece before its first and behind its last whole vector (slab side):
    // 32 byte-tasks per piece
    for (uint32_t task = tid; task < n_p * 32; task += PACK_THREADS) {
        const uint32_t r = task >> 5, idx = task & 31;
        const uint64_t pb = tab_b[wave][r], pe = tab_e[wave][r];
        const uint64_t up = (pb + 15) & ~15ull, dn = pe & ~15ull;
        uint64_t y;
        bool mine;
        if (idx < 16) {
            y = pb + idx;
            mine = y < (pe < up ? pe : up);
        } else {
            y = (up > dn ? up : dn) + (idx - 16);
            mine = y < pe;
        }
        if (mine) {
            uint8_t *gq = tab_g[wave][r] + y;
            if (unpack) *gq = slab[y]; else slab[y] = *gq;
        }
    }
}

uint64_t tc_pack_tile_count(uint64_t total) { return (total + PACK_TILE - 1) / PACK_TILE; }

hipError_t tc_launch_pack_index(const uint64_t *slab_off, uint32_t n, uint64_t total, uint32_t *tile_first, hipStream_t s)
{
    const uint64_t tiles = tc_pack_tile_count(total);
    if (n == 0 || tiles == 0) return hipSuccess;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tc_pack_index_kernel, dim3((uint32_t)((tiles + 255) / 256)), dim3(256), 0, s, slab_off, n, tiles,
                       (uint32_t)PACK_TILE, tile_first);
    return hipGetLastError();
}

hipError_t tc_launch_pack(void *slab, const void *const *ptrs, const uint64_t *bytes, const uint64_t *slab_off,
                          uint32_t n, uint64_t total, int unpack, const uint32_t *tile_first, hipStream_t s)
{
    const uint64_t tiles = tc_pack_tile_count(total);
    if (n == 0 || tiles == 0) return hipSuccess;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(tc_pack_kernel, dim3((uint32_t)tiles), dim3(PACK_THREADS), 0, s, (uint8_t *)slab,
                       (uint8_t *const *)ptrs, bytes, slab_off, n, total, unpack, tile_first);
    return hipGetLastError();
}

// ===========================================================================
// Pack / unpack for callers that cannot allocate (code under HIP graph capture,
// serving loops, harnesses that forbid hipMalloc): the tile index, which tc_pack
// takes as a workspace argument, lives in a file-scope device array instead.
//
// In host code the array's name is only a stand-in for the symbol; the address a
// kernel can use is asked for once per device (hipGetSymbolAddress with that
// device current; every GPU holds its own copy at its own address) and kept.
// Every call on a GPU shares that GPU's array.  Nothing in it has to start at
// zero: the index kernel writes every entry the pack kernel of the same call
// reads, in stream order.  Calls that overlap on one GPU (two streams, two
// threads) race on it.
// ===========================================================================
#define PACK_STATIC_TILES (TC_PACK_STATIC_MAX_BYTES / PACK_TILE)
static __device__ __align__(256) uint32_t scratch[PACK_STATIC_TILES];     // 1 MiB per GPU, held until the process ends

static hipError_t pack_static_scratch(uint32_t **out)
{
    static std::mutex mu;
    static uint32_t *ptr[64];                               // per device, nullptr until asked for
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> g(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = (uint32_t *)p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

extern "C" int tc_pack_static(void *slab, const void *const *ptrs, const uint64_t *bytes, const uint64_t *slab_off,
                              uint32_t n, uint64_t total, int unpack, void *stream)
{
    if (total > TC_PACK_STATIC_MAX_BYTES) return TC_E_CAPACITY;          // the index would not fit the array
    if (n == 0 || total == 0) return TC_OK;
    if (!slab || !ptrs || !bytes || !slab_off) return TC_E_ARG;
    if ((uintptr_t)slab & 15) return TC_E_ARG;
    uint32_t *index = nullptr;
    if (pack_static_scratch(&index) != hipSuccess) return TC_E_HIP;
    const uint64_t tiles = tc_pack_tile_count(total);
    if (tiles > PACK_STATIC_TILES) return TC_E_CAPACITY;
    hipStream_t s = (hipStream_t)stream;
    if (tc_launch_pack_index(slab_off, n, total, index, s) != hipSuccess) return TC_E_HIP;
    if (tc_launch_pack(slab, ptrs, bytes, slab_off, n, total, unpack ? 1 : 0, index, s) != hipSuccess) return TC_E_HIP;
    return TC_OK;
}
