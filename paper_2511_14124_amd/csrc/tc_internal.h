// Internal declarations shared by the planner, the runtime and the kernels of
// libtc.so.  Nothing here is part of the public ABI (see include/tc.h).
#pragma once

#include <stdint.h>
#include <string>
#include <vector>

#include <hip/hip_runtime.h>

#include "tc.h"

#define TC_INF 0xFFFFFFFFu

// ---------------------------------------------------------------------------
// host-side plan (Sec. 3.2 - 3.3)
// ---------------------------------------------------------------------------
struct TcProfile {
    uint32_t n_tensors = 0, n_steps = 0;
    std::vector<uint64_t> bytes;          // per tensor
    std::vector<uint8_t> group, kind;
    std::vector<uint32_t> rows_tensor;    // prefetch table, execution order
    std::vector<uint8_t> rows_rw;
    std::vector<uint32_t> row_begin;      // n_steps + 1 entries
    std::vector<uint64_t> step_ns;        // modelled compute per step
    std::vector<uint32_t> occ_ptr, occ_rows;   // CSR: rows using tensor t
    std::vector<uint32_t> first_use;
    std::vector<uint32_t> class_of;
    // per class
    std::vector<uint64_t> class_bytes;
    std::vector<uint32_t> class_group, count, used, step_max;
};

struct TcPools {
    std::vector<uint64_t> stride, hbm_off, host_off;
    std::vector<uint32_t> gpu_count, cpu_count;
    std::vector<uint32_t> gpu_base, cpu_base;   // first entry of class s in the flat owner tables
    uint64_t hbm_total = 0, host_total = 0;
    uint32_t gpu_slots = 0, cpu_slots = 0;
};

struct TcPlacement {
    std::vector<uint8_t> final_tier;
    std::vector<uint32_t> slot;
    std::vector<uint64_t> file_off;
    std::vector<uint32_t> order;                // tensors in placement order
    std::vector<uint32_t> member_ptr, members;  // CSR: placement order within each class
    uint64_t file_total = 0;
};

int tc_build_profile(TcProfile &p, const tc_tensor_desc *t, uint32_t n_t, const tc_event *ev,
                     uint64_t n_ev, std::string &err);
int tc_build_pools(const TcProfile &p, const tc_budget &b, TcPools &out, std::string &err);
void tc_build_placement(const TcProfile &p, const TcPools &pools, TcPlacement &out);

// ---------------------------------------------------------------------------
// device-side tables of the decision kernel
// ---------------------------------------------------------------------------
struct TcDevTables {
    // immutable after tc_bind_memory
    const uint32_t *rows_tensor;
    const uint32_t *row_begin;
    const uint32_t *occ_ptr;
    const uint32_t *occ_rows;
    const uint32_t *class_of;
    const uint32_t *final_tier;
    const uint32_t *gpu_count, *cpu_count, *gpu_base, *cpu_base;
    const uint32_t *member_ptr, *members;
    uint32_t n_rows, n_steps, n_tensors, n_classes;
    uint32_t flags;                             // tc_budget.flags
    const uint8_t *rows_rw;                     // R/W flags of the profiled rows
    // mutable scheduler state
    uint32_t *cur, *gslot, *cslot, *dirty, *moved;
    uint32_t *undefined;                        // allocated without fetch, not written yet
    uint32_t *gpu_owner, *gpu_freed, *cpu_owner, *cpu_freed, *designated;
    uint32_t *scalars;                          // [0] cursor, [1] call id, [2] iteration
};

// one decision, as the kernel reports it (16 bytes)
struct TcOpRec {
    uint32_t tensor, src_slot, dst_slot;
    uint8_t op, phase, src_tier, dst_tier;
};

// what the decision kernel reports for one hook call (pinned host memory);
// the call's op records are written to a separate array
struct TcDecideOut {
    uint32_t n_ops, hits, misses, fails;
    uint32_t cursor, iteration, overflow, undefined_reads;
    uint32_t slots[TC_MAX_STEP_TENSORS];
};

struct TcStepArgs {
    uint32_t ids[TC_MAX_STEP_TENSORS];
    uint8_t rw[TC_MAX_STEP_TENSORS];
    uint32_t n, step, phase, cap;
};

// a window of steps decided by one launch (lists in device memory)
#define TC_WINDOW_MAX 256
struct TcWindowArgs {
    const uint32_t *step_ptr;                   // n_steps + 1 offsets into ids / rw
    const uint32_t *ids;
    const uint8_t *rw;
    uint32_t first, count;                      // steps first .. first+count-1
    uint32_t cap;                               // op records the window may write
    uint32_t n_calls;                           // hook calls to decide: 2 * count, or fewer to stop inside the window
};

// ---------------------------------------------------------------------------
// migration kernel
// ---------------------------------------------------------------------------
// One exchange unit: up to two copies that share one index space.  Every lane
// loads its 16 bytes of both sources before it stores either, so "out" may
// read the buffer "in" overwrites (a tensor leaving a GPU buffer while another
// arrives in it) and the two host buffers may be one (a swap).
struct TcUnit {
    const uint8_t *out_src;
    uint8_t *out_dst;
    const uint8_t *in_src;
    uint8_t *in_dst;
    uint64_t bytes;
    uint64_t chunk0;                            // first work chunk of this unit in the launch
};

#define TC_MOVER_MAX_UNITS 48
struct TcMoverArgs {
    TcUnit u[TC_MOVER_MAX_UNITS];
    uint64_t n_chunks;
    uint32_t n_units;
    uint32_t chunk_bytes;
    uint32_t *tickets;                          // device: two words, both zero before the stream's first launch
    uint32_t slot;                              // 0 or 1: set by the launcher, alternates between launches
    uint32_t xcc;                               // the XCD whose workgroups do the work
    uint32_t n_xcd;                             // XCDs the dispatcher deals workgroups to (grid = workgroups x n_xcd)
    // Dependencies resolved on the GPU (progress nullptr: none).  The launch may be queued before the modules
    // it has to wait for have run; its working workgroups wait until the word at `progress` has reached
    // need_seq (tc_signal_kernel, queued on the compute stream behind those modules, raises it).  The wait
    // is bounded: after spin_ticks of the 100 MHz wall clock a waiter gives up, raises *fault and the launch
    // moves nothing (the host reports it; the data is then not to be trusted).  (That a launch is done is
    // signalled the same way, by a tc_signal_kernel queued behind it on its own stream, and waited for by a
    // tc_wait_kernel in front of the module that needs it.)
    const uint32_t *progress;
    uint32_t *fault;                            // pinned host word the host reads
    uint32_t *gave_up;                          // device word: set with *fault, makes every later waiter give up at once
    uint32_t need_seq;
    uint64_t spin_ticks;
};

struct TcStampArgs {
    uint8_t *ptr[TC_MAX_STEP_TENSORS];
    uint64_t bytes[TC_MAX_STEP_TENSORS];
    uint32_t tensor[TC_MAX_STEP_TENSORS];
    uint8_t whole[TC_MAX_STEP_TENSORS];         // written whole (filled), not stamped
    uint32_t n, iteration, step;
    uint64_t busy_ns;
};

// launchers (tc_kernels.hip)
hipError_t tc_launch_decide(const TcDevTables &T, const TcStepArgs &a, TcDecideOut *out, TcOpRec *ops, hipStream_t s);
hipError_t tc_launch_decide_window(const TcDevTables &T, const TcWindowArgs &w, TcDecideOut *out, TcOpRec *ops,
                                   hipStream_t s);
// workgroups: how many should work (the launch has n_xcd times as many, those on other XCDs exit)
// where the dispatcher puts workgroups on the current device (probed once): XCD of workgroup 0, number of XCDs
hipError_t tc_mover_topology(uint32_t *xcc, uint32_t *n_xcd);
hipError_t tc_launch_zero_tickets(uint32_t *tickets, hipStream_t s);   // both counters to zero, by a kernel
// launches: how many launches have used a.tickets so far (all on one stream, in order); counted up here
hipError_t tc_launch_mover(TcMoverArgs &a, uint32_t workgroups, hipStream_t s, uint64_t *launches);
// raises the word at `word` to seq (never lowers it), one lane, on stream s
hipError_t tc_launch_signal(uint32_t *word, uint32_t seq, hipStream_t s);
// waits on stream s until the word at `word` has reached seq, at most spin_ticks of the 100 MHz clock (then *fault = 2)
hipError_t tc_launch_wait(const uint32_t *word, uint32_t seq, uint64_t spin_ticks, uint32_t *fault, uint32_t *gave_up,
                          hipStream_t s);
hipError_t tc_launch_stamp(const TcStampArgs &a, hipStream_t s);
hipError_t tc_launch_fill(void *dst, uint64_t bytes, uint32_t tensor, uint32_t seed, hipStream_t s);
uint64_t tc_pack_tile_count(uint64_t total);
hipError_t tc_launch_pack_index(const uint64_t *slab_off, uint32_t n, uint64_t total, uint32_t *tile_first, hipStream_t s);
hipError_t tc_launch_pack(void *slab, const void *const *ptrs, const uint64_t *bytes, const uint64_t *slab_off,
                          uint32_t n, uint64_t total, int unpack, const uint32_t *tile_first, hipStream_t s);
