// Host planner: the tensor characteristic analyzer (Sec. 3.2), the cache
// allocator (Sec. 3.3.1, Alg. 1-2 and the region layout of Step 3) and the
// tensor allocator (Sec. 3.3.2).  Pure integer host code, run once per
// workload before training starts, as in the paper.
#include "tc_internal.h"

#include <algorithm>
#include <map>
#include <numeric>

typedef unsigned __int128 u128;

int tc_build_profile(TcProfile &p, const tc_tensor_desc *t, uint32_t n_t, const tc_event *ev,
                     uint64_t n_ev, std::string &err)
{
    p = TcProfile();
    p.n_tensors = n_t;
    p.bytes.resize(n_t);
    p.group.resize(n_t);
    p.kind.resize(n_t);
    for (uint32_t i = 0; i < n_t; ++i) {
        if (t[i].bytes < 16) { err = "tensor smaller than 16 bytes"; return TC_E_ARG; }
        if (t[i].group > 1) { err = "tensor group must be 0 or 1"; return TC_E_ARG; }
        p.bytes[i] = t[i].bytes;
        p.group[i] = t[i].group;
        p.kind[i] = t[i].kind;
    }
    if (n_ev >= TC_INF) { err = "too many events"; return TC_E_ARG; }
    // the last event names the last step only if the events are in order: look before the tables are sized by it
    for (uint64_t i = 1; i < n_ev; ++i)
        if (ev[i].step < ev[i - 1].step) { err = "events are not ordered by step"; return TC_E_ARG; }
    if (n_ev && ev[n_ev - 1].step >= TC_MAX_STEPS) { err = "step index beyond TC_MAX_STEPS"; return TC_E_ARG; }
    p.n_steps = n_ev ? ev[n_ev - 1].step + 1 : 0;
    // Prefetch table (Sec. 3.2.1): rows in execution order; a tensor a step
    // names twice is one row whose flags are OR-ed.
    p.row_begin.assign(p.n_steps + 1, 0);
    p.step_ns.assign(p.n_steps, 0);
    std::vector<uint32_t> row_of(n_t, TC_INF);     // row of tensor t within the step being built
    uint32_t cur_step = 0;
    uint32_t step_first_row = 0;
    for (uint64_t i = 0; i < n_ev; ++i) {
        const tc_event &e = ev[i];
        if (e.step < cur_step) { err = "events are not ordered by step"; return TC_E_ARG; }
        if (e.tensor >= n_t) { err = "event names an unknown tensor"; return TC_E_ARG; }
        if (e.rw < 1 || e.rw > 3) { err = "event rw must be R, W or RW"; return TC_E_ARG; }
        while (cur_step < e.step) {
            ++cur_step;
            p.row_begin[cur_step] = (uint32_t)p.rows_tensor.size();
            step_first_row = p.row_begin[cur_step];
        }
        p.step_ns[e.step] = e.compute_ns;
        uint32_t r = row_of[e.tensor];
        if (r != TC_INF && r >= step_first_row) {
            p.rows_rw[r] |= e.rw;
        } else {
            row_of[e.tensor] = (uint32_t)p.rows_tensor.size();
            p.rows_tensor.push_back(e.tensor);
            p.rows_rw.push_back(e.rw);
        }
    }
    for (uint32_t k = cur_step + 1; k <= p.n_steps; ++k) p.row_begin[k] = (uint32_t)p.rows_tensor.size();
    const uint32_t n_rows = (uint32_t)p.rows_tensor.size();

    // per-tensor use lists
    p.occ_ptr.assign(n_t + 1, 0);
    for (uint32_t r = 0; r < n_rows; ++r) p.occ_ptr[p.rows_tensor[r] + 1]++;
    for (uint32_t i = 0; i < n_t; ++i) p.occ_ptr[i + 1] += p.occ_ptr[i];
    p.occ_rows.resize(n_rows);
    {
        std::vector<uint32_t> fill(p.occ_ptr.begin(), p.occ_ptr.end() - 1);
        for (uint32_t r = 0; r < n_rows; ++r) p.occ_rows[fill[p.rows_tensor[r]]++] = r;
    }
    p.first_use.resize(n_t);
    for (uint32_t i = 0; i < n_t; ++i)
        p.first_use[i] = p.occ_ptr[i + 1] > p.occ_ptr[i] ? p.occ_rows[p.occ_ptr[i]] : TC_INF;

    // size classes: distinct (bytes, group), ascending (Sec. 3.2.2: the
    // dictionary TC; the two groups are sized in separate runs of Alg. 2)
    std::map<std::pair<uint64_t, uint32_t>, uint32_t> keys;
    for (uint32_t i = 0; i < n_t; ++i) keys[{p.bytes[i], p.group[i]}] = 0;
    uint32_t n_c = 0;
    for (auto &kv : keys) {
        kv.second = n_c++;
        p.class_bytes.push_back(kv.first.first);
        p.class_group.push_back(kv.first.second);
    }
    p.class_of.resize(n_t);
    p.count.assign(n_c, 0);
    p.used.assign(n_c, 0);
    p.step_max.assign(n_c, 0);
    for (uint32_t i = 0; i < n_t; ++i) {
        uint32_t s = keys[{p.bytes[i], p.group[i]}];
        p.class_of[i] = s;
        p.count[s]++;
        if (p.first_use[i] != TC_INF) p.used[s]++;
    }
    std::vector<uint32_t> per(n_c);
    for (uint32_t k = 0; k < p.n_steps; ++k) {
        std::fill(per.begin(), per.end(), 0u);
        for (uint32_t r = p.row_begin[k]; r < p.row_begin[k + 1]; ++r) per[p.class_of[p.rows_tensor[r]]]++;
        for (uint32_t s = 0; s < n_c; ++s) p.step_max[s] = std::max(p.step_max[s], per[s]);
    }
    return TC_OK;
}

// One output of Alg. 2 for a set of (size, count) pairs: Alg. 1's share of the
// size, times the available memory, divided by the size, rounded down, capped.
// TSD[s]*avail/s = count*avail/total exactly, so no fraction is ever formed.
static void buffer_count(const std::vector<uint64_t> &size, const std::vector<uint32_t> &count,
                         uint64_t avail, const std::vector<uint32_t> &cap, std::vector<uint32_t> &out)
{
    u128 total = 0;
    for (size_t i = 0; i < size.size(); ++i) total += (u128)size[i] * count[i];
    out.resize(size.size());
    for (size_t i = 0; i < size.size(); ++i) {
        u128 n = total ? ((u128)count[i] * avail) / total : 0;
        out[i] = (uint32_t)std::min<u128>(n, cap[i]);
    }
}

int tc_build_pools(const TcProfile &p, const tc_budget &b, TcPools &out, std::string &err)
{
    const uint32_t n_c = (uint32_t)p.count.size();
    uint32_t align = b.align ? b.align : 256;
    if (align < 16 || (align & (align - 1))) { err = "align must be a power of two >= 16"; return TC_E_ARG; }
    out = TcPools();
    out.stride.resize(n_c);
    for (uint32_t s = 0; s < n_c; ++s) out.stride[s] = (p.class_bytes[s] + align - 1) / align * align;

    if (b.flags & TC_SMALLEST_FIRST) {
        // The placement the paper argues against (Sec. 3.1, Sec. 3.3.2: large tensors live below the
        // GPU whatever their place in the execution order), as an ablation: beyond the working-set
        // floor, GPU memory goes to the classes in ascending size, each taking what it can use.
        out.gpu_count.resize(n_c);
        u128 reserved = 0;
        for (uint32_t s = 0; s < n_c; ++s) {
            out.gpu_count[s] = (b.flags & TC_LITERAL_ALG2) ? 0 : std::min(p.step_max[s], p.used[s]);
            reserved += (u128)out.gpu_count[s] * out.stride[s];
        }
        if (reserved > b.hbm_bytes) { err = "HBM budget below the per-step working set"; return TC_E_CAPACITY; }
        uint64_t left = b.hbm_bytes - (uint64_t)reserved;
        for (uint32_t s = 0; s < n_c; ++s) {               // classes are ascending by (bytes, group)
            const uint64_t more = std::min<uint64_t>(p.used[s] - out.gpu_count[s], left / out.stride[s]);
            out.gpu_count[s] += (uint32_t)more;
            left -= more * out.stride[s];
        }
    } else if (b.flags & TC_LITERAL_ALG2) {
        buffer_count(out.stride, p.used, b.hbm_bytes, p.used, out.gpu_count);
    } else {
        // working-set floor: step_max buffers per class first, Alg. 2 on the rest
        std::vector<uint32_t> floor_(n_c), rest(n_c), extra;
        u128 reserved = 0;
        for (uint32_t s = 0; s < n_c; ++s) {
            floor_[s] = std::min(p.step_max[s], p.used[s]);
            rest[s] = p.used[s] - floor_[s];
            reserved += (u128)floor_[s] * out.stride[s];
        }
        if (reserved > b.hbm_bytes) { err = "HBM budget below the per-step working set"; return TC_E_CAPACITY; }
        buffer_count(out.stride, rest, b.hbm_bytes - (uint64_t)reserved, rest, extra);
        out.gpu_count.resize(n_c);
        for (uint32_t s = 0; s < n_c; ++s) out.gpu_count[s] = floor_[s] + extra[s];
    }
    out.cpu_count.assign(n_c, 0);
    for (uint32_t g = 0; g < 2; ++g) {
        std::vector<uint64_t> size;
        std::vector<uint32_t> cnt, cap, got, idx;
        for (uint32_t s = 0; s < n_c; ++s)
            if (p.class_group[s] == g) {
                idx.push_back(s);
                size.push_back(out.stride[s]);
                cnt.push_back(p.count[s]);
                cap.push_back(p.count[s] - out.gpu_count[s]);
            }
        buffer_count(size, cnt, b.host_bytes[g], cap, got);
        for (size_t i = 0; i < idx.size(); ++i) out.cpu_count[idx[i]] = got[i];
    }
    // Step 3: classes ascending, offsets are running sums; buffer k of class s
    // is at off[s] + k*stride[s].
    out.hbm_off.resize(n_c);
    out.host_off.resize(n_c);
    out.gpu_base.resize(n_c);
    out.cpu_base.resize(n_c);
    for (uint32_t s = 0; s < n_c; ++s) {
        out.hbm_off[s] = out.hbm_total;
        out.host_off[s] = out.host_total;
        out.gpu_base[s] = out.gpu_slots;
        out.cpu_base[s] = out.cpu_slots;
        out.hbm_total += (uint64_t)out.gpu_count[s] * out.stride[s];
        out.host_total += (uint64_t)out.cpu_count[s] * out.stride[s];
        out.gpu_slots += out.gpu_count[s];
        out.cpu_slots += out.cpu_count[s];
    }
    return TC_OK;
}

void tc_build_placement(const TcProfile &p, const TcPools &pools, TcPlacement &out)
{
    const uint32_t n_t = p.n_tensors, n_c = (uint32_t)p.count.size();
    out = TcPlacement();
    out.order.resize(n_t);
    std::iota(out.order.begin(), out.order.end(), 0u);
    // execution order; tensors the profiled iteration never used come last, by id
    std::stable_sort(out.order.begin(), out.order.end(),
                     [&](uint32_t a, uint32_t b) { return p.first_use[a] < p.first_use[b]; });
    out.final_tier.assign(n_t, TC_NVME);
    out.slot.assign(n_t, TC_NONE);
    std::vector<uint32_t> gpu_next(n_c, 0), cpu_next(n_c, 0);
    for (uint32_t t : out.order) {
        uint32_t s = p.class_of[t];
        if (p.first_use[t] != TC_INF && gpu_next[s] < pools.gpu_count[s]) {
            out.final_tier[t] = TC_GPU;
            out.slot[t] = gpu_next[s]++;
        } else if (cpu_next[s] < pools.cpu_count[s]) {
            out.final_tier[t] = TC_CPU;
            out.slot[t] = cpu_next[s]++;
        }
    }
    out.file_off.resize(n_t);
    uint64_t off = 0;
    for (uint32_t t = 0; t < n_t; ++t) {
        out.file_off[t] = off;
        off += (p.bytes[t] + 4095) / 4096 * 4096;
    }
    out.file_total = off;
    out.member_ptr.assign(n_c + 1, 0);
    for (uint32_t t = 0; t < n_t; ++t) out.member_ptr[p.class_of[t] + 1]++;
    for (uint32_t s = 0; s < n_c; ++s) out.member_ptr[s + 1] += out.member_ptr[s];
    out.members.resize(n_t);
    std::vector<uint32_t> fill(out.member_ptr.begin(), out.member_ptr.end() - 1);
    for (uint32_t t : out.order) out.members[fill[p.class_of[t]]++] = t;
}
