// Stand-alone entry points of libtc.so: batched copy and exchange over the
// migration kernel, pack / unpack.  They need no context.
#include "tc_internal.h"

#include <stdint.h>

// Ticket counters for the stand-alone movers: two words from the stream-ordered
// allocator, cleared on the stream by a small kernel, freed on the stream behind
// the launches.
namespace {
struct StreamTickets {
    uint32_t *p = nullptr;
    hipStream_t s;
    uint64_t launches = 0;
    uint32_t xcc = 0, n_xcd = 1;
    explicit StreamTickets(hipStream_t stream) : s(stream)
    {
        if (tc_mover_topology(&xcc, &n_xcd) != hipSuccess) return;
        if (hipMallocAsync((void **)&p, 256, s) != hipSuccess) { p = nullptr; return; }
        if (tc_launch_zero_tickets(p, s) != hipSuccess) { (void)hipFreeAsync(p, s); p = nullptr; }
    }
    ~StreamTickets() { if (p) (void)hipFreeAsync(p, s); }
};
} // namespace

extern "C" int tc_copy_batch(const tc_segment *segs, uint32_t n, void *stream, uint32_t workgroups,
                             uint32_t chunk_bytes)
{
    if (!segs && n) return TC_E_ARG;
    if (!workgroups) workgroups = 12;
    if (!chunk_bytes) chunk_bytes = 16384;
    if (chunk_bytes % 4096 || workgroups > 8192) return TC_E_ARG;
    for (uint32_t k = 0; k < n; ++k)
        if (segs[k].bytes && (!segs[k].src || !segs[k].dst || ((((uintptr_t)segs[k].src) | ((uintptr_t)segs[k].dst)) & 15)))
            return TC_E_ARG;
    StreamTickets tk((hipStream_t)stream);
    if (!tk.p) return TC_E_HIP;
    uint32_t i = 0;
    while (i < n) {
        TcMoverArgs a{};
        a.chunk_bytes = chunk_bytes;
        a.tickets = tk.p;
        a.xcc = tk.xcc;
        a.n_xcd = tk.n_xcd;
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
        if (tc_launch_mover(a, workgroups, (hipStream_t)stream, &tk.launches) != hipSuccess) return TC_E_HIP;
    }
    return TC_OK;
}

extern "C" int tc_exchange_batch(const tc_segment *out, const tc_segment *in, uint32_t n, void *stream,
                                 uint32_t workgroups, uint32_t chunk_bytes)
{
    if ((!out || !in) && n) return TC_E_ARG;
    if (!workgroups) workgroups = 12;
    if (!chunk_bytes) chunk_bytes = 16384;
    if (chunk_bytes % 4096 || workgroups > 8192) return TC_E_ARG;
    for (uint32_t k = 0; k < n; ++k) {
        if (out[k].bytes && in[k].bytes && out[k].bytes != in[k].bytes) return TC_E_ARG;
        if (out[k].bytes && (!out[k].src || !out[k].dst || ((((uintptr_t)out[k].src) | ((uintptr_t)out[k].dst)) & 15))) return TC_E_ARG;
        if (in[k].bytes && (!in[k].src || !in[k].dst || ((((uintptr_t)in[k].src) | ((uintptr_t)in[k].dst)) & 15))) return TC_E_ARG;
    }
    StreamTickets tk((hipStream_t)stream);
    if (!tk.p) return TC_E_HIP;
    uint32_t i = 0;
    while (i < n) {
        TcMoverArgs a{};
        a.chunk_bytes = chunk_bytes;
        a.tickets = tk.p;
        a.xcc = tk.xcc;
        a.n_xcd = tk.n_xcd;
        for (; i < n && a.n_units < TC_MOVER_MAX_UNITS; ++i) {
            const uint64_t bytes = out[i].bytes ? out[i].bytes : in[i].bytes;
            if (!bytes) continue;
            if (out[i].bytes && in[i].bytes && out[i].bytes != in[i].bytes) return TC_E_ARG;
            TcUnit &u = a.u[a.n_units];
            if (out[i].bytes) {
                if (!out[i].src || !out[i].dst || ((((uintptr_t)out[i].src) | ((uintptr_t)out[i].dst)) & 15)) return TC_E_ARG;
                u.out_src = (const uint8_t *)out[i].src;
                u.out_dst = (uint8_t *)out[i].dst;
            }
            if (in[i].bytes) {
                if (!in[i].src || !in[i].dst || ((((uintptr_t)in[i].src) | ((uintptr_t)in[i].dst)) & 15)) return TC_E_ARG;
                u.in_src = (const uint8_t *)in[i].src;
                u.in_dst = (uint8_t *)in[i].dst;
            }
            u.bytes = bytes;
            u.chunk0 = a.n_chunks;
            a.n_chunks += (bytes + chunk_bytes - 1) / chunk_bytes;
            a.n_units++;
        }
        if (tc_launch_mover(a, workgroups, (hipStream_t)stream, &tk.launches) != hipSuccess) return TC_E_HIP;
    }
    return TC_OK;
}

extern "C" uint64_t tc_pack_tiles(uint64_t total_bytes) { return tc_pack_tile_count(total_bytes); }

extern "C" int tc_pack_index(const uint64_t *slab_off, uint32_t n, uint64_t total, uint32_t *tile_first, void *stream)
{
    if ((!slab_off || !tile_first) && n && total) return TC_E_ARG;
    return tc_launch_pack_index(slab_off, n, total, tile_first, (hipStream_t)stream) == hipSuccess ? TC_OK : TC_E_HIP;
}

extern "C" int tc_pack(void *slab, const void *const *ptrs, const uint64_t *bytes, const uint64_t *slab_off,
                       uint32_t n, uint64_t total, const uint32_t *tile_first, void *stream)
{
    if ((!slab || !ptrs || !bytes || !slab_off) && n) return TC_E_ARG;
    if ((uintptr_t)slab & 15) return TC_E_ARG;
    return tc_launch_pack(slab, ptrs, bytes, slab_off, n, total, 0, tile_first, (hipStream_t)stream) == hipSuccess
               ? TC_OK : TC_E_HIP;
}

extern "C" int tc_unpack(const void *slab, void *const *ptrs, const uint64_t *bytes, const uint64_t *slab_off,
                         uint32_t n, uint64_t total, const uint32_t *tile_first, void *stream)
{
    if ((!slab || !ptrs || !bytes || !slab_off) && n) return TC_E_ARG;
    if ((uintptr_t)slab & 15) return TC_E_ARG;
    return tc_launch_pack((void *)slab, (const void *const *)ptrs, bytes, slab_off, n, total, 1, tile_first,
                          (hipStream_t)stream) == hipSuccess ? TC_OK : TC_E_HIP;
}
