// Stand-alone probe of the host link under duplex load, XCD by XCD (gfx950).
//
// Part 1: one exchange launch (a GPU buffer goes out to pinned memory while
// another pinned buffer comes in, 16 KiB blocks handed out by a ticket
// counter), every workgroup noting for each of its blocks the XCD it runs on
// and how long the block took: the table shows how unevenly the XCDs are served
// when workgroups are spread over all of them.
// Part 2: the same exchange with the working workgroups confined to chosen XCDs
// (mask) and in varying number, by launch size.
//
// This is the experiment behind the migration kernel's placement (all working
// workgroups on one XCD, a dozen of them).  Built by the package's build step
// into link_xcd_probe.bin; run it on the GPU machine without arguments.
#include <hip/hip_runtime.h>

#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <vector>

#define CHECK(x)                                                              \
    do {                                                                      \
        hipError_t e_ = (x);                                                  \
        if (e_ != hipSuccess) {                                               \
            printf("%s: %s\n", #x, hipGetErrorString(e_));                    \
            return 1;                                                         \
        }                                                                     \
    } while (0)

#define THREADS 256
#define UNROLL 4
#define BLOCK_BYTES (THREADS * UNROLL * 16)

struct Rec {
    unsigned long long t0, t1;      // wall_clock64 (100 MHz) before the block's loads, after its stores were acknowledged
    unsigned xcc;
};

// every workgroup on an XCD of `mask` takes blocks from the ticket counter until none are left
__global__ __launch_bounds__(THREADS) void exchange(const uint4 *out_src, uint4 *out_dst, const uint4 *in_src,
                                                    uint4 *in_dst, unsigned n_blocks, unsigned *ticket, unsigned mask,
                                                    Rec *rec)
{
    unsigned xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    xcc &= 15u;
    if (!((mask >> xcc) & 1u)) return;
    __shared__ unsigned next;
    for (;;) {
        __syncthreads();
        if (threadIdx.x == 0) next = atomicAdd(ticket, 1u);
        __syncthreads();
        const unsigned b = next;
        if (b >= n_blocks) break;
        const size_t base = (size_t)b * THREADS * UNROLL + threadIdx.x;
        uint4 vo[UNROLL], vi[UNROLL];
        const unsigned long long t0 = (unsigned long long)wall_clock64();
        for (int j = 0; j < UNROLL; ++j) vi[j] = in_src[base + j * THREADS];
        for (int j = 0; j < UNROLL; ++j) vo[j] = out_src[base + j * THREADS];
        for (int j = 0; j < UNROLL; ++j) out_dst[base + j * THREADS] = vo[j];
        for (int j = 0; j < UNROLL; ++j) in_dst[base + j * THREADS] = vi[j];
        if (rec) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (threadIdx.x == 0) rec[b] = Rec{t0, (unsigned long long)wall_clock64(), xcc};
        }
    }
}

int main()
{
    const size_t max_bytes = 256ull << 20;
    uint4 *hbm, *host_a, *host_b;
    unsigned *ticket;
    Rec *rec;
    CHECK(hipMalloc(&hbm, max_bytes));
    CHECK(hipHostMalloc(&host_a, max_bytes, 0));
    CHECK(hipHostMalloc(&host_b, max_bytes, 0));
    CHECK(hipMalloc(&ticket, 256));
    CHECK(hipMalloc(&rec, (max_bytes / BLOCK_BYTES) * sizeof(Rec)));
    CHECK(hipMemset(hbm, 1, max_bytes));
    memset(host_a, 2, max_bytes);
    memset(host_b, 3, max_bytes);
    hipStream_t s;
    CHECK(hipStreamCreate(&s));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));

    // ---- part 1: who gets served
    for (unsigned mask : {0xFFu, 0x01u}) {
        const size_t bytes = 64ull << 20;
        const unsigned n_blocks = (unsigned)(bytes / BLOCK_BYTES);
        const unsigned grid = mask == 0xFFu ? 64 : 96;        // 64 workgroups over 8 XCDs, or 12 on XCD 0
        for (int r = 0; r < 3; ++r) {
            CHECK(hipMemsetAsync(ticket, 0, 4, s));
            hipLaunchKernelGGL(exchange, dim3(grid), dim3(THREADS), 0, s, hbm, host_a, host_b, hbm, n_blocks, ticket, mask,
                               rec);
        }
        CHECK(hipStreamSynchronize(s));
        std::vector<Rec> h(n_blocks);
        CHECK(hipMemcpy(h.data(), rec, n_blocks * sizeof(Rec), hipMemcpyDeviceToHost));
        unsigned long long first = ~0ull, last = 0;
        double sum[16] = {0}, worst[16] = {0};
        unsigned cnt[16] = {0};
        for (const Rec &x : h) {
            first = std::min(first, x.t0);
            last = std::max(last, x.t1);
            const double us = (x.t1 - x.t0) / 100.0;
            sum[x.xcc] += us;
            worst[x.xcc] = std::max(worst[x.xcc], us);
            cnt[x.xcc]++;
        }
        printf("exchange of 64 MiB per direction, %s: %.0f us = %.1f GB/s per direction\n",
               mask == 0xFFu ? "64 workgroups dealt over all XCDs" : "12 workgroups on XCD 0", (last - first) / 100.0,
               bytes / ((last - first) * 10.0));
        for (int x = 0; x < 16; ++x)
            if (cnt[x])
                printf("  XCD %d: %5u blocks of 16 KiB, %6.1f us per block on average, %6.1f us the slowest\n", x, cnt[x],
                       sum[x] / cnt[x], worst[x]);
    }

    // ---- part 2: launch time by size, for placements of the working workgroups
    struct Variant { const char *name; unsigned mask, grid; };
    const Variant variants[] = {
        {"64 workgroups, all XCDs", 0xFF, 64},   {"16 workgroups, all XCDs", 0xFF, 16},  {"16 workgroups, XCDs 6 and 7", 0xC0, 64},
        {"16 workgroups, XCDs 0 and 1", 0x03, 64}, {"8 workgroups, XCD 7", 0x80, 64},    {"12 workgroups, XCD 7", 0x80, 96},
        {"12 workgroups, XCD 0", 0x01, 96},      {"16 workgroups, XCD 0", 0x01, 128},    {"32 workgroups, XCD 0", 0x01, 256},
    };
    const size_t sizes_mb[] = {1, 4, 16, 64, 256};
    printf("\nexchange launches by size: us per launch (GB/s per direction), best of 8\n");
    for (const Variant &v : variants) {
        printf("%-30s", v.name);
        for (size_t mb : sizes_mb) {
            const size_t bytes = mb << 20;
            float best = 1e9f;
            for (int r = 0; r < 8; ++r) {
                CHECK(hipMemsetAsync(ticket, 0, 4, s));
                CHECK(hipEventRecord(e0, s));
                hipLaunchKernelGGL(exchange, dim3(v.grid), dim3(THREADS), 0, s, hbm, host_a, host_b, hbm,
                                   (unsigned)(bytes / BLOCK_BYTES), ticket, v.mask, (Rec *)nullptr);
                CHECK(hipEventRecord(e1, s));
                CHECK(hipEventSynchronize(e1));
                float ms;
                CHECK(hipEventElapsedTime(&ms, e0, e1));
                best = std::min(best, ms);
            }
            printf("  %3zu MiB %7.0f (%4.1f)", mb, best * 1e3, bytes / (best * 1e6));
        }
        printf("\n");
    }
    return 0;
}
