/*
 * The C ABI used from plain C99, without Python or PyTorch: the CPU-GPU
 * offloading example of Sec. 3.4.1 of the 10Cache paper (six equal tensors,
 * three GPU buffers, three CPU buffers, forward 1..6 then backward 6..1).
 *
 * The program checks the tier contents the paper's text states after the
 * events it names (GPU {2,3,4} after tensor 1, GPU {4,5,6} after tensor 3, no
 * movement after 4, 5 and 6), that every access is a hit, and that every
 * tensor's bytes survive the twelve migrations.  Exit code 0 = all checks
 * passed; each failed check prints a line.
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "tc.h"

#define N 6
#define BYTES 512

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { printf("FAIL: " __VA_ARGS__); printf("\n"); failures++; } } while (0)
#define TC(call) do { int rc_ = (call); if (rc_ != TC_OK) { printf("FAIL: %s -> %d (%s: %s)\n", #call, rc_, tc_strerror(rc_), tc_last_error(ctx)); return 1; } } while (0)
#define HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { printf("FAIL: %s -> %s\n", #call, hipGetErrorString(e_)); return 1; } } while (0)

static unsigned gpu_set(tc_ctx *ctx)
{
    uint8_t tier[N];
    unsigned m = 0;
    if (tc_dump_state(ctx, tier, NULL, NULL) != TC_OK) return 0xFFFFFFFFu;
    for (int t = 0; t < N; ++t) if (tier[t] == TC_GPU) m |= 1u << t;
    return m;
}

int main(void)
{
    tc_ctx *ctx = NULL;
    TC(tc_create(&ctx));

    tc_tensor_desc desc[N];
    memset(desc, 0, sizeof desc);
    for (int t = 0; t < N; ++t) desc[t].bytes = BYTES;
    tc_event ev[2 * N];
    memset(ev, 0, sizeof ev);
    for (int k = 0; k < 2 * N; ++k) {
        ev[k].step = (uint32_t)k;
        ev[k].tensor = (uint32_t)(k < N ? k : 2 * N - 1 - k);
        ev[k].rw = TC_R;
    }
    TC(tc_profile_order(ctx, desc, N, ev, 2 * N));

    tc_budget b;
    memset(&b, 0, sizeof b);
    b.hbm_bytes = 3 * BYTES;
    b.host_bytes[0] = 3 * BYTES;
    b.flags = TC_LITERAL_ALG2;
    tc_pool_plan plan;
    tc_pool_class cls[4];
    TC(tc_plan_pools(ctx, &b, &plan, cls, 4));
    CHECK(plan.n_classes == 1 && cls[0].gpu_count == 3 && cls[0].cpu_count == 3, "pool plan: %u classes, G=%u C=%u",
          plan.n_classes, cls[0].gpu_count, cls[0].cpu_count);
    tc_placement place[N];
    TC(tc_plan_schedule(ctx, place));
    for (int t = 0; t < N; ++t)
        CHECK(place[t].final_tier == (t < 3 ? TC_GPU : TC_CPU) && place[t].slot == (uint32_t)(t % 3),
              "placement of tensor %d: tier %u buffer %u", t + 1, place[t].final_tier, place[t].slot);

    void *hbm = NULL, *pinned = NULL;
    hipStream_t migrate, compute;
    HIP(hipMalloc(&hbm, plan.hbm_total));
    HIP(hipHostMalloc(&pinned, plan.host_total, 0));
    HIP(hipStreamCreateWithFlags(&migrate, hipStreamNonBlocking));
    HIP(hipStreamCreateWithFlags(&compute, hipStreamNonBlocking));
    TC(tc_bind_memory(ctx, hbm, plan.hbm_total, pinned, plan.host_total, NULL, 0, -1, migrate, 0));

    static uint8_t payload[N][BYTES], back[BYTES];
    for (int t = 0; t < N; ++t) {
        for (int i = 0; i < BYTES; ++i) payload[t][i] = (uint8_t)(31 * t + 7 * i + (i >> 5));
        TC(tc_load_tensor(ctx, (uint32_t)t, payload[t]));
    }

    /* GPU contents are compared as masks: bit t set = tensor t+1 is in a GPU buffer */
    for (int k = 0; k < 2 * N; ++k) {
        uint32_t id = ev[k].tensor;
        uint8_t rw = TC_R;
        void *ptr = NULL;
        TC(tc_migrate_step(ctx, (uint32_t)k, TC_PRE, &id, &rw, 1, compute, &ptr));
        CHECK(ptr != NULL, "step %d: tensor %u has no GPU buffer", k, id + 1);
        /* the "module": read the tensor through the pointer the hook returned */
        HIP(hipMemcpyAsync(back, ptr, BYTES, hipMemcpyDeviceToHost, compute));
        HIP(hipStreamSynchronize(compute));
        CHECK(memcmp(back, payload[id], BYTES) == 0, "step %d: tensor %u read through its buffer differs", k, id + 1);
        TC(tc_migrate_step(ctx, (uint32_t)k, TC_POST, &id, &rw, 1, compute, NULL));
        if (k < N) {            /* the forward states the text prints */
            const unsigned want = k == 0 ? 0x0E : k == 1 ? 0x1C : 0x38;
            CHECK(gpu_set(ctx) == want, "after forward of tensor %d the GPU holds mask 0x%02X, text says 0x%02X", k + 1,
                  gpu_set(ctx), want);
        }
    }
    CHECK(gpu_set(ctx) == 0x07, "after the backward pass the GPU holds mask 0x%02X, not tensors 1-3", gpu_set(ctx));
    TC(tc_end_iteration(ctx, compute));
    TC(tc_synchronize(ctx));

    tc_stats st;
    TC(tc_cache_stats(ctx, &st));
    CHECK(st.hits == 12 && st.misses == 0 && st.fails == 0, "hits %llu misses %llu", (unsigned long long)st.hits,
          (unsigned long long)st.misses);
    CHECK(st.n_ops[TC_OP_PREFETCH] == 6 && st.n_ops[TC_OP_EVICT] == 6, "prefetches %llu evictions %llu",
          (unsigned long long)st.n_ops[TC_OP_PREFETCH], (unsigned long long)st.n_ops[TC_OP_EVICT]);
    CHECK(st.bytes_h2d == 6 * BYTES && st.bytes_d2h == 6 * BYTES, "bytes h2d %llu d2h %llu",
          (unsigned long long)st.bytes_h2d, (unsigned long long)st.bytes_d2h);
    for (int t = 0; t < N; ++t) {
        TC(tc_read_tensor(ctx, (uint32_t)t, back));
        CHECK(memcmp(back, payload[t], BYTES) == 0, "tensor %d bytes differ after the iteration", t + 1);
    }
    uint64_t n_log = 0;
    TC(tc_dump_oplog(ctx, 0, NULL, 0, &n_log));
    CHECK(n_log == 12, "op log has %llu records", (unsigned long long)n_log);

    TC(tc_destroy(ctx));
    HIP(hipStreamDestroy(migrate));
    HIP(hipStreamDestroy(compute));
    HIP(hipFree(hbm));
    HIP(hipHostFree(pinned));
    printf(failures ? "tc_example: %d check(s) failed\n" : "tc_example: ok\n", failures);
    return failures ? 1 : 0;
}
