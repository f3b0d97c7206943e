/*
 * The two-tier mode of the C ABI from plain C99, without Python or PyTorch: the
 * optimizer-state example of Sec. 3.4.2 of the 10Cache paper (states of eight
 * tensors, five of them in the CPU cache, three on the file tier; once a
 * tensor's update is complete it is evicted and the next absent one is
 * prefetched while the CPU computes).
 *
 * The "update" adds 1 to every float of a tensor's state through the host
 * pointer the PRE call returned.  The program checks what the figure fixes
 * (the cache holds T2..T6 once T1's update is complete), that no access
 * misses, the op counts of two sweeps, and that every state ends at its
 * initial value plus two wherever it lives.  Exit code 0 = all checks passed.
 */
#define _POSIX_C_SOURCE 200809L
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <unistd.h>

#include "tc.h"

#define N 8
#define FLOATS 1024
#define BYTES (FLOATS * sizeof(float))
#define SWEEPS 2

static int failures = 0;
#define CHECK(cond, ...) do { if (!(cond)) { printf("FAIL: " __VA_ARGS__); printf("\n"); failures++; } } while (0)
#define TC(call) do { int rc_ = (call); if (rc_ != TC_OK) { printf("FAIL: %s -> %d (%s: %s)\n", #call, rc_, tc_strerror(rc_), tc_last_error(ctx)); return 1; } } while (0)
#define HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { printf("FAIL: %s -> %s\n", #call, hipGetErrorString(e_)); return 1; } } while (0)

static unsigned cached_set(tc_ctx *ctx)
{
    uint8_t tier[N];
    unsigned m = 0;
    if (tc_dump_state(ctx, tier, NULL, NULL) != TC_OK) return 0xFFFFFFFFu;
    for (int t = 0; t < N; ++t) if (tier[t] == TC_GPU) m |= 1u << t;      /* TC_GPU names the fast tier */
    return m;
}

int main(void)
{
    tc_ctx *ctx = NULL;
    TC(tc_create(&ctx));

    tc_tensor_desc desc[N];
    memset(desc, 0, sizeof desc);
    for (int t = 0; t < N; ++t) { desc[t].bytes = BYTES; desc[t].group = 1; }
    tc_event ev[N];
    memset(ev, 0, sizeof ev);
    for (int k = 0; k < N; ++k) { ev[k].step = (uint32_t)k; ev[k].tensor = (uint32_t)k; ev[k].rw = TC_R | TC_W; }
    TC(tc_profile_order(ctx, desc, N, ev, N));

    tc_budget b;
    memset(&b, 0, sizeof b);
    b.hbm_bytes = 5 * BYTES;                    /* the budget of the fast tier: here the CPU cache */
    tc_pool_plan plan;
    tc_pool_class cls[2];
    TC(tc_plan_pools(ctx, &b, &plan, cls, 2));
    CHECK(plan.n_classes == 1 && cls[0].gpu_count == 5 && cls[0].cpu_count == 0 && plan.host_total == 0,
          "pool plan: %u classes, fast %u, host %u", plan.n_classes, cls[0].gpu_count, cls[0].cpu_count);
    tc_placement place[N];
    TC(tc_plan_schedule(ctx, place));
    for (int t = 0; t < N; ++t)
        CHECK(place[t].final_tier == (t < 5 ? TC_GPU : TC_NVME), "placement of T%d: tier %u", t + 1, place[t].final_tier);

    char path[] = "/tmp/tc_opt_example_XXXXXX";
    int fd = mkstemp(path);
    CHECK(fd >= 0, "mkstemp failed");
    if (fd < 0) return 1;
    unlink(path);
    CHECK(ftruncate(fd, (off_t)plan.file_total) == 0, "ftruncate failed");

    void *cache = NULL;
    hipStream_t migrate;
    HIP(hipHostMalloc(&cache, plan.hbm_total, 0));
    HIP(hipStreamCreateWithFlags(&migrate, hipStreamNonBlocking));
    TC(tc_bind_memory(ctx, cache, plan.hbm_total, NULL, 0, NULL, 0, fd, migrate, TC_BIND_HOST_TIER));

    static float init[N][FLOATS], back[FLOATS];
    for (int t = 0; t < N; ++t) {
        for (int i = 0; i < FLOATS; ++i) init[t][i] = (float)(100 * t) + (float)i * 0.25f;
        TC(tc_load_tensor(ctx, (uint32_t)t, init[t]));
    }

    for (int sweep = 0; sweep < SWEEPS; ++sweep) {
        for (int k = 0; k < N; ++k) {
            uint32_t id = (uint32_t)k;
            uint8_t rw = TC_R | TC_W;
            void *ptr = NULL;
            TC(tc_migrate_step(ctx, (uint32_t)k, TC_PRE, &id, &rw, 1, NULL, &ptr));
            CHECK(ptr != NULL, "sweep %d: T%d has no buffer", sweep, k + 1);
            if (!ptr) return 1;
            float *state = (float *)ptr;                    /* host memory: the CPU updates it in place */
            CHECK(state[3] == init[k][3] + (float)sweep, "sweep %d: T%d arrived with %f", sweep, k + 1, (double)state[3]);
            for (int i = 0; i < FLOATS; ++i) state[i] += 1.0f;
            TC(tc_migrate_step(ctx, (uint32_t)k, TC_POST, &id, &rw, 1, NULL, NULL));
            if (sweep == 0 && k == 0)
                CHECK(cached_set(ctx) == 0x3E, "once T1's update is complete the cache holds mask 0x%02X, the figure says T2..T6",
                      cached_set(ctx));
        }
        TC(tc_end_iteration(ctx, NULL));
        CHECK(cached_set(ctx) == 0x1F, "after the restore the cache holds mask 0x%02X, not T1..T5", cached_set(ctx));
    }
    TC(tc_synchronize(ctx));

    tc_stats st;
    TC(tc_cache_stats(ctx, &st));
    CHECK(st.hits == SWEEPS * N && st.misses == 0 && st.fails == 0, "hits %llu misses %llu", (unsigned long long)st.hits,
          (unsigned long long)st.misses);
    /* per sweep: T1..T3 make room for T6..T8, the restore returns T1..T3 in place of three of T4..T8 */
    CHECK(st.n_ops[TC_OP_WRITEBACK] == SWEEPS * 6 && st.n_ops[TC_OP_PREFETCH] == SWEEPS * 6 && st.n_ops[TC_OP_EVICT] == 0,
          "write-backs %llu prefetches %llu", (unsigned long long)st.n_ops[TC_OP_WRITEBACK],
          (unsigned long long)st.n_ops[TC_OP_PREFETCH]);
    CHECK(st.bytes_file_write == SWEEPS * 6 * BYTES && st.bytes_file_read == SWEEPS * 6 * BYTES, "file bytes w %llu r %llu",
          (unsigned long long)st.bytes_file_write, (unsigned long long)st.bytes_file_read);
    for (int t = 0; t < N; ++t) {
        TC(tc_read_tensor(ctx, (uint32_t)t, back));
        int same = 1;
        for (int i = 0; i < FLOATS; ++i) same = same && back[i] == init[t][i] + (float)SWEEPS;
        CHECK(same, "state of T%d is not its initial value plus %d", t + 1, SWEEPS);
    }

    TC(tc_destroy(ctx));
    HIP(hipStreamDestroy(migrate));
    HIP(hipHostFree(cache));
    close(fd);
    printf(failures ? "tc_opt_example: %d check(s) failed\n" : "tc_opt_example: ok\n", failures);
    return failures ? 1 : 0;
}
