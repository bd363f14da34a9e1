// Host-side exercise of the C ABI for the sanitizer run of tests/test_sanitizers.py (no GPU).
//
// Linked against a build of api.hip / bookkeeping.hip / aggregate.hip whose HOST code carries
// AddressSanitizer and UndefinedBehaviorSanitizer.  Part 1: calls that the argument checks refuse.
// Part 2, only on a machine WITHOUT a GPU: calls with plausible sizes and made-up (never
// dereferenced on the host) device addresses, which run all the host-side carving and job-building
// code up to the first kernel launch, where the runtime reports that there is no device.  With a
// GPU present part 2 is skipped: made-up addresses must never reach a kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "fastgl_agg.h"

#define MUST(cond) do { if (!(cond)) { fprintf(stderr, "check failed at line %d: %s (%s)\n", __LINE__, #cond, fastgl_last_error()); exit(2); } } while (0)

int main()
{
    void *fake = (void *)(uintptr_t)0x7f0000001000ull;       // 256-byte aligned, never touched
    const int32_t *ip = (const int32_t *)fake, *ix = (const int32_t *)fake;
    // ---- part 1: refusals
    MUST(fastgl_block_aggregate_fwd(ip, ix, nullptr, -1, 4, 4, 8, FASTGL_AGG_SUM, FASTGL_F32, fake, fake, nullptr, fake, 1 << 20, nullptr) == FASTGL_ERR_INVALID_ARG);
    MUST(fastgl_block_aggregate_bwd(ip, ix, nullptr, 4, 4, 4, 0, FASTGL_AGG_SUM, FASTGL_F32, fake, fake, nullptr, fake, 1 << 20, nullptr) == FASTGL_ERR_INVALID_ARG);
    MUST(fastgl_block_aggregate_fwd(ip, ix, nullptr, 4, 4, 4, 8, FASTGL_AGG_SUM, FASTGL_F32, fake, fake, nullptr, fake, 16, nullptr) == FASTGL_ERR_WORKSPACE);
    MUST(fastgl_block_aggregate_fwd(ip, ix, nullptr, 4, (int64_t)1 << 31, 4, 8, FASTGL_AGG_SUM, FASTGL_F32, fake, fake, nullptr, fake, 1 << 20, nullptr) == FASTGL_ERR_UNSUPPORTED);
    fastgl_plan *plan = nullptr;
    MUST(fastgl_block_plan_create(ip, ix, 4, 4, 4, 0, fake, 1 << 30, nullptr, &plan) == FASTGL_ERR_INVALID_ARG && !plan);
    MUST(fastgl_block_plan_create(ip, ix, 4, 4, 4, FASTGL_PLAN_ALL, fake, 8, nullptr, &plan) == FASTGL_ERR_WORKSPACE && !plan);
    MUST(fastgl_gather_rows(fake, 10, (const int64_t *)fake, 3, 0, FASTGL_F32, fake, nullptr) == FASTGL_ERR_INVALID_ARG);
    MUST(fastgl_block_plan_bytes(-1, 0, 0) == 0);
    for (int64_t e : {0ll, 1ll, 255ll, 256ll, 257ll, 100000ll, 2000000000ll})
        for (int64_t n : {0ll, 1ll, 1000ll, 2000000000ll}) {
            MUST(fastgl_block_plan_bytes(n, n, e) >= 256);
            MUST(fastgl_block_workspace_bytes(n, n, e, 100, FASTGL_F32) >= fastgl_block_plan_bytes(n, n, e));
        }
    // ---- part 2: host-side code up to the first launch
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0) {
        printf("abi host driver: refusals clean; a GPU is present, launch-reaching calls skipped\n");
        return 0;
    }
    (void)hipGetLastError();
    fastgl_block_desc blocks[FASTGL_MAX_PLAN_BATCH];
    fastgl_plan *plans[FASTGL_MAX_PLAN_BATCH];
    for (int i = 0; i < FASTGL_MAX_PLAN_BATCH; ++i) {
        blocks[i].indptr = ip; blocks[i].indices = ix;
        blocks[i].num_dst = 1 + 977 * i; blocks[i].num_src = 3 + 40001 * i; blocks[i].num_edges = (int64_t)i * i * 99991;
        blocks[i].parts = (i % 3 == 0) ? FASTGL_PLAN_FWD : (i % 3 == 1) ? (FASTGL_PLAN_ALL | FASTGL_PLAN_PERM) : (FASTGL_PLAN_FWD | FASTGL_PLAN_SRC_DEG | FASTGL_PLAN_SHORT_DST_ROWS);
        blocks[i].plan_mem = fake;
        blocks[i].plan_bytes = fastgl_block_plan_bytes(blocks[i].num_dst, blocks[i].num_src, blocks[i].num_edges);
    }
    for (int n : {1, 2, 5, FASTGL_MAX_PLAN_BATCH}) {
        fastgl_status st = fastgl_block_plan_create_many(n, blocks, nullptr, plans);
        MUST(st == FASTGL_ERR_HIP);                                   // no device: the first launch fails
        for (int i = 0; i < n; ++i) MUST(plans[i] == nullptr);
    }
    for (int64_t feat : {1ll, 7ll, 100ll, 602ll, 4096ll})
        for (int dt = 0; dt < 2; ++dt)
            for (int mode = 0; mode < 3; ++mode) {
                const int64_t nd = 5000, ns = 9000, ne = 77777;
                const size_t ws = fastgl_block_workspace_bytes(nd, ns, ne, feat, (fastgl_dtype)dt);
                MUST(fastgl_block_aggregate_fwd(ip, ix, nullptr, nd, ns, ne, feat, (fastgl_agg_mode)mode, (fastgl_dtype)dt, fake, fake, nullptr, fake, ws, nullptr) == FASTGL_ERR_HIP);
                MUST(fastgl_block_aggregate_bwd(ip, ix, (const float *)fake, nd, ns, ne, feat, (fastgl_agg_mode)mode, (fastgl_dtype)dt, fake, fake, nullptr, fake, ws, nullptr) == FASTGL_ERR_HIP);
            }
    MUST(fastgl_gather_rows(fake, 1000, (const int64_t *)fake, 10, 128, FASTGL_BF16, fake, nullptr) == FASTGL_ERR_HIP);
    printf("abi host driver: clean\n");
    return 0;
}
