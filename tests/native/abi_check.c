/* Uses the library from plain C through include/vccl.h only: the header must be valid
 * C11, the host-only entry points must work without a device, and calls that need a
 * context must fail with VCCL_ERR_NOT_INIT.  Exit status 0 = all checks passed. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "vccl.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "line %d: check failed: %s (last error: %s)\n", __LINE__, #cond, \
                    vccl_last_error());                                    \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main(void)
{
    /* nothing works before vccl_init, and says so */
    void *one[1] = {(void *)0x1000};
    CHECK(vccl_alltoall(one, one, 16, 1, VCCL_MODE_CU, NULL) == VCCL_ERR_NOT_INIT);
    CHECK(strlen(vccl_last_error()) > 0);
    CHECK(vccl_finalize() == VCCL_ERR_NOT_INIT);
    CHECK(vccl_set_option("cu_unroll", "2") == VCCL_ERR_NOT_INIT);

    /* planner, host only: 2 ranks, equal blocks of 4 KiB, fake 1 KiB-aligned addresses */
    enum { P = 2 };
    const uint64_t c = 4096;
    void *send[P] = {(void *)0x10000000, (void *)0x20000000};
    void *recv[P] = {(void *)0x30000000, (void *)0x40000000};
    uint64_t cnt[P * P], sdis[P * P], rdis[P * P];
    for (int a = 0; a < P; ++a)
        for (int b = 0; b < P; ++b) {
            cnt[a * P + b] = c;
            sdis[a * P + b] = (uint64_t)b * c;
            rdis[a * P + b] = (uint64_t)b * c;
        }
    vccl_plan_desc d[8];
    int n = -1, aligned = -1;
    uint32_t gx = 0, gy = 0, tile = 0;
    CHECK(vccl_plan_alltoallv(send, cnt, sdis, recv, cnt, rdis, P, 1, 64, d, 8, &n, &gx, &gy, &tile, &aligned) ==
          VCCL_OK);
    CHECK(n == 4 && gy == 4 && aligned == 1 && tile == 1024 && gx == 4);
    /* rotated order: 0->0, 1->1, then 1->0, 0->1 */
    CHECK(d[0].src == 0x10000000u && d[0].dst == 0x30000000u);
    CHECK(d[1].src == 0x20000000u + c && d[1].dst == 0x40000000u + c);
    CHECK(d[2].src == 0x20000000u && d[2].dst == 0x30000000u + c);
    CHECK(d[3].src == 0x10000000u + c && d[3].dst == 0x40000000u);
    for (int i = 0; i < 4; ++i) CHECK(d[i].bytes == c && d[i].head == 0 && d[i].lead == 0);
    /* a count mismatch is an error of its own */
    cnt[1] = c + 1;
    CHECK(vccl_plan_alltoallv(send, cnt, sdis, recv, cnt, rdis, P, 1, 64, d, 8, &n, &gx, &gy, &tile, &aligned) ==
          VCCL_ERR_COUNT_MISMATCH);

    /* window monitor, host only: 3 messages of 1 MB, one per microsecond */
    vccl_monitor *m = vccl_monitor_create(8, 10000000ull);
    CHECK(m != NULL);
    vccl_monitor_sample s;
    for (uint64_t i = 0; i < 3; ++i) {
        CHECK(vccl_monitor_post(m, i, 1000000, i * 1000) == VCCL_OK);
        CHECK(vccl_monitor_complete(m, i, i * 1000 + 1000, &s) == VCCL_OK);
    }
    uint64_t msgs = 0, anomalies = 99;
    CHECK(vccl_monitor_totals(m, &msgs, &anomalies, &s) == VCCL_OK);
    CHECK(msgs == 3 && anomalies == 0);
    /* each message: 1 MB in 1 us = 1e12 bytes per second; the window of 3 the same */
    CHECK(s.bw_message > 0.99e12 && s.bw_message < 1.01e12);
    vccl_monitor_destroy(m);
    printf("abi ok\n");
    return 0;
}
