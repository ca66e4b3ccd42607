/* The library without Python or PyTorch: a plain C program (HIP runtime for device
 * memory only) runs AlltoAll on both data paths, AlltoAllv with byte-granular
 * segments, and a SendRecv ring, and compares every receive buffer with the CPU
 * oracle (linked in as a shared library).  argv[1], if given, selects the
 * copy-engine ordering ("memops", "event" or "host").  Exit status 0 = all results right. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "vccl.h"

int oracle_alltoallv(const uint8_t *const *send, const uint64_t *sendcounts, const uint64_t *sdispls,
                     uint8_t *const *recv, const uint64_t *recvcounts, const uint64_t *rdispls, int P,
                     int threads);
int oracle_alltoall(const uint8_t *const *send, uint8_t *const *recv, uint64_t c, int P, int threads);
int oracle_sendrecv(const uint8_t *const *send, const uint64_t *sendbytes, const int *send_to,
                    uint8_t *const *recv, const uint64_t *recvbytes, const int *recv_from, int P);

#define HIPCHECK(x)                                                                        \
    do {                                                                                   \
        hipError_t e_ = (x);                                                               \
        if (e_ != hipSuccess) {                                                            \
            fprintf(stderr, "line %d: %s: %s\n", __LINE__, #x, hipGetErrorString(e_));     \
            return 2;                                                                      \
        }                                                                                  \
    } while (0)
#define VCHECK(x)                                                                          \
    do {                                                                                   \
        int r_ = (x);                                                                      \
        if (r_ != VCCL_OK) {                                                               \
            fprintf(stderr, "line %d: %s = %d: %s\n", __LINE__, #x, r_, vccl_last_error()); \
            return 3;                                                                      \
        }                                                                                  \
    } while (0)

enum { P = 5 };
#define SENTINEL 0xA5

static uint64_t mix(uint64_t x)   /* any fixed byte pattern will do for this check */
{
    x ^= x >> 33; x *= 0xff51afd7ed558ccdull; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ull; x ^= x >> 33;
    return x;
}

static int compare(const char *what, uint8_t *const *dev, uint8_t *const *want, const uint64_t *sizes)
{
    for (int r = 0; r < P; ++r) {
        uint8_t *got = (uint8_t *)malloc(sizes[r] ? sizes[r] : 1);
        if (hipMemcpy(got, dev[r], sizes[r], hipMemcpyDeviceToHost) != hipSuccess) return 2;
        for (uint64_t i = 0; i < sizes[r]; ++i)
            if (got[i] != want[r][i]) {
                fprintf(stderr, "%s: recv[%d] differs at byte %llu: got %02x, want %02x\n", what, r,
                        (unsigned long long)i, got[i], want[r][i]);
                free(got);
                return 1;
            }
        free(got);
    }
    printf("%s: ok\n", what);
    return 0;
}

int main(int argc, char **argv)
{
    const uint64_t c = 300000 - 300000 % 16, cap = (uint64_t)P * c + 64;
    HIPCHECK(hipSetDevice(0));
    VCHECK(vccl_init(0, 16));
    if (argc > 1) VCHECK(vccl_set_option("ce_sync", argv[1]));
    hipStream_t stream;
    HIPCHECK(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));

    uint8_t *hs[P], *hw[P], *ds[P], *dr[P];
    uint64_t sizes[P];
    for (int s = 0; s < P; ++s) {
        hs[s] = (uint8_t *)malloc(cap);
        hw[s] = (uint8_t *)malloc(cap);
        for (uint64_t i = 0; i < cap; ++i) hs[s][i] = (uint8_t)mix(((uint64_t)s << 40) ^ i);
        HIPCHECK(hipMalloc((void **)&ds[s], cap));
        HIPCHECK(hipMalloc((void **)&dr[s], cap));
        HIPCHECK(hipMemcpy(ds[s], hs[s], cap, hipMemcpyHostToDevice));
        sizes[s] = cap;
    }
    int rc = 0;
    /* AlltoAll, equal blocks, both paths */
    for (int mode = VCCL_MODE_CU; mode <= VCCL_MODE_CE && !rc; ++mode) {
        for (int r = 0; r < P; ++r) {
            HIPCHECK(hipMemset(dr[r], SENTINEL, cap));
            memset(hw[r], SENTINEL, cap);
        }
        HIPCHECK(hipDeviceSynchronize());
        VCHECK(vccl_alltoall((void *const *)ds, (void *const *)dr, c, P, (vccl_mode)mode, stream));
        HIPCHECK(hipStreamSynchronize(stream));
        if (oracle_alltoall((const uint8_t *const *)hs, hw, c, P, 1)) return 4;
        rc = compare(mode == VCCL_MODE_CU ? "alltoall, compute units" : "alltoall, copy engines", dr, hw, sizes);
    }
    /* AlltoAllv, byte-granular counts and displacements, both paths */
    uint64_t sc[P * P], sd[P * P], rcn[P * P], rd[P * P];
    for (int s = 0; s < P; ++s) {
        uint64_t off = 3;
        for (int r = 0; r < P; ++r) {
            sc[s * P + r] = (s + r) % 4 == 0 ? 0 : 1000 + 7777 * (uint64_t)((s * 3 + r) % 11);
            sd[s * P + r] = off;
            off += sc[s * P + r] + 5;
        }
    }
    for (int r = 0; r < P; ++r) {
        uint64_t off = 1;
        for (int s = 0; s < P; ++s) {
            rcn[r * P + s] = sc[s * P + r];
            rd[r * P + s] = off;
            off += rcn[r * P + s] + 9;
        }
    }
    for (int mode = VCCL_MODE_CU; mode <= VCCL_MODE_CE && !rc; ++mode) {
        for (int r = 0; r < P; ++r) {
            HIPCHECK(hipMemset(dr[r], SENTINEL, cap));
            memset(hw[r], SENTINEL, cap);
        }
        HIPCHECK(hipDeviceSynchronize());
        VCHECK(vccl_alltoallv((void *const *)ds, sc, sd, (void *const *)dr, rcn, rd, P, (vccl_mode)mode, stream));
        HIPCHECK(hipStreamSynchronize(stream));
        if (oracle_alltoallv((const uint8_t *const *)hs, sc, sd, hw, rcn, rd, P, 1)) return 4;
        rc = compare(mode == VCCL_MODE_CU ? "alltoallv, compute units" : "alltoallv, copy engines", dr, hw, sizes);
    }
    /* SendRecv ring, every mode */
    int to[P], from[P];
    uint64_t nb[P];
    for (int s = 0; s < P; ++s) {
        to[s] = (s + 1) % P;
        from[s] = (s + P - 1) % P;
        nb[s] = 1000003;
    }
    for (int mode = VCCL_MODE_CU; mode <= VCCL_MODE_CU_STAGED && !rc; ++mode) {
        for (int r = 0; r < P; ++r) {
            HIPCHECK(hipMemset(dr[r], SENTINEL, cap));
            memset(hw[r], SENTINEL, cap);
        }
        HIPCHECK(hipDeviceSynchronize());
        VCHECK(vccl_sendrecv((void *const *)ds, nb, to, (void *const *)dr, nb, from, P, (vccl_mode)mode, stream));
        if (mode == VCCL_MODE_CU_STAGED) VCHECK(vccl_sendrecv_staged_status());
        HIPCHECK(hipStreamSynchronize(stream));
        if (oracle_sendrecv((const uint8_t *const *)hs, nb, to, hw, nb, from, P)) return 4;
        rc = compare(mode == VCCL_MODE_CU ? "ring, compute units"
                                          : mode == VCCL_MODE_CE ? "ring, copy engines" : "ring, staged", dr, hw, sizes);
    }
    char kind[32] = "", sync[32] = "";
    vccl_get_option("ce_kind", kind, sizeof(kind));
    vccl_get_option("ce_sync", sync, sizeof(sync));
    printf("copy-engine back end: %s, ordering: %s\n", kind, sync);
    HIPCHECK(hipStreamDestroy(stream));
    VCHECK(vccl_finalize());
    for (int s = 0; s < P; ++s) {
        HIPCHECK(hipFree(ds[s]));
        HIPCHECK(hipFree(dr[s]));
        free(hs[s]);
        free(hw[s]);
    }
    if (!rc) printf("native ok\n");
    return rc;
}
