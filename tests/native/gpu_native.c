/* The library without Python or PyTorch: a plain C program (HIP runtime for device
 * memory only) runs AlltoAll on both data paths, AlltoAllv with byte-granular
 * segments, a SendRecv ring, an AlltoAll over receive buffers at a constant stride
 * (pitched engine copies), and the MoE pack -> exchange -> inverse exchange -> un-permute
 * round trip, and compares every result with the CPU oracle (linked in as a shared
 * library); the co-run probe reports its clocks.  argv[1], if given, selects the
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
int oracle_moe_pack(const uint8_t *x, const int32_t *ids, int64_t T, int K, uint64_t row_bytes, int E,
                    uint8_t *packed, int64_t *order, uint64_t *cnt);
int oracle_moe_exchange_layout(const uint64_t *cnt, int P, int E, int experts_per_rank, uint64_t row_bytes,
                               uint64_t *sendcounts, uint64_t *sdispls, uint64_t *recvcounts, uint64_t *rdispls);

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
    setvbuf(stdout, NULL, _IOLBF, 0);   /* progress lines reach a pipe as they are printed */
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
    /* AlltoAll on the copy engines into receive buffers that are slices of one allocation:
     * one pitched copy per rank (forced, whatever the library would choose for this shape) */
    if (!rc) {
        const uint64_t cb = 4096 + 32, stride = (uint64_t)P * cb + 256;
        uint8_t *slab, *dslab[P];
        uint64_t ssz[P];
        HIPCHECK(hipMalloc((void **)&slab, stride * P));
        HIPCHECK(hipMemset(slab, SENTINEL, stride * P));
        for (int r = 0; r < P; ++r) {
            dslab[r] = slab + (uint64_t)r * stride;
            ssz[r] = stride;                      /* the gap behind each rank buffer is compared too */
            memset(hw[r], SENTINEL, cap);
        }
        HIPCHECK(hipDeviceSynchronize());
        char before[32] = "", after[32] = "";
        VCHECK(vccl_get_option("ce_pitched_copies", before, sizeof(before)));
        VCHECK(vccl_set_option("ce_pitched", "2"));
        VCHECK(vccl_alltoall((void *const *)ds, (void *const *)dslab, cb, P, VCCL_MODE_CE, stream));
        HIPCHECK(hipStreamSynchronize(stream));
        VCHECK(vccl_set_option("ce_pitched", "1"));
        VCHECK(vccl_get_option("ce_pitched_copies", after, sizeof(after)));
        if (oracle_alltoall((const uint8_t *const *)hs, hw, cb, P, 1)) return 4;
        rc = compare("alltoall, pitched engine copies", dslab, hw, ssz);
        if (!rc && atoll(after) - atoll(before) != P) {
            fprintf(stderr, "expected %d pitched copies, counted %lld\n", P, atoll(after) - atoll(before));
            rc = 1;
        }
        HIPCHECK(hipFree(slab));
    }
    /* MoE dispatch and combine: pack -> AlltoAllv -> AlltoAllv back -> un-permute gives every
     * token's row back once per slot; the packed rows, the counts and what each rank receives
     * are the oracle's */
    if (!rc) {
        enum { T = 700, K = 4, E = 20, EPR = E / P };
        const uint64_t row = 1040;
        const uint64_t xb = (uint64_t)T * row, pb = xb * K;
        uint8_t *hx[P], *hp[P], *dx[P], *dp[P], *dout[P], *drecv[P], *hrecv[P];
        int32_t *hid[P], *did[P];
        uint64_t cnt[P * E], *dcnt, lsc[P * P], lsd[P * P], lrc[P * P], lrd[P * P], psz[P], rsz[P], xsz[P];
        uint64_t osc[P * P], osd[P * P], orc[P * P], ord_[P * P];
        int64_t *order = (int64_t *)malloc(sizeof(int64_t) * T * K);   /* the oracle's pair order, not used here */
        HIPCHECK(hipMalloc((void **)&dcnt, sizeof(cnt)));
        for (int s = 0; s < P; ++s) {
            hx[s] = (uint8_t *)malloc(xb);
            hp[s] = (uint8_t *)malloc(pb);
            hid[s] = (int32_t *)malloc(sizeof(int32_t) * T * K);
            for (uint64_t i = 0; i < xb; ++i) hx[s][i] = (uint8_t)mix(((uint64_t)(s + 17) << 40) ^ i);
            for (int t = 0; t < T; ++t)
                for (int k = 0; k < K; ++k)   /* K distinct experts per token */
                    hid[s][t * K + k] = (int32_t)((mix((uint64_t)s * 1000003u + (uint64_t)t) % E + (uint64_t)k * 5u) % E);
            HIPCHECK(hipMalloc((void **)&dx[s], xb));
            HIPCHECK(hipMalloc((void **)&dp[s], pb));
            HIPCHECK(hipMalloc((void **)&dout[s], pb));
            HIPCHECK(hipMalloc((void **)&did[s], sizeof(int32_t) * T * K));
            HIPCHECK(hipMemcpy(dx[s], hx[s], xb, hipMemcpyHostToDevice));
            HIPCHECK(hipMemcpy(did[s], hid[s], sizeof(int32_t) * T * K, hipMemcpyHostToDevice));
            HIPCHECK(hipMemset(dp[s], SENTINEL, pb));
            if (oracle_moe_pack(hx[s], hid[s], T, K, row, E, hp[s], order, cnt + s * E)) return 4;
            psz[s] = pb;
            xsz[s] = xb;
        }
        VCHECK(vccl_moe_pack((const void *const *)dx, (const int32_t *const *)did, P, T, K, row, E,
                             (void *const *)dp, dcnt, NULL, NULL, stream));
        HIPCHECK(hipStreamSynchronize(stream));
        rc = compare("moe pack", dp, hp, psz);
        uint64_t gcnt[P * E];
        HIPCHECK(hipMemcpy(gcnt, dcnt, sizeof(gcnt), hipMemcpyDeviceToHost));
        if (!rc && memcmp(gcnt, cnt, sizeof(cnt))) {
            fprintf(stderr, "moe pack: counts differ from the oracle's\n");
            rc = 1;
        }
        VCHECK(vccl_moe_exchange_layout(cnt, P, E, EPR, row, lsc, lsd, lrc, lrd));
        if (oracle_moe_exchange_layout(cnt, P, E, EPR, row, osc, osd, orc, ord_)) return 4;
        if (!rc && (memcmp(lsc, osc, sizeof(osc)) || memcmp(lsd, osd, sizeof(osd)) || memcmp(lrc, orc, sizeof(orc)) ||
                    memcmp(lrd, ord_, sizeof(ord_)))) {
            fprintf(stderr, "moe exchange layout differs from the oracle's\n");
            rc = 1;
        }
        for (int r = 0; r < P; ++r) {
            rsz[r] = 16;
            for (int s = 0; s < P; ++s) rsz[r] += lrc[r * P + s];
            HIPCHECK(hipMalloc((void **)&drecv[r], rsz[r]));
            HIPCHECK(hipMemset(drecv[r], SENTINEL, rsz[r]));
            hrecv[r] = (uint8_t *)malloc(rsz[r]);
            memset(hrecv[r], SENTINEL, rsz[r]);
        }
        for (int mode = VCCL_MODE_CU; mode <= VCCL_MODE_CE && !rc; ++mode) {
            for (int r = 0; r < P; ++r) HIPCHECK(hipMemset(drecv[r], SENTINEL, rsz[r]));
            HIPCHECK(hipDeviceSynchronize());
            VCHECK(vccl_alltoallv((void *const *)dp, lsc, lsd, (void *const *)drecv, lrc, lrd, P, (vccl_mode)mode, stream));
            HIPCHECK(hipStreamSynchronize(stream));
            if (oracle_alltoallv((const uint8_t *const *)hp, lsc, lsd, hrecv, lrc, lrd, P, 1)) return 4;
            rc = compare(mode == VCCL_MODE_CU ? "moe exchange, compute units" : "moe exchange, copy engines", drecv,
                         hrecv, rsz);
        }
        if (!rc) {   /* the way back: the receive description as the send description, then the un-permute */
            for (int s = 0; s < P; ++s) HIPCHECK(hipMemset(dp[s], SENTINEL, pb));
            VCHECK(vccl_alltoallv((void *const *)drecv, lrc, lrd, (void *const *)dp, lsc, lsd, P, VCCL_MODE_CE, stream));
            VCHECK(vccl_moe_unpack((const void *const *)dp, (const int32_t *const *)did, P, T, K, row, E,
                                   (void *const *)dout, stream));
            HIPCHECK(hipStreamSynchronize(stream));
            for (int s = 0; s < P; ++s)      /* row t*K+k of out[s] is row t of x[s] */
                for (int t = 0; t < T; ++t)
                    for (int k = 0; k < K; ++k) memcpy(hp[s] + ((uint64_t)t * K + k) * row, hx[s] + (uint64_t)t * row, row);
            rc = compare("moe combine (inverse exchange + un-permute)", dout, hp, psz);
        }
        (void)xsz;
        for (int s = 0; s < P; ++s) {
            HIPCHECK(hipFree(dx[s])); HIPCHECK(hipFree(dp[s])); HIPCHECK(hipFree(dout[s])); HIPCHECK(hipFree(did[s]));
            HIPCHECK(hipFree(drecv[s]));
            free(hx[s]); free(hp[s]); free(hid[s]); free(hrecv[s]);
        }
        HIPCHECK(hipFree(dcnt));
        free(order);
    }
    /* the co-run probe with its clocks: shader ticks and real-time ticks per workgroup */
    if (!rc) {
        const int wgs = vccl_device_cu_count(), khz = vccl_device_wall_clock_khz();
        float *dprobe;
        uint64_t *dclk, *hclk = (uint64_t *)malloc(sizeof(uint64_t) * 2 * (size_t)wgs);
        HIPCHECK(hipMalloc((void **)&dprobe, sizeof(float) * 256 * (size_t)wgs));
        HIPCHECK(hipMalloc((void **)&dclk, sizeof(uint64_t) * 2 * (size_t)wgs));
        VCHECK(vccl_fma_probe_clocks(dprobe, dclk, (uint32_t)wgs, 256, 20000, stream));
        HIPCHECK(hipStreamSynchronize(stream));
        HIPCHECK(hipMemcpy(hclk, dclk, sizeof(uint64_t) * 2 * (size_t)wgs, hipMemcpyDeviceToHost));
        if (wgs < 1 || khz < 1000 || !hclk[0] || !hclk[1]) {
            fprintf(stderr, "probe clocks: %d workgroups, %d kHz, ticks %llu / %llu\n", wgs, khz,
                    (unsigned long long)hclk[0], (unsigned long long)hclk[1]);
            rc = 1;
        } else {
            printf("probe: workgroup 0 ran %.3f ms at %.0f MHz shader clock\n", (double)hclk[1] / khz,
                   (double)hclk[0] / (double)hclk[1] * khz * 1e-3);
        }
        free(hclk);
        HIPCHECK(hipFree(dprobe));
        HIPCHECK(hipFree(dclk));
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
