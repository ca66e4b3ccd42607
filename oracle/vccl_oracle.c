/*
 * CPU oracle for the P2P data movement behind SendRecv and AlltoAll(v).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * primitives compute, used to check the GPU library and as a reported host
 * baseline.  It shares no code with the GPU path and the GPU path never calls
 * it.  Everything is an element loop over bytes; nothing is blocked, fused or
 * reordered beyond an optional split of the outermost destination-rank loop
 * over threads (each destination rank owns its own receive buffer, so the
 * split changes no result).
 *
 * What is followed:
 *   - SendRecv and AlltoAll are the reduction-free P2P primitives of the paper
 *     (Section 1, Challenge 1; Section 2.1 "Distributed LLM Training").
 *   - In pipeline parallelism a stage sends to the next stage and receives
 *     from the previous one (Section 3.2, "Improve overlaps in PP").
 *   - NCCL's intra-node path moves data in chunks through a receiver chunk
 *     buffer (Section 2.2, intra-node two-step pattern); the staged routine
 *     below models that FIFO.  The zero-copy form (Section 3.2, item 1) is the
 *     direct application-buffer to application-buffer copy of oracle_sendrecv.
 *   - MoE uses AlltoAll for token routing (Section 2.1) in a dispatch phase
 *     (Section 6); the pack is the permutation that makes every destination's
 *     rows contiguous.
 * With P virtual ranks in one memory the exchange law is
 *     recv[r][rdispls[r][s] + i] = send[s][sdispls[s][r] + i],  i < count(s -> r).
 *
 * Pins: every routine here is pinned by tests/test_oracle_*.py (identity at
 * P = 1, NumPy axis swap, NumPy roll, NumPy stable argsort / bincount,
 * involution, conservation, untouched gaps, hand-worked fixtures, exhaustive
 * tiny cases; unpack(pack(x)) = each row K times and a hand-worked fixture for the
 * un-permute; the per-rank pack against NumPy's unique over (rank, token) keys, its
 * reduction to the per-expert pack when no two slots share a rank, and a hand-worked
 * fixture).  No routine is "parity unpinned".
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum {
    ORACLE_OK = 0,
    ORACLE_ERR_ARG = -1,
    ORACLE_ERR_COUNT_MISMATCH = -2,
    ORACLE_ERR_FIFO = -3
};

/* AlltoAllv.  sendcounts/sdispls are [P][P] row-major indexed [s][r];
 * recvcounts/rdispls are [P][P] indexed [r][s]; all in bytes.  Bytes of recv[r]
 * that no segment covers are left as they were. */
int oracle_alltoallv(const uint8_t *const *send, const uint64_t *sendcounts, const uint64_t *sdispls,
                     uint8_t *const *recv, const uint64_t *recvcounts, const uint64_t *rdispls,
                     int P, int threads)
{
    if (P < 1) return ORACLE_ERR_ARG;
    for (int s = 0; s < P; ++s)
        for (int r = 0; r < P; ++r)
            if (sendcounts[(size_t)s * P + r] != recvcounts[(size_t)r * P + s])
                return ORACLE_ERR_COUNT_MISMATCH;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static, 1)
    for (int r = 0; r < P; ++r) {
        for (int s = 0; s < P; ++s) {
            const uint64_t n = recvcounts[(size_t)r * P + s];
            const uint8_t *src = send[s] + sdispls[(size_t)s * P + r];
            uint8_t *dst = recv[r] + rdispls[(size_t)r * P + s];
            for (uint64_t i = 0; i < n; ++i) dst[i] = src[i];
        }
    }
    return ORACLE_OK;
}

/* AlltoAll with equal blocks of c bytes: block r of send[s] becomes block s of recv[r]. */
int oracle_alltoall(const uint8_t *const *send, uint8_t *const *recv, uint64_t c, int P, int threads)
{
    if (P < 1) return ORACLE_ERR_ARG;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static, 1)
    for (int r = 0; r < P; ++r)
        for (int s = 0; s < P; ++s)
            for (uint64_t i = 0; i < c; ++i)
                recv[r][(uint64_t)s * c + i] = send[s][(uint64_t)r * c + i];
    return ORACLE_OK;
}

/* SendRecv, zero-copy form.  Rank s sends sendbytes[s] bytes from send[s] to rank
 * send_to[s]; rank r receives recvbytes[r] bytes into recv[r] from rank recv_from[r].
 * send_to must be a permutation, recv_from its inverse, and the byte counts of the
 * two ends of every connection must agree. */
int oracle_sendrecv(const uint8_t *const *send, const uint64_t *sendbytes, const int *send_to,
                    uint8_t *const *recv, const uint64_t *recvbytes, const int *recv_from, int P)
{
    if (P < 1) return ORACLE_ERR_ARG;
    for (int s = 0; s < P; ++s) {
        const int r = send_to[s];
        if (r < 0 || r >= P) return ORACLE_ERR_ARG;
        if (recv_from[r] != s) return ORACLE_ERR_ARG;
        if (sendbytes[s] != recvbytes[r]) return ORACLE_ERR_COUNT_MISMATCH;
    }
    for (int s = 0; s < P; ++s) {
        uint8_t *dst = recv[send_to[s]];
        for (uint64_t i = 0; i < sendbytes[s]; ++i) dst[i] = send[s][i];
    }
    return ORACLE_OK;
}

/* One connection of the staged (chunk-buffer) SendRecv: the sender copies chunk k
 * into FIFO slot k mod slots and advances head; the receiver copies the slot into
 * the destination and advances tail; the sender may not run more than `slots`
 * chunks ahead.  `schedule` is a bit string consumed one bit per step (wrapping
 * after schedule_bits): 1 asks the sender to move, 0 the receiver; a side that
 * cannot move yields to the other.  max_occupancy (may be NULL) gets the largest
 * head - tail seen.  The last chunk may be short. */
int oracle_sendrecv_staged(const uint8_t *src, uint8_t *dst, uint64_t nbytes, uint64_t chunk_bytes,
                           int slots, uint8_t *fifo, const uint8_t *schedule, uint64_t schedule_bits,
                           uint64_t *max_occupancy)
{
    if (chunk_bytes == 0 || slots < 1) return ORACLE_ERR_ARG;
    const uint64_t nchunks = (nbytes + chunk_bytes - 1) / chunk_bytes;
    uint64_t head = 0, tail = 0, step = 0, peak = 0;
    while (tail < nchunks) {
        int want_sender = 1;
        if (schedule && schedule_bits) {
            const uint64_t b = step % schedule_bits;
            want_sender = (schedule[b >> 3] >> (b & 7)) & 1;
        }
        ++step;
        const int sender_can = head < nchunks && head - tail < (uint64_t)slots;
        const int receiver_can = tail < head;
        if (!sender_can && !receiver_can) return ORACLE_ERR_FIFO;
        const int move_sender = want_sender ? sender_can : !receiver_can;
        if (move_sender) {
            const uint64_t k = head, off = k * chunk_bytes;
            const uint64_t n = nbytes - off < chunk_bytes ? nbytes - off : chunk_bytes;
            uint8_t *slot = fifo + (k % (uint64_t)slots) * chunk_bytes;
            for (uint64_t i = 0; i < n; ++i) slot[i] = src[off + i];
            ++head;
        } else {
            const uint64_t k = tail, off = k * chunk_bytes;
            const uint64_t n = nbytes - off < chunk_bytes ? nbytes - off : chunk_bytes;
            const uint8_t *slot = fifo + (k % (uint64_t)slots) * chunk_bytes;
            for (uint64_t i = 0; i < n; ++i) dst[off + i] = slot[i];
            ++tail;
        }
        if (head < tail || head - tail > (uint64_t)slots) return ORACLE_ERR_FIFO;
        if (head - tail > peak) peak = head - tail;
    }
    if (max_occupancy) *max_occupancy = peak;
    return ORACLE_OK;
}

/* MoE dispatch pack of one source rank.  The T*K (token, slot) pairs, taken in
 * order p = t*K + k, are stably sorted by their expert id ids[p]; row j of
 * `packed` is the row of x belonging to the token of the j-th pair in that order.
 * order[j] gets the pair index p, cnt[e] the number of pairs routed to expert e. */
int oracle_moe_pack(const uint8_t *x, const int32_t *ids, int64_t T, int K, uint64_t row_bytes,
                    int E, uint8_t *packed, int64_t *order, uint64_t *cnt)
{
    if (T < 0 || K < 1 || E < 1) return ORACLE_ERR_ARG;
    const int64_t npairs = T * (int64_t)K;
    for (int64_t p = 0; p < npairs; ++p)
        if (ids[p] < 0 || ids[p] >= E) return ORACLE_ERR_ARG;
    int64_t j = 0;
    for (int e = 0; e < E; ++e) {
        cnt[e] = 0;
        for (int64_t p = 0; p < npairs; ++p) {
            if (ids[p] == e) {
                order[j++] = p;
                ++cnt[e];
            }
        }
    }
    for (j = 0; j < npairs; ++j) {
        const uint8_t *row = x + (uint64_t)(order[j] / K) * row_bytes;
        uint8_t *out = packed + (uint64_t)j * row_bytes;
        for (uint64_t i = 0; i < row_bytes; ++i) out[i] = row[i];
    }
    return ORACLE_OK;
}

/* MoE combine, un-permute step: the inverse of oracle_moe_pack's row movement.
 * `packed` holds T*K rows in the packed order that ids defines (stable sort of the
 * pairs by expert id); row p = t*K + k of `out` receives the packed row at the
 * position pair p has in that order.  The combine phase mirrors dispatch (paper
 * Section 6); summing the K rows of a token is a reduction and not modelled. */
int oracle_moe_unpack(const uint8_t *packed, const int32_t *ids, int64_t T, int K, uint64_t row_bytes,
                      int E, uint8_t *out)
{
    if (T < 0 || K < 1 || E < 1) return ORACLE_ERR_ARG;
    const int64_t npairs = T * (int64_t)K;
    for (int64_t p = 0; p < npairs; ++p)
        if (ids[p] < 0 || ids[p] >= E) return ORACLE_ERR_ARG;
    int64_t j = 0;   /* position in the packed order */
    for (int e = 0; e < E; ++e) {
        for (int64_t p = 0; p < npairs; ++p) {
            if (ids[p] != e) continue;
            const uint8_t *row = packed + (uint64_t)j * row_bytes;
            uint8_t *dst = out + (uint64_t)p * row_bytes;
            for (uint64_t i = 0; i < row_bytes; ++i) dst[i] = row[i];
            ++j;
        }
    }
    return ORACLE_OK;
}

/* MoE dispatch pack with one row per (token, destination rank): the reading of
 * the dispatch phase (paper Section 6) in which a token whose experts share a
 * rank crosses the fabric once.  Expert e lives on rank e / experts_per_rank;
 * R = E / experts_per_rank destination ranks.  For r = 0..R-1 in turn and, inside,
 * t = 0..T-1 in turn: if any of the K slots of token t routes to rank r, the row
 * of t is appended to `packed`.  row_token[j] is the token of packed row j,
 * cnt[r] the number of rows bound for rank r, slot_row[t*K + k] the packed row
 * that serves slot k of token t, *rows the total. */
int oracle_moe_pack_dedup(const uint8_t *x, const int32_t *ids, int64_t T, int K, uint64_t row_bytes,
                          int E, int experts_per_rank, uint8_t *packed, int64_t *row_token,
                          uint64_t *cnt, int64_t *slot_row, int64_t *rows)
{
    if (T < 0 || K < 1 || E < 1 || experts_per_rank < 1 || E % experts_per_rank) return ORACLE_ERR_ARG;
    const int R = E / experts_per_rank;
    for (int64_t p = 0; p < T * (int64_t)K; ++p)
        if (ids[p] < 0 || ids[p] >= E) return ORACLE_ERR_ARG;
    int64_t j = 0;
    for (int r = 0; r < R; ++r) {
        cnt[r] = 0;
        for (int64_t t = 0; t < T; ++t) {
            int hit = 0;
            for (int k = 0; k < K; ++k) {
                if (ids[t * K + k] / experts_per_rank == r) {
                    hit = 1;
                    slot_row[t * K + k] = j;
                }
            }
            if (!hit) continue;
            const uint8_t *row = x + (uint64_t)t * row_bytes;
            uint8_t *out = packed + (uint64_t)j * row_bytes;
            for (uint64_t i = 0; i < row_bytes; ++i) out[i] = row[i];
            row_token[j] = t;
            ++cnt[r];
            ++j;
        }
    }
    *rows = j;
    return ORACLE_OK;
}

/* Count and displacement matrices of the exchange that follows the pack.
 * cnt is [P][E] (per source rank, per expert).  Expert e lives on rank
 * e / experts_per_rank.  sendcounts[s][r] = row_bytes * (rows of s routed to r's
 * experts); sdispls[s][.] is the exclusive prefix sum over r (rank s's packed
 * buffer is already in destination order); recvcounts[r][s] = sendcounts[s][r];
 * rdispls[r][.] is the exclusive prefix sum over s (segments land in source-rank
 * order). */
int oracle_moe_exchange_layout(const uint64_t *cnt, int P, int E, int experts_per_rank,
                               uint64_t row_bytes, uint64_t *sendcounts, uint64_t *sdispls,
                               uint64_t *recvcounts, uint64_t *rdispls)
{
    if (P < 1 || experts_per_rank < 1 || E != P * experts_per_rank) return ORACLE_ERR_ARG;
    for (int s = 0; s < P; ++s) {
        for (int r = 0; r < P; ++r) {
            uint64_t rows = 0;
            for (int e = r * experts_per_rank; e < (r + 1) * experts_per_rank; ++e)
                rows += cnt[(size_t)s * E + e];
            sendcounts[(size_t)s * P + r] = rows * row_bytes;
        }
        uint64_t acc = 0;
        for (int r = 0; r < P; ++r) {
            sdispls[(size_t)s * P + r] = acc;
            acc += sendcounts[(size_t)s * P + r];
        }
    }
    for (int r = 0; r < P; ++r) {
        uint64_t acc = 0;
        for (int s = 0; s < P; ++s) {
            recvcounts[(size_t)r * P + s] = sendcounts[(size_t)s * P + r];
            rdispls[(size_t)r * P + s] = acc;
            acc += recvcounts[(size_t)r * P + s];
        }
    }
    return ORACLE_OK;
}
