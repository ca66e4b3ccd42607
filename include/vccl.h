/*
 * vccl.h - C boundary of the MI355X-native P2P data-movement library.
 *
 * The library moves the bytes behind the reduction-free P2P primitives SendRecv
 * and AlltoAll(v) (paper Section 1, Challenge 1; Section 2.1) for P virtual
 * ranks whose buffers all live in ONE device's HBM:
 *
 *     recv[r][rdispls[r][s] + i] = send[s][sdispls[s][r] + i]   for i < count(s -> r)
 *
 * Two data paths exist for every primitive:
 *   VCCL_MODE_CU  a compute-unit copy kernel on the caller's stream (the kind of
 *                 SM-consuming P2P kernel the paper sets out to remove, Section 2.2);
 *   VCCL_MODE_CE  SDMA copy engines driven by a host proxy thread (the paper's SM-free
 *                 P2P, Section 3.2 items 1-3).  The data never touches a compute unit.
 *                 What keeps stream order is chosen by option "ce_sync", and what
 *                 each choice dispatches depends on the HIP runtime (measured with
 *                 rocprofv3, kernel trace and SQ_WAVES):
 *                   "event"   readiness by an event the proxy polls, completion by a
 *                             stream wait-value operation.  With GPU_STREAMOPS_CP_WAIT=1
 *                             in the environment when the HIP runtime starts, the
 *                             command processor carries the wait out itself: NO kernel
 *                             is dispatched and the call does not block.  This is the
 *                             default whenever the process runs with that setting; the
 *                             library asks for it at load time (it sets the variable
 *                             unless it is already set), which is in time if the
 *                             library is loaded before the process's first HIP call -
 *                             a program that links it, or a Python process that
 *                             imports the package before anything touches the GPU.
 *                             Read-only option "ce_wait_on_cp" tells what vccl_init found.
 *                   "memops"  readiness by a stream write-value operation as well (the
 *                             paper's proxyReadyEvent).  The runtime carries the write
 *                             out with a one-lane helper kernel (a few microseconds),
 *                             and - without the setting above - the wait with another
 *                             that holds one wavefront slot for the length of the
 *                             transfer.  Default when the setting is absent.
 *                   "host"    no stream operation: the calling thread blocks until the
 *                             copies are done.  Nothing is dispatched.
 *
 * Conventions
 *   - Every pointer named *_dev / every element of a buffer-pointer array is a
 *     DEVICE address on the device given to vccl_init.  The pointer arrays
 *     themselves, and all count / displacement / peer arrays, are HOST memory;
 *     they are read during the call only (the library copies what it needs).
 *   - Counts and displacements are BYTES (uint64_t).  Any byte alignment is
 *     handled; 16-byte aligned addresses and lengths take the fast path.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     are asynchronous to the host, start after all work already enqueued on
 *     `stream`, and work enqueued on `stream` afterwards sees the completed
 *     receive buffers (the ordering contract of Section 3.2 item 3).
 *   - The caller owns all data buffers.  Bytes of a receive buffer that no
 *     segment covers are never written.  Send and receive regions must not
 *     overlap (in-place exchange is not supported); receive segments must not
 *     overlap each other.  With option "check"="1" the library verifies this
 *     and returns VCCL_ERR_OVERLAP.
 *   - Every function returns VCCL_OK (0) or a negative vccl_status.  On error
 *     nothing that moves data has been enqueued (a failing copy-engine call may leave
 *     an event record or a stream write of a sequence number nobody waits for), and
 *     vccl_last_error() describes the cause.
 *   - Calls may be made from several host threads; calls on different streams
 *     may overlap on the device.
 *   - VCCL_MODE_CE calls (and vccl_p2p_send / vccl_p2p_recv) on a stream that is capturing
 *     a graph return VCCL_ERR_UNSUPPORTED: a host thread carries each such call out once, a
 *     replayed graph would not reach it.
 */
#ifndef VCCL_H
#define VCCL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    VCCL_MODE_CU = 0,        /* compute-unit copy kernel, application buffer to application buffer */
    VCCL_MODE_CE = 1,        /* copy engines + host proxy thread; no kernel in the default ordering */
    VCCL_MODE_CU_STAGED = 2  /* vccl_sendrecv only: two-step copy through the chunk FIFO */
} vccl_mode;

typedef enum {
    VCCL_OK = 0,
    VCCL_ERR_ARG = -1,            /* null pointer with non-zero size, P out of range, bad mode/peer table */
    VCCL_ERR_COUNT_MISMATCH = -2, /* sender's and receiver's byte counts disagree */
    VCCL_ERR_OVERLAP = -3,        /* overlapping receive segments or send/recv aliasing ("check"="1") */
    VCCL_ERR_HIP = -4,            /* a HIP runtime call failed; message holds hipGetErrorString */
    VCCL_ERR_NOT_INIT = -5,       /* vccl_init has not been called (or vccl_finalize has) */
    VCCL_ERR_UNSUPPORTED = -6,    /* mode not available for this primitive / device */
    VCCL_ERR_TIMEOUT = -7         /* a bounded wait gave up: the staged FIFO's device-side wait, vccl_p2p_connect's
                                     deadline; also a call on a cross-process connection that was aborted */
} vccl_status;

/* Largest number of virtual ranks vccl_init accepts. */
#define VCCL_MAX_RANKS 256

/* Create the library context on `device`: internal copy streams and events, the
 * descriptor staging ring and the two host proxy threads of the copy-engine path
 * (the CPU proxy of Section 3.2, which drives the engines, and the receiving side of
 * the SendRecv handshake).  max_ranks bounds P of later calls
 * (1 .. VCCL_MAX_RANKS).  Calling it again after vccl_finalize is allowed;
 * calling it twice without is VCCL_ERR_ARG. */
int vccl_init(int device, int max_ranks);

/* Wait for every operation handed to the library, stop the proxy threads and free
 * everything the library owns.  Caller buffers are untouched. */
int vccl_finalize(void);

/* Message of the last failing call made by THIS thread (library-owned storage,
 * valid until the thread's next failing call).  Never NULL. */
const char *vccl_last_error(void);

/* Tuning and test knobs; unknown keys or unparsable values give VCCL_ERR_ARG
 * (silently ignored settings are the configuration hazard of Section 5).
 * Keys: "cu_unroll" (16-byte vectors per lane per tile: 1,2,4,8,16),
 *       "cu_wg_per_cu" (0 = one workgroup per tile; 1..16 = that many grid-striding
 *                        workgroups per compute unit),
 *       "cu_max_wg" (cap on the copy grid, 0 = none; the co-run study sweeps it),
 *       "cu_nontemporal" (0 plain accesses, 1 non-temporal loads and stores, 2 non-temporal
 *                         loads and device-scope stores), "cu_threads" (64 | 128 | 256 lanes per
 *                         workgroup of the copy kernels), "cu_fast_path" (0/1: allow the all-aligned kernel),
 *       "ce_kind" (copy-engine back end: "sdma" = SDMA engines driven
 *       through the HSA runtime with stream write/wait-value ordering, the default when the
 *       device supports it; "hip_nocu" / "hip_default" = hipMemcpyAsync on internal streams
 *       with event ordering, kind hipMemcpyDeviceToDeviceNoCU / hipMemcpyDeviceToDevice),
 *       "ce_streams" (1..8 internal streams of the hip_* back ends),
 *       "ce_sync" (sdma back end only: "event", "memops" or "host", see VCCL_MODE_CE above),
 *       "ce_wait_on_cp" (read-only: 1 if GPU_STREAMOPS_CP_WAIT was set to a non-zero value
 *       when vccl_init ran),
 *       "ce_engines" (read-only: SDMA engines found),
 *       "ce_engine_bytes" (read-only: bytes handed to each engine since vccl_init, comma
 *       separated; the pieces of an operation go to the engine with the fewest bytes),
 *       "ce_errors" (read-only: copy-engine operations that could not move all of their bytes
 *       after the call had returned - a piece that every engine refused and that the HIP copy
 *       issued in its place could not move either, or a cross-process transfer that was
 *       mismatched or aborted; the next copy-engine call then fails once with
 *       VCCL_ERR_HIP, and vccl_finalize returns VCCL_ERR_HIP if any went unreported),
 *       "ce_refused" (read-only: pieces that no engine took and that went through the HIP
 *       copy instead, before the operation's stream was released),
 *       "ce_test_refuse" (test hook, 0..131071: bit i < 16 makes the proxy treat engine i as
 *       refusing every copy, bit 16 makes it treat every pitched copy as refused - its rows
 *       then go as plain copies),
 *       "ce_proxy_poll" (0, default: while operations are in flight the sender proxy polls
 *       around the time each is expected to complete - what operations of the same shape took
 *       before, a model of the engines for a shape not yet seen - and sleeps in between;
 *       1: it polls without pause, as the proxy of Section 3.1 does, which keeps one host core busy),
 *       "ce_pitched" (vccl_alltoall on the sdma back end when the rank buffers of one side are
 *       16-byte aligned slices of one allocation at a constant stride and the block size is a
 *       multiple of 16: the P blocks of a rank are then ONE pitched engine copy, P copies per
 *       exchange in place of P * P; the engines need microseconds per copy whatever its size,
 *       and the runtime runs pitched copies one after another on one engine.  1, default: take
 *       pitched copies where they are expected to finish first - many ranks, small blocks;
 *       0: never; 2: wherever the layout allows),
 *       "ce_pitched_copies" (read-only: pitched copies issued since vccl_init),
 *       "ce_max_engines" (0 = all; else use only that many engines),
 *       "p2p_close_wait_ms" (0..3600000, default 10000: see vccl_p2p_close),
 *       "check" (0/1 overlap validation),
 *       "moe_gather_variant" (row gather of vccl_moe_pack: 208 / 308 = one workgroup of 8
 *       wavefronts per 2 KiB piece of a token's row, one wavefront per slot, non-temporal /
 *       plain stores (the per-rank pack uses 408 / 508 in their place); 408 / 508 = one
 *       wavefront per 2 KiB piece looping over the slots, non-temporal / plain stores;
 *       4, 8, 16 = one wavefront per token holding that many vectors per lane,
 *       non-temporal stores; 108, 116 = the same with plain stores),
 *       "moe_gather_full" (1, default: rows that are whole 2 KiB pieces with slot counts that
 *       are whole groups of 8 take gather kernels without bounds tests; 0: always the
 *       checked kernels),
 *       "moe_unpack_variant" (row un-permute of vccl_moe_unpack: 0 = one workgroup per row,
 *       1 / 2 = one wavefront per 1 KiB tile with non-temporal / device-scope stores,
 *       3 = one wavefront per two tiles, device-scope stores),
 *       "fifo_chunk_bytes", "fifo_slots", "fifo_wg_per_conn" (sender / receiver workgroup
 *       pairs per connection, default 32; fewer when the
 *       pairs of all connections would exceed two workgroups per compute unit),
 *       "fifo_spin_limit" (polls before a staged wait gives up),
 *       "fifo_scoped" (1, default: FIFO memory is read and written with device-scope
 *       accesses and the chunk counters move relaxed; 0: plain accesses ordered by a
 *       release on the sender's counter and an acquire on the receiver's poll, which
 *       costs a cache write-back / invalidate per workgroup and chunk).
 * vccl_get_option writes the current value as text into out[0..cap). */
int vccl_set_option(const char *key, const char *value);
int vccl_get_option(const char *key, char *out, int cap);

/* SendRecv (pipeline-parallel activations, Section 3.2 "Improve overlaps in PP";
 * the zero-copy application-buffer transfer of Section 3.2 item 1).
 * Rank s sends sendbytes[s] bytes from sendbuf[s] to rank send_to[s]; rank r
 * receives recvbytes[r] bytes into recvbuf[r] from rank recv_from[r].  send_to
 * must be a permutation of 0..P-1 and recv_from its inverse (VCCL_ERR_ARG), and
 * sendbytes[s] must equal recvbytes[send_to[s]] (VCCL_ERR_COUNT_MISMATCH).
 * VCCL_MODE_CU / VCCL_MODE_CE copy directly; VCCL_MODE_CU_STAGED models NCCL's
 * intra-node two-step path (Section 2.2): sender workgroups copy chunks into a
 * library-owned FIFO of "fifo_slots" slots of "fifo_chunk_bytes", receiver
 * workgroups copy them out, the sender never running more than the slot count
 * ahead.  The FIFO is allocated on first use. */
int vccl_sendrecv(void *const *sendbuf, const uint64_t *sendbytes, const int *send_to,
                  void *const *recvbuf, const uint64_t *recvbytes, const int *recv_from,
                  int P, vccl_mode mode, void *stream);

/* Waits (on the host) for the VCCL_MODE_CU_STAGED operations issued so far and returns
 * VCCL_ERR_TIMEOUT if, since the last time this was asked, one of them had a bounded
 * device-side FIFO wait give up (its data is then incomplete), VCCL_OK otherwise.
 * The staged call itself does not wait for the device: operations queue behind each
 * other on the device (one at a time owns the FIFO), whatever streams they are on. */
int vccl_sendrecv_staged_status(void);

/* The receiver-owned handshake record of a SendRecv connection in copy-engine mode
 * (Section 3.2: receiverRegAddr, receiverReady, copyStarted, copyDone).  The
 * paper's 1-bit flags are kept as sequence numbers that only grow: operation n on
 * the connection is ready / started / done once the field has reached n.  Any
 * output pointer may be NULL. */
int vccl_p2p_reginfo(int receiver_rank, uint64_t *receiver_ready, uint64_t *copy_started,
                     uint64_t *copy_done, void **receiver_reg_addr);

/* SendRecv between two PROCESSES on the device (the paper's intra-node design, Section
 * 3.2): the receiver registers an application buffer once - vccl_p2p_export creates the
 * receiver-owned handshake record (receiverRegAddr, receiverReady, copyStarted, copyDone,
 * kept as sequence numbers) in POSIX shared memory under `name` ("/" + up to 199
 * characters) and puts the buffer's IPC handle into it; the sender maps record and buffer
 * once with vccl_p2p_connect (waits up to timeout_s for the export to appear).  recvbuf_dev
 * is device memory of this process (any address inside one allocation; the allocation
 * must be smaller than 2 GiB) and stays the receiver's: it must outlive the connection.
 * Transfer n of a connection is the n-th vccl_p2p_recv on one side and the n-th
 * vccl_p2p_send on the other:
 *   vccl_p2p_recv(conn, offset, bytes, stream)  once `stream` has reached the call (earlier
 *     work that reads the buffer is done) and transfer n-1 has started, the receiver's proxy
 *     publishes "n goes to buffer + offset, bytes long" and raises receiverReady; work
 *     enqueued on `stream` afterwards runs when the record shows copyDone >= n.
 *   vccl_p2p_send(conn, sendbuf_dev, bytes, stream)  once `stream` has reached the call and
 *     the record shows receiverReady = n, the sender's proxy marks copyStarted, moves the
 *     bytes with the copy engines straight from sendbuf_dev into the receiver's buffer, and
 *     marks copyDone; `stream` resumes then.
 * Neither call blocks the host (ordering as for VCCL_MODE_CE, "ce_sync"), no kernel runs
 * in either process.  If the two sides disagree on the byte count, nothing is copied, the
 * record counts a mismatch and the sender's next copy-engine call fails.  A send without
 * a matching recv waits, as it would between two machines - until either side calls
 * vccl_p2p_abort (a peer that died, a deadline that passed): every outstanding transfer of
 * the connection in either process then ends without copying, its stream is released, the
 * failure is reported by the next copy-engine call, and later sends / receives on the
 * connection return VCCL_ERR_TIMEOUT.  vccl_p2p_record reads the
 * record from either side (any pointer may be NULL).  vccl_p2p_close waits for this
 * process's outstanding copy-engine operations - for at most 10 seconds (option
 * "p2p_close_wait_ms"): if transfers of the
 * connection are still outstanding then (the peer never posted its side), it aborts the
 * connection as vccl_p2p_abort does and returns VCCL_ERR_TIMEOUT after cleaning up - then
 * unmaps, and (receiver) removes the name.
 * Needs the "sdma" copy-engine back end. */
typedef struct vccl_p2p_conn vccl_p2p_conn;
int vccl_p2p_export(const char *name, void *recvbuf_dev, uint64_t capacity, vccl_p2p_conn **out);
int vccl_p2p_connect(const char *name, double timeout_s, vccl_p2p_conn **out);
int vccl_p2p_recv(vccl_p2p_conn *conn, uint64_t offset, uint64_t bytes, void *stream);
int vccl_p2p_send(vccl_p2p_conn *conn, const void *sendbuf_dev, uint64_t bytes, void *stream);
int vccl_p2p_record(vccl_p2p_conn *conn, uint64_t *receiver_ready, uint64_t *copy_started,
                    uint64_t *copy_done, uint64_t *reg_offset, uint64_t *mismatches);
int vccl_p2p_abort(vccl_p2p_conn *conn);
int vccl_p2p_close(vccl_p2p_conn *conn);

/* AlltoAll with equal blocks (MoE token routing, Section 2.1): block r
 * (bytes_per_peer bytes at offset r*bytes_per_peer) of sendbuf[s] becomes block s
 * of recvbuf[r].  Every buffer holds at least P*bytes_per_peer bytes.
 * In VCCL_MODE_CU with 16-byte aligned buffers and block size (or at most 64
 * segments otherwise) the call is one kernel launch with no allocation, copy or
 * wait around it, so it may be recorded into a HIP graph on a capturing stream. */
int vccl_alltoall(void *const *sendbuf, void *const *recvbuf, uint64_t bytes_per_peer,
                  int P, vccl_mode mode, void *stream);

/* AlltoAllv (the dispatch / combine exchange of Section 6).  sendcounts and
 * sdispls are [P][P] row-major indexed [s][r]; recvcounts and rdispls are [P][P]
 * indexed [r][s].  sendcounts[s][r] must equal recvcounts[r][s]
 * (VCCL_ERR_COUNT_MISMATCH - a distributed library would hang instead).
 * Zero-length segments are legal and their displacements are ignored. */
int vccl_alltoallv(void *const *sendbuf, const uint64_t *sendcounts, const uint64_t *sdispls,
                   void *const *recvbuf, const uint64_t *recvcounts, const uint64_t *rdispls,
                   int P, vccl_mode mode, void *stream);

/* Host-only view of the planner of the compute-unit path (needs no device and no
 * vccl_init; buffer addresses are never dereferenced).  For an AlltoAllv
 * description it reports the copy descriptors in launch order - non-empty segments,
 * destination-major with the source rotated by the destination index (the incast
 * counter-measure, Section 6), long segments cut into pieces of equal tile count -
 * and the launch grid: grid_x tiles of *tile_bytes = 16 * cu_unroll * cu_threads
 * bytes per descriptor, grid_y descriptors.
 * head is the number of leading bytes copied bytewise before the destination is
 * 16-byte aligned.  Tiles are cut where the destination address is a multiple of
 * *tile_bytes: lead is the number of 16-byte vectors between the last such multiple
 * and dst + head, and a descriptor has ceil(((bytes - head) / 16 + lead) /
 * (*tile_bytes / 16)) tiles, at least one.  all_aligned tells whether the fast
 * kernel applies.  out may be NULL to query the count. */
typedef struct {
    uint64_t src, dst, bytes;
    uint32_t head, lead;
} vccl_plan_desc;
int vccl_plan_alltoallv(void *const *sendbuf, const uint64_t *sendcounts, const uint64_t *sdispls,
                        void *const *recvbuf, const uint64_t *recvcounts, const uint64_t *rdispls,
                        int P, int cu_unroll, int cu_threads, vccl_plan_desc *out, int out_cap,
                        int *n_out, uint32_t *grid_x, uint32_t *grid_y, uint32_t *tile_bytes,
                        int *all_aligned);

/* MoE dispatch pack (Section 2.1 token routing; Section 6 dispatch phase) for all
 * P source ranks in one call.  For rank s, x[s] holds `tokens` rows of row_bytes
 * bytes (row_bytes a multiple of 16, rows 16-byte aligned) and expert_ids[s] holds
 * tokens*topk int32 expert ids in [0, num_experts), row-major [token][slot].  The
 * tokens*topk (token, slot) pairs are stably sorted by expert id (ties keep
 * token-then-slot order) and packed[s] receives one copy of the token's row per
 * pair, in that order, so that the rows for each destination rank are contiguous.
 * counts_dev (device, uint64 [P][num_experts]) receives the number of pairs per
 * expert; if counts_host is not NULL it must be pinned host memory of the same
 * shape and an asynchronous copy of the counts is enqueued after the kernels
 * (synchronise `stream` before reading it).  Ids outside the range are counted
 * in *bad_ids_dev (device uint32, may be NULL) and their pairs are dropped.
 * Runs on compute units only (it is index arithmetic plus a gather). */
int vccl_moe_pack(const void *const *x, const int32_t *const *expert_ids, int P, int tokens,
                  int topk, uint64_t row_bytes, int num_experts, void *const *packed,
                  uint64_t *counts_dev, uint64_t *counts_host, uint32_t *bad_ids_dev, void *stream);

/* vccl_moe_pack for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * result and stream semantics as vccl_moe_pack (without the pinned copy of the
 * counts), but nothing is allocated or freed, on the device or through any library:
 * the index data of the call (per-block histograms, one destination row per pair, the
 * table of rank pointers) lives in a fixed 8 MiB array that is part of the library's
 * device image (each device the library runs on holds it until the process ends).
 * Limits: P <= 16, and 256-byte pointer table + 4 * (P * ceil(tokens*topk / 2048) *
 * num_experts + P * tokens * topk + 2 * P * num_experts + 4) bytes must fit into the
 * 8 MiB (P = 8, 8192 tokens, top-8 of 256 experts needs 2.3 MiB); beyond that the call
 * returns VCCL_ERR_UNSUPPORTED and enqueues nothing.  All calls on one device share the
 * array: a call may start only after the previous vccl_moe_pack_noalloc on that device
 * has finished or on the same stream; calls that overlap on one device race.  Nothing
 * in the array has to be cleared between calls (every word a call reads it has written
 * first). */
int vccl_moe_pack_noalloc(const void *const *x, const int32_t *const *expert_ids, int P, int tokens,
                          int topk, uint64_t row_bytes, int num_experts, void *const *packed,
                          uint64_t *counts_dev, uint32_t *bad_ids_dev, void *stream);

/* MoE dispatch pack with one row per (token, destination rank): the reading of the
 * dispatch phase (Section 6) in which a token whose experts share a rank crosses the
 * fabric once.  Expert e lives on rank e / experts_per_rank (experts_per_rank divides
 * num_experts; R = num_experts / experts_per_rank destination ranks).  For every
 * source rank s the (token, rank) pairs with at least one slot routed to that rank
 * are ordered by rank, then token, and packed[s] (room for tokens * min(topk, R)
 * rows) receives the token's row for each.  counts_dev (device uint64 [P][R]) and
 * the optional pinned counts_host receive the rows per destination rank - with
 * vccl_moe_exchange_layout(counts, P, R, 1, row_bytes) they describe the exchange
 * that follows.  slot_row may be NULL; else it is a host array of P device pointers
 * (entries may be NULL), each to tokens*topk uint32: slot_row[s][t*topk + k] = the
 * packed row that serves slot k of token t (0xffffffff for an out-of-range id), which
 * is what the receiving side needs to fan a row out to its experts.  Out-of-range
 * ids are counted in *bad_ids_dev (may be NULL) and dropped.  Other arguments and
 * stream semantics as vccl_moe_pack. */
int vccl_moe_pack_per_rank(const void *const *x, const int32_t *const *expert_ids, int P, int tokens,
                           int topk, uint64_t row_bytes, int num_experts, int experts_per_rank,
                           void *const *packed, uint64_t *counts_dev, uint64_t *counts_host,
                           uint32_t *const *slot_row, uint32_t *bad_ids_dev, void *stream);

/* Fused MoE dispatch: the pack and the exchange in one pass - the zero-copy idea of
 * Section 3.2 (item 1: move data between application buffers directly, no staging
 * buffer) applied to the dispatch phase of Section 6.  Every row goes from x[s]
 * straight to the place in recv[r] where vccl_moe_pack + vccl_moe_exchange_layout +
 * vccl_alltoallv would have put it (segments in source-rank order, inside a segment
 * by expert id, token, slot), so each row is written once and no packed buffer
 * exists.  num_experts must equal P * experts_per_rank.  recv[r] (device, 16-byte
 * aligned) has room for recv_capacity_rows[r] rows (host array); rows beyond a
 * buffer's capacity are not written and status_dev[1] becomes non-zero.
 * status_dev (device uint32 [2], may be NULL, zeroed by the caller): [0] counts
 * out-of-range ids (their pairs are dropped), [1] flags an overflow.  counts_dev
 * (device uint64 [P][num_experts], may be NULL) receives the pairs per expert.
 * layout_dev (device uint64 [4][P][P], required) receives sendcounts, sdispls,
 * recvcounts, rdispls in bytes, as the two-step form would use them - rdispls and
 * recvcounts tell the receiver where each source's rows are; layout_host, if not
 * NULL, is pinned host memory of the same shape that gets an asynchronous copy.
 * One call, no host synchronisation inside.  Compute units only. */
int vccl_moe_dispatch_fused(const void *const *x, const int32_t *const *expert_ids, int P, int tokens,
                            int topk, uint64_t row_bytes, int num_experts, int experts_per_rank,
                            void *const *recv, const uint64_t *recv_capacity_rows, uint64_t *counts_dev,
                            uint64_t *layout_dev, uint64_t *layout_host, uint32_t *status_dev,
                            void *stream);

/* Fused MoE combine: the way back in one pass (Section 6: the combine phase mirrors
 * dispatch; Section 3.2 item 1: no staging buffer).  back[r] holds, for rank r, the
 * rows it received in the dispatch (in the order vccl_moe_dispatch_fused or pack +
 * exchange delivered them, typically after the experts changed their contents),
 * back_capacity_rows[r] rows of room (host array; a pair whose row would lie beyond
 * it is skipped).  Row t*topk + k of out[s] (tokens*topk rows, 16-byte aligned)
 * receives the row of pair (t, k) of source rank s - what the inverse vccl_alltoallv
 * followed by vccl_moe_unpack would produce.  Rows of pairs with out-of-range ids are
 * left untouched.  The weighted sum over a token's rows is a reduction and not part
 * of this library. */
int vccl_moe_combine_fused(const void *const *back, const uint64_t *back_capacity_rows,
                           const int32_t *const *expert_ids, int P, int tokens, int topk,
                           uint64_t row_bytes, int num_experts, int experts_per_rank, void *const *out,
                           void *stream);

/* MoE combine, un-permute step (Section 6: the combine phase mirrors dispatch).  The
 * inverse of vccl_moe_pack for all P ranks: packed[s] holds tokens*topk rows in the
 * packed order defined by expert_ids[s] (for instance the rows that came back
 * through vccl_alltoallv with the receive description used as the send description);
 * row t*topk + k of out[s] receives the packed row that pair (t, k) had been sent
 * to.  Rows of pairs with out-of-range ids are left untouched.  Pure data movement:
 * the weighted sum over the topk rows of a token is a reduction and not part of
 * this library.  Same alignment rules as vccl_moe_pack. */
int vccl_moe_unpack(const void *const *packed, const int32_t *const *expert_ids, int P, int tokens,
                    int topk, uint64_t row_bytes, int num_experts, void *const *out, void *stream);

/* Host-side planner step between pack and exchange: from counts [P][num_experts]
 * (host) build the four [P][P] byte matrices for vccl_alltoallv.  Expert e lives on
 * rank e / experts_per_rank; sdispls / rdispls are exclusive prefix sums (packed
 * rows are already in destination order; received segments land in source-rank
 * order).  num_experts must equal P*experts_per_rank. */
int vccl_moe_exchange_layout(const uint64_t *counts, int P, int num_experts, int experts_per_rank,
                             uint64_t row_bytes, uint64_t *sendcounts, uint64_t *sdispls,
                             uint64_t *recvcounts, uint64_t *rdispls);

/* HBM ceiling probe, a measurement aid: plain streaming kernels in the launch shapes of
 * the copy paths, for finding what the device gives to read-only, write-only, copy
 * and scattered-row-write traffic - the rooflines the copy kernel (Appendix A: the
 * P2P copy that occupies compute units) and the MoE row movement (Section 6) are
 * held against.  One workgroup of `threads` lanes handles vecs_per_lane consecutive
 * 16-byte vectors per lane; accepted shapes: 64x1, 64x2, 64x4, 64x16, 256x1, 256x4,
 * 448x2.  kind 0: read `bytes` from src (dst = any 64-byte device buffer, not
 * written); 1: write `bytes` to dst; 2: copy `bytes` from src to dst; 3: write n_rows
 * whole rows of row_bytes to dst, the i-th at row row_index[i] (device uint32 array,
 * values below the number of rows dst holds; NULL = row i).  Buffers are device
 * memory, 16-byte aligned; what is written is a fixed pattern.  Asynchronous on
 * `stream`; timing is the caller's. */
int vccl_hbm_probe(int kind, const void *src, void *dst, uint64_t bytes, int threads, int vecs_per_lane,
                   const uint32_t *row_index, uint64_t n_rows, uint64_t row_bytes, void *stream);

/* Co-run probe (Appendix E: a compute kernel forming one wave of workgroups over
 * all compute units, slowed by co-resident communication warps).  Launches a
 * register-only FP32 FMA kernel of `workgroups` x `threads` (threads a multiple of
 * 64, at most 1024) running `iters` dependent FMA rounds per lane; out_dev (device,
 * workgroups*threads floats) receives one value per lane so the work cannot be
 * elided.  workgroups = 0 selects one workgroup per compute unit. */
int vccl_fma_probe(float *out_dev, uint32_t workgroups, uint32_t threads, uint64_t iters,
                   void *stream);

/* The same probe, reporting for every workgroup how long it ran on two counters of the
 * chip: clocks_dev (device, 2 * workgroups uint64, 8-byte aligned) receives per workgroup
 * the elapsed ticks of the shader clock, which the chip's power management raises and
 * lowers, and of the constant-rate real-time counter (vccl_device_wall_clock_khz ticks
 * per millisecond).  A probe that takes longer beside a transfer with the same shader
 * ticks was slowed down by a lower clock; one with more shader ticks was held up inside
 * its compute units (the mechanism Appendix E describes). */
int vccl_fma_probe_clocks(float *out_dev, uint64_t *clocks_dev, uint32_t workgroups, uint32_t threads,
                          uint64_t iters, void *stream);

/* Rate of the device's constant real-time counter in kHz (negative: error code). */
int vccl_device_wall_clock_khz(void);

/* Window-based bandwidth monitor (Section 3.4), host-only and usable on its own:
 * feed it the post and completion times of messages (nanoseconds on any monotonic
 * clock, calls in non-decreasing time order) and it returns, per completion, the
 * per-message estimate bytes/(t2-t1), the sliding-window estimate (sum of the bytes
 * of the last `window` completed messages over the span from their earliest post to
 * their latest completion; the paper deploys window = 8), the bytes still
 * outstanding, and the anomaly flag: window estimate below half the mean of the
 * estimates of the `history_ns` that precede the current window AND outstanding
 * bytes above twice the largest amount seen in that span (the paper uses about
 * 10 ms).  Bandwidths are in bytes per second.  vccl_monitor_create returns NULL on
 * bad arguments.  The copy-engine proxy runs one monitor per primitive over the
 * operations it issues (vccl_proxy_monitor: primitive 0 = SendRecv, 1 = AlltoAll(v)). */
typedef struct vccl_monitor vccl_monitor;
typedef struct {
    uint64_t t_ns;
    double bw_message;
    double bw_window;
    uint64_t outstanding;
    int anomaly;
} vccl_monitor_sample;
vccl_monitor *vccl_monitor_create(int window, uint64_t history_ns);
void vccl_monitor_destroy(vccl_monitor *m);
int vccl_monitor_post(vccl_monitor *m, uint64_t id, uint64_t bytes, uint64_t t_post_ns);
int vccl_monitor_complete(vccl_monitor *m, uint64_t id, uint64_t t_done_ns, vccl_monitor_sample *out);
int vccl_monitor_totals(vccl_monitor *m, uint64_t *messages, uint64_t *anomalies, vccl_monitor_sample *last);
int vccl_proxy_monitor(int primitive, uint64_t *messages, uint64_t *anomalies, vccl_monitor_sample *last);

/* Counters of the copy-engine proxy since vccl_init: operations, copies issued,
 * bytes, and nanoseconds the proxy spent issuing.  Any pointer may be NULL. */
int vccl_proxy_stats(uint64_t *ops, uint64_t *copies, uint64_t *bytes, uint64_t *issue_ns);

/* Processor time, in nanoseconds, that the sender proxy thread (which drives the
 * copy engines and polls for completion) and the receiver proxy thread (the
 * receiving side of the SendRecv handshake) have used since vccl_init: the cost the
 * paper's CPU-utilisation measurement (Section 4.1) charges to moving control from
 * the GPU to host threads.  The threads sleep while nothing is in flight and poll
 * while something is.  Either pointer may be NULL. */
int vccl_proxy_cpu_time(uint64_t *sender_ns, uint64_t *receiver_ns);

/* Number of compute units of the initialised device (for sizing probes). */
int vccl_device_cu_count(void);

#ifdef __cplusplus
}
#endif
#endif /* VCCL_H */
