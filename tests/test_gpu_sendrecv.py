"""GPU parity: SendRecv ring (direct on compute units, copy engines, staged FIFO)."""
import contextlib

import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import SENTINEL, assert_same, require_gpu, stream_handle, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vccl():
    require_gpu()
    import paper_2510_00991_amd as v
    v.vccl_init(0, 64)
    yield v
    v.vccl_finalize()


MODES = ["cu", "ce", "staged", "staged_fenced"]


def _modes(v):
    return {"cu": v.MODE_CU, "ce": v.MODE_CE, "staged": v.MODE_CU_STAGED, "staged_fenced": v.MODE_CU_STAGED}


@contextlib.contextmanager
def _protocol(v, mode):
    """The staged mode has two synchronisation protocols: device-scope accesses to
    the FIFO (default) and plain accesses ordered by release / acquire fences."""
    saved = v.vccl_get_option("fifo_scoped")
    v.vccl_set_option("fifo_scoped", 0 if mode == "staged_fenced" else 1)
    try:
        yield _modes(v)[mode]
    finally:
        v.vccl_set_option("fifo_scoped", saved)


def _ring(torch, v, mode, sizes, misalign=0, stream=None):
    P = len(sizes)
    to, frm = wl.ring_peers(P)
    send_np = [wl.payload_bytes(wl.config_seed(4), s, sizes[s] + 5) for s in range(P)]
    rbytes = [sizes[frm[r]] for r in range(P)]
    recv_np = [np.full(rbytes[r] + 9, SENTINEL, dtype=np.uint8) for r in range(P)]
    send = [to_dev(torch, a, misalign) for a in send_np]
    recv = [to_dev(torch, a, (misalign * 3) % 16) for a in recv_np]
    v.vccl_sendrecv(send, sizes, to, recv, rbytes, frm, P, mode, stream_handle(torch, stream))
    if mode == v.MODE_CU_STAGED:
        v.vccl_sendrecv_staged_status()
    torch.cuda.synchronize()
    oracle.sendrecv(send_np, sizes, to, recv_np, rbytes, frm)
    for r in range(P):
        assert_same(to_host(recv[r]), recv_np[r], f"recv[{r}]")


@pytest.mark.parametrize("mode", MODES)
def test_ring_small_and_ragged(vccl, mode):
    torch = require_gpu()
    with _protocol(vccl, mode) as m:
        _ring(torch, vccl, m, [100000, 0, 7, 65536, 1 << 20])
        _ring(torch, vccl, m, [12345], misalign=0)
        _ring(torch, vccl, m, [3 * 524288 + 17, 524288, 524287], misalign=0)


@pytest.mark.parametrize("mode", MODES)
def test_ring_unaligned_buffers(vccl, mode):
    torch = require_gpu()
    with _protocol(vccl, mode) as m:
        _ring(torch, vccl, m, [700001, 33, 524288 + 1, 99999], misalign=5)
        _ring(torch, vccl, m, [524288 * 2 + 3, 17, 524288 - 16, 4099], misalign=11)


@pytest.mark.parametrize("mode", MODES)
def test_config4_ring_p8_64m_full_size(vccl, mode):
    """8 stages, one 64 MiB activation (1 x 4096 x 8192 bf16, N(0,1)) per stage,
    512 KiB chunks through 8 FIFO slots in staged mode."""
    torch = require_gpu()
    P = 8
    n = wl.pp_message_bytes(1, 4096, 8192, 2)
    assert n == 64 << 20
    to, frm = wl.ring_peers(P)
    send_np = [wl.normal_bf16_bits(wl.config_seed(4), s, n // 2).view(np.uint8) for s in range(P)]
    send = [to_dev(torch, a) for a in send_np]
    recv = [torch.full((n,), SENTINEL, dtype=torch.uint8, device="cuda") for _ in range(P)]
    with _protocol(vccl, mode) as m:
        vccl.vccl_sendrecv(send, [n] * P, to, recv, [n] * P, frm, P, m, stream_handle(torch))
        if m == vccl.MODE_CU_STAGED:
            vccl.vccl_sendrecv_staged_status()
        torch.cuda.synchronize()
    recv_np = [np.empty(n, dtype=np.uint8) for _ in range(P)]
    oracle.sendrecv(send_np, [n] * P, to, recv_np, [n] * P, frm)
    for r in range(P):
        assert_same(to_host(recv[r]), recv_np[r], f"recv[{r}]")


def test_ring_sdma_host_sync(vccl):
    torch = require_gpu()
    saved = vccl.vccl_get_option("ce_sync")
    try:
        for sync in ("host", "event", "memops"):
            vccl.vccl_set_option("ce_sync", sync)
            _ring(torch, vccl, vccl.MODE_CE, [700001, 33, 524288 + 1, 0, 99999], misalign=3)
    finally:
        vccl.vccl_set_option("ce_sync", saved)


@pytest.mark.parametrize("scoped", [1, 0])
def test_staged_equals_oracle_fifo_model(vccl, scoped):
    """Different chunk / slot settings give the same bytes as the oracle's FIFO model,
    under either synchronisation protocol."""
    torch = require_gpu()
    n = 200000
    src_np = wl.payload_bytes(3, 0, n)
    keys = ("fifo_chunk_bytes", "fifo_slots", "fifo_wg_per_conn", "fifo_scoped")
    saved = {k: vccl.vccl_get_option(k) for k in keys}
    for chunk, slots, wg in ((4096, 1, 1), (8192, 3, 4), (65536, 8, 16), (4096, 2, 64)):
        vccl.vccl_set_option("fifo_chunk_bytes", chunk)
        vccl.vccl_set_option("fifo_slots", slots)
        vccl.vccl_set_option("fifo_wg_per_conn", wg)
        vccl.vccl_set_option("fifo_scoped", scoped)
        try:
            src = to_dev(torch, src_np)
            dst = to_dev(torch, np.full(n, SENTINEL, np.uint8))
            vccl.vccl_sendrecv([src], [n], [0], [dst], [n], [0], 1, vccl.MODE_CU_STAGED,
                               stream_handle(torch))
            vccl.vccl_sendrecv_staged_status()
            want = np.full(n, SENTINEL, np.uint8)
            oracle.sendrecv_staged(src_np, want, n, chunk, slots)
            assert_same(to_host(dst), want, f"chunk {chunk} slots {slots}")
        finally:
            for k, val in saved.items():
                vccl.vccl_set_option(k, val)


@pytest.mark.parametrize("scoped", [1, 0])
def test_staged_transfers_in_a_row_never_read_a_stale_slot(vccl, scoped):
    """The FIFO slots are reused by every chunk and every call.  Twelve rings in a row,
    each with its own payload and each wrapping the 8 slots twice, all arrive whole: a
    receiver that took a slot's bytes from a cache instead of from the sender's latest
    write would deliver the previous chunk's or the previous call's data."""
    torch = require_gpu()
    P, n = 8, 8 << 20
    to, frm = wl.ring_peers(P)
    saved = vccl.vccl_get_option("fifo_scoped")
    vccl.vccl_set_option("fifo_scoped", scoped)
    try:
        recv = [torch.full((n,), SENTINEL, dtype=torch.uint8, device="cuda") for _ in range(P)]
        for it in range(12):
            send = [to_dev(torch, wl.payload_bytes(4100 + it, s, n)) for s in range(P)]
            vccl.vccl_sendrecv(send, [n] * P, to, recv, [n] * P, frm, P, vccl.MODE_CU_STAGED, stream_handle(torch))
            vccl.vccl_sendrecv_staged_status()
            torch.cuda.synchronize()
            for r in range(P):
                assert torch.equal(recv[r], send[frm[r]]), f"round {it}, recv[{r}]"
            if it == 0:     # the device-side comparison itself, pinned to the oracle once
                want = [np.zeros(n, np.uint8) for _ in range(P)]
                oracle.sendrecv([to_host(t) for t in send], [n] * P, to, want, [n] * P, frm)
                for r in range(P):
                    assert_same(to_host(recv[r]), want[r], f"recv[{r}]")
    finally:
        vccl.vccl_set_option("fifo_scoped", saved)


def test_staged_calls_do_not_wait_for_the_device(vccl):
    """Staged calls on a stream that a long kernel holds back, and on eleven other
    streams, all return while that kernel still runs.  Operations on different
    streams get FIFO memory of their own while the library has some to give (eight at
    a time) and queue behind each other beyond that; every one arrives whole."""
    torch = require_gpu()
    P, n, calls = 4, 2 << 20, 14
    to, frm = wl.ring_peers(P)
    sends = [[to_dev(torch, wl.payload_bytes(4300 + i, s, n)) for s in range(P)] for i in range(calls)]
    recvs = [[to_dev(torch, np.full(n, SENTINEL, np.uint8)) for _ in range(P)] for _ in range(calls)]
    streams = [torch.cuda.Stream() for _ in range(12)]
    held = streams[0]
    sink = torch.zeros(256 * 256, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    vccl.vccl_fma_probe(sink, 256, 256, 120000, int(held.cuda_stream))       # about 18 ms of compute
    probe_done = torch.cuda.Event()
    probe_done.record(held)
    for i in range(calls):
        st = streams[i % len(streams)]
        vccl.vccl_sendrecv(sends[i], [n] * P, to, recvs[i], [n] * P, frm, P, vccl.MODE_CU_STAGED,
                           int(st.cuda_stream))
    still_running = not probe_done.query()
    vccl.vccl_sendrecv_staged_status()
    torch.cuda.synchronize()
    assert still_running, "the staged calls waited for the kernel on the held stream"
    for i in range(calls):
        want = [np.zeros(n, np.uint8) for _ in range(P)]
        oracle.sendrecv([to_host(t) for t in sends[i]], [n] * P, to, want, [n] * P, frm)
        for r in range(P):
            assert_same(to_host(recvs[i][r]), want[r], f"transfer {i}, recv[{r}]")


def test_staged_wait_gives_up_when_its_poll_budget_runs_out(vccl):
    """Failure path of the staged FIFO, forced from the host: with a poll budget of one
    and a single slow sender workgroup per connection, the receiver's bounded wait runs
    out long before the first chunk is there.  The kernel still ends by itself, the
    status call reports the time-out, and the next staged transfer with the normal
    budget is complete and right."""
    torch = require_gpu()
    P, n = 2, 8 << 20
    to, frm = wl.ring_peers(P)
    send_np = [wl.payload_bytes(77, s, n) for s in range(P)]
    send = [to_dev(torch, a) for a in send_np]
    recv = [to_dev(torch, np.full(n, SENTINEL, np.uint8)) for _ in range(P)]
    keys = ("fifo_spin_limit", "fifo_chunk_bytes", "fifo_slots", "fifo_wg_per_conn")
    saved = {k: vccl.vccl_get_option(k) for k in keys}
    try:
        for k, val in (("fifo_spin_limit", 1), ("fifo_chunk_bytes", 64 << 20), ("fifo_slots", 1),
                       ("fifo_wg_per_conn", 1)):
            vccl.vccl_set_option(k, val)
        vccl.vccl_sendrecv(send, [n] * P, to, recv, [n] * P, frm, P, vccl.MODE_CU_STAGED, stream_handle(torch))
        with pytest.raises(vccl.VcclError) as e:
            vccl.vccl_sendrecv_staged_status()
        assert e.value.code == -7
        torch.cuda.synchronize()            # the grid has drained by itself
    finally:
        for k, val in saved.items():
            vccl.vccl_set_option(k, val)
    for r in range(P):
        recv[r].fill_(SENTINEL)
    vccl.vccl_sendrecv(send, [n] * P, to, recv, [n] * P, frm, P, vccl.MODE_CU_STAGED, stream_handle(torch))
    vccl.vccl_sendrecv_staged_status()
    torch.cuda.synchronize()
    want = [np.zeros(n, np.uint8) for _ in range(P)]
    oracle.sendrecv(send_np, [n] * P, to, want, [n] * P, frm)
    for r in range(P):
        assert_same(to_host(recv[r]), want[r], f"recv[{r}] after the time-out")


def test_ce_handshake_record_advances(vccl):
    """Copy-engine SendRecv walks receiverReady -> copyStarted -> copyDone on the
    receiver's record and publishes the receive buffer's address in it."""
    torch = require_gpu()
    P, n = 3, 1 << 16
    to, frm = wl.ring_peers(P)
    send = [to_dev(torch, wl.payload_bytes(8, s, n)) for s in range(P)]
    recv = [to_dev(torch, np.zeros(n, np.uint8)) for _ in range(P)]
    before = [vccl.vccl_p2p_reginfo(r) for r in range(P)]
    for it in range(1, 4):
        vccl.vccl_sendrecv(send, [n] * P, to, recv, [n] * P, frm, P, vccl.MODE_CE, stream_handle(torch))
        torch.cuda.synchronize()
        import time
        deadline = time.time() + 5
        while time.time() < deadline:
            now = [vccl.vccl_p2p_reginfo(r) for r in range(P)]
            if all(now[r][2] == before[r][2] + it for r in range(P)):
                break
            time.sleep(0.001)
        for r in range(P):
            ready, started, done, addr = now[r]
            assert ready == before[r][0] + it and started == ready and done == ready
            assert addr == recv[r].data_ptr()
    st = vccl.vccl_proxy_stats()
    assert st["ops"] >= 3 and st["bytes"] >= 3 * P * n
    # both proxy threads have run, and neither can have used more processor time than
    # has passed since the module's fixture initialised the library
    cpu = vccl.vccl_proxy_cpu_time()
    assert cpu["sender_ns"] > 0 and cpu["receiver_ns"] > 0
    again = vccl.vccl_proxy_cpu_time()
    assert again["sender_ns"] >= cpu["sender_ns"] and again["receiver_ns"] >= cpu["receiver_ns"]


@pytest.mark.parametrize("kind,sync", [("sdma", "memops"), ("sdma", "event"), ("hip_default", "memops")])
def test_ce_connection_keeps_order_with_many_transfers_outstanding(vccl, kind, sync):
    """Several copy-engine SendRecv calls on the same connections are handed over
    without any wait in between (the calling thread only draws sequence numbers), the
    first of them on a stream that is held back by a long kernel and the rest on a
    second, idle stream.  Every transfer arrives whole in its own receive buffers, a
    connection hands its transfers to the copy engines in the order they were posted
    (a transfer whose stream is ready early waits for its turn), and each record
    has advanced by the number of transfers."""
    torch = require_gpu()
    import time
    P, n, calls = 4, 1 << 20, 6
    to, frm = wl.ring_peers(P)
    sends = [[to_dev(torch, wl.payload_bytes(300 + i, s, n)) for s in range(P)] for i in range(calls)]
    recvs = [[to_dev(torch, np.full(n, SENTINEL, np.uint8)) for _ in range(P)] for _ in range(calls)]
    before = [vccl.vccl_p2p_reginfo(r) for r in range(P)]
    held, idle = torch.cuda.Stream(), torch.cuda.Stream()
    sink = torch.zeros(256 * 256, dtype=torch.float32, device="cuda")
    saved = (vccl.vccl_get_option("ce_kind"), vccl.vccl_get_option("ce_sync"))
    vccl.vccl_set_option("ce_kind", kind)
    vccl.vccl_set_option("ce_sync", sync)
    try:
        torch.cuda.synchronize()
        vccl.vccl_fma_probe(sink, 256, 256, 60000, int(held.cuda_stream))       # about 9 ms of compute
        probe_done = torch.cuda.Event()
        probe_done.record(held)
        t0 = time.perf_counter()
        vccl.vccl_sendrecv(sends[0], [n] * P, to, recvs[0], [n] * P, frm, P, vccl.MODE_CE, int(held.cuda_stream))
        for i in range(1, calls):
            vccl.vccl_sendrecv(sends[i], [n] * P, to, recvs[i], [n] * P, frm, P, vccl.MODE_CE,
                               int(idle.cuda_stream))
        issue_s = time.perf_counter() - t0
        still_running = not probe_done.query()
        torch.cuda.synchronize()
    finally:
        vccl.vccl_set_option("ce_kind", saved[0])
        vccl.vccl_set_option("ce_sync", saved[1])
    for i in range(calls):
        want = [np.zeros(n, np.uint8) for _ in range(P)]
        oracle.sendrecv([to_host(t) for t in sends[i]], [n] * P, to, want, [n] * P, frm)
        for r in range(P):
            assert_same(to_host(recvs[i][r]), want[r], f"transfer {i}, recv[{r}]")
    deadline = time.time() + 5
    while time.time() < deadline:
        now = [vccl.vccl_p2p_reginfo(r) for r in range(P)]
        if all(now[r][2] == before[r][2] + calls for r in range(P)):
            break
        time.sleep(0.001)
    for r in range(P):
        assert now[r][0] == now[r][1] == now[r][2] == before[r][0] + calls
    if kind == "sdma":
        # nothing in the sdma hand-over waits for the device: all calls return while the kernel still runs
        assert still_running, f"handing over {calls} transfers took {issue_s * 1e3:.2f} ms: the held stream's kernel had ended"


@pytest.mark.parametrize("kind,sync", [("sdma", "memops"), ("sdma", "event"), ("sdma", "host"), ("hip_nocu", "memops")])
def test_opposite_directions_on_two_held_streams_all_complete(vccl, kind, sync):
    """The traffic pattern behind the deadlock the paper met with host callbacks (Section
    3.2, item 3): two independent streams carry SendRecv in opposite directions between
    the same pair of ranks, and each transfer is posted while a long kernel still holds
    its own and the other stream.  A runtime that serialises the two streams' host-side
    work stalls here; the proxy treats every operation on its own: all transfers complete
    with the right bytes, and one whose stream becomes ready early is not held up by an
    earlier-posted one whose stream is still busy."""
    torch = require_gpu()
    import time
    n, rounds = (2 << 20) + 48, 3
    fwd = ([1, 0], [1, 0])                               # send_to, recv_from for the pair (0 -> 1 and 1 -> 0)
    a_np = [wl.payload_bytes(7100 + i, 0, n) for i in range(rounds)]      # rank 0 -> rank 1, stream A
    b_np = [wl.payload_bytes(7200 + i, 1, n) for i in range(rounds)]      # rank 1 -> rank 0, stream B
    a_src = [to_dev(torch, x) for x in a_np]
    b_src = [to_dev(torch, x) for x in b_np]
    a_dst = [to_dev(torch, np.full(n + 16, SENTINEL, np.uint8)) for _ in range(rounds)]
    b_dst = [to_dev(torch, np.full(n + 16, SENTINEL, np.uint8)) for _ in range(rounds)]
    null = torch.zeros(16, dtype=torch.uint8, device="cuda")
    A, B = torch.cuda.Stream(), torch.cuda.Stream()
    sink = [torch.zeros(256 * 256, dtype=torch.float32, device="cuda") for _ in range(2)]
    saved = (vccl.vccl_get_option("ce_kind"), vccl.vccl_get_option("ce_sync"))
    vccl.vccl_set_option("ce_kind", kind)
    vccl.vccl_set_option("ce_sync", sync)
    try:
        torch.cuda.synchronize()
        vccl.vccl_fma_probe(sink[0], 128, 256, 20000, int(A.cuda_stream))       # about 3 ms: A is ready first
        vccl.vccl_fma_probe(sink[1], 128, 256, 200000, int(B.cuda_stream))      # about 30 ms
        b_probe_done = torch.cuda.Event()
        b_probe_done.record(B)
        a_first_done = torch.cuda.Event()
        t0 = time.perf_counter()
        for i in range(rounds):
            if not (sync == "host" and i == 0):
                # B's transfer is posted first, while both streams are held
                vccl.vccl_sendrecv([null, b_src[i]], [0, n], fwd[0], [b_dst[i], null], [n, 0], fwd[1], 2,
                                   vccl.MODE_CE, int(B.cuda_stream))
            vccl.vccl_sendrecv([a_src[i], null], [n, 0], fwd[0], [null, a_dst[i]], [0, n], fwd[1], 2,
                               vccl.MODE_CE, int(A.cuda_stream))
            if i == 0:
                a_first_done.record(A)
                if sync == "host":     # a blocking caller can post B's transfer only now
                    vccl.vccl_sendrecv([null, b_src[i]], [0, n], fwd[0], [b_dst[i], null], [n, 0], fwd[1], 2,
                                       vccl.MODE_CE, int(B.cuda_stream))
        posted_s = time.perf_counter() - t0
        a_first_done.synchronize()
        b_still_held = not b_probe_done.query()
        torch.cuda.synchronize()
    finally:
        vccl.vccl_set_option("ce_kind", saved[0])
        vccl.vccl_set_option("ce_sync", saved[1])
    for i in range(rounds):
        want_a, want_b = np.full(n + 16, SENTINEL, np.uint8), np.full(n + 16, SENTINEL, np.uint8)
        oracle.sendrecv([a_np[i], np.zeros(0, np.uint8)], [n, 0], fwd[0], [np.zeros(0, np.uint8), want_a], [0, n], fwd[1])
        oracle.sendrecv([np.zeros(0, np.uint8), b_np[i]], [0, n], fwd[0], [want_b, np.zeros(0, np.uint8)], [n, 0], fwd[1])
        assert_same(to_host(a_dst[i]), want_a, f"round {i}: rank 0 -> 1")
        assert_same(to_host(b_dst[i]), want_b, f"round {i}: rank 1 -> 0")
    if kind == "sdma" and sync != "host":
        # A's first transfer (posted second) finished while B's kernel, and with it B's
        # earlier-posted transfer, was still waiting.  (The hipMemcpyAsync back end shares
        # its internal streams between operations and only has to complete.)
        assert b_still_held, f"posting took {posted_s * 1e3:.1f} ms; A's transfer waited for B's stream"


def test_proxy_window_monitor_sees_copy_engine_operations(vccl):
    """The proxy feeds one window monitor per primitive with the operations it
    issues: message counts advance and the window estimate is a sane copy rate."""
    torch = require_gpu()
    P, n = 4, 8 << 20
    to, frm = wl.ring_peers(P)
    send = [to_dev(torch, wl.payload_bytes(18, s, n)) for s in range(P)]
    recv = [to_dev(torch, np.zeros(n, np.uint8)) for _ in range(P)]
    before = [vccl.vccl_proxy_monitor(k) for k in (0, 1)]
    st = stream_handle(torch)
    for _ in range(12):
        vccl.vccl_sendrecv(send, [n] * P, to, recv, [n] * P, frm, P, vccl.MODE_CE, st)
    for _ in range(5):
        vccl.vccl_alltoall(send, recv, n // P, P, vccl.MODE_CE, st)
    torch.cuda.synchronize()
    import time
    deadline = time.time() + 5
    while time.time() < deadline:
        after = [vccl.vccl_proxy_monitor(k) for k in (0, 1)]
        if after[0]["messages"] == before[0]["messages"] + 12 and after[1]["messages"] == before[1]["messages"] + 5:
            break
        time.sleep(0.001)
    assert after[0]["messages"] == before[0]["messages"] + 12
    assert after[1]["messages"] == before[1]["messages"] + 5
    for k in (0, 1):
        bw = after[k]["last"]["bw_window"]
        assert 1e9 < bw < 2e12, bw            # between 1 GB/s and 2 TB/s of copy rate
        assert after[k]["last"]["outstanding"] == 0
    with pytest.raises(vccl.VcclError):
        vccl.vccl_proxy_monitor(2)
