"""GPU parity: SendRecv ring (direct on compute units, copy engines, staged FIFO)."""
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


def _modes(v):
    return {"cu": v.MODE_CU, "ce": v.MODE_CE, "staged": v.MODE_CU_STAGED}


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


@pytest.mark.parametrize("mode", ["cu", "ce", "staged"])
def test_ring_small_and_ragged(vccl, mode):
    torch = require_gpu()
    m = _modes(vccl)[mode]
    _ring(torch, vccl, m, [100000, 0, 7, 65536, 1 << 20])
    _ring(torch, vccl, m, [12345], misalign=0)
    _ring(torch, vccl, m, [3 * 524288 + 17, 524288, 524287], misalign=0)


@pytest.mark.parametrize("mode", ["cu", "ce", "staged"])
def test_ring_unaligned_buffers(vccl, mode):
    torch = require_gpu()
    _ring(torch, vccl, _modes(vccl)[mode], [700001, 33, 524288 + 1, 99999], misalign=5)


@pytest.mark.parametrize("mode", ["cu", "ce", "staged"])
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
    m = _modes(vccl)[mode]
    vccl.vccl_sendrecv(send, [n] * P, to, recv, [n] * P, frm, P, m, stream_handle(torch))
    if mode == "staged":
        vccl.vccl_sendrecv_staged_status()
    torch.cuda.synchronize()
    recv_np = [np.empty(n, dtype=np.uint8) for _ in range(P)]
    oracle.sendrecv(send_np, [n] * P, to, recv_np, [n] * P, frm)
    for r in range(P):
        assert_same(to_host(recv[r]), recv_np[r], f"recv[{r}]")


def test_ring_sdma_host_sync(vccl):
    torch = require_gpu()
    vccl.vccl_set_option("ce_sync", "host")
    try:
        _ring(torch, vccl, vccl.MODE_CE, [700001, 33, 524288 + 1, 0, 99999], misalign=3)
    finally:
        vccl.vccl_set_option("ce_sync", "memops")


def test_staged_equals_oracle_fifo_model(vccl):
    """Different chunk / slot settings give the same bytes as the oracle's FIFO model."""
    torch = require_gpu()
    n = 200000
    src_np = wl.payload_bytes(3, 0, n)
    for chunk, slots, wg in ((4096, 1, 1), (8192, 3, 4), (65536, 8, 16)):
        vccl.vccl_set_option("fifo_chunk_bytes", chunk)
        vccl.vccl_set_option("fifo_slots", slots)
        vccl.vccl_set_option("fifo_wg_per_conn", wg)
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
            vccl.vccl_set_option("fifo_chunk_bytes", 524288)
            vccl.vccl_set_option("fifo_slots", 8)
            vccl.vccl_set_option("fifo_wg_per_conn", 8)


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
