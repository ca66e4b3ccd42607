"""Error behaviour of the boundary on a live context (nothing may be enqueued on error)."""
import numpy as np
import pytest

from gpu_util import SENTINEL, require_gpu, stream_handle, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vccl():
    require_gpu()
    import paper_2510_00991_amd as v
    v.vccl_init(0, 8)
    yield v
    v.vccl_finalize()


def test_double_init_and_reinit(vccl):
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_init(0, 8)
    assert e.value.code == -1
    assert vccl.vccl_device_cu_count() > 0


def test_argument_errors(vccl):
    torch = require_gpu()
    x = to_dev(torch, np.zeros(64, np.uint8))
    y = to_dev(torch, np.full(64, SENTINEL, np.uint8))
    st = stream_handle(torch)
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_alltoall([x] * 9, [y] * 9, 4, 9, vccl.MODE_CU, st)        # P > max_ranks
    assert e.value.code == -1
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_alltoall([x], [y], 4, 1, 7, st)                           # unknown mode
    assert e.value.code == -1
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_alltoall([x], [y], 4, 1, vccl.MODE_CU_STAGED, st)         # staged is SendRecv only
    assert e.value.code == -6
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_alltoall([0], [y], 4, 1, vccl.MODE_CU, st)                # NULL with bytes
    assert e.value.code == -1
    c = np.array([[1, 2], [3, 4]], np.uint64)
    d = np.zeros((2, 2), np.uint64)
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_alltoallv([x, x], c, d, [y, y], c, d, 2, vccl.MODE_CU, st)  # not transposed
    assert e.value.code == -2 and "sendcounts[0][1]" in e.value.message
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_sendrecv([x, x], [8, 8], [1, 1], [y, y], [8, 8], [0, 0], 2, vccl.MODE_CU, st)
    assert e.value.code == -1
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_sendrecv([x, x], [8, 4], [1, 0], [y, y], [8, 8], [1, 0], 2, vccl.MODE_CE, st)
    assert e.value.code == -2
    torch.cuda.synchronize()
    assert (to_host(y) == SENTINEL).all(), "a failing call must not write"


def test_unknown_or_bad_options_fail_loudly(vccl):
    for k, val in (("no_such_knob", "1"), ("cu_unroll", "3"), ("cu_unroll", "x"), ("ce_streams", "0"),
                   ("ce_kind", "dma"), ("fifo_chunk_bytes", "1000"), ("check", "-1")):
        with pytest.raises(vccl.VcclError) as e:
            vccl.vccl_set_option(k, val)
        assert e.value.code == -1, (k, val)
    vccl.vccl_set_option("ce_streams", 2)
    assert vccl.vccl_get_option("ce_streams") == "2"
    vccl.vccl_set_option("ce_streams", 4)
    assert vccl.vccl_get_option("ce_kind") == "sdma"
    assert int(vccl.vccl_get_option("ce_engines")) >= 1
    with pytest.raises(vccl.VcclError):
        vccl.vccl_set_option("ce_engines", 4)


def test_overlap_check(vccl):
    torch = require_gpu()
    buf = to_dev(torch, np.arange(256, dtype=np.uint8))
    out = to_dev(torch, np.full(256, SENTINEL, np.uint8))
    st = stream_handle(torch)
    one = np.full((2, 2), 32, np.uint64)
    sd = np.array([[0, 32], [0, 32]], np.uint64)
    rd_overlapping = np.array([[0, 16], [64, 96]], np.uint64)
    vccl.vccl_set_option("check", 1)
    try:
        with pytest.raises(vccl.VcclError) as e:   # two receive segments overlap
            vccl.vccl_alltoallv([buf, buf], one, sd, [out, out], one, rd_overlapping, 2, vccl.MODE_CU, st)
        assert e.value.code == -3
        with pytest.raises(vccl.VcclError) as e:   # in place
            vccl.vccl_alltoall([buf], [buf], 64, 1, vccl.MODE_CE, st)
        assert e.value.code == -3
        rd_ok = np.array([[0, 32], [64, 96]], np.uint64)
        vccl.vccl_alltoallv([buf, buf], one, sd, [out, out], one, rd_ok, 2, vccl.MODE_CU, st)
    finally:
        vccl.vccl_set_option("check", 0)
    torch.cuda.synchronize()


def test_finalize_with_operations_in_flight_drains_them_and_init_works_again(vccl):
    """vccl_finalize while copy-engine and compute-unit operations are still queued behind
    a long kernel: it waits for them (nothing is dropped, nothing hangs), the bytes are
    right, and a new context can be created afterwards.  (The module's context is
    re-created at the end for the tests that follow.)"""
    import oracle
    import workloads as wl
    from gpu_util import assert_same
    torch = require_gpu()
    P, c = 4, 1 << 18
    send_np = [wl.payload_bytes(31, s, P * c) for s in range(P)]
    send = [to_dev(torch, a) for a in send_np]
    recv_ce = [to_dev(torch, np.full(P * c, SENTINEL, np.uint8)) for _ in range(P)]
    recv_cu = [to_dev(torch, np.full(P * c, SENTINEL, np.uint8)) for _ in range(P)]
    sink = torch.zeros(256 * 256, dtype=torch.float32, device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    vccl.vccl_fma_probe(sink, 256, 256, 30000, int(s1.cuda_stream))          # a few ms of compute first
    vccl.vccl_alltoall(send, recv_ce, c, P, vccl.MODE_CE, int(s1.cuda_stream))
    vccl.vccl_fma_probe(sink, 256, 256, 30000, int(s2.cuda_stream))
    vccl.vccl_alltoall(send, recv_cu, c, P, vccl.MODE_CU, int(s2.cuda_stream))
    try:
        vccl.vccl_finalize()
        torch.cuda.synchronize()
        want = [np.zeros(P * c, np.uint8) for _ in range(P)]
        oracle.alltoall(send_np, want, c)
        for r in range(P):
            assert_same(to_host(recv_ce[r]), want[r], f"copy-engine recv[{r}]")
            assert_same(to_host(recv_cu[r]), want[r], f"compute-unit recv[{r}]")
        with pytest.raises(vccl.VcclError) as e:
            vccl.vccl_alltoall(send, recv_cu, c, P, vccl.MODE_CU, stream_handle(torch))
        assert e.value.code == -5
    finally:
        vccl.vccl_init(0, 8)
    for r in range(P):
        recv_cu[r].fill_(SENTINEL)
    vccl.vccl_alltoall(send, recv_cu, c, P, vccl.MODE_CE, stream_handle(torch))
    torch.cuda.synchronize()
    for r in range(P):
        assert_same(to_host(recv_cu[r]), want[r], f"recv[{r}] on the new context")


def test_copy_engine_error_counter_is_readable_and_read_only(vccl):
    torch = require_gpu()
    x = [to_dev(torch, np.arange(4096, dtype=np.uint8).repeat(1)) for _ in range(2)]
    y = [to_dev(torch, np.zeros(4096, np.uint8)) for _ in range(2)]
    vccl.vccl_alltoall(x, y, 2048, 2, vccl.MODE_CE, stream_handle(torch))
    torch.cuda.synchronize()
    assert int(vccl.vccl_get_option("ce_errors")) == 0
    with pytest.raises(vccl.VcclError):
        vccl.vccl_set_option("ce_errors", 0)
