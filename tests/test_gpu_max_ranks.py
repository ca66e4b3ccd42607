"""GPU parity at the largest rank count the library accepts (P = 256: 65 536 segments, more
than a launch grid has rows, so workgroups stride over descriptors) and just below it."""
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
    v.vccl_init(0, 256)      # VCCL_MAX_RANKS
    yield v
    v.vccl_finalize()


@pytest.mark.parametrize("P,c,mode", [(256, 64, "cu"), (256, 48, "cu"), (200, 80, "cu"), (128, 256, "cu"),
                                      (128, 4096, "ce")])
def test_alltoall_many_ranks(vccl, P, c, mode):
    torch = require_gpu()
    send_np = [wl.payload_bytes(4000 + P, s, P * c) for s in range(P)]
    want = [np.full(P * c + 16, SENTINEL, dtype=np.uint8) for _ in range(P)]
    oracle.alltoall(send_np, want, c, threads=8)
    # one allocation per side, rank buffers are slices of it (256 separate tensors are slow to make)
    big_s = torch.from_numpy(np.concatenate(send_np)).cuda()
    big_r = torch.full((P * (P * c + 16),), SENTINEL, dtype=torch.uint8, device="cuda")
    send = [big_s[s * P * c:(s + 1) * P * c] for s in range(P)]
    recv = [big_r[r * (P * c + 16):(r + 1) * (P * c + 16)] for r in range(P)]
    m = vccl.MODE_CU if mode == "cu" else vccl.MODE_CE
    vccl.vccl_alltoall(send, recv, c, P, m, stream_handle(torch))
    torch.cuda.synchronize()
    got = to_host(big_r).reshape(P, P * c + 16)
    for r in range(P):
        assert_same(got[r], want[r], f"recv[{r}]")


def test_alltoallv_256_ranks_random_layout(vccl):
    torch = require_gpu()
    P = 256
    lay = wl.random_layout(4242, P, 300, align=1, zero_fraction=0.5)
    send_np = [wl.payload_bytes(4300, s, int(lay["send_sizes"][s])) for s in range(P)]
    recv_np = [np.full(int(lay["recv_sizes"][r]), SENTINEL, dtype=np.uint8) for r in range(P)]
    soff = np.concatenate(([0], np.cumsum([a.size + 16 for a in send_np])))
    roff = np.concatenate(([0], np.cumsum([a.size + 16 for a in recv_np])))
    big_s = torch.zeros(int(soff[-1]), dtype=torch.uint8, device="cuda")
    big_r = torch.full((int(roff[-1]),), SENTINEL, dtype=torch.uint8, device="cuda")
    for s in range(P):
        if send_np[s].size:
            big_s[int(soff[s]):int(soff[s]) + send_np[s].size].copy_(torch.from_numpy(send_np[s]))
    send = [big_s[int(soff[s]):int(soff[s]) + send_np[s].size] for s in range(P)]
    recv = [big_r[int(roff[r]):int(roff[r]) + recv_np[r].size] for r in range(P)]
    send_ptrs = [int(big_s.data_ptr()) + int(soff[s]) for s in range(P)]
    recv_ptrs = [int(big_r.data_ptr()) + int(roff[r]) for r in range(P)]
    vccl.vccl_alltoallv(send_ptrs, lay["sendcounts"], lay["sdispls"], recv_ptrs, lay["recvcounts"], lay["rdispls"],
                        P, vccl.MODE_CU, stream_handle(torch))
    torch.cuda.synchronize()
    oracle.alltoallv(send_np, lay["sendcounts"], lay["sdispls"], recv_np, lay["recvcounts"], lay["rdispls"],
                     threads=8)
    host = to_host(big_r)
    for r in range(P):
        assert_same(host[int(roff[r]):int(roff[r]) + recv_np[r].size], recv_np[r], f"recv[{r}]")
        assert (host[int(roff[r]) + recv_np[r].size:int(roff[r + 1])] == SENTINEL).all()


@pytest.mark.parametrize("P,mode", [(100, "staged"), (256, "staged"), (256, "cu"), (100, "ce")])
def test_sendrecv_ring_many_ranks(vccl, P, mode):
    """A ring over more connections than the staged kernel carries in its arguments
    (the table path) and up to the rank limit; every rank a different message size."""
    torch = require_gpu()
    to, frm = wl.ring_peers(P)
    sizes = [int(4096 + 1000 * (s % 7) + (s % 3)) for s in range(P)]
    send_np = [wl.payload_bytes(4500 + P, s, sizes[s]) for s in range(P)]
    rbytes = [sizes[frm[r]] for r in range(P)]
    want = [np.full(rbytes[r] + 8, SENTINEL, dtype=np.uint8) for r in range(P)]
    oracle.sendrecv(send_np, sizes, to, want, rbytes, frm)
    send = [to_dev(torch, a) for a in send_np]
    recv = [to_dev(torch, np.full(rbytes[r] + 8, SENTINEL, dtype=np.uint8)) for r in range(P)]
    m = {"cu": vccl.MODE_CU, "ce": vccl.MODE_CE, "staged": vccl.MODE_CU_STAGED}[mode]
    for _ in range(2):      # the second staged call reuses the table of the first
        vccl.vccl_sendrecv(send, sizes, to, recv, rbytes, frm, P, m, stream_handle(torch))
    if mode == "staged":
        vccl.vccl_sendrecv_staged_status()
    torch.cuda.synchronize()
    for r in range(P):
        assert_same(to_host(recv[r]), want[r], f"recv[{r}]")


def test_rank_count_above_the_limit_is_rejected(vccl):
    torch = require_gpu()
    P = 257
    z = np.zeros((P, P), dtype=np.uint64)
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_alltoallv([0] * P, z, z, [0] * P, z, z, P, vccl.MODE_CU, stream_handle(torch))
    assert e.value.code == -1
