"""GPU parity, randomised but seeded: many small AlltoAllv / SendRecv / MoE cases with
random layouts, buffer offsets, kernel options and data paths, each compared with
the CPU oracle bit for bit (whole buffers, sentinel-filled)."""
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


def _options(rng, v):
    opts = {"cu_unroll": int(rng.choice([1, 2, 4, 8, 16])), "cu_threads": int(rng.choice([64, 128, 256])),
            "cu_nontemporal": int(rng.choice([0, 1, 2])), "cu_fast_path": int(rng.choice([0, 1]))}
    if rng.random() < 0.25:
        opts["cu_max_wg"] = int(rng.choice([1, 7, 64, 300]))
    saved = {k: v.vccl_get_option(k) for k in opts}
    for k, val in opts.items():
        v.vccl_set_option(k, val)
    return opts, saved


def _restore(v, saved):
    for k, val in saved.items():
        v.vccl_set_option(k, val)


@pytest.mark.parametrize("case", range(40))
def test_alltoallv_random_case(vccl, case):
    torch = require_gpu()
    rng = np.random.Generator(np.random.PCG64(9000 + case))
    P = int(rng.integers(1, 13))
    scale = int(rng.choice([40, 3000, 70000, 400000]))
    align = int(rng.choice([1, 1, 16]))
    lay = wl.random_layout(9100 + case, P, scale, align=align, zero_fraction=float(rng.choice([0.0, 0.2, 0.6])))
    send_np = [wl.payload_bytes(9200 + case, s, int(lay["send_sizes"][s])) for s in range(P)]
    # offsets: byte-granular for byte-granular layouts, multiples of 16 (off the tile boundary) otherwise
    step = 1 if align == 1 else 16
    ms = [int(rng.integers(0, 70)) * step for _ in range(P)]
    mr = [int(rng.integers(0, 70)) * step for _ in range(P)]
    mode = vccl.MODE_CE if rng.random() < 0.3 else vccl.MODE_CU
    opts, saved = _options(rng, vccl)
    try:
        send = [to_dev(torch, send_np[s], ms[s]) for s in range(P)]
        recv_np = [np.full(int(lay["recv_sizes"][r]), SENTINEL, dtype=np.uint8) for r in range(P)]
        recv = [to_dev(torch, recv_np[r], mr[r]) for r in range(P)]
        vccl.vccl_alltoallv(send, lay["sendcounts"], lay["sdispls"], recv, lay["recvcounts"], lay["rdispls"],
                            P, mode, stream_handle(torch))
        torch.cuda.synchronize()
    finally:
        _restore(vccl, saved)
    oracle.alltoallv(send_np, lay["sendcounts"], lay["sdispls"], recv_np, lay["recvcounts"], lay["rdispls"])
    for r in range(P):
        assert_same(to_host(recv[r]), recv_np[r], f"case {case} {opts} mode {mode} recv[{r}]")


@pytest.mark.parametrize("case", range(12))
def test_sendrecv_random_permutation(vccl, case):
    """SendRecv over a random permutation of the ranks (not only the ring), random sizes
    including zero, every mode."""
    torch = require_gpu()
    rng = np.random.Generator(np.random.PCG64(9500 + case))
    P = int(rng.integers(1, 10))
    to = rng.permutation(P).astype(np.int32)
    frm = np.empty(P, dtype=np.int32)
    frm[to] = np.arange(P, dtype=np.int32)
    sizes = [int(rng.choice([0, 1, 15, 4096, 100001, 1 << 20])) for _ in range(P)]
    send_np = [wl.payload_bytes(9600 + case, s, sizes[s]) for s in range(P)]
    rbytes = [sizes[int(frm[r])] for r in range(P)]
    recv_np = [np.full(rbytes[r] + 5, SENTINEL, dtype=np.uint8) for r in range(P)]
    mode = [vccl.MODE_CU, vccl.MODE_CE, vccl.MODE_CU_STAGED][case % 3]
    send = [to_dev(torch, send_np[s], int(rng.integers(0, 16))) for s in range(P)]
    recv = [to_dev(torch, recv_np[r], int(rng.integers(0, 16))) for r in range(P)]
    vccl.vccl_sendrecv(send, sizes, to, recv, rbytes, frm, P, mode, stream_handle(torch))
    if mode == vccl.MODE_CU_STAGED:
        vccl.vccl_sendrecv_staged_status()
    torch.cuda.synchronize()
    oracle.sendrecv(send_np, sizes, to, recv_np, rbytes, frm)
    for r in range(P):
        assert_same(to_host(recv[r]), recv_np[r], f"case {case} mode {mode} recv[{r}]")


@pytest.mark.parametrize("case", range(10))
def test_moe_random_case(vccl, case):
    """Random MoE shapes through pack, per-rank pack and the fused dispatch."""
    torch = require_gpu()
    rng = np.random.Generator(np.random.PCG64(9800 + case))
    P = int(rng.integers(1, 9))
    epr = int(rng.integers(1, 9))
    E = P * epr
    K = int(rng.integers(1, min(E, 12) + 1))
    T = int(rng.choice([1, 37, 513, 2100]))
    row = 16 * int(rng.choice([1, 3, 17, 129, 896]))
    x_np = [wl.payload_bytes(9900 + case, s, T * row) for s in range(P)]
    ids_np = [wl.zipf_topk_expert_ids(9900 + case, s, T, K, E) for s in range(P)]
    x = [to_dev(torch, a) for a in x_np]
    ids = [torch.from_numpy(a.reshape(-1).copy()).cuda() for a in ids_np]
    st = stream_handle(torch)
    # per-slot pack
    packed = [torch.full((T * K * row,), SENTINEL, dtype=torch.uint8, device="cuda") for _ in range(P)]
    counts = torch.zeros((P, E), dtype=torch.int64, device="cuda")
    vccl.vccl_moe_pack(x, ids, P, T, K, row, E, packed, counts, None, None, st)
    # per-rank pack
    packed_r = [torch.full((T * min(K, P) * row,), SENTINEL, dtype=torch.uint8, device="cuda") for _ in range(P)]
    counts_r = torch.zeros((P, P), dtype=torch.int64, device="cuda")
    slot_row = [torch.zeros(T * K, dtype=torch.int32, device="cuda") for _ in range(P)]
    vccl.vccl_moe_pack_per_rank(x, ids, P, T, K, row, E, epr, packed_r, counts_r, None, slot_row, None, st)
    torch.cuda.synchronize()
    opk = [oracle.moe_pack(x_np[s], ids_np[s], row, E) for s in range(P)]
    lay = oracle.moe_exchange_layout(np.stack([o[2] for o in opk]), epr, row)
    want = [np.zeros(int(lay["recvcounts"][r].sum()), np.uint8) for r in range(P)]
    oracle.alltoallv([o[0] for o in opk], lay["sendcounts"], lay["sdispls"], want, lay["recvcounts"], lay["rdispls"])
    for s in range(P):
        assert_same(to_host(packed[s]), opk[s][0], f"case {case} packed[{s}]")
        assert np.array_equal(counts[s].cpu().numpy().astype(np.uint64), opk[s][2])
        pk, _, cnt, srow = oracle.moe_pack_dedup(x_np[s], ids_np[s], row, E, epr)
        got = to_host(packed_r[s])
        assert_same(got[:pk.size], pk, f"case {case} per-rank packed[{s}]")
        assert (got[pk.size:] == SENTINEL).all()
        assert np.array_equal(counts_r[s].cpu().numpy().astype(np.uint64), cnt)
        assert np.array_equal(to_host(slot_row[s]).view(np.uint32).astype(np.int64), srow)
    # fused dispatch into exactly sized buffers
    rows = np.array([w.size // row for w in want], dtype=np.uint64)
    recv = [torch.full((int(rows[r]) * row + 16,), SENTINEL, dtype=torch.uint8, device="cuda") for r in range(P)]
    layout = torch.zeros((4, P, P), dtype=torch.int64, device="cuda")
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    vccl.vccl_moe_dispatch_fused(x, ids, P, T, K, row, E, epr, recv, rows, None, layout, None, status, st)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, 0]
    for r in range(P):
        got = to_host(recv[r])
        assert_same(got[:want[r].size], want[r], f"case {case} fused recv[{r}]")
        assert (got[want[r].size:] == SENTINEL).all()
