"""GPU parity: AlltoAll / AlltoAllv through the C boundary against the CPU oracle,
bit for bit, whole buffers (bytes no segment covers must keep the sentinel)."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import SENTINEL, assert_same, require_gpu, stream_handle, to_dev, to_host

pytestmark = pytest.mark.gpu

MODES = ["cu", "ce"]


@pytest.fixture(scope="module")
def vccl():
    require_gpu()
    import paper_2510_00991_amd as v
    v.vccl_init(0, 64)
    yield v
    v.vccl_finalize()


def _mode(v, name):
    return {"cu": v.MODE_CU, "ce": v.MODE_CE}[name]


def _run_v(torch, v, lay, send_np, mode, misalign_send=None, misalign_recv=None, stream=None):
    P = len(send_np)
    ms = misalign_send or [0] * P
    mr = misalign_recv or [0] * P
    send = [to_dev(torch, send_np[s], ms[s]) for s in range(P)]
    recv_np = [np.full(int(lay["recv_sizes"][r]), SENTINEL, dtype=np.uint8) for r in range(P)]
    recv = [to_dev(torch, recv_np[r], mr[r]) for r in range(P)]
    v.vccl_alltoallv(send, lay["sendcounts"], lay["sdispls"], recv, lay["recvcounts"], lay["rdispls"],
                     P, mode, stream_handle(torch, stream))
    torch.cuda.synchronize()
    oracle.alltoallv(send_np, lay["sendcounts"], lay["sdispls"], recv_np, lay["recvcounts"],
                     lay["rdispls"])
    for r in range(P):
        assert_same(to_host(recv[r]), recv_np[r], f"recv[{r}]")
    for s in range(P):
        assert_same(to_host(send[s]), send_np[s], f"send[{s}] must be unchanged")


@pytest.mark.parametrize("mode", MODES)
def test_config1_alltoall_p4_64k(vccl, mode):
    """P = 4, equal 64 KiB blocks, uint8 payload from the seeded generator."""
    torch = require_gpu()
    P, c = 4, 65536
    seed = wl.config_seed(1)
    send_np = [wl.payload_bytes(seed, s, P * c) for s in range(P)]
    recv_np = [np.full(P * c, SENTINEL, dtype=np.uint8) for _ in range(P)]
    send = [to_dev(torch, a) for a in send_np]
    recv = [to_dev(torch, a) for a in recv_np]
    vccl.vccl_alltoall(send, recv, c, P, _mode(vccl, mode), stream_handle(torch))
    torch.cuda.synchronize()
    oracle.alltoall(send_np, recv_np, c)
    for r in range(P):
        assert_same(to_host(recv[r]), recv_np[r], f"recv[{r}]")


@pytest.mark.parametrize("mode", MODES)
def test_config2_alltoall_p8_16m_full_size(vccl, mode):
    """P = 8, 16 MiB per peer (1 GiB sent), random 16-bit patterns; the launch
    configuration is the one the benchmark times."""
    torch = require_gpu()
    P, c = 8, 16 << 20
    seed = wl.config_seed(2)
    send_np = [wl.payload_bytes(seed, s, P * c) for s in range(P)]
    send = [to_dev(torch, a) for a in send_np]
    recv = [torch.full((P * c,), SENTINEL, dtype=torch.uint8, device="cuda") for _ in range(P)]
    vccl.vccl_alltoall(send, recv, c, P, _mode(vccl, mode), stream_handle(torch))
    torch.cuda.synchronize()
    recv_np = [np.empty(P * c, dtype=np.uint8) for _ in range(P)]
    oracle.alltoall(send_np, recv_np, c, threads=8)
    for r in range(P):
        assert_same(to_host(recv[r]), recv_np[r], f"recv[{r}]")


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("seed", range(8))
def test_alltoallv_random_layouts(vccl, mode, seed):
    """Random P in 1..9, counts with zeros, shuffled unaligned segments with gaps,
    buffers starting at odd device addresses."""
    torch = require_gpu()
    rng = np.random.Generator(np.random.PCG64(1000 + seed))
    P = int(rng.integers(1, 10))
    max_count = int(rng.choice([40, 3000, 70000, 300000]))
    lay = wl.random_layout(2000 + seed, P, max_count, align=1)
    send_np = [wl.payload_bytes(seed, s, int(lay["send_sizes"][s])) for s in range(P)]
    _run_v(torch, vccl, lay, send_np, _mode(vccl, mode),
           misalign_send=[int(x) for x in rng.integers(0, 16, P)],
           misalign_recv=[int(x) for x in rng.integers(0, 16, P)])


@pytest.mark.parametrize("mode", MODES)
def test_alltoallv_aligned_layout_spans_tiles(vccl, mode):
    """16-byte aligned fast path: segments of several tiles plus a ragged tail."""
    torch = require_gpu()
    lay = wl.random_layout(77, 5, 700000, align=16, zero_fraction=0.1)
    send_np = [wl.payload_bytes(78, s, int(lay["send_sizes"][s])) for s in range(5)]
    _run_v(torch, vccl, lay, send_np, _mode(vccl, mode))


def test_every_relative_misalignment_cu(vccl):
    """All 16 x 16 (source, destination) address residues modulo 16 in one call:
    segment s -> r reads at residue r and writes at residue s, and its length
    leaves a head, several LDS rounds of body and a tail."""
    torch = require_gpu()
    P = 16
    n = 40000 + 13
    stride = n + 64
    counts = np.full((P, P), n, dtype=np.uint64)
    sd = np.zeros((P, P), dtype=np.uint64)
    rd = np.zeros((P, P), dtype=np.uint64)
    for a in range(P):
        for b in range(P):
            sd[a, b] = b * stride + ((b - (b * stride)) % 16)        # residue b in rank a's buffer
            rd[a, b] = b * stride + ((b - (b * stride)) % 16)        # residue b in rank a's buffer
    lay = {"sendcounts": counts, "sdispls": sd, "recvcounts": counts.copy(), "rdispls": rd,
           "send_sizes": np.full(P, P * stride + 32), "recv_sizes": np.full(P, P * stride + 32)}
    send_np = [wl.payload_bytes(5, s, int(lay["send_sizes"][s])) for s in range(P)]
    _run_v(torch, vccl, lay, send_np, vccl.MODE_CU)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("c", [4096, 65536])
def test_config5_p64_sweep_points(vccl, mode, c):
    """P = 64 (4096 segments, the device descriptor table path) at two sweep sizes."""
    torch = require_gpu()
    P = 64
    seed = wl.config_seed(5)
    send_np = [wl.payload_bytes(seed, s, P * c) for s in range(P)]
    recv_np = [np.full(P * c, SENTINEL, dtype=np.uint8) for _ in range(P)]
    send = [to_dev(torch, a) for a in send_np]
    recv = [to_dev(torch, a) for a in recv_np]
    vccl.vccl_alltoall(send, recv, c, P, _mode(vccl, mode), stream_handle(torch))
    torch.cuda.synchronize()
    oracle.alltoall(send_np, recv_np, c, threads=4)
    for r in range(P):
        assert_same(to_host(recv[r]), recv_np[r], f"recv[{r}]")


def test_config5_p64_1mib_sampled_destinations(vccl):
    """P = 64 at 1 MiB per peer (4 GiB sent, the launch shape the sweep times): the
    receive buffers of sampled destination ranks are checked in full against the
    oracle, which is run on the reduced exchange "everything bound for rank r"."""
    torch = require_gpu()
    P, c = 64, 1 << 20
    seed = wl.config_seed(5)
    send_np = [wl.payload_bytes(seed, s, P * c) for s in range(P)]
    send = [torch.from_numpy(a).cuda() for a in send_np]
    for mode in ("cu", "ce"):
        recv = [torch.full((P * c,), SENTINEL, dtype=torch.uint8, device="cuda") for _ in range(P)]
        vccl.vccl_alltoall(send, recv, c, P, _mode(vccl, mode), stream_handle(torch))
        torch.cuda.synchronize()
        for r in (0, 17, 63):
            counts = np.zeros((P, P), dtype=np.uint64)
            counts[:, r] = c
            sd = np.zeros((P, P), dtype=np.uint64)
            sd[:, r] = r * c
            rd = np.zeros((P, P), dtype=np.uint64)
            rd[r, :] = np.arange(P, dtype=np.uint64) * np.uint64(c)
            want = [np.zeros(16, np.uint8) for _ in range(P)]
            want[r] = np.full(P * c, SENTINEL, dtype=np.uint8)
            oracle.alltoallv(send_np, counts, sd, want, counts.T.copy(), rd, threads=1)
            assert_same(to_host(recv[r]), want[r], f"{mode} recv[{r}]")
        del recv
        torch.cuda.empty_cache()


@pytest.mark.parametrize("k", range(11))
def test_config5_p64_every_sweep_size(vccl, k):
    """P = 64 at every size of the sweep, 4 KiB ... 4 MiB per peer (up to 16 GiB sent), both
    data paths.  The payload is produced on the device (seeded), too large to build on the
    host at the upper sizes; the whole result is checked on the device against the exchange
    law block by block (recv[r] block s == send[s] block r, nothing else touched), and one
    destination rank per size is brought to the host and checked against the oracle."""
    torch = require_gpu()
    P, c = 64, 4096 << k
    g = torch.Generator(device="cuda")
    g.manual_seed(wl.config_seed(5) + k)
    send = [torch.randint(0, 256, (P * c,), dtype=torch.uint8, device="cuda", generator=g) for _ in range(P)]
    r_chk = (7 * k + 3) % P
    send_blocks = [to_host(send[s][r_chk * c:(r_chk + 1) * c]) for s in range(P)]   # everything bound for r_chk
    want = np.full(P * c + 16, SENTINEL, dtype=np.uint8)
    cnt = np.zeros((P, P), dtype=np.uint64)
    cnt[:, r_chk] = c
    z = np.zeros((P, P), dtype=np.uint64)
    rd = np.zeros((P, P), dtype=np.uint64)
    rd[r_chk, :] = np.arange(P, dtype=np.uint64) * np.uint64(c)
    dummy = [np.zeros(16, np.uint8) for _ in range(P)]
    dummy[r_chk] = want
    oracle.alltoallv(send_blocks, cnt, z, dummy, cnt.T.copy(), rd, threads=4)
    for mode in ("cu", "ce"):
        recv = [torch.full((P * c + 16,), SENTINEL, dtype=torch.uint8, device="cuda") for _ in range(P)]
        vccl.vccl_alltoall(send, recv, c, P, _mode(vccl, mode), stream_handle(torch))
        torch.cuda.synchronize()
        for r in range(P):
            got = recv[r][:P * c].view(P, c)
            ref = torch.stack([send[s][r * c:(r + 1) * c] for s in range(P)]) if c <= (1 << 16) else None
            if ref is not None:
                assert torch.equal(got, ref), f"{mode} recv[{r}]"
            else:
                for s in range(P):
                    assert torch.equal(got[s], send[s][r * c:(r + 1) * c]), f"{mode} recv[{r}] block {s}"
            assert bool((recv[r][P * c:] == SENTINEL).all()), f"{mode} recv[{r}] tail"
        assert_same(to_host(recv[r_chk]), want, f"{mode} recv[{r_chk}] against the oracle")
        del recv
    del send
    torch.cuda.empty_cache()


def _with_options(v, opts, fn):
    saved = {k: v.vccl_get_option(k) for k in opts}
    for k, val in opts.items():
        v.vccl_set_option(k, val)
    try:
        fn()
    finally:
        for k, val in saved.items():
            v.vccl_set_option(k, val)


@pytest.mark.parametrize("P,c", [(9, 16), (16, 4096 + 16), (37, 50000 - 50000 % 16), (64, 1 << 20)])
def test_alltoall_pointer_table_kernel(vccl, P, c):
    """Equal-block AlltoAll above 8 ranks derives its segments in the kernel from
    the rank pointers (no descriptor upload); odd P, ragged last tile, and the same
    call with the fast path switched off must all agree with the oracle."""
    torch = require_gpu()
    send_np = [wl.payload_bytes(600 + P, s, P * c) for s in range(P)]
    want = [np.full(P * c + 32, SENTINEL, dtype=np.uint8) for _ in range(P)]
    oracle.alltoall(send_np, want, c, threads=4)
    send = [to_dev(torch, a) for a in send_np]
    for fast in (1, 0):
        recv = [to_dev(torch, np.full(P * c + 32, SENTINEL, dtype=np.uint8)) for _ in range(P)]
        _with_options(vccl, {"cu_fast_path": fast},
                      lambda: vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CU, stream_handle(torch)))
        torch.cuda.synchronize()
        for r in range(P):
            assert_same(to_host(recv[r]), want[r], f"fast={fast} recv[{r}]")


def test_p40_alltoallv_table_path_non_uniform(vccl):
    """More than 64 descriptors of different lengths: the device descriptor table
    and the early exit of workgroups past a short descriptor."""
    torch = require_gpu()
    lay = wl.random_layout(4242, 40, 90000, align=16, zero_fraction=0.3)
    send_np = [wl.payload_bytes(9, s, int(lay["send_sizes"][s])) for s in range(40)]
    _run_v(torch, vccl, lay, send_np, vccl.MODE_CU)
    _with_options(vccl, {"cu_unroll": 1}, lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CU))


@pytest.mark.parametrize("mode", MODES)
def test_skewed_layout_is_cut_into_pieces(vccl, mode):
    """One 40 MB segment among tiny ones, all unaligned: the planner cuts the long
    segment into pieces; heads, tails and cut points must all land exactly."""
    torch = require_gpu()
    P = 4
    counts = np.full((P, P), 9001, dtype=np.uint64)
    counts[2, 1] = 40_000_003
    counts[0, 3] = 0
    counts[3, 3] = 5
    sd = np.zeros((P, P), dtype=np.uint64)
    rd = np.zeros((P, P), dtype=np.uint64)
    ssz, rsz = [], []
    for a in range(P):
        pos = 3
        for b in range(P):
            sd[a, b] = pos
            pos += int(counts[a, b]) + 7
        ssz.append(pos)
        pos = 11
        for b in range(P):
            rd[a, b] = pos
            pos += int(counts[b, a]) + 5
        rsz.append(pos)
    lay = {"sendcounts": counts, "sdispls": sd, "recvcounts": counts.T.copy(), "rdispls": rd,
           "send_sizes": np.array(ssz), "recv_sizes": np.array(rsz)}
    send_np = [wl.payload_bytes(12, s, ssz[s]) for s in range(P)]
    _run_v(torch, vccl, lay, send_np, _mode(vccl, mode))


def test_copy_engines_share_a_skewed_exchange_by_bytes(vccl):
    """An AlltoAllv in which one destination takes most of the bytes (the incast of a
    skewed MoE dispatch): the copy-engine path cuts the long segments and hands every
    piece to the engine with the fewest bytes, so no engine ends up with much more than
    its share (round-robin over the segments put all the long ones on two engines)."""
    torch = require_gpu()
    P = 8
    counts = np.full((P, P), 1 << 20, dtype=np.uint64)
    counts[:, 0] = 96 << 20                       # everyone sends 96 MiB to rank 0
    sd = np.zeros((P, P), dtype=np.uint64)
    rd = np.zeros((P, P), dtype=np.uint64)
    sd[:, 1:] = np.cumsum(counts[:, :-1], axis=1)
    rc = counts.T.copy()
    rd[:, 1:] = np.cumsum(rc[:, :-1], axis=1)
    lay = {"sendcounts": counts, "sdispls": sd, "recvcounts": rc, "rdispls": rd,
           "send_sizes": counts.sum(axis=1), "recv_sizes": rc.sum(axis=1)}
    send_np = [wl.payload_bytes(15, s, int(lay["send_sizes"][s])) for s in range(P)]
    before = [int(x) for x in vccl.vccl_get_option("ce_engine_bytes").split(",")]
    _run_v(torch, vccl, lay, send_np, vccl.MODE_CE)
    after = [int(x) for x in vccl.vccl_get_option("ce_engine_bytes").split(",")]
    got = np.array(after) - np.array(before)
    assert got.sum() == int(counts.sum())
    assert len(got) == int(vccl.vccl_get_option("ce_engines"))
    assert got.max() <= 1.25 * got.mean(), got.tolist()


@pytest.mark.parametrize("opts", [{"cu_max_wg": 1}, {"cu_max_wg": 8}, {"cu_max_wg": 100},
                                  {"cu_wg_per_cu": 1}, {"cu_wg_per_cu": 8}])
def test_capped_grid_strides_over_descriptors_and_tiles(vccl, opts):
    """A grid smaller than the tile count (the co-run study caps it) still copies everything."""
    torch = require_gpu()
    lay = wl.random_layout(555, 6, 400000, align=1, zero_fraction=0.2)
    send_np = [wl.payload_bytes(13, s, int(lay["send_sizes"][s])) for s in range(6)]
    _with_options(vccl, opts, lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CU))
    lay = wl.random_layout(556, 12, 30000, align=16, zero_fraction=0.0)    # 144 descriptors: table path
    send_np = [wl.payload_bytes(14, s, int(lay["send_sizes"][s])) for s in range(12)]
    _with_options(vccl, opts, lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CU))


@pytest.mark.parametrize("unroll", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("nt", [0, 1, 2])
def test_copy_kernel_variants(vccl, unroll, nt):
    """Every unroll and access policy of the general kernel (byte-granular layout) and of
    the all-aligned kernel at both workgroup sizes (16-byte layout, ragged last tiles)."""
    torch = require_gpu()
    lay = wl.random_layout(31, 4, 500000, align=1)
    send_np = [wl.payload_bytes(32, s, int(lay["send_sizes"][s])) for s in range(4)]
    _with_options(vccl, {"cu_unroll": unroll, "cu_nontemporal": nt},
                  lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CU))
    lay = wl.random_layout(33, 5, 300000, align=16, zero_fraction=0.1)
    send_np = [wl.payload_bytes(34, s, int(lay["send_sizes"][s])) for s in range(5)]
    for threads in (64, 128, 256):
        _with_options(vccl, {"cu_unroll": unroll, "cu_nontemporal": nt, "cu_threads": threads},
                      lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CU))
        P, c = 11, 70000 - 70000 % 16       # pointer-table kernel
        a2a_np = [wl.payload_bytes(35, s, P * c) for s in range(P)]
        want = [np.full(P * c + 32, SENTINEL, dtype=np.uint8) for _ in range(P)]
        oracle.alltoall(a2a_np, want, c, threads=4)
        send = [to_dev(torch, a) for a in a2a_np]
        recv = [to_dev(torch, np.full(P * c + 32, SENTINEL, dtype=np.uint8)) for _ in range(P)]
        _with_options(vccl, {"cu_unroll": unroll, "cu_nontemporal": nt, "cu_threads": threads},
                      lambda: vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CU, stream_handle(torch)))
        torch.cuda.synchronize()
        for r in range(P):
            assert_same(to_host(recv[r]), want[r], f"threads={threads} recv[{r}]")


@pytest.mark.parametrize("shift_send,shift_recv", [(16, 16), (528, 0), (0, 1008), (48, 4080)])
def test_buffers_off_the_tile_boundary(vccl, shift_send, shift_recv):
    """16-byte aligned buffers that start between tile boundaries: tiles are cut at
    destination multiples of the tile size, so the first tile of a segment is short
    (all-aligned kernel, general kernel, and the pointer-table kernel)."""
    torch = require_gpu()
    P = 5
    lay = wl.random_layout(71, P, 300000, align=16, zero_fraction=0.1)
    send_np = [wl.payload_bytes(72, s, int(lay["send_sizes"][s])) for s in range(P)]
    ms, mr = [shift_send] * P, [shift_recv] * P
    for threads in (64, 256):
        _with_options(vccl, {"cu_threads": threads},
                      lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CU, ms, mr))
    _with_options(vccl, {"cu_fast_path": 0}, lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CU, ms, mr))
    _with_options(vccl, {"cu_unroll": 4}, lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CU, ms, mr))
    lay1 = wl.random_layout(73, P, 200000, align=1)          # byte-granular counts on shifted buffers
    send1 = [wl.payload_bytes(74, s, int(lay1["send_sizes"][s])) for s in range(P)]
    _run_v(torch, vccl, lay1, send1, vccl.MODE_CU, ms, mr)
    P, c = 11, 70000 - 70000 % 16                             # pointer-table kernel
    a2a_np = [wl.payload_bytes(75, s, P * c) for s in range(P)]
    want = [np.full(P * c + 32, SENTINEL, dtype=np.uint8) for _ in range(P)]
    oracle.alltoall(a2a_np, want, c, threads=4)
    send = [to_dev(torch, a, shift_send) for a in a2a_np]
    for unroll in (1, 2):
        recv = [to_dev(torch, np.full(P * c + 32, SENTINEL, dtype=np.uint8), shift_recv) for _ in range(P)]
        _with_options(vccl, {"cu_unroll": unroll},
                      lambda: vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CU, stream_handle(torch)))
        torch.cuda.synchronize()
        for r in range(P):
            assert_same(to_host(recv[r]), want[r], f"unroll={unroll} recv[{r}]")


@pytest.mark.parametrize("kind", ["hip_nocu", "hip_default"])
def test_event_ordered_copy_backends_are_bit_exact_too(vccl, kind):
    """The hipMemcpyAsync back ends of the copy-engine mode (event ordering)."""
    torch = require_gpu()
    lay = wl.random_layout(91, 5, 200000, align=1)
    send_np = [wl.payload_bytes(92, s, int(lay["send_sizes"][s])) for s in range(5)]
    _with_options(vccl, {"ce_kind": kind}, lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CE))
    _with_options(vccl, {"ce_kind": kind, "ce_streams": 1},
                  lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CE))


@pytest.mark.parametrize("seed", [3, 5])
def test_sdma_host_sync_mode(vccl, seed):
    """SDMA back end without stream memory operations (the call blocks until done)."""
    torch = require_gpu()
    rng = np.random.Generator(np.random.PCG64(seed))
    P = int(rng.integers(2, 8))
    lay = wl.random_layout(700 + seed, P, 150000, align=1)
    send_np = [wl.payload_bytes(seed, s, int(lay["send_sizes"][s])) for s in range(P)]
    _with_options(vccl, {"ce_sync": "host"}, lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CE))
    _with_options(vccl, {"ce_sync": "host", "ce_max_engines": 1},
                  lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CE))


@pytest.mark.parametrize("sync", ["memops", "event"])
def test_engines_that_refuse_a_copy_are_passed_over(vccl, sync):
    """The error path of the SDMA back end, forced from the host (option ce_test_refuse
    makes the proxy treat the listed engines as refusing every copy): with some engines
    refusing, their pieces go to the others; with all of them refusing, the pieces are
    copied through the HIP runtime before the operation completes.  Either way the call's
    stream is released only with complete receive buffers, and no error is left behind."""
    torch = require_gpu()
    lay = wl.random_layout(4100, 6, 3 << 20, align=16)
    send_np = [wl.payload_bytes(4101, s, int(lay["send_sizes"][s])) for s in range(6)]
    refused0 = int(vccl.vccl_get_option("ce_refused"))
    errors0 = int(vccl.vccl_get_option("ce_errors"))
    _with_options(vccl, {"ce_sync": sync, "ce_test_refuse": 0x5555},
                  lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CE))
    assert int(vccl.vccl_get_option("ce_refused")) == refused0, "another engine takes a refused piece"
    _with_options(vccl, {"ce_sync": sync, "ce_test_refuse": 0xFFFF},
                  lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CE))
    assert int(vccl.vccl_get_option("ce_refused")) > refused0, "no engine left: the pieces took the HIP copy"
    assert int(vccl.vccl_get_option("ce_errors")) == errors0
    assert int(vccl.vccl_get_option("ce_test_refuse")) == 0


def test_proxy_sleeping_on_its_estimates_and_polling_without_pause(vccl):
    """The sender proxy sleeps until an operation is about due (what operations of the same
    shape took before; a model for a shape not yet seen) or, with ce_proxy_poll = 1, polls
    without pause as the proxy of Section 3.1 does.  The same exchange repeated under both,
    with a shape change in between so that remembered and first-seen shapes alternate: right
    bytes every time."""
    torch = require_gpu()
    with pytest.raises(vccl.VcclError):
        vccl.vccl_set_option("ce_proxy_poll", 2)
    lays = [wl.random_layout(4200 + k, 5, size, align=16) for k, size in enumerate((64 << 10, 1 << 20, 6 << 20))]
    sends = [[wl.payload_bytes(4300 + k, s, int(lay["send_sizes"][s])) for s in range(5)]
             for k, lay in enumerate(lays)]
    for poll in (0, 1, 0):
        for rep in range(3):
            for lay, send_np in zip(lays, sends):
                _with_options(vccl, {"ce_proxy_poll": poll},
                              lambda: _run_v(torch, vccl, lay, send_np, vccl.MODE_CE))
    assert vccl.vccl_get_option("ce_proxy_poll") == "0"


def test_small_message_alltoall_on_the_copy_engines(vccl):
    """An AlltoAll of many small blocks on the copy engines (2304 copies of 4 KiB + 16 B,
    one per block): right bytes, also when some engines refuse and their pieces are offered
    to the others."""
    torch = require_gpu()
    P, c = 48, 4096 + 16
    send_np = [wl.payload_bytes(6100, s, P * c) for s in range(P)]
    want = [np.full(P * c + 32, SENTINEL, dtype=np.uint8) for _ in range(P)]
    oracle.alltoall(send_np, want, c, threads=4)
    send = [to_dev(torch, a) for a in send_np]
    st = stream_handle(torch)
    copies0 = vccl.vccl_proxy_stats()["copies"]
    for refuse in (0, 0x0A0A):
        recv = [to_dev(torch, np.full(P * c + 32, SENTINEL, np.uint8)) for _ in range(P)]
        _with_options(vccl, {"ce_test_refuse": refuse},
                      lambda: vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CE, st))
        torch.cuda.synchronize()
        for r in range(P):
            assert_same(to_host(recv[r]), want[r], f"refuse={refuse:#x} recv[{r}]")
    assert vccl.vccl_proxy_stats()["copies"] - copies0 == 2 * P * P
    assert int(vccl.vccl_get_option("ce_errors")) == 0


@pytest.mark.parametrize("side", ["recv", "send", "both"])
def test_pitched_copies_for_buffers_at_a_constant_stride(vccl, side):
    """Equal-block AlltoAll on the copy engines when the rank buffers of one side are slices of
    one allocation at a constant stride: the P blocks of a rank go as ONE pitched copy (P in
    place of P * P).  Right bytes for either side (or both) at a constant stride, with gaps
    between the rank buffers left untouched; the same when every pitched copy is refused and
    its rows go as plain copies; nothing pitched when switched off or when no side qualifies."""
    torch = require_gpu()
    P, c, gap = 24, 4096 + 48, 256
    send_np = [wl.payload_bytes(6300, s, P * c) for s in range(P)]
    want = [np.full(P * c, SENTINEL, dtype=np.uint8) for _ in range(P)]
    oracle.alltoall(send_np, want, c, threads=4)
    st = stream_handle(torch)

    def buffers(strided, fill):
        if strided:
            slab = torch.full((P, P * c + gap), SENTINEL, dtype=torch.uint8, device="cuda")
            views = [slab[r, :P * c] for r in range(P)]
        else:
            slab = None
            views = [torch.full((P * c + 16 * (r % 3),), SENTINEL, dtype=torch.uint8, device="cuda")[:P * c] for r in range(P)]
        if fill is not None:
            for r in range(P):
                views[r].copy_(torch.from_numpy(fill[r]))
        return slab, views

    _, send = buffers(side in ("send", "both"), send_np)
    for mode_opt, refuse, expect_pitched in ((2, 0, P), (2, 0x10000, 0), (0, 0, 0)):
        slab, recv = buffers(side in ("recv", "both"), None)
        before = int(vccl.vccl_get_option("ce_pitched_copies"))
        copies0 = vccl.vccl_proxy_stats()["copies"]
        _with_options(vccl, {"ce_pitched": mode_opt, "ce_test_refuse": refuse},
                      lambda: vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CE, st))
        torch.cuda.synchronize()
        what = f"side={side} ce_pitched={mode_opt} refuse={refuse:#x}"
        for r in range(P):
            assert_same(to_host(recv[r]), want[r], f"{what} recv[{r}]")
        if slab is not None:
            assert bool((slab[:, P * c:] == SENTINEL).all()), what + ": bytes between the rank buffers"
        assert int(vccl.vccl_get_option("ce_pitched_copies")) - before == expect_pitched, what
        assert vccl.vccl_proxy_stats()["copies"] - copies0 == (P if expect_pitched else P * P), what
    assert int(vccl.vccl_get_option("ce_errors")) == 0


@pytest.mark.parametrize("P,c", [(2, 16), (3, 1 << 20), (5, 65536 + 16), (64, 48)])
def test_pitched_copies_at_the_edges_of_their_shapes(vccl, P, c):
    """Forced pitched copies for the smallest exchange, for wide rows, for a width that is no
    power of two and for many ranks with tiny blocks: whatever the runtime makes of a shape -
    it may take the pitched copy or refuse it, in which case the rows go as plain copies -
    the bytes are right and nothing is left in error."""
    torch = require_gpu()
    send_np = [wl.payload_bytes(6500 + P, s, P * c) for s in range(P)]
    want = [np.full(P * c, SENTINEL, dtype=np.uint8) for _ in range(P)]
    oracle.alltoall(send_np, want, c, threads=2)
    send = [to_dev(torch, a) for a in send_np]
    slab = torch.full((P, P * c + 64), SENTINEL, dtype=torch.uint8, device="cuda")
    recv = [slab[r, :P * c] for r in range(P)]
    before = int(vccl.vccl_get_option("ce_pitched_copies"))
    _with_options(vccl, {"ce_pitched": 2}, lambda: vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CE, stream_handle(torch)))
    torch.cuda.synchronize()
    for r in range(P):
        assert_same(to_host(recv[r]), want[r], f"P={P} c={c} recv[{r}]")
    assert bool((slab[:, P * c:] == SENTINEL).all())
    assert int(vccl.vccl_get_option("ce_pitched_copies")) - before in (0, P)
    assert int(vccl.vccl_get_option("ce_errors")) == 0


def test_pitched_copies_are_chosen_where_they_pay(vccl):
    """With the default setting the library takes pitched copies for many ranks and small
    blocks (P = 64, 4 KiB: 64 copies in place of 4096) and plain ones for large blocks or few
    ranks; rank buffers that are not at a constant stride always go as plain copies."""
    torch = require_gpu()
    st = stream_handle(torch)
    for P, c, pitched in ((64, 4096, True), (64, 64 << 10, False), (8, 4096, False)):
        send_np = [wl.payload_bytes(6400 + P, s, P * c) for s in range(P)]
        want = [np.full(P * c, SENTINEL, dtype=np.uint8) for _ in range(P)]
        oracle.alltoall(send_np, want, c, threads=4)
        send = [to_dev(torch, a) for a in send_np]
        slab = torch.full((P, P * c), SENTINEL, dtype=torch.uint8, device="cuda")
        recv = [slab[r] for r in range(P)]
        before = int(vccl.vccl_get_option("ce_pitched_copies"))
        vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CE, st)
        torch.cuda.synchronize()
        for r in range(P):
            assert_same(to_host(recv[r]), want[r], f"P={P} c={c} recv[{r}]")
        assert int(vccl.vccl_get_option("ce_pitched_copies")) - before == (P if pitched else 0), (P, c)
    with pytest.raises(vccl.VcclError):
        vccl.vccl_set_option("ce_pitched", 3)
    with pytest.raises(vccl.VcclError):
        vccl.vccl_set_option("ce_pitched_copies", 1)


def test_many_copy_engine_operations_in_flight(vccl):
    """Several copy-engine calls queued back to back on two streams before any
    synchronisation: operation slots are recycled and every result is right."""
    torch = require_gpu()
    P, c = 4, 256 << 10
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    send = [[torch.from_numpy(wl.payload_bytes(100 + k, s, P * c)).cuda() for s in range(P)] for k in range(2)]
    recv = [[torch.zeros(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)] for _ in range(2)]
    torch.cuda.synchronize()
    for it in range(40):
        k = it % 2
        vccl.vccl_alltoall(send[k], recv[k], c, P, vccl.MODE_CE, stream_handle(torch, streams[k]))
    torch.cuda.synchronize()
    for k in range(2):
        want = [np.zeros(P * c, np.uint8) for _ in range(P)]
        oracle.alltoall([wl.payload_bytes(100 + k, s, P * c) for s in range(P)], want, c)
        for r in range(P):
            assert_same(to_host(recv[k][r]), want[r], f"stream {k} recv[{r}]")


@pytest.mark.parametrize("mode", MODES)
def test_edge_cases(vccl, mode):
    torch = require_gpu()
    m = _mode(vccl, mode)
    # P = 1 is the identity
    x_np = wl.payload_bytes(1, 0, 1000)
    x = to_dev(torch, x_np, 3)
    y = to_dev(torch, np.full(1000, SENTINEL, np.uint8), 5)
    vccl.vccl_alltoall([x], [y], 1000, 1, m, stream_handle(torch))
    torch.cuda.synchronize()
    assert_same(to_host(y), x_np, "P=1 identity")
    # all-zero counts: nothing happens, NULL buffers are fine
    z = np.zeros((3, 3), dtype=np.uint64)
    vccl.vccl_alltoallv([0, 0, 0], z, z, [0, 0, 0], z, z, 3, m, stream_handle(torch))
    # zero bytes per peer
    vccl.vccl_alltoall([x], [y], 0, 1, m, stream_handle(torch))
    # single-byte segments
    one = np.ones((2, 2), dtype=np.uint64)
    d = np.array([[0, 1], [0, 1]], dtype=np.uint64)
    s_np = [np.array([10, 11], np.uint8), np.array([20, 21], np.uint8)]
    s_dev = [to_dev(torch, a, 1) for a in s_np]
    r_dev = [to_dev(torch, np.full(3, SENTINEL, np.uint8), 7) for _ in range(2)]
    vccl.vccl_alltoallv(s_dev, one, d, r_dev, one, d, 2, m, stream_handle(torch))
    torch.cuda.synchronize()
    assert to_host(r_dev[0]).tolist() == [10, 20, SENTINEL]
    assert to_host(r_dev[1]).tolist() == [11, 21, SENTINEL]


@pytest.mark.parametrize("mode", MODES + ["ce_host", "ce_event", "ce_memops", "ce_hip"])
def test_stream_ordering(vccl, mode):
    """The exchange starts after earlier work on the caller's stream and later work
    on that stream sees the received data (a side stream, repeated)."""
    torch = require_gpu()
    opts = {"ce_host": {"ce_sync": "host"}, "ce_event": {"ce_sync": "event"}, "ce_memops": {"ce_sync": "memops"},
            "ce_hip": {"ce_kind": "hip_nocu"}}.get(mode, {})
    saved = {k: vccl.vccl_get_option(k) for k in opts}
    for k, val in opts.items():
        vccl.vccl_set_option(k, val)
    try:
        _stream_ordering_body(torch, vccl, vccl.MODE_CU if mode == "cu" else vccl.MODE_CE)
    finally:
        for k, val in saved.items():
            vccl.vccl_set_option(k, val)


def _stream_ordering_body(torch, vccl, m):
    P, c = 4, 1 << 20
    side = torch.cuda.Stream()
    send = [torch.zeros(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
    recv = [torch.zeros(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
    snap = [torch.zeros(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
    torch.cuda.synchronize()
    for it in range(1, 6):
        with torch.cuda.stream(side):
            for s in range(P):
                send[s].fill_(it * 10 + s)                       # producer on the same stream
            vccl.vccl_alltoall(send, recv, c, P, m, stream_handle(torch, side))
            for r in range(P):
                snap[r].copy_(recv[r])                           # consumer on the same stream
        side.synchronize()
        for r in range(P):
            got = to_host(snap[r]).reshape(P, c)
            for s in range(P):
                assert (got[s] == it * 10 + s).all(), (m, it, r, s)


@pytest.mark.parametrize("mode,nthreads", [("cu", 4), ("ce", 4), ("cu", 12)])
def test_concurrent_callers_on_their_own_streams(vccl, mode, nthreads):
    """Several host threads (once more of them than the descriptor staging ring has
    slots), each with its own stream and buffers, call the library at the same time
    (the C boundary promises thread safety); every result is right."""
    import threading
    torch = require_gpu()
    P, c, rounds = 12, 96 << 10, 6                    # 144 descriptors: the shared staging ring is used
    m = _mode(vccl, mode)
    data = []
    for t in range(nthreads):
        lay = wl.random_layout(3000 + t, P, c, align=16, zero_fraction=0.1)
        send_np = [wl.payload_bytes(40 + t, s, int(lay["send_sizes"][s])) for s in range(P)]
        want = [np.full(int(lay["recv_sizes"][r]), SENTINEL, dtype=np.uint8) for r in range(P)]
        oracle.alltoallv(send_np, lay["sendcounts"], lay["sdispls"], want, lay["recvcounts"], lay["rdispls"])
        send = [to_dev(torch, a) for a in send_np]
        recv = [to_dev(torch, np.full(int(lay["recv_sizes"][r]), SENTINEL, dtype=np.uint8)) for r in range(P)]
        data.append((lay, send, recv, want, torch.cuda.Stream()))
    torch.cuda.synchronize()
    errors = []

    def worker(t):
        try:
            lay, send, recv, want, stream = data[t]
            for _ in range(rounds):
                vccl.vccl_alltoallv(send, lay["sendcounts"], lay["sdispls"], recv, lay["recvcounts"],
                                    lay["rdispls"], P, m, stream_handle(torch, stream))
            stream.synchronize()
        except Exception as e:          # noqa: BLE001 - reported below
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(nthreads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=60)
    assert not errors, errors
    assert not any(th.is_alive() for th in threads)
    torch.cuda.synchronize()
    for t in range(nthreads):
        lay, send, recv, want, _ = data[t]
        for r in range(P):
            assert_same(to_host(recv[r]), want[r], f"thread {t} recv[{r}]")


@pytest.mark.parametrize("P,c", [(8, 1 << 16), (20, 4096)])
def test_cu_path_replays_from_a_hip_graph(vccl, P, c):
    """The compute-unit AlltoAll with its descriptors in the kernel arguments (P = 8) or
    derived from the rank pointers (P = 20) is a single launch with no allocation, copy
    or wait around it, so it can be captured in a HIP graph.  The graph is replayed
    several times on fresh inputs, with eager work and synchronisations in between,
    and every replay is checked against the oracle."""
    torch = require_gpu()
    send = [torch.zeros(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
    recv = [torch.zeros(P * c + 32, dtype=torch.uint8, device="cuda") for _ in range(P)]
    vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CU, stream_handle(torch))      # eager warm-up
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CU, stream_handle(torch))
    for rep in range(3):
        send_np = [wl.payload_bytes(800 + rep, s, P * c) for s in range(P)]
        for s in range(P):
            send[s].copy_(torch.from_numpy(send_np[s]))
        for r in range(P):
            recv[r].fill_(SENTINEL)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want = [np.full(P * c + 32, SENTINEL, dtype=np.uint8) for _ in range(P)]
        oracle.alltoall(send_np, want, c, threads=4)
        for r in range(P):
            assert_same(to_host(recv[r]), want[r], f"replay {rep} recv[{r}]")


def test_copy_engine_calls_refuse_a_capturing_stream(vccl):
    """A copy-engine call is carried out once by a host thread, so it cannot live in a graph:
    on a capturing stream it fails before anything is recorded, the capture itself stays
    valid, and the compute-unit call recorded beside it replays."""
    torch = require_gpu()
    P, c = 4, 4096
    send_np = [wl.payload_bytes(880, s, P * c) for s in range(P)]
    send = [to_dev(torch, a) for a in send_np]
    recv = [torch.full((P * c,), SENTINEL, dtype=torch.uint8, device="cuda") for _ in range(P)]
    vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CU, stream_handle(torch))      # eager warm-up
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        with pytest.raises(vccl.VcclError) as e:
            vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CE, stream_handle(torch))
        assert e.value.code == -6
        with pytest.raises(vccl.VcclError):
            vccl.vccl_sendrecv(send, [c] * P, [1, 0, 3, 2], recv, [c] * P, [1, 0, 3, 2], P, vccl.MODE_CE,
                               stream_handle(torch))
        vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CU, stream_handle(torch))
    for r in range(P):
        recv[r].fill_(SENTINEL)
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    want = [np.full(P * c, SENTINEL, dtype=np.uint8) for _ in range(P)]
    oracle.alltoall(send_np, want, c, threads=2)
    for r in range(P):
        assert_same(to_host(recv[r]), want[r], f"replayed recv[{r}]")
    vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CE, stream_handle(torch))      # outside a capture it works as ever
    torch.cuda.synchronize()
    assert int(vccl.vccl_get_option("ce_errors")) == 0


@pytest.mark.parametrize("kind,sync", [("sdma", "memops"), ("sdma", "event"), ("sdma", "host"), ("hip_nocu", "memops")])
def test_kernels_after_a_copy_engine_exchange_read_fresh_data(vccl, kind, sync):
    """Cache coherence of the copy-engine path: the receive buffers are small enough to
    stay in the L2 caches, a kernel writes and another reads them right before the
    exchange (so their old contents are cached), the copy engines then write them
    behind the caches' back, and a compute kernel on the same stream reads them right
    after.  It must see the new bytes, iteration after iteration.  The bytes to send
    are themselves produced by a kernel right before the exchange: the engines must
    read what that kernel wrote, not what memory held before."""
    torch = require_gpu()
    P, c = 4, 1 << 16
    st = torch.cuda.current_stream()
    send = [torch.zeros(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
    recv = [torch.zeros(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
    saved = (vccl.vccl_get_option("ce_kind"), vccl.vccl_get_option("ce_sync"))
    vccl.vccl_set_option("ce_kind", kind)
    vccl.vccl_set_option("ce_sync", sync)
    try:
        for it in range(25):
            send_np = [wl.payload_bytes(5000 + it, s, P * c) for s in range(P)]
            for s in range(P):
                send[s].copy_(torch.from_numpy(np.bitwise_not(send_np[s])), non_blocking=False)
            for s in range(P):
                send[s].bitwise_not_()          # a kernel produces the bytes to send right before the exchange
            touched = []
            for r in range(P):
                recv[r].fill_(it & 0xFF)                       # a kernel writes the old contents
                touched.append(recv[r].to(torch.int32).sum())    # and a kernel reads them
            vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CE, int(st.cuda_stream))
            seen = [recv[r] ^ 0 for r in range(P)]               # compute kernels read right behind the exchange
            sums = [recv[r].to(torch.int64).sum() for r in range(P)]
            torch.cuda.synchronize()
            want = [np.zeros(P * c, dtype=np.uint8) for _ in range(P)]
            oracle.alltoall(send_np, want, c)
            for r in range(P):
                assert int(touched[r].item()) == (it & 0xFF) * P * c
                assert_same(to_host(seen[r]), want[r], f"iteration {it} recv[{r}] as a kernel saw it")
                assert int(sums[r].item()) == int(want[r].astype(np.int64).sum())
    finally:
        vccl.vccl_set_option("ce_kind", saved[0])
        vccl.vccl_set_option("ce_sync", saved[1])
