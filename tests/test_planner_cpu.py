"""Host logic of the compute-unit path, on the CPU: the planner's descriptors must
tile every non-empty segment exactly once, in the rotated order, with cuts on
destination addresses that are multiples of the tile size and a launch grid that
wastes little."""
import numpy as np
import pytest

import paper_2510_00991_amd as vccl
import workloads as wl

TILE = 4096        # bytes per tile at cu_unroll = 1


def _fake_buffers(P, sizes, rng, align=1):
    """Disjoint fake device address ranges (never dereferenced by the planner)."""
    base = 0x7F0000000000
    out = []
    for i in range(P):
        off = int(rng.integers(0, 16)) if align == 1 else 0
        out.append(base + off)
        base += ((int(sizes[i]) + 4096 + 255) // 256) * 256 + 1 << 0
        base = (base + 4095) // 4096 * 4096
    return out


def _tiles(desc, tile_bytes):
    """Tiles start where the destination is a multiple of the tile size; `lead`
    vectors of the first tile lie before the body of the segment."""
    tv = tile_bytes // 16
    nv = (int(desc["bytes"]) - int(desc["head"])) // 16
    lead = ((int(desc["dst"]) + int(desc["head"])) // 16) % tv
    assert int(desc["lead"]) == lead
    return max(1, -(-(nv + lead) // tv))


def _check_plan(lay, send, recv, unroll=1, threads=64):
    P = len(send)
    desc, gx, gy, tile_bytes, aligned = vccl.vccl_plan_alltoallv(
        send, lay["sendcounts"], lay["sdispls"], recv, lay["recvcounts"], lay["rdispls"], P, unroll, threads)
    # walk the descriptors in order against the segments in rotated order
    i = 0
    for k in range(P):
        for r in range(P):
            s = (r + k) % P
            n = int(lay["recvcounts"][r, s])
            if n == 0:
                continue
            src = send[s] + int(lay["sdispls"][s, r])
            dst = recv[r] + int(lay["rdispls"][r, s])
            covered = 0
            first = True
            while covered < n:
                d = desc[i]
                assert int(d["src"]) == src + covered and int(d["dst"]) == dst + covered, (k, r, i)
                assert int(d["bytes"]) > 0
                want_head = min(int(d["bytes"]), (16 - (int(d["dst"]) % 16)) % 16)
                assert int(d["head"]) == want_head
                if not first:
                    assert int(d["dst"]) % tile_bytes == 0 and want_head == 0, "cuts fall on tile boundaries"
                covered += int(d["bytes"])
                first = False
                i += 1
            assert covered == n
    assert i == len(desc), "descriptors beyond the segments"
    if len(desc):
        want_aligned = all(int(d["src"]) % 16 == 0 and int(d["dst"]) % 16 == 0 and int(d["bytes"]) % 16 == 0
                           for d in desc)
        assert aligned == want_aligned
        assert tile_bytes == unroll * 16 * threads
        tiles = [_tiles(d, tile_bytes) for d in desc]
        assert gx == max(tiles) and gy == len(desc)
        waste = gx * len(desc) - sum(tiles)
        assert waste <= sum(tiles) / 16 + len(desc) * 64 + 64, (gx, len(desc), sum(tiles))
    return desc, gx, gy


@pytest.mark.parametrize("seed", range(10))
def test_random_layouts_are_tiled_exactly(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    P = int(rng.integers(1, 12))
    lay = wl.random_layout(seed, P, int(rng.choice([50, 5000, 300000])), align=int(rng.choice([1, 16])))
    send = _fake_buffers(P, lay["send_sizes"], rng)
    recv = _fake_buffers(P, lay["recv_sizes"], rng)
    recv = [a + (1 << 40) for a in recv]
    _check_plan(lay, send, recv, unroll=int(rng.choice([1, 2, 8])), threads=int(rng.choice([64, 128, 256])))


def test_equal_blocks_are_not_cut_and_use_the_fast_kernel():
    P, c = 8, 16 << 20
    lay = wl.equal_layout(P, c)
    send = [0x7F0000000000 + i * (1 << 30) for i in range(P)]
    recv = [0x7E0000000000 + i * (1 << 30) for i in range(P)]
    desc, gx, gy, tile_bytes, aligned = vccl.vccl_plan_alltoallv(send, lay["sendcounts"], lay["sdispls"], recv,
                                                                 lay["recvcounts"], lay["rdispls"], P, 1, 256)
    assert len(desc) == 64 and tile_bytes == TILE and gx == c // TILE and gy == 64 and aligned
    # rotated order: the first P descriptors are the self segments 0->0, 1->1, ...
    for r in range(P):
        assert int(desc[r]["src"]) == send[r] + r * c and int(desc[r]["dst"]) == recv[r] + r * c
    # the next P come from the next rank around the ring
    for r in range(P):
        s = (r + 1) % P
        assert int(desc[P + r]["src"]) == send[s] + r * c and int(desc[P + r]["dst"]) == recv[r] + s * c


def test_skewed_segments_are_cut_into_equal_pieces():
    """A MoE-like skew: one 1 GiB segment among 63 of 16 MiB."""
    P = 8
    counts = np.full((P, P), 16 << 20, dtype=np.uint64)
    counts[0, 0] = 1 << 30
    disp = np.zeros((P, P), dtype=np.uint64)
    for a in range(P):
        disp[a] = np.cumsum(counts[a]) - counts[a]
    rdisp = np.zeros((P, P), dtype=np.uint64)
    for a in range(P):
        rdisp[a] = np.cumsum(counts.T[a]) - counts.T[a]
    lay = {"sendcounts": counts, "sdispls": disp, "recvcounts": counts.T.copy(), "rdispls": rdisp}
    send = [0x7F0000000000 + i * (1 << 32) for i in range(P)]
    recv = [0x7E0000000000 + i * (1 << 32) for i in range(P)]
    desc, gx, gy = _check_plan(lay, send, recv)
    assert len(desc) > 64, "the long segment must have been cut"
    assert gx < (1 << 30) // TILE, "the grid must not be sized by the uncut long segment"
    assert len(desc) <= 8192 + 64


@pytest.mark.parametrize("shift", [16, 528, 1008, 4080])
@pytest.mark.parametrize("threads", [64, 256])
def test_shifted_buffers_keep_tiles_on_destination_multiples(shift, threads):
    """16-byte aligned buffers that do not start on a tile boundary: the fast kernel still
    applies, every descriptor carries its lead, and cuts of the skewed segment land on
    multiples of the tile size."""
    P = 4
    counts = np.full((P, P), (3 << 20) + 48, dtype=np.uint64)
    counts[1, 2] = (200 << 20) + 16
    disp = np.zeros((P, P), dtype=np.uint64)
    rdisp = np.zeros((P, P), dtype=np.uint64)
    for a in range(P):
        disp[a] = np.cumsum(counts[a]) - counts[a]
        rdisp[a] = np.cumsum(counts.T[a]) - counts.T[a]
    lay = {"sendcounts": counts, "sdispls": disp, "recvcounts": counts.T.copy(), "rdispls": rdisp}
    send = [0x7F0000000000 + i * (1 << 32) + shift for i in range(P)]
    recv = [0x7E0000000000 + i * (1 << 32) + 2 * shift for i in range(P)]
    desc, gx, gy = _check_plan(lay, send, recv, unroll=1, threads=threads)
    assert len(desc) > 16, "the long segment must have been cut"
    assert any(int(d["lead"]) for d in desc)


def test_zero_segments_and_errors():
    P = 3
    z = np.zeros((P, P), dtype=np.uint64)
    desc, gx, gy, tile_bytes, aligned = vccl.vccl_plan_alltoallv([0] * P, z, z, [0] * P, z, z, P, 1)
    assert len(desc) == 0
    c = np.array([[1, 2, 0], [0, 0, 0], [0, 0, 0]], dtype=np.uint64)
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_plan_alltoallv([64] * P, c, z, [1024] * P, c, z, P, 1)     # not transposed
    assert e.value.code == -2
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_plan_alltoallv([0] * P, c, z, [1024] * P, c.T.copy(), z, P, 1)   # NULL with bytes
    assert e.value.code == -1
    with pytest.raises(vccl.VcclError):
        vccl.vccl_plan_alltoallv([64] * P, z, z, [64] * P, z, z, P, 3)       # bad unroll
    with pytest.raises(vccl.VcclError):
        vccl.vccl_plan_alltoallv([64] * P, z, z, [64] * P, z, z, P, 1, 32)   # bad workgroup size
