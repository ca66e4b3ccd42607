"""The entry point that allocates nothing (vccl_moe_pack_noalloc) against the
allocating one (vccl_moe_pack), bit for bit: two calls in a row through the C
boundary, the second with a smaller input, so that whatever the first call left
in the library's static device array is still there when the second one runs."""
import numpy as np
import pytest

import workloads as wl
from gpu_util import SENTINEL, require_gpu, stream_handle, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vccl():
    require_gpu()
    import paper_2510_00991_amd as v
    v.vccl_init(0, 64)
    yield v
    v.vccl_finalize()


def _both(torch, v, P, T, K, E, row, seed):
    """Runs the allocating and the non-allocating pack on the same inputs; returns
    (packed, counts, bad) of each as host arrays."""
    x_np = [wl.payload_bytes(seed, s, T * row) for s in range(P)]
    ids_np = [wl.zipf_topk_expert_ids(seed, s, T, K, E).copy() for s in range(P)]
    ids_np[0][T // 2, K - 1] = E + 3                  # one out-of-range id: counted and dropped by both
    x = [to_dev(torch, a) for a in x_np]
    ids = [torch.from_numpy(a.reshape(-1).copy()).cuda() for a in ids_np]
    st = stream_handle(torch)
    res = []
    for fn in ("vccl_moe_pack", "vccl_moe_pack_noalloc"):
        packed = [torch.full((T * K * row + 32,), SENTINEL, dtype=torch.uint8, device="cuda") for _ in range(P)]
        counts = torch.full((P, E), -1, dtype=torch.int64, device="cuda")
        bad = torch.zeros(1, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        if fn == "vccl_moe_pack":
            v.vccl_moe_pack(x, ids, P, T, K, row, E, packed, counts, None, bad, st)
        else:
            v.vccl_moe_pack_noalloc(x, ids, P, T, K, row, E, packed, counts, bad, st)
        torch.cuda.synchronize()
        res.append(([p.cpu().numpy() for p in packed], counts.cpu().numpy(), int(bad.item())))
    return res


def test_no_alloc_pack_equals_the_allocating_pack_twice_in_a_row(vccl):
    torch = require_gpu()
    # first call: several histogram blocks, a row longer than one 2 KiB piece; second: smaller in every dimension
    for shape in ((8, 2049, 8, 256, 4112), (3, 130, 4, 12, 272)):
        P, T, K, E, row = shape
        (pk_a, cnt_a, bad_a), (pk_n, cnt_n, bad_n) = _both(torch, vccl, P, T, K, E, row, 4242 + T)
        assert bad_a == bad_n == 1
        assert np.array_equal(cnt_a, cnt_n), shape
        assert int(cnt_n.sum()) == P * T * K - 1
        for s in range(P):
            assert np.array_equal(pk_a[s], pk_n[s]), (shape, s)
        assert (pk_n[0][-32:] == SENTINEL).all()


def test_no_alloc_pack_rejects_what_does_not_fit(vccl):
    torch = require_gpu()
    st = stream_handle(torch)
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    ids = torch.zeros(64, dtype=torch.int32, device="cuda")
    counts = torch.zeros((32, 1024), dtype=torch.int64, device="cuda")
    # more ranks than the static pointer table holds
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_moe_pack_noalloc([dummy] * 17, [ids] * 17, 17, 1, 1, 16, 17, [dummy] * 17, counts, None, st)
    assert e.value.code == -6 and "at most 16 ranks" in e.value.message
    # index data beyond the 8 MiB array: nothing is enqueued, the buffers are never touched
    with pytest.raises(vccl.VcclError) as e:
        vccl.vccl_moe_pack_noalloc([dummy] * 16, [ids] * 16, 16, 1 << 20, 8, 16, 1024, [dummy] * 16, counts, None, st)
    assert e.value.code == -6 and "static scratch" in e.value.message
    torch.cuda.synchronize()
