"""GPU parity of the 1F1B pipeline emulation (the paper's Section 3.2, "Improve
overlaps in PP": 8 microbatches over 4 workers, every stage sending its activation
to the next stage and its gradient to the previous one with SendRecv): what a
stage consumes is, byte for byte, what the oracle's SendRecv delivers from the
stage that produced it, in every transfer mode."""
import numpy as np
import pytest

import oracle
import workloads as wl
from gpu_util import SENTINEL, assert_same, require_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vccl():
    require_gpu()
    import paper_2510_00991_amd as v
    v.vccl_init(0, 64)
    yield v
    v.vccl_finalize()


def _payload(n):
    def make(kind, stage, m):
        # one seeded stream per (direction, stage, microbatch)
        return wl.payload_bytes(wl.config_seed(4) + (1 if kind == "B" else 0), stage * 64 + m, n)
    return make


def _expected(stages, micro, n, payload):
    """Every transfer of one iteration through the oracle, with the peer tables of the
    emulation: forward link i carries rank i -> i+1, backward link i rank S+i -> S+i-1."""
    from paper_2510_00991_amd.harness import pipeline_links
    PR, fwd, bwd = pipeline_links(stages)
    want = {}
    for kind, (to, frm) in (("F", fwd), ("B", bwd)):
        for i in range(stages):
            if (kind == "F" and i == stages - 1) or (kind == "B" and i == 0):
                continue
            s_rank = i if kind == "F" else stages + i
            r_rank = to[s_rank]
            for m in range(micro):
                send = [np.zeros(0, np.uint8)] * PR
                recv = [np.zeros(0, np.uint8)] * PR
                sb, rb = [0] * PR, [0] * PR
                send[s_rank], sb[s_rank] = payload(kind, i, m), n
                recv[r_rank], rb[r_rank] = np.full(n, SENTINEL, np.uint8), n
                oracle.sendrecv(send, sb, to, recv, rb, frm)
                to_stage = i + 1 if kind == "F" else i - 1
                want[(kind, to_stage, m)] = recv[r_rank]
    return want


@pytest.mark.parametrize("stages,micro", [(2, 8), (4, 8), (4, 3)])
def test_1f1b_arrivals_match_the_oracle(vccl, stages, micro):
    torch = require_gpu()
    from paper_2510_00991_amd.harness import pipeline_1f1b
    n = 3 * (512 << 10) + 4096 + 48          # three whole FIFO chunks and a ragged one
    payload = _payload(n)
    want = _expected(stages, micro, n, payload)
    assert len(want) == 2 * (stages - 1) * micro
    res = pipeline_1f1b(torch, stages=stages, micro=micro, act_bytes=n, fwd_iters=300,
                        modes=("cu_path", "cu_staged_fifo", "copy_engine"), payload=payload)
    for mode in ("cu_path", "cu_staged_fifo", "copy_engine"):
        got = res["arrivals"][mode]
        assert set(got) == set(want), mode
        for key in sorted(want):
            assert_same(got[key].numpy(), want[key], f"{mode}: what stage {key[1]} consumes for {key[0]}{key[2]}")
    # distinct payloads: a transfer that delivered another microbatch's or link's bytes would differ
    keys = sorted(want)
    assert not np.array_equal(want[keys[0]], want[keys[1]])


def test_1f1b_copy_engine_ordering_modes(vccl):
    """The same check on the copy-engine path under each of its stream-ordering mechanisms."""
    torch = require_gpu()
    from paper_2510_00991_amd.harness import pipeline_1f1b
    n = (1 << 20) + 16
    payload = _payload(n)
    want = _expected(2, 4, n, payload)
    saved = (vccl.vccl_get_option("ce_kind"), vccl.vccl_get_option("ce_sync"))
    try:
        for kind, sync in (("sdma", "memops"), ("sdma", "host"), ("hip_nocu", "memops")):
            vccl.vccl_set_option("ce_kind", kind)
            vccl.vccl_set_option("ce_sync", sync)
            res = pipeline_1f1b(torch, stages=2, micro=4, act_bytes=n, fwd_iters=300,
                                modes=("copy_engine",), payload=payload)
            got = res["arrivals"]["copy_engine"]
            for key in sorted(want):
                assert_same(got[key].numpy(), want[key], f"{kind}/{sync}: {key}")
    finally:
        vccl.vccl_set_option("ce_kind", saved[0])
        vccl.vccl_set_option("ce_sync", saved[1])
