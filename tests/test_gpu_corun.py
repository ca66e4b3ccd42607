"""Co-run behaviour: the FMA probe runs, and the copy-engine path makes progress
while a compute kernel holds every wavefront slot of every compute unit (a copy
kernel could not start then; copy engines can)."""
import time

import numpy as np
import pytest

import workloads as wl
from gpu_util import require_gpu, stream_handle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vccl():
    require_gpu()
    import paper_2510_00991_amd as v
    v.vccl_init(0, 16)
    yield v
    v.vccl_finalize()


def test_fma_probe_runs_and_scales_with_iterations(vccl):
    torch = require_gpu()
    cu = vccl.vccl_device_cu_count()
    out = torch.zeros(cu * 256, dtype=torch.float32, device="cuda")
    st = stream_handle(torch)
    ts = []
    for iters in (2000, 8000):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        vccl.vccl_fma_probe(out, 0, 256, iters, st)
        torch.cuda.synchronize()
        a.record()
        vccl.vccl_fma_probe(out, 0, 256, iters, st)
        b.record()
        torch.cuda.synchronize()
        ts.append(a.elapsed_time(b))
    assert torch.isfinite(out).all() and float(out.abs().sum()) > 0
    assert 3.0 < ts[1] / ts[0] < 5.0, ts          # compute-bound: time follows the iteration count
    with pytest.raises(vccl.VcclError):
        vccl.vccl_fma_probe(out, 0, 100, 10, st)  # threads must be a multiple of 64


@pytest.mark.parametrize("kind", ["sdma", "sdma_event", "sdma_host_sync", "hip_nocu"])
def test_copy_engine_progresses_while_all_wave_slots_are_busy(vccl, kind):
    """The acceptance test for "zero compute units": with every wavefront slot of
    the device held by a long compute kernel, the SDMA back end still completes an
    AlltoAll long before that kernel ends.  The hipMemcpyAsync(NoCU) back end is
    measured and reported only: whether it needs compute units depends on the HIP
    runtime in the process."""
    torch = require_gpu()
    vccl.vccl_set_option("ce_kind", "hip_nocu" if kind == "hip_nocu" else "sdma")
    saved_sync = vccl.vccl_get_option("ce_sync")
    vccl.vccl_set_option("ce_sync", {"sdma_host_sync": "host", "sdma_event": "event"}.get(kind, "memops"))
    cu = vccl.vccl_device_cu_count()
    P, c = 8, 4 << 20
    send = [torch.from_numpy(wl.payload_bytes(9, s, P * c)).cuda() for s in range(P)]
    recv = [torch.zeros(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
    wgs = cu * 8                                   # 8 x 256 lanes = all 32 wavefront slots of a CU
    out = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
    comp, comm = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    # size the compute kernel to roughly 40 ms
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(comp):
        a.record()
        vccl.vccl_fma_probe(out, wgs, 256, 2000, stream_handle(torch, comp))
        b.record()
    torch.cuda.synchronize()
    iters = int(2000 * 40.0 / max(a.elapsed_time(b), 0.05))
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c1 = torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(comp):
        a0.record()
        vccl.vccl_fma_probe(out, wgs, 256, iters, stream_handle(torch, comp))
        a1.record()
    time.sleep(0.005)                              # the compute kernel now owns the device
    assert not a1.query(), "compute kernel finished too early for the test to mean anything"
    with torch.cuda.stream(comm):
        vccl.vccl_alltoall(send, recv, c, P, vccl.MODE_CE, stream_handle(torch, comm))
        c1.record()
    torch.cuda.synchronize()
    t_compute = a0.elapsed_time(a1)
    t_copy_done = a0.elapsed_time(c1)
    vccl.vccl_set_option("ce_kind", "sdma")
    vccl.vccl_set_option("ce_sync", saved_sync)
    print(f"[{kind}] compute kernel {t_compute:.1f} ms; copy-engine AlltoAll finished "
          f"{t_copy_done:.1f} ms after the kernel started")
    if kind.startswith("sdma"):
        assert t_copy_done < 0.7 * t_compute, (t_copy_done, t_compute)
    for r, s in ((0, 5), (7, 7), (3, 0)):
        assert torch.equal(recv[r][s * c:(s + 1) * c], send[s][r * c:(r + 1) * c])


def test_hbm_probe_kernels_touch_exactly_what_they_should(vccl):
    """The ceiling probes are measurement aids, but they must move what they claim to: the
    copy copies, the write fills exactly `bytes`, the row writer puts whole rows at the
    indexed positions and nothing else, in every accepted launch shape."""
    torch = require_gpu()
    import numpy as np
    st = int(torch.cuda.current_stream().cuda_stream)
    n = (1 << 20) + 4096 + 16
    for threads, vecs in ((64, 1), (64, 2), (64, 4), (64, 16), (256, 1), (256, 4), (448, 2)):
        src = torch.randint(0, 256, (n + 64,), dtype=torch.uint8, device="cuda")
        dst = torch.full((n + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        vccl.vccl_hbm_probe(2, src, dst, n, threads, vecs, None, 0, 0, st)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src[:n]) and bool((dst[n:] == 0xA5).all()), (threads, vecs)
        dst.fill_(0xA5)
        vccl.vccl_hbm_probe(1, None, dst, n, threads, vecs, None, 0, 0, st)
        vccl.vccl_hbm_probe(0, src, dst[n:], n, threads, vecs, None, 0, 0, st)     # reads only: the sink stays
        torch.cuda.synchronize()
        assert bool((dst[n:] == 0xA5).all())
        words = dst[:n].cpu().numpy().view(np.uint32).reshape(-1, 4)
        assert (words[:, 2] == 0x5A5A5A5A).all() and (words[:, 3] == 0xA5A5A5A5).all(), (threads, vecs)
        # rows: 7 rows of 1 040 bytes into a buffer of 16 rows, at chosen positions
        row, total_rows = 1040, 16
        idx = torch.tensor([3, 0, 15, 7, 9, 1, 12], dtype=torch.int32, device="cuda")
        buf = torch.full((row * total_rows,), 0xA5, dtype=torch.uint8, device="cuda")
        vccl.vccl_hbm_probe(3, None, buf, 0, threads, vecs, idx, idx.numel(), row, st)
        torch.cuda.synchronize()
        got = buf.cpu().numpy().reshape(total_rows, row)
        for r in range(total_rows):
            if r in idx.cpu().tolist():
                w = got[r].view(np.uint32).reshape(-1, 4)
                assert (w[:, 2] == 0x5A5A5A5A).all() and (w[:, 0] == idx.cpu().tolist().index(r)).all(), (threads, vecs, r)
            else:
                assert (got[r] == 0xA5).all(), (threads, vecs, r)
    with pytest.raises(vccl.VcclError):
        vccl.vccl_hbm_probe(2, src, dst, n, 128, 3, None, 0, 0, st)


def test_probe_reports_its_shader_ticks_and_real_time(vccl):
    """vccl_fma_probe_clocks: per workgroup, shader-clock ticks that follow the work (twice the
    rounds, twice the ticks) and real-time ticks that agree with the event timing."""
    torch = require_gpu()
    wgs = vccl.vccl_device_cu_count()
    khz = vccl.vccl_device_wall_clock_khz()
    assert 1000 <= khz <= 10_000_000
    out = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
    clk = torch.zeros((wgs, 2), dtype=torch.int64, device="cuda")
    st = stream_handle(torch)
    seen = {}
    for iters in (20000, 40000):
        vccl.vccl_fma_probe_clocks(out, clk, wgs, 256, iters, st)       # warm
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        vccl.vccl_fma_probe_clocks(out, clk, wgs, 256, iters, st)
        b.record()
        torch.cuda.synchronize()
        k = clk.cpu().numpy()
        assert (k > 0).all()
        seen[iters] = (float(np.median(k[:, 0])), float(np.median(k[:, 1])), a.elapsed_time(b))
        ms_from_ticks = float(k[:, 1].max()) / khz
        assert 0.8 * seen[iters][2] < ms_from_ticks < 1.05 * seen[iters][2], (ms_from_ticks, seen[iters])
        mhz = seen[iters][0] / seen[iters][1] * khz * 1e-3
        assert 300.0 < mhz < 4000.0, mhz
    assert 1.9 < seen[40000][0] / seen[20000][0] < 2.1, seen
    with pytest.raises(vccl.VcclError):
        vccl.vccl_fma_probe_clocks(out, None, wgs, 256, 10, st)


def test_copy_engine_traffic_leaves_the_probe_alone_and_a_copy_kernel_does_not(vccl):
    """The co-run protocol's outcome on the config-2 exchange (P = 8 x 16 MiB, random
    payload), with bounds that leave room to what is measured: the compute-bound probe loses
    at most 3 % beside copy-engine traffic (measured: under 0.5 %) and more than that beside the
    full-grid copy kernel (measured: about a third), while both transfers move their bytes at
    their usual rate.  The probe's own counters say where the time goes: in neither case is
    it held up inside its compute units (its shader ticks stay within 3 %); beside the copy
    kernel the chip runs its shaders at a lower clock."""
    torch = require_gpu()
    from paper_2510_00991_amd.harness import CoRun, time_region
    P, c = 8, 16 << 20
    send = [torch.from_numpy(wl.payload_bytes(wl.config_seed(2), s, P * c)).cuda() for s in range(P)]
    recv = [torch.empty(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
    sp, rp = vccl.pointer_array(send), vccl.pointer_array(recv)
    co = CoRun(torch, iters=60000)
    moved = 2.0 * P * P * c
    res = {}
    for name, mode, pairs in (("ce", vccl.MODE_CE, 16), ("cu", vccl.MODE_CU, 6)):
        fn = lambda sh, m=mode: vccl.vccl_alltoall(sp, rp, c, P, m, sh)
        per = time_region(torch, lambda: fn(stream_handle(torch)), 5, 2)[0] / 5
        res[name] = co.beside(fn, moved, per, reps=pairs)
    assert res["ce"]["slowdown_pct"] <= 3.0, res["ce"]
    assert res["cu"]["slowdown_pct"] >= 3.0, res["cu"]
    assert res["ce"]["comm_GBps_while_corunning"] > 1000.0, res["ce"]
    assert res["cu"]["comm_GBps_while_corunning"] > 4000.0, res["cu"]
    for name in ("ce", "cu"):
        assert abs(res[name]["probe_shader_ticks_pct"]) < 3.0, res[name]
    assert res["cu"]["shader_clock_MHz_beside"] < 0.99 * res["cu"]["shader_clock_MHz_alone"], res["cu"]
    assert res["ce"]["shader_clock_MHz_beside"] > 0.97 * res["ce"]["shader_clock_MHz_alone"], res["ce"]
