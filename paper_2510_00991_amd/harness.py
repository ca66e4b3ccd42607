"""Measurement harness around the C boundary: event timing, the co-run slowdown
protocol (a compute-bound FMA kernel timed alone and beside a transfer, the
effect the paper describes in Appendix E), the pipeline SendRecv ring and the
P = 64 message-size sweep.  PyTorch is used for device memory, streams and
events only; every byte is moved by libvccl.

CLI:  python -m paper_2510_00991_amd.harness ring|sweep|pipeline|ceilings|all  [--json FILE]
"""
from __future__ import annotations

import argparse
import json
import statistics
import sys
import time

import numpy as np

from . import binding as v


def _ev(torch):
    return torch.cuda.Event(enable_timing=True)


def time_calls(torch, fn, steps, warmup):
    """(wall seconds for `steps` back-to-back calls, per-call device seconds from
    events recorded on the current stream around each call)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(_ev(torch), _ev(torch)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, [a.elapsed_time(b) * 1e-3 for a, b in ev]


def time_region(torch, fn, steps, warmup):
    """(wall seconds, device seconds) for `steps` back-to-back calls: the host clock
    between two device synchronisations, and one pair of events on the current stream
    around the whole train of calls.  Nothing is recorded between the calls, so the
    launches follow each other as they would in an application (an event between two
    kernels costs about 5 us of dispatch each on this device)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    a, b = _ev(torch), _ev(torch)
    t0 = time.perf_counter()
    a.record()
    for _ in range(steps):
        fn()
    b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, a.elapsed_time(b) * 1e-3


class CoRun:
    """FMA probe on its own stream, timed alone and while `comm_fn` keeps another
    stream busy.  slowdown = (T_with - T_alone) / T_alone.  Every probe also reports the
    shader-clock ticks and the real-time ticks its workgroups ran for, which splits a
    slowdown into its two possible causes: more shader ticks (the probe was held up
    inside its compute units) or the same ticks at a lower shader clock."""

    def __init__(self, torch, iters=60000, threads=256, workgroups=0):
        self.torch = torch
        self.iters, self.threads, self.workgroups = iters, threads, workgroups
        self.cu = v.vccl_device_cu_count()
        n = (workgroups or self.cu) * threads
        self.out = torch.zeros(n, dtype=torch.float32, device="cuda")
        self.clocks = torch.zeros((workgroups or self.cu, 2), dtype=torch.int64, device="cuda")
        self.wall_khz = v.vccl_device_wall_clock_khz()
        self.comp = torch.cuda.Stream()
        self.comm = torch.cuda.Stream()
        self._alone = None

    def comm_stream_handle(self) -> int:
        return int(self.comm.cuda_stream)

    def _probe(self):
        torch = self.torch
        a, b = _ev(torch), _ev(torch)
        with torch.cuda.stream(self.comp):
            a.record()
            v.vccl_fma_probe_clocks(self.out, self.clocks, self.workgroups, self.threads, self.iters,
                                    int(self.comp.cuda_stream))
            b.record()
        return a, b

    def _ticks(self):
        """(shader-clock ticks, real-time ticks) of the probe launched last: medians over its workgroups."""
        k = self.clocks.cpu().numpy()
        return float(np.median(k[:, 0])), float(np.median(k[:, 1]))

    def _time_alone(self, ticks=None):
        """Probe preceded by an untimed probe, so that the timed one always starts
        with the compute units already busy and the clocks settled."""
        self._probe()
        a, b = self._probe()
        self.comp.synchronize()
        if ticks is not None:
            ticks.append(self._ticks())
        return a.elapsed_time(b) * 1e-3

    def alone(self, reps=10):
        if self._alone is None:
            self._time_alone()
            self._alone = statistics.median(self._time_alone() for _ in range(reps))
        return self._alone

    def beside(self, comm_fn, comm_bytes_per_call, comm_seconds_per_call, reps=20):
        """comm_fn(stream_handle) enqueues one transfer on the given stream.  Each
        repetition is a pair: the probe alone and the probe beside the transfers, in
        alternating order from pair to pair (alone first, then beside first) so that
        whatever the measurement before leaves behind - clocks, power state, engines
        winding down - falls on both sides equally.  In both cases the timed probe
        directly follows an untimed one, and the transfers are held back until that
        untimed probe has finished, so both timed probes start from the same state; the
        device is idle (every stream synchronised, so every copy-engine operation has
        been completed by the proxy) before each measurement.  The slowdown is the
        median of the per-pair ratios; the quartiles and extremes of those ratios are
        reported with it."""
        torch = self.torch
        t_guess = self.alone()
        n_comm = max(1, int(1.25 * t_guess / max(comm_seconds_per_call, 1e-6)) + 1)
        sh = self.comm_stream_handle()
        alone, both, comm_t = [], [], []
        ticks_alone, ticks_both = [], []

        def timed_beside():
            self._probe()                                   # untimed lead-in
            gate = torch.cuda.Event()
            gate.record(self.comp)
            self.comm.wait_event(gate)
            c0, c1 = _ev(torch), _ev(torch)
            with torch.cuda.stream(self.comm):
                c0.record()
                for _ in range(n_comm):
                    comm_fn(sh)
                c1.record()
            a, b = self._probe()
            torch.cuda.synchronize()
            both.append(a.elapsed_time(b) * 1e-3)
            comm_t.append(c0.elapsed_time(c1) * 1e-3)
            ticks_both.append(self._ticks())

        for i in range(reps):
            torch.cuda.synchronize()
            if i % 2 == 0:
                alone.append(self._time_alone(ticks_alone))
                torch.cuda.synchronize()
                timed_beside()
            else:
                timed_beside()
                torch.cuda.synchronize()
                alone.append(self._time_alone(ticks_alone))
        t_alone = statistics.median(alone)
        t_with = statistics.median(both)
        tc = statistics.median(comm_t)
        ratios = sorted(b / a for a, b in zip(alone, both))
        q = statistics.quantiles(ratios, n=4) if len(ratios) >= 4 else [ratios[0], statistics.median(ratios), ratios[-1]]
        pct = lambda r: 100.0 * (r - 1.0)
        mhz = lambda t: statistics.median(c / r for c, r in t) * self.wall_khz * 1e-3
        return {"alone_ms": t_alone * 1e3, "corun_ms": t_with * 1e3,
                # the two possible causes of a slowdown, from the probe's own counters
                "probe_shader_ticks_pct": pct(statistics.median(b[0] / a[0] for a, b in zip(ticks_alone, ticks_both))),
                "shader_clock_MHz_alone": mhz(ticks_alone), "shader_clock_MHz_beside": mhz(ticks_both),
                "slowdown_pct": pct(statistics.median(ratios)), "slowdown_pct_mean": pct(statistics.mean(ratios)),
                "slowdown_pct_q1": pct(q[0]), "slowdown_pct_q3": pct(q[2]),
                "slowdown_pct_min": pct(ratios[0]), "slowdown_pct_max": pct(ratios[-1]),
                "alone_ms_min": min(alone) * 1e3, "alone_ms_max": max(alone) * 1e3,
                "pairs": reps,
                "comm_calls": n_comm, "comm_ms": tc * 1e3,
                "comm_GBps_while_corunning": comm_bytes_per_call * n_comm / tc / 1e9}


def _set(opts):
    saved = {k: v.vccl_get_option(k) for k in opts}
    for k, val in opts.items():
        v.vccl_set_option(k, val)
    return saved


def ring_corun(torch, P=8, nbytes=64 << 20, cu_grids=(8, 16, 32, 64, 256), steps=5):
    """Pipeline SendRecv ring (P stages, one activation per stage) in every mode:
    copy GB/s alone, and the FMA probe's slowdown beside it; for the direct
    compute-unit mode also over a capped copy grid."""
    import workloads as wl   # seeded inputs

    send = [torch.from_numpy(wl.normal_bf16_bits(wl.config_seed(4), s, nbytes // 2).view("uint8")).cuda()
            for s in range(P)]
    recv = [torch.zeros(nbytes, dtype=torch.uint8, device="cuda") for _ in range(P)]
    to, frm = wl.ring_peers(P)
    st = int(torch.cuda.current_stream().cuda_stream)
    co = CoRun(torch)
    rows = []

    def run(name, mode, algo_factor, opts=None):
        saved = _set(opts or {})
        try:
            fn = lambda s=st: v.vccl_sendrecv(send, [nbytes] * P, to, recv, [nbytes] * P, frm, P, mode, s)
            wall, _ = time_region(torch, fn, steps, 2)
            per = wall / steps
            moved = 2.0 * P * nbytes
            row = {"mode": name, "ms": per * 1e3, "GBps_effective": moved / per / 1e9,
                   "GBps_algorithmic": algo_factor * moved / per / 1e9}
            row.update(co.beside(lambda s: v.vccl_sendrecv(send, [nbytes] * P, to, recv, [nbytes] * P,
                                                           frm, P, mode, s), moved, per))
            if mode == v.MODE_CU_STAGED:
                v.vccl_sendrecv_staged_status()
            rows.append(row)
        finally:
            _set(saved)

    run("cu_direct", v.MODE_CU, 1.0)
    for g in cu_grids:
        run(f"cu_direct_grid{g}", v.MODE_CU, 1.0, {"cu_max_wg": g, "cu_unroll": 8, "cu_threads": 256})
    run("cu_staged_fifo", v.MODE_CU_STAGED, 2.0)
    run("copy_engine", v.MODE_CE, 1.0)
    return {"workload": f"SendRecv ring, {P} stages x {nbytes >> 20} MiB, FMA probe on all CUs",
            "probe": {"workgroups": co.cu, "threads": co.threads, "iters": co.iters}, "rows": rows}


def sweep_p64(torch, P=64, sizes=None, with_corun=True, max_bytes_per_side=16 << 30):
    """AlltoAll over P virtual ranks for per-peer sizes 4 KiB .. 4 MiB: both paths'
    bandwidth and the probe's slowdown beside each."""
    import workloads as wl

    sizes = [c for c in (sizes or [4096 << k for k in range(11)]) if P * P * c <= max_bytes_per_side]
    co = CoRun(torch) if with_corun else None
    st = int(torch.cuda.current_stream().cuda_stream)
    rows = []
    # The buffers of every size are allocated before the first measurement and freed
    # after the last (about 64 GiB in all): after device memory has been freed the copy
    # engines of this device run at about 60 % of their rate for a second or two, which
    # would distort the size measured next.
    bufs = {}
    for c in sizes:
        send = [torch.empty(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
        recv = [torch.empty(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
        for s in range(P):     # seeded payload: one MiB per rank, repeated through the buffer (the power a
            n = min(P * c, 1 << 20)   # transfer draws, and with it what it costs its neighbours, depends on the values)
            send[s].view(-1, n).copy_(torch.from_numpy(wl.payload_bytes(wl.config_seed(5), s, n)).cuda())
        # For small blocks the copy-engine path is also given receive buffers that are slices of
        # one allocation (a constant stride between the ranks), the layout that lets it take one
        # pitched copy per rank in place of P plain ones.
        slab = ([b[:P * c] for b in torch.empty((P, P * c + 4096), dtype=torch.uint8, device="cuda").unbind(0)]
                if c <= 32 << 10 else None)
        bufs[c] = (send, recv, slab)
    for c in sizes:
        send, recv, slab = bufs[c]
        send_p, recv_p = v.pointer_array(send), v.pointer_array(recv)   # marshalled once, not per call
        slab_p = v.pointer_array(slab) if slab is not None else recv_p
        moved = 2.0 * P * P * c
        row = {"bytes_per_peer": c, "total_sent_MiB": P * P * c / (1 << 20)}
        for name, mode in (("cu", v.MODE_CU), ("ce", v.MODE_CE)):
            to = slab_p if name == "ce" else recv_p
            fn = lambda s=st, m=mode, to=to: v.vccl_alltoall(send_p, to, c, P, m, s)
            k = 10 if name == "cu" else 3
            # keep the device busy for ~50 ms first: the memory clocks of an idle
            # device ramp up slowly under copy-engine traffic alone
            t_warm = time.perf_counter()
            while time.perf_counter() - t_warm < 0.05:
                fn()
                torch.cuda.synchronize()
            t = statistics.median(time_region(torch, fn, k, 1)[0] for _ in range(3)) / k
            row[name] = {"us": t * 1e6, "GBps": moved / t / 1e9}
            if name == "ce":     # the same call with plain copies only (one per block)
                v.vccl_set_option("ce_pitched", 0)
                tp = statistics.median(time_region(torch, fn, k, 1)[0] for _ in range(3)) / k
                v.vccl_set_option("ce_pitched", 1)
                row[name]["us_plain_copies"] = tp * 1e6
                row[name]["receive_buffers"] = "slices of one allocation" if slab is not None else "separate allocations"
            if co is not None:
                row[name].update(co.beside(lambda s, m=mode, to=to: v.vccl_alltoall(send_p, to, c, P, m, s),
                                           moved, t, reps=8))
        # What one device of P does in this exchange: its own P outgoing blocks (the other
        # ranks' blocks are the work of their devices' engines or compute units).
        one = np.zeros((P, P), dtype=np.uint64)
        one[0, :] = c
        displs = np.tile(np.arange(P, dtype=np.uint64) * np.uint64(c), (P, 1))
        for name, mode in (("cu", v.MODE_CU), ("ce", v.MODE_CE)):
            fn = lambda s=st, m=mode: v.vccl_alltoallv(send_p, one, displs, recv_p, one.T.copy(), displs, P, m, s)
            t = statistics.median(time_region(torch, fn, 10, 2)[0] for _ in range(3)) / 10
            row[name]["one_rank_share_us"] = t * 1e6
            row[name]["one_rank_share_GBps"] = 2.0 * P * c / t / 1e9
        rows.append(row)
    del send, recv, slab, bufs
    torch.cuda.empty_cache()
    return {"workload": f"AlltoAll sweep, P={P}, per-peer 4 KiB..4 MiB", "rows": rows}


def hbm_ceilings(torch, gib=(1, 7), reps=10):
    """What the device gives plain streaming kernels, for the rooflines of the copy
    paths: read-only, write-only, copy, and whole 14 KiB rows written in order or to
    permuted row positions (the MoE pack's write pattern), in several launch shapes.
    GB/s = bytes read + bytes written."""
    st = int(torch.cuda.current_stream().cuda_stream)
    rows_out = []

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        ev = [(_ev(torch), _ev(torch)) for _ in range(reps)]
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return statistics.median(a.elapsed_time(b) * 1e-3 for a, b in ev)

    sink = torch.zeros(64, dtype=torch.uint8, device="cuda")
    for g in gib:
        n = g << 30
        import workloads as wl
        a = torch.empty(n, dtype=torch.uint8, device="cuda")      # seeded payload, one MiB repeated
        a.view(-1, 1 << 20).copy_(torch.from_numpy(wl.payload_bytes(wl.config_seed(2), 0, 1 << 20)).cuda())
        b = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(2)
        for kind, name, moved in ((0, "read", n), (1, "write", n), (2, "copy", 2 * n)):
            for threads, vecs in ((64, 1), (64, 2), (64, 4), (64, 16), (256, 1), (256, 4)):
                dst = sink if kind == 0 else b
                t = timed(lambda: v.vccl_hbm_probe(kind, a, dst, n, threads, vecs, None, 0, 0, st))
                rows_out.append({"pattern": name, "GiB": g, "lanes": threads, "vectors_per_lane": vecs,
                                 "us": t * 1e6, "GBps": moved / t / 1e9})
        del a
        # whole rows of 14 336 bytes (config 3), in order and to permuted positions
        row = 14336
        n_rows = n // row
        gen = torch.Generator(device="cuda")
        gen.manual_seed(12345)
        perm = torch.randperm(n_rows, device="cuda", generator=gen).to(torch.int32)
        for order, idx in (("rows in order", None), ("rows permuted", perm)):
            for threads, vecs in ((64, 2), (256, 1), (448, 2), (64, 16)):
                t = timed(lambda: v.vccl_hbm_probe(3, None, b, 0, threads, vecs, idx, n_rows, row, st))
                rows_out.append({"pattern": "write " + order, "GiB": g, "lanes": threads, "vectors_per_lane": vecs,
                                 "us": t * 1e6, "GBps": n_rows * row / t / 1e9})
        del b, perm
        torch.cuda.empty_cache()
    return {"workload": "HBM ceiling probes (vccl_hbm_probe)", "rows": rows_out}


def p2p_sweep(torch, sizes=None, reps=20):
    """One pair of ranks exchanging one message each way (rank 0 -> 1 and 1 -> 0) over
    message sizes 1 KiB .. 256 MiB in every SendRecv mode: the time from the call to the
    completion of the caller's stream (median over single calls on an idle device) and
    the rate of a train of calls.  The shape of the paper's point-to-point evaluation
    (Section 4.1): bandwidth for large messages, latency for small ones."""
    import workloads as wl

    sizes = sizes or [1 << k for k in range(10, 29, 2)]
    P = 2
    to, frm = wl.ring_peers(P)
    st = int(torch.cuda.current_stream().cuda_stream)
    top = max(sizes)
    send = [torch.from_numpy(wl.payload_bytes(wl.config_seed(4), s, min(top, 1 << 20))).cuda().repeat(
        (top + (1 << 20) - 1) >> 20)[:top].contiguous() for s in range(P)]
    recv = [torch.zeros(top, dtype=torch.uint8, device="cuda") for _ in range(P)]
    send_p, recv_p = v.pointer_array(send), v.pointer_array(recv)
    modes = (("cu_direct", v.MODE_CU, {}),
             ("cu_staged_fifo", v.MODE_CU_STAGED, {}),
             ("copy_engine_event", v.MODE_CE, {"ce_kind": "sdma", "ce_sync": "event"}),
             ("copy_engine_memops", v.MODE_CE, {"ce_kind": "sdma", "ce_sync": "memops"}),
             ("copy_engine_host_sync", v.MODE_CE, {"ce_kind": "sdma", "ce_sync": "host"}))
    rows = []
    for n in sizes:
        row = {"bytes": n}
        for name, mode, opts in modes:
            saved = _set(opts)
            try:
                fn = lambda: v.vccl_sendrecv(send_p, [n] * P, to, recv_p, [n] * P, frm, P, mode, st)
                fn()
                torch.cuda.synchronize()
                lat = []
                for _ in range(reps):
                    t0 = time.perf_counter()
                    fn()
                    torch.cuda.synchronize()
                    lat.append(time.perf_counter() - t0)
                k = 10 if n <= (16 << 20) else 4
                wall = statistics.median(time_region(torch, fn, k, 1)[0] for _ in range(5))
                if mode == v.MODE_CU_STAGED:
                    v.vccl_sendrecv_staged_status()
                row[name] = {"call_to_completion_us": statistics.median(lat) * 1e6,
                             "train_us_per_call": wall / k * 1e6,
                             "GBps": 2.0 * P * n / (wall / k) / 1e9}
            finally:
                _set(saved)
        rows.append(row)
    return {"workload": "SendRecv between one pair of ranks, one message each way, 1 KiB .. 256 MiB "
                        "(GB/s = bytes read + bytes written)", "rows": rows}


def _schedule_1f1b(stages, micro):
    """Per stage, the 1F1B order of ("F", m) / ("B", m) steps (warm-up forwards,
    then one forward one backward, then the remaining backwards)."""
    out = []
    for i in range(stages):
        w = min(stages - 1 - i, micro)
        ops = [("F", m) for m in range(w)]
        for j in range(micro - w):
            ops += [("F", w + j), ("B", j)]
        ops += [("B", m) for m in range(micro - w, micro)]
        out.append(ops)
    return out


def pipeline_links(stages):
    """Peer tables of the pipeline emulation: every link is a connection of its own (its
    own pair of virtual ranks), as between real pipeline stages.  Forward links use ranks
    0..S-1 (stage i sends from rank i to rank i+1), backward links ranks S..2S-1 (stage i
    sends from rank S+i to rank S+i-1).  Sharing one pair of ranks would queue all links
    behind each other, because a connection carries its transfers in the order they were
    posted.  Returns (ranks, (send_to, recv_from) of a forward transfer, the same of a
    backward transfer)."""
    S = stages
    up = [(r + 1) % S if r < S else S + (r - S + 1) % S for r in range(2 * S)]
    down = [(r - 1) % S if r < S else S + (r - S - 1) % S for r in range(2 * S)]
    return 2 * S, (up, down), (down, up)


def pipeline_1f1b(torch, stages=4, micro=8, act_bytes=128 << 20, fwd_iters=4000, reps=5, modes=None,
                  payload=None):
    """Emulation of the paper's pipeline figure (1F1B, 8 microbatches, 4 workers) on
    one device: every stage computes on its own stream with the FMA probe sized to a
    quarter of the compute units (forward = fwd_iters rounds, backward twice that),
    activations go to the next stage and gradients to the previous one through
    vccl_sendrecv on per-link streams.  Reports the iteration time per transfer mode
    and without any transfer, and the paper's gain I = (T_n - T_v) / (T_v + alpha)
    with alpha = 0 (no data-parallel traffic here), T_n the compute-unit path (also given
    with T_n the staged chunk-FIFO path, the kernel-driven two-step baseline).

    `modes` restricts the run to some of "no_transfer", "cu_path", "cu_path_capped_32wg",
    "cu_staged_fifo", "copy_engine".  With `payload` (a function (kind, stage, microbatch)
    -> act_bytes uint8 values, kind "F" for the activation stage `stage` sends forward, "B"
    for the gradient it sends backward) the run carries real data: a stage's step writes
    its payload into the send buffer on the compute stream behind its compute kernel, and
    the receiving stage copies what has arrived out of its receive buffer at the start of
    the step that consumes it, on its own compute stream.  The result then holds, per
    mode, "arrivals": {(kind, receiving stage, microbatch): bytes as a CPU tensor}, every
    transfer with a buffer of its own."""
    cu = v.vccl_device_cu_count()
    wg = max(1, cu // stages)
    sched = _schedule_1f1b(stages, micro)
    comp = [torch.cuda.Stream() for _ in range(stages)]
    link_f = [torch.cuda.Stream() for _ in range(stages)]     # stage i -> i+1
    link_b = [torch.cuda.Stream() for _ in range(stages)]     # stage i -> i-1
    outs = [torch.zeros(wg * 256, dtype=torch.float32, device="cuda") for _ in range(stages)]
    nbuf = micro if payload is not None else 2

    def bufs():
        return [[torch.zeros(act_bytes, dtype=torch.uint8, device="cuda") for _ in range(nbuf)]
                for _ in range(stages)]

    src_f, dst_f, src_b, dst_b = bufs(), bufs(), bufs(), bufs()
    null = torch.zeros(16, dtype=torch.uint8, device="cuda")
    pay = {}
    if payload is None:
        # timing runs move activation-like values (N(0,1) as bf16), not zeros: the power a
        # transfer draws, and with it what it costs the compute beside it, depends on the values
        import workloads as wl
        n = min(act_bytes, 4 << 20) & ~1
        for i, per_stage in enumerate(src_f + src_b):
            block = torch.from_numpy(wl.normal_bf16_bits(wl.config_seed(4), i, n // 2).view("uint8")).cuda()
            for buf in per_stage:
                buf[:(act_bytes // n) * n].view(-1, n).copy_(block)
    if payload is not None:
        for i in range(stages):
            for m in range(micro):
                if i < stages - 1:
                    pay[("F", i, m)] = torch.as_tensor(payload("F", i, m), dtype=torch.uint8).cuda()
                if i > 0:
                    pay[("B", i, m)] = torch.as_tensor(payload("B", i, m), dtype=torch.uint8).cuda()

    PR, fwd_tables, bwd_tables = pipeline_links(stages)
    S = stages

    def transfer(mode, src, dst, stream, stage, forward):
        sendbuf, recvbuf = [null] * PR, [null] * PR
        sb, rb = [0] * PR, [0] * PR
        if forward:
            s_rank, r_rank = stage, stage + 1
            to, frm = fwd_tables
        else:
            s_rank, r_rank = S + stage, S + stage - 1
            to, frm = bwd_tables
        sendbuf[s_rank], sb[s_rank] = src, act_bytes
        recvbuf[r_rank], rb[r_rank] = dst, act_bytes
        v.vccl_sendrecv(sendbuf, sb, to, recvbuf, rb, frm, PR, mode, int(stream.cuda_stream))

    def iteration(mode, got=None):
        """Enqueue one whole iteration; returns the wall time from the first launch to
        the completion of every stream."""
        done = {}                      # (kind, stage, m) -> event after the step's compute
        arrived = {}                   # (kind, stage, m) -> event after the step's input has landed
        pos = [0] * stages
        if payload is not None:
            for group in (dst_f, dst_b, src_f, src_b):
                for per_stage in group:
                    for t in per_stage:
                        t.fill_(0xA5)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        progress = True
        while progress:
            progress = False
            for i in range(stages):
                while pos[i] < len(sched[i]):
                    kind, m = sched[i][pos[i]]
                    need = None
                    if kind == "F" and i > 0:
                        need = ("F", i, m)
                    if kind == "B" and i < stages - 1:
                        need = ("B", i, m)
                    if need is not None and mode is not None and need not in arrived:
                        break
                    if need is not None and mode is None:
                        dep = ("F", i - 1, m) if kind == "F" else ("B", i + 1, m)
                        if dep not in done:
                            break
                        comp[i].wait_event(done[dep])
                    elif need is not None:
                        comp[i].wait_event(arrived[need])
                        if got is not None:     # what this step consumes, as the compute stream sees it
                            inbox = dst_f[i - 1][m % nbuf] if kind == "F" else dst_b[i + 1][m % nbuf]
                            with torch.cuda.stream(comp[i]):
                                got[need] = inbox.clone()
                    v.vccl_fma_probe(outs[i], wg, 256, fwd_iters * (1 if kind == "F" else 2),
                                     int(comp[i].cuda_stream))
                    sends = mode is not None and ((kind == "F" and i < stages - 1) or (kind == "B" and i > 0))
                    if sends and payload is not None:   # the step's result, written behind its compute
                        outbox = src_f[i][m % nbuf] if kind == "F" else src_b[i][m % nbuf]
                        with torch.cuda.stream(comp[i]):
                            outbox.copy_(pay[(kind, i, m)], non_blocking=True)
                    e = torch.cuda.Event()
                    e.record(comp[i])
                    done[(kind, i, m)] = e
                    if mode is not None:
                        if kind == "F" and i < stages - 1:
                            link_f[i].wait_event(e)
                            transfer(mode, src_f[i][m % nbuf], dst_f[i][m % nbuf], link_f[i], i, True)
                            a = torch.cuda.Event()
                            a.record(link_f[i])
                            arrived[("F", i + 1, m)] = a
                        if kind == "B" and i > 0:
                            link_b[i].wait_event(e)
                            transfer(mode, src_b[i][m % nbuf], dst_b[i][m % nbuf], link_b[i], i, False)
                            a = torch.cuda.Event()
                            a.record(link_b[i])
                            arrived[("B", i - 1, m)] = a
                    pos[i] += 1
                    progress = True
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    table = (("no_transfer", None, {}), ("cu_path", v.MODE_CU, {}),
             ("cu_path_capped_32wg", v.MODE_CU, {"cu_max_wg": 32, "cu_unroll": 8, "cu_threads": 256}),
             ("cu_staged_fifo", v.MODE_CU_STAGED, {}),
             ("copy_engine", v.MODE_CE, {}))
    rows, arrivals = {}, {}
    for name, mode, opts in table:
        if modes is not None and name not in modes:
            continue
        saved = _set(opts)
        try:
            if payload is not None and mode is not None:
                got = {}
                rows[name] = iteration(mode, got) * 1e3
                arrivals[name] = {k: t.cpu() for k, t in got.items()}
            else:
                iteration(mode)
                rows[name] = statistics.median(iteration(mode) for _ in range(reps)) * 1e3
            if mode == v.MODE_CU_STAGED:
                v.vccl_sendrecv_staged_status()
        finally:
            _set(saved)
    out = {"workload": f"1F1B, {stages} stages x {micro} microbatches, {act_bytes} bytes per transfer, "
                       f"FMA probe {wg} workgroups per stage, forward {fwd_iters} rounds",
           "iteration_ms": rows}
    if "cu_path" in rows and "copy_engine" in rows:
        out["gain_I_pct"] = 100.0 * (rows["cu_path"] - rows["copy_engine"]) / rows["copy_engine"]
    if "cu_staged_fifo" in rows and "copy_engine" in rows:
        out["gain_I_pct_over_staged_fifo"] = 100.0 * (rows["cu_staged_fifo"] - rows["copy_engine"]) / rows["copy_engine"]
    if "no_transfer" in rows:
        out["overhead_vs_no_transfer_pct"] = {k: 100.0 * (val - rows["no_transfer"]) / rows["no_transfer"]
                                              for k, val in rows.items() if k != "no_transfer"}
    if payload is not None:
        out["arrivals"] = arrivals
    return out


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["ring", "sweep", "pipeline", "ceilings", "p2p", "all"])
    ap.add_argument("--ceiling-gib", default="1,7", help="buffer sizes of the ceiling probes, GiB, comma separated")
    ap.add_argument("--json", default=None)
    ap.add_argument("--no-corun", action="store_true")
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        print("harness: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)
    v.vccl_init(0, 64)
    out = {}
    try:
        if args.what in ("ring", "all"):
            out["ring"] = ring_corun(torch)
            print(json.dumps(out["ring"]), flush=True)
        if args.what in ("pipeline", "all"):
            # 4 stages need 12 streams, which share this box's 4 hardware queues; the
            # 2-stage runs (4 streams) show the schedule without that false sharing
            out["pipeline"] = [pipeline_1f1b(torch, stages=4, fwd_iters=4000),
                               pipeline_1f1b(torch, stages=4, fwd_iters=40000, reps=3),
                               pipeline_1f1b(torch, stages=2, fwd_iters=4000),
                               pipeline_1f1b(torch, stages=2, fwd_iters=40000)]
            print(json.dumps(out["pipeline"]), flush=True)
        if args.what in ("ceilings", "all"):
            out["ceilings"] = hbm_ceilings(torch, gib=tuple(int(x) for x in args.ceiling_gib.split(",")))
        if args.what in ("p2p", "all"):
            out["p2p"] = p2p_sweep(torch)
            print(json.dumps(out["p2p"]), flush=True)
        if args.what in ("sweep", "all"):
            out["sweep"] = sweep_p64(torch, with_corun=not args.no_corun)
            print(json.dumps(out["sweep"]), flush=True)
    finally:
        v.vccl_finalize()
    if args.json:
        with open(args.json, "w") as f:
            json.dump(out, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
