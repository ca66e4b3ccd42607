#!/usr/bin/env python3
"""Benchmark of the P2P data-movement path on one MI355X.

A step is one AlltoAll of the headline workload (P = 8 virtual ranks, 16 MiB per
peer, 1 GiB sent, random 16-bit patterns) through the C boundary on the
compute-unit copy path: host planning, launch and the copy itself.  The metric is
achieved GB/s counted as bytes read plus bytes written, set against the HBM peak.
The same run also reports the copy-engine path on the same workload, the co-run
slowdown each path causes to a compute-bound FMA kernel (headline workload, the
SendRecv ring in every mode, four points of the P = 64 message sweep), the MoE
dispatch and combine, and the CPU oracle timed on the host cores.

Prints ONE JSON line.  `python bench.py --gpus 1 --steps K --warmup W`.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Imported before anything touches the GPU: the package asks the HIP runtime to carry out
# stream waits in the command processor (no helper kernel on the copy-engine path).
from paper_2510_00991_amd.harness import time_calls, time_region  # noqa: E402  (timing helpers)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
CSRC = os.path.join(ROOT, "paper_2510_00991_amd", "csrc")


def cpu_baseline(P, c, budget_s=12.0):
    """The oracle, as it stands, on the host cores: the destination-rank loop
    spread over min(P, cores) threads; a bounded number of passes."""
    import numpy as np

    import oracle
    import workloads as wl

    cores = min(P, len(os.sched_getaffinity(0)))
    send = [wl.payload_bytes(wl.config_seed(2), s, P * c) for s in range(P)]
    recv = [np.empty(P * c, dtype=np.uint8) for _ in range(P)]
    oracle.alltoall(send, recv, c, threads=cores)        # touch pages
    t_end = time.perf_counter() + budget_s
    times = []
    while time.perf_counter() < t_end and len(times) < 60:     # about 2 s on 8 cores: 10-20 s of processor time
        t0 = time.perf_counter()
        oracle.alltoall(send, recv, c, threads=cores)
        times.append(time.perf_counter() - t0)
    t1 = time.perf_counter()
    oracle.alltoall(send, recv, c, threads=1)
    single = time.perf_counter() - t1
    gb = 2.0 * P * P * c / 1e9
    return {"value": gb / statistics.median(times), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{len(times)} passes of the full P={P}, {c >> 20} MiB-per-peer AlltoAll "
                      f"({P * P * c >> 20} MiB sent per pass), bytes read + written",
            "single_core_GBps": gb / single}


def headline(torch, v, a2a_cu, args, algo_bytes, P, c, send, recv):
    """The timed region of the benchmark: K AlltoAll calls on the compute-unit path."""
    # One call is one launch of the copy kernel (64 descriptors travel as kernel
    # arguments), so the device time of the train of K calls divided by K is the
    # kernel's average duration in the timed region.
    wall, dev = time_region(torch, a2a_cu, args.steps, args.warmup)
    ms_per_step = wall / args.steps * 1e3
    value = algo_bytes / (wall / args.steps) / 1e9
    kern = dev / args.steps
    achieved = algo_bytes / kern / 1e9
    # the same kernel with an event pair around every single call (outside the timed
    # region: the events themselves delay the next launch)
    _, per = time_calls(torch, a2a_cu, min(args.steps, 20), 0)
    out = {
        "metric": "AlltoAll(v) achieved GB/s (R+W) vs HBM peak; co-run compute slowdown %",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "AlltoAll P=8 virtual ranks, 16 MiB per peer (1 GiB sent), "
                               "bf16 payload as random 16-bit patterns, compute-unit copy path",
                   "P": P, "bytes_per_peer": c, "mode": "cu",
                   "cu_unroll": int(v.vccl_get_option("cu_unroll")),
                   "cu_threads": int(v.vccl_get_option("cu_threads")),
                   "cu_nontemporal": int(v.vccl_get_option("cu_nontemporal")),
                   "cu_wg_per_cu": int(v.vccl_get_option("cu_wg_per_cu"))},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(),
                     "traffic_source": "committed rocprofv3 counter summary (profiles/), not this run",
                     "kernel": "copy_aligned_kernel", "kernel_us": kern * 1e6,
                     "kernel_us_single_calls": statistics.mean(per) * 1e6,
                     "algorithmic_bytes": algo_bytes},
        "frac_of_hbm_peak": value / HBM_PEAK_GBS,
    }
    # correctness spot check of what was just timed: block s of recv[r] is block r of send[s]
    for r, s in ((0, 7), (5, 2)):
        assert torch.equal(recv[r][s * c:(s + 1) * c], send[s][r * c:(r + 1) * c])
    return out, kern


def _summary_fields(name, sources):
    """`key: value` fields of a committed profiler summary; None when the file is missing or
    the sources it was taken from have changed since (the summary carries their hash)."""
    try:
        fields = {}
        for line in open(os.path.join(ROOT, "profiles", name)):
            if ":" in line:
                k, val = line.split(":", 1)
                fields[k.strip()] = val.strip()
        digest = hashlib.sha256(b"".join(open(os.path.join(CSRC, n), "rb").read() for n in sources)).hexdigest()
        if fields.get("kernel_source_sha256", fields.get("source_sha256")) != digest:
            return None
        return fields
    except OSError:
        return None


def measured_traffic():
    """HBM bytes per launch of the headline kernel from the committed counter
    summary (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known size); None
    when there is no summary or the kernel source has changed since it was taken."""
    f = _summary_fields("copy_aligned_kernel_alltoall_p8_16MiB_pmc.txt", ("copy_kernel.hip", "device_util.h"))
    try:
        return float(f["traffic_bytes_per_launch"]) if f else None
    except (KeyError, ValueError):
        return None


def copy_engine_dispatches(sync):
    """Kernel dispatches and wavefronts (SQ_WAVES) per copy-engine call in the given ordering
    mode, from the committed counter summary; None when the proxy source has changed since."""
    f = _summary_fields("copy_engine_sq_waves.txt", ("proxy.cpp",))
    if not f:
        return None
    try:
        return {"dispatches_per_call": float(f[f"dispatches_per_call_{sync}"]),
                "sq_waves_per_call": float(f[f"sq_waves_per_call_{sync}"]),
                "source": "committed rocprofv3 --pmc SQ_WAVES summary (profiles/), not this run"}
    except (KeyError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--legs", default="cu,ce,small,corun,sendrecv,sweep,moe,cpu",
                    help="comma list of legs to run: cu (always), ce, small, corun, sendrecv, sweep, moe, cpu, "
                         "calib (a plain 1 GiB device copy, used to scale profiler counters)")
    ap.add_argument("--ce-sync", default="default", choices=["default", "memops", "event", "host"],
                    help="ordering of the copy-engine path: the library's default for this process, stream "
                         "write/wait-value operations, event + wait-value, or none (the call blocks)")
    ap.add_argument("--pairs", type=int, default=20, help="alone/beside pairs per co-run figure of a compute-unit path")
    ap.add_argument("--ce-pairs", type=int, default=60,
                    help="pairs per co-run figure of the copy-engine path: its effect is looked for at the tenth of a "
                         "per cent, below the probe's own run-to-run scatter (a few per cent of all probes run 4-5 %% "
                         "long, alone or not), so it gets more pairs")
    args = ap.parse_args()
    legs = set(x.strip() for x in args.legs.split(",") if x.strip())
    unknown = legs - {"cu", "ce", "small", "corun", "sendrecv", "sweep", "moe", "cpu", "calib"}
    if unknown:
        print(f"bench.py: unknown legs {sorted(unknown)}", file=sys.stderr)
        sys.exit(2)
    if args.gpus != 1:
        print("bench.py: this path is built and measured on ONE GPU (P virtual ranks in one HBM); "
              "--gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2510_00991_amd as v
    import workloads as wl
    from paper_2510_00991_amd.harness import CoRun

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    v.vccl_init(0, 64)
    if args.ce_sync != "default":
        v.vccl_set_option("ce_sync", args.ce_sync)
    ce_sync = v.vccl_get_option("ce_sync")
    out = {}
    try:
        P, c = 8, 16 << 20
        total = P * P * c
        seed = wl.config_seed(2)
        send = [torch.from_numpy(wl.payload_bytes(seed, s, P * c)).cuda() for s in range(P)]
        recv = [torch.zeros(P * c, dtype=torch.uint8, device="cuda") for _ in range(P)]
        st = int(torch.cuda.current_stream().cuda_stream)
        algo_bytes = 2.0 * total                          # every byte is read once and written once
        # Buffers of the P = 64 sweep: allocated before the first copy-engine measurement and
        # freed after the last (after device memory has been freed the copy engines of this
        # device run at about 60 % of their rate for a second or two).
        P5, sweep_sizes = 64, (4 << 10, 16 << 10, 64 << 10, 4 << 20)
        sweep_bufs = {}
        if "sweep" in legs:
            for c5 in sweep_sizes:
                s5 = [torch.empty(P5 * c5, dtype=torch.uint8, device="cuda") for _ in range(P5)]
                r5 = [torch.empty(P5 * c5, dtype=torch.uint8, device="cuda") for _ in range(P5)]
                for s in range(P5):     # seeded payload: one MiB per rank, repeated through the buffer (what a
                    n = min(P5 * c5, 1 << 20)   # transfer costs its neighbours depends on the values it moves)
                    s5[s].view(-1, n).copy_(torch.from_numpy(wl.payload_bytes(wl.config_seed(5), s, n)).cuda())
                # for small blocks the copy-engine path also gets receive buffers that are slices of one
                # allocation (a constant stride between the ranks): one pitched copy per rank, not 64 plain ones
                slab5 = ([b[:P5 * c5] for b in torch.empty((P5, P5 * c5 + 4096), dtype=torch.uint8, device="cuda").unbind(0)]
                         if c5 <= 32 << 10 else None)
                sweep_bufs[c5] = (s5, r5, slab5)

        def a2a_cu():
            v.vccl_alltoall(send, recv, c, P, v.MODE_CU, st)

        def a2a_ce():
            v.vccl_alltoall(send, recv, c, P, v.MODE_CE, st)

        if "cu" not in legs:      # profiling runs that isolate another leg
            out = {"metric": None, "value": None, "note": "headline leg skipped (--legs)"}
            kern = 350e-6
        else:
            out, kern = headline(torch, v, a2a_cu, args, algo_bytes, P, c, send, recv)

        if "calib" in legs:
            a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            b = torch.empty_like(a)
            w, _ = time_region(torch, lambda: b.copy_(a), 5, 2)
            out["calib_copy_1GiB"] = {"GBps": 2.0 * (1 << 30) / (w / 5) / 1e9, "launches": 7}
        if "ce" in legs:
            k_ce = max(3, min(args.steps, 10))
            cpu0 = v.vccl_proxy_cpu_time()
            wall_ce, _ = time_region(torch, a2a_ce, k_ce, 2)
            cpu1 = v.vccl_proxy_cpu_time()
            proxy_ms = (cpu1["sender_ns"] - cpu0["sender_ns"] + cpu1["receiver_ns"] - cpu0["receiver_ns"]) * 1e-6
            out["copy_engine"] = {"GBps": algo_bytes / (wall_ce / k_ce) / 1e9,
                                  "ms_per_step": wall_ce / k_ce * 1e3, "steps": k_ce,
                                  "kind": v.vccl_get_option("ce_kind"), "sync": ce_sync,
                                  "stream_wait_in_command_processor": int(v.vccl_get_option("ce_wait_on_cp")),
                                  "engines": int(v.vccl_get_option("ce_engines")),
                                  "kernels": copy_engine_dispatches(ce_sync),
                                  # processor time of the proxy threads over warm-up + timed calls
                                  "proxy_cpu_ms_per_step": proxy_ms / (k_ce + 2),
                                  "proxy_cpu_ms_per_GB_moved": proxy_ms / ((k_ce + 2) * total / 1e9)}
            for r, s in ((1, 6), (7, 0)):
                assert torch.equal(recv[r][s * c:(s + 1) * c], send[s][r * c:(r + 1) * c])
        co = CoRun(torch) if legs & {"corun", "sendrecv", "sweep"} else None
        if "corun" in legs:
            # co-run: FMA probe alone vs beside each path (protocol in harness.CoRun)
            cor_cu = co.beside(lambda sh: v.vccl_alltoall(send, recv, c, P, v.MODE_CU, sh), algo_bytes, kern,
                               reps=args.pairs)
            # the same path with its grid capped to one workgroup per compute unit
            # (4 wavefronts of 8 vectors per lane each, so that 256 workgroups can keep HBM busy)
            v.vccl_set_option("cu_max_wg", co.cu)
            v.vccl_set_option("cu_unroll", 8)
            v.vccl_set_option("cu_threads", 256)
            wcap, _ = time_region(torch, a2a_cu, 5, 2)
            cor_cap = co.beside(lambda sh: v.vccl_alltoall(send, recv, c, P, v.MODE_CU, sh), algo_bytes, wcap / 5,
                                reps=args.pairs)
            cor_cap["GBps_alone"] = algo_bytes / (wcap / 5) / 1e9
            # and to a quarter of that: 64 workgroups
            v.vccl_set_option("cu_max_wg", 64)
            wcap64, _ = time_region(torch, a2a_cu, 3, 1)
            cor_cap64 = co.beside(lambda sh: v.vccl_alltoall(send, recv, c, P, v.MODE_CU, sh), algo_bytes,
                                  wcap64 / 3, reps=args.pairs)
            cor_cap64["GBps_alone"] = algo_bytes / (wcap64 / 3) / 1e9
            # and to 32: about the rate of the copy engines, for a comparison at equal bytes per second
            v.vccl_set_option("cu_max_wg", 32)
            wcap32, _ = time_region(torch, a2a_cu, 3, 1)
            cor_cap32 = co.beside(lambda sh: v.vccl_alltoall(send, recv, c, P, v.MODE_CU, sh), algo_bytes,
                                  wcap32 / 3, reps=args.ce_pairs)
            cor_cap32["GBps_alone"] = algo_bytes / (wcap32 / 3) / 1e9
            v.vccl_set_option("cu_max_wg", 0)
            v.vccl_set_option("cu_unroll", 1)
            v.vccl_set_option("cu_threads", 64)
            wce, _ = time_region(torch, a2a_ce, 3, 1)
            cor_ce = co.beside(lambda sh: v.vccl_alltoall(send, recv, c, P, v.MODE_CE, sh), algo_bytes, wce / 3,
                               reps=args.ce_pairs)
            out["corun"] = {"probe": f"FMA kernel, {co.cu} workgroups x {co.threads} threads, "
                                     f"{co.iters} rounds of 64 FMAs per lane",
                            "protocol": f"{args.pairs} alone/beside pairs per compute-unit figure, {args.ce_pairs} per "
                                        "copy-engine figure, in alternating order; median, mean and quartiles of the "
                                        "paired ratios; probe_shader_ticks_pct = change of the probe's own shader-clock "
                                        "tick count (held up inside compute units), shader_clock_MHz_* = its ticks per "
                                        "real-time tick (the chip lowering its clock)",
                            "cu_path": cor_cu, "cu_path_capped_1wg_per_cu": cor_cap,
                            "cu_path_capped_64wg": cor_cap64, "cu_path_capped_32wg": cor_cap32,
                            "copy_engine_path": cor_ce}
        if "small" in legs:
            # the small configuration (P = 4 x 64 KiB, 2 MiB of traffic): too small for a rate, so the time from
            # the call to the completion of the stream on an idle device, both paths, median of 30 single calls
            P1, c1 = 4, 64 << 10
            s1 = [torch.from_numpy(wl.payload_bytes(wl.config_seed(1), s, P1 * c1)).cuda() for s in range(P1)]
            r1 = [torch.zeros(P1 * c1, dtype=torch.uint8, device="cuda") for _ in range(P1)]
            s1p, r1p = v.pointer_array(s1), v.pointer_array(r1)
            small = {}
            for name, mode in (("cu", v.MODE_CU), ("ce", v.MODE_CE)):
                lat = []
                for _ in range(32):
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    v.vccl_alltoall(s1p, r1p, c1, P1, mode, st)
                    torch.cuda.synchronize()
                    lat.append(time.perf_counter() - t0)
                small[name + "_call_to_completion_us"] = statistics.median(lat[2:]) * 1e6
                for r, s in ((1, 3), (2, 0)):
                    assert torch.equal(r1[r][s * c1:(s + 1) * c1], s1[s][r * c1:(r + 1) * c1])
            out["alltoall_p4_64KiB"] = small
        if "sendrecv" in legs:
            # SendRecv ring, 8 stages x 64 MiB: rate and probe slowdown in every mode
            n = 64 << 20
            to, frm = wl.ring_peers(P)
            send_p, recv_p = v.pointer_array(send), v.pointer_array(recv)    # marshalled once, not per call
            sr = {}
            for name, mode in (("cu_direct", v.MODE_CU), ("cu_staged", v.MODE_CU_STAGED),
                               ("copy_engine", v.MODE_CE)):
                fn = lambda sh=st, m=mode: v.vccl_sendrecv(send_p, [n] * P, to, recv_p, [n] * P, frm, P, m, sh)
                # median of three trains: the copy engines' rate wanders from train to train
                k = 20   # calls per train: the one synchronisation at its end weighs 1/20 per call
                runs = sorted((time_region(torch, fn, k, 2) for _ in range(3)), key=lambda t: t[0])
                w, dev = runs[1]
                sr[name] = {"GBps": 2.0 * P * n / (w / k) / 1e9, "ms": w / k * 1e3, "calls_per_train": k,
                            # device time of the train / calls: for the kernel modes one call is one launch
                            "device_us_per_call": dev / k * 1e6,
                            "GBps_device": 2.0 * P * n / (dev / k) / 1e9}
                if co is not None and "corun" in legs:
                    sr[name]["corun"] = co.beside(fn, 2.0 * P * n, w / 5,
                                                  reps=args.ce_pairs if mode == v.MODE_CE else max(8, args.pairs // 2))
            v.vccl_sendrecv_staged_status()
            for r in (0, 5):
                assert torch.equal(recv[r][:n], send[frm[r]][:n])
            out["sendrecv_ring_8x64MiB"] = sr
        if "sweep" in legs:
            # four points of the P = 64 message sweep: both paths' rate and the probe's slowdown, and
            # what one device of the 64 does in the exchange (its own 64 outgoing blocks)
            rows = []
            for c5 in sweep_sizes:
                s5, r5, slab5 = sweep_bufs[c5]
                sp, rp = v.pointer_array(s5), v.pointer_array(r5)
                slab_p = v.pointer_array(slab5) if slab5 is not None else rp
                moved = 2.0 * P5 * P5 * c5
                row = {"bytes_per_peer": c5}
                for name, mode in (("cu", v.MODE_CU), ("ce", v.MODE_CE)):
                    to = slab_p if name == "ce" else rp
                    fn = lambda sh=st, m=mode, to=to: v.vccl_alltoall(sp, to, c5, P5, m, sh)
                    k = 10 if name == "cu" else 3
                    t = statistics.median(time_region(torch, fn, k, 2)[0] for _ in range(3)) / k
                    row[name] = {"us": t * 1e6, "GBps": moved / t / 1e9}
                    if name == "ce":     # the same call with plain copies only (one per block)
                        v.vccl_set_option("ce_pitched", 0)
                        tp = statistics.median(time_region(torch, fn, k, 2)[0] for _ in range(3)) / k
                        v.vccl_set_option("ce_pitched", 1)
                        row[name]["us_plain_copies"] = tp * 1e6
                        row[name]["receive_buffers"] = ("slices of one allocation" if slab5 is not None
                                                        else "separate allocations")
                    if "corun" in legs:
                        row[name]["corun"] = co.beside(fn, moved, t,
                                                       reps=args.ce_pairs // 2 if name == "ce" else max(8, args.pairs // 2))
                for r, s in ((3, 60), (63, 1)):     # block r of send[s] is block s of recv[r]
                    for dst in (r5, slab5 or r5):
                        assert torch.equal(dst[r][s * c5:(s + 1) * c5], s5[s][r * c5:(r + 1) * c5])
                one = np.zeros((P5, P5), dtype=np.uint64)
                one[0, :] = c5
                displs = np.tile(np.arange(P5, dtype=np.uint64) * np.uint64(c5), (P5, 1))
                for name, mode in (("cu", v.MODE_CU), ("ce", v.MODE_CE)):
                    fn = lambda sh=st, m=mode: v.vccl_alltoallv(sp, one, displs, rp, one.T.copy(), displs, P5, m, sh)
                    row[name]["one_rank_share_us"] = statistics.median(
                        time_region(torch, fn, 10, 2)[0] for _ in range(3)) / 10 * 1e6
                rows.append(row)
            out["alltoall_sweep_p64"] = rows
        if "moe" in legs:
            # MoE pack, config 3 shapes
            T, K, E, H = 8192, 8, 256, 7168
            row = H * 2
            x = [torch.from_numpy(wl.normal_bf16_bits(wl.config_seed(3), s, T * H).view(np.uint8)).cuda()
                 for s in range(P)]
            ids = [torch.from_numpy(wl.zipf_topk_expert_ids(wl.config_seed(3), s, T, K, E).reshape(-1).copy()).cuda()
                   for s in range(P)]
            packed = [torch.empty(T * K * row, dtype=torch.uint8, device="cuda") for _ in range(P)]
            counts = torch.zeros((P, E), dtype=torch.int64, device="cuda")
            counts_h = torch.zeros((P, E), dtype=torch.int64).pin_memory()
            fn = lambda: v.vccl_moe_pack(x, ids, P, T, K, row, E, packed, counts, counts_h, None, st)
            w, _ = time_region(torch, fn, 5, 2)
            pack_bytes = P * (T * row + T * K * 4 + T * K * row)
            lay = v.vccl_moe_exchange_layout(counts_h.numpy().astype(np.uint64), P, E, E // P, row)
            rcv = [torch.empty(int(lay["recvcounts"][r].sum()), dtype=torch.uint8, device="cuda")
                   for r in range(P)]
            fx = lambda: v.vccl_alltoallv(packed, lay["sendcounts"], lay["sdispls"], rcv,
                                          lay["recvcounts"], lay["rdispls"], P, v.MODE_CU, st)
            wx, _ = time_region(torch, fx, 5, 2)
            # the same exchange on the copy engines (incast on rank 0: 5 of the 7 GiB land there)
            fxe = lambda: v.vccl_alltoallv(packed, lay["sendcounts"], lay["sdispls"], rcv,
                                           lay["recvcounts"], lay["rdispls"], P, v.MODE_CE, st)
            wxe, _ = time_region(torch, fxe, 2, 1)
            outp = [torch.empty(T * K * row, dtype=torch.uint8, device="cuda") for _ in range(P)]
            fu = lambda: v.vccl_moe_unpack(packed, ids, P, T, K, row, E, outp, st)
            wu, _ = time_region(torch, fu, 5, 2)
            out["moe_combine_unpack"] = {"GBps": 2.0 * P * T * K * row / (wu / 5) / 1e9, "ms": wu / 5 * 1e3}
            out["moe_dispatch"] = {
                "pack_GBps": pack_bytes / (w / 5) / 1e9, "pack_ms": w / 5 * 1e3,
                "pack_frac_of_hbm_peak": pack_bytes / (w / 5) / 1e9 / HBM_PEAK_GBS,
                "exchange_GBps": 2.0 * float(lay["sendcounts"].sum()) / (wx / 5) / 1e9,
                "exchange_ms": wx / 5 * 1e3,
                "exchange_copy_engine_GBps": 2.0 * float(lay["sendcounts"].sum()) / (wxe / 2) / 1e9,
                "exchange_copy_engine_ms": wxe / 2 * 1e3,
                "recv_bytes_per_rank": [int(lay["recvcounts"][r].sum()) for r in range(P)]}
            # the same dispatch with one row per (token, destination rank)
            counts_r = torch.zeros((P, P), dtype=torch.int64, device="cuda")
            counts_rh = torch.zeros((P, P), dtype=torch.int64).pin_memory()
            fr = lambda: v.vccl_moe_pack_per_rank(x, ids, P, T, K, row, E, E // P, packed, counts_r, counts_rh,
                                                  None, None, st)
            wr, _ = time_region(torch, fr, 5, 2)
            rows_r = int(counts_rh.numpy().sum())
            lay_r = v.vccl_moe_exchange_layout(counts_rh.numpy().astype(np.uint64), P, P, 1, row)
            fxr = lambda: v.vccl_alltoallv(packed, lay_r["sendcounts"], lay_r["sdispls"], rcv,
                                           lay_r["recvcounts"], lay_r["rdispls"], P, v.MODE_CU, st)
            wxr, _ = time_region(torch, fxr, 5, 2)
            out["moe_dispatch_per_rank"] = {
                "rows": rows_r, "rows_per_slot_form": P * T * K,
                "pack_GBps": (P * (T * row + T * K * 4) + rows_r * row) / (wr / 5) / 1e9, "pack_ms": wr / 5 * 1e3,
                "exchange_GBps": 2.0 * float(lay_r["sendcounts"].sum()) / (wxr / 5) / 1e9,
                "exchange_ms": wxr / 5 * 1e3,
                "recv_bytes_per_rank": [int(lay_r["recvcounts"][r].sum()) for r in range(P)]}
            # pack and exchange fused: rows written once, straight into the receive buffers
            cap = np.array([int(lay["recvcounts"][r].sum()) // row for r in range(P)], dtype=np.uint64)
            layout_d = torch.zeros((4, P, P), dtype=torch.int64, device="cuda")
            status_d = torch.zeros(2, dtype=torch.int32, device="cuda")
            ff = lambda: v.vccl_moe_dispatch_fused(x, ids, P, T, K, row, E, E // P, rcv, cap, counts, layout_d,
                                                   None, status_d, st)
            wf, _ = time_region(torch, ff, 5, 2)
            assert status_d.cpu().tolist() == [0, 0]
            out["moe_dispatch_fused"] = {"GBps": pack_bytes / (wf / 5) / 1e9, "ms": wf / 5 * 1e3,
                                         "frac_of_hbm_peak": pack_bytes / (wf / 5) / 1e9 / HBM_PEAK_GBS,
                                         "two_step_ms": (w + wx) / 5 * 1e3}
            # the way back fused: inverse exchange + un-permute in one pass
            fc = lambda: v.vccl_moe_combine_fused(rcv, cap, ids, P, T, K, row, E, E // P, outp, st)
            wc, _ = time_region(torch, fc, 5, 2)
            out["moe_combine_fused"] = {"GBps": 2.0 * P * T * K * row / (wc / 5) / 1e9, "ms": wc / 5 * 1e3,
                                        "two_step_ms": (wx + wu) / 5 * 1e3}
            # spot check of what was timed last: the fused round trip gives every token's row back K times
            t_chk = 4097
            for s in (0, 6):
                got = outp[s].view(T, K, row)[t_chk]
                assert torch.equal(got, x[s].view(T, row)[t_chk].expand(K, row))
            del x, ids, packed, rcv, outp
        del send, recv, sweep_bufs
        torch.cuda.empty_cache()
    finally:
        v.vccl_finalize()

    out["cpu_baseline"] = cpu_baseline(8, 16 << 20) if "cpu" in legs else None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
