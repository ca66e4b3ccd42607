"""ctypes binding with the same names as the C boundary in ``include/vccl.h``.

Buffers are passed as sequences of device addresses (``int``) or of objects with
a ``data_ptr()`` method (torch tensors); count tables as anything NumPy can turn
into ``uint64``; streams as an ``int`` handle (``torch.cuda.current_stream().cuda_stream``)
or ``None`` for the null stream.  Nothing is computed here.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

MODE_CU = 0
MODE_CE = 1
MODE_CU_STAGED = 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libvccl.so")
_lib: Optional[ctypes.CDLL] = None

_u64p = ctypes.POINTER(ctypes.c_uint64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_vpp = ctypes.POINTER(ctypes.c_void_p)

EXPORTS = {
    "vccl_init": (ctypes.c_int, [ctypes.c_int, ctypes.c_int]),
    "vccl_finalize": (ctypes.c_int, []),
    "vccl_last_error": (ctypes.c_char_p, []),
    "vccl_set_option": (ctypes.c_int, [ctypes.c_char_p, ctypes.c_char_p]),
    "vccl_get_option": (ctypes.c_int, [ctypes.c_char_p, ctypes.c_char_p, ctypes.c_int]),
    "vccl_sendrecv": (ctypes.c_int, [_vpp, _u64p, _i32p, _vpp, _u64p, _i32p, ctypes.c_int,
                                     ctypes.c_int, ctypes.c_void_p]),
    "vccl_sendrecv_staged_status": (ctypes.c_int, []),
    "vccl_p2p_reginfo": (ctypes.c_int, [ctypes.c_int, _u64p, _u64p, _u64p, _vpp]),
    "vccl_p2p_export": (ctypes.c_int, [ctypes.c_char_p, ctypes.c_void_p, ctypes.c_uint64, _vpp]),
    "vccl_p2p_connect": (ctypes.c_int, [ctypes.c_char_p, ctypes.c_double, _vpp]),
    "vccl_p2p_recv": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p]),
    "vccl_p2p_send": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]),
    "vccl_p2p_record": (ctypes.c_int, [ctypes.c_void_p, _u64p, _u64p, _u64p, _u64p, _u64p]),
    "vccl_p2p_abort": (ctypes.c_int, [ctypes.c_void_p]),
    "vccl_p2p_close": (ctypes.c_int, [ctypes.c_void_p]),
    "vccl_alltoall": (ctypes.c_int, [_vpp, _vpp, ctypes.c_uint64, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_void_p]),
    "vccl_alltoallv": (ctypes.c_int, [_vpp, _u64p, _u64p, _vpp, _u64p, _u64p, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_void_p]),
    "vccl_plan_alltoallv": (ctypes.c_int, [_vpp, _u64p, _u64p, _vpp, _u64p, _u64p, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                           ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_uint32),
                                           ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint32),
                                           ctypes.POINTER(ctypes.c_int)]),
    "vccl_moe_pack": (ctypes.c_int, [_vpp, _vpp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_uint64, ctypes.c_int, _vpp, ctypes.c_void_p,
                                     ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "vccl_moe_pack_noalloc": (ctypes.c_int, [_vpp, _vpp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                             ctypes.c_uint64, ctypes.c_int, _vpp, ctypes.c_void_p,
                                             ctypes.c_void_p, ctypes.c_void_p]),
    "vccl_moe_pack_per_rank": (ctypes.c_int, [_vpp, _vpp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_uint64, ctypes.c_int, ctypes.c_int, _vpp,
                                              ctypes.c_void_p, ctypes.c_void_p, _vpp, ctypes.c_void_p,
                                              ctypes.c_void_p]),
    "vccl_moe_dispatch_fused": (ctypes.c_int, [_vpp, _vpp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                               ctypes.c_uint64, ctypes.c_int, ctypes.c_int, _vpp, _u64p,
                                               ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_void_p]),
    "vccl_moe_combine_fused": (ctypes.c_int, [_vpp, _u64p, _vpp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.c_uint64, ctypes.c_int, ctypes.c_int, _vpp,
                                              ctypes.c_void_p]),
    "vccl_moe_unpack": (ctypes.c_int, [_vpp, _vpp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_uint64, ctypes.c_int, _vpp, ctypes.c_void_p]),
    "vccl_moe_exchange_layout": (ctypes.c_int, [_u64p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_uint64, _u64p, _u64p, _u64p, _u64p]),
    "vccl_hbm_probe": (ctypes.c_int, [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_uint64,
                                      ctypes.c_uint64, ctypes.c_void_p]),
    "vccl_fma_probe": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint32,
                                      ctypes.c_uint64, ctypes.c_void_p]),
    "vccl_fma_probe_clocks": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint32,
                                             ctypes.c_uint64, ctypes.c_void_p]),
    "vccl_device_wall_clock_khz": (ctypes.c_int, []),
    "vccl_monitor_create": (ctypes.c_void_p, [ctypes.c_int, ctypes.c_uint64]),
    "vccl_monitor_destroy": (None, [ctypes.c_void_p]),
    "vccl_monitor_post": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64]),
    "vccl_monitor_complete": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_void_p]),
    "vccl_monitor_totals": (ctypes.c_int, [ctypes.c_void_p, _u64p, _u64p, ctypes.c_void_p]),
    "vccl_proxy_monitor": (ctypes.c_int, [ctypes.c_int, _u64p, _u64p, ctypes.c_void_p]),
    "vccl_proxy_stats": (ctypes.c_int, [_u64p, _u64p, _u64p, _u64p]),
    "vccl_proxy_cpu_time": (ctypes.c_int, [_u64p, _u64p]),
    "vccl_device_cu_count": (ctypes.c_int, []),
}


class VcclError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"vccl status {code}: {message}")
        self.code = code
        self.message = message


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load libvccl.so (built in-tree by ``paper_2510_00991_amd/build.py``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2510_00991_amd.build` "
                "(there is no fallback path)")
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(rv: int) -> int:
    if rv < 0:
        raise VcclError(rv, vccl_last_error())
    return rv


def _addr(b) -> int:
    if b is None:
        return 0
    if hasattr(b, "data_ptr"):
        return int(b.data_ptr())
    return int(b)


def _ptrs(bufs: Sequence):
    if isinstance(bufs, ctypes.Array):   # already marshalled by pointer_array()
        return bufs
    arr = (ctypes.c_void_p * len(bufs))()
    for i, b in enumerate(bufs):
        arr[i] = _addr(b)
    return arr


def pointer_array(bufs: Sequence):
    """The host array of device pointers a call takes, built once: pass it in place of
    the list of tensors when the same buffers are used call after call (marshalling
    P tensors costs more than a small exchange)."""
    return _ptrs(bufs)


def _u64(a, shape=None) -> np.ndarray:
    m = np.ascontiguousarray(a, dtype=np.uint64)
    if shape is not None and m.shape != shape:
        raise ValueError(f"expected shape {shape}, got {m.shape}")
    return m


def _p64(a: np.ndarray):
    return a.ctypes.data_as(_u64p)


def _stream(s) -> ctypes.c_void_p:
    return ctypes.c_void_p(int(s) if s else 0)


def vccl_last_error() -> str:
    return load().vccl_last_error().decode("utf-8", "replace")


def vccl_init(device: int = 0, max_ranks: int = 64) -> None:
    _check(load().vccl_init(device, max_ranks))


def vccl_finalize() -> None:
    _check(load().vccl_finalize())


def vccl_set_option(key: str, value) -> None:
    _check(load().vccl_set_option(key.encode(), str(value).encode()))


def vccl_get_option(key: str) -> str:
    buf = ctypes.create_string_buffer(512)
    _check(load().vccl_get_option(key.encode(), buf, 512))
    return buf.value.decode()


def vccl_device_cu_count() -> int:
    return _check(load().vccl_device_cu_count())


def vccl_sendrecv(sendbuf, sendbytes, send_to, recvbuf, recvbytes, recv_from, P: int, mode: int,
                  stream=None) -> None:
    sb, rb = _u64(sendbytes, (P,)), _u64(recvbytes, (P,))
    st = np.ascontiguousarray(send_to, dtype=np.int32)
    rf = np.ascontiguousarray(recv_from, dtype=np.int32)
    if st.shape != (P,) or rf.shape != (P,) or len(sendbuf) != P or len(recvbuf) != P:
        raise ValueError("per-rank arrays must have P entries")
    _check(load().vccl_sendrecv(_ptrs(sendbuf), _p64(sb), st.ctypes.data_as(_i32p), _ptrs(recvbuf),
                                _p64(rb), rf.ctypes.data_as(_i32p), P, mode, _stream(stream)))


def vccl_sendrecv_staged_status() -> None:
    _check(load().vccl_sendrecv_staged_status())


def vccl_p2p_reginfo(receiver_rank: int):
    """(receiverReady, copyStarted, copyDone, receiverRegAddr) of one connection."""
    a, b, c = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
    p = ctypes.c_void_p()
    _check(load().vccl_p2p_reginfo(receiver_rank, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                   ctypes.byref(p)))
    return a.value, b.value, c.value, p.value or 0


def vccl_p2p_export(name: str, recvbuf, capacity: int) -> int:
    """Receiver side of a connection between two processes; returns the connection handle."""
    h = ctypes.c_void_p()
    _check(load().vccl_p2p_export(name.encode(), ctypes.c_void_p(_addr(recvbuf)), int(capacity), ctypes.byref(h)))
    return h.value


def vccl_p2p_connect(name: str, timeout_s: float = 30.0) -> int:
    h = ctypes.c_void_p()
    _check(load().vccl_p2p_connect(name.encode(), float(timeout_s), ctypes.byref(h)))
    return h.value


def vccl_p2p_recv(conn: int, offset: int, nbytes: int, stream=None) -> None:
    _check(load().vccl_p2p_recv(ctypes.c_void_p(conn), int(offset), int(nbytes), _stream(stream)))


def vccl_p2p_send(conn: int, sendbuf, nbytes: int, stream=None) -> None:
    _check(load().vccl_p2p_send(ctypes.c_void_p(conn), ctypes.c_void_p(_addr(sendbuf)), int(nbytes), _stream(stream)))


def vccl_p2p_record(conn: int):
    """(receiverReady, copyStarted, copyDone, receiverRegOffset, mismatches) of a cross-process connection."""
    v = [ctypes.c_uint64() for _ in range(5)]
    _check(load().vccl_p2p_record(ctypes.c_void_p(conn), *[ctypes.byref(x) for x in v]))
    return tuple(x.value for x in v)


def vccl_p2p_abort(conn: int) -> None:
    _check(load().vccl_p2p_abort(ctypes.c_void_p(conn)))


def vccl_p2p_close(conn: int) -> None:
    _check(load().vccl_p2p_close(ctypes.c_void_p(conn)))


def vccl_alltoall(sendbuf, recvbuf, bytes_per_peer: int, P: int, mode: int, stream=None) -> None:
    if len(sendbuf) != P or len(recvbuf) != P:
        raise ValueError("per-rank arrays must have P entries")
    _check(load().vccl_alltoall(_ptrs(sendbuf), _ptrs(recvbuf), int(bytes_per_peer), P, mode,
                                _stream(stream)))


def vccl_alltoallv(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P: int, mode: int,
                   stream=None) -> None:
    if len(sendbuf) != P or len(recvbuf) != P:
        raise ValueError("per-rank arrays must have P entries")
    sc, sd, rc, rd = (_u64(m, (P, P)) for m in (sendcounts, sdispls, recvcounts, rdispls))
    _check(load().vccl_alltoallv(_ptrs(sendbuf), _p64(sc), _p64(sd), _ptrs(recvbuf), _p64(rc),
                                 _p64(rd), P, mode, _stream(stream)))


def vccl_plan_alltoallv(sendbuf, sendcounts, sdispls, recvbuf, recvcounts, rdispls, P: int,
                        cu_unroll: int = 1, cu_threads: int = 64):
    """Planner only (no device needed).  Returns (descriptors, grid_x, grid_y, tile_bytes,
    all_aligned); descriptors is a structured array with fields src, dst, bytes, head, lead."""
    sc, sd, rc, rd = (_u64(m, (P, P)) for m in (sendcounts, sdispls, recvcounts, rdispls))
    n, gx, gy, al = ctypes.c_int(), ctypes.c_uint32(), ctypes.c_uint32(), ctypes.c_int()
    tb = ctypes.c_uint32()
    args = (_ptrs(sendbuf), _p64(sc), _p64(sd), _ptrs(recvbuf), _p64(rc), _p64(rd), P, cu_unroll, cu_threads)
    _check(load().vccl_plan_alltoallv(*args, None, 0, ctypes.byref(n), ctypes.byref(gx), ctypes.byref(gy),
                                      ctypes.byref(tb), ctypes.byref(al)))
    dt = np.dtype([("src", np.uint64), ("dst", np.uint64), ("bytes", np.uint64), ("head", np.uint32),
                   ("lead", np.uint32)])
    out = np.zeros(max(1, n.value), dtype=dt)
    _check(load().vccl_plan_alltoallv(*args, ctypes.c_void_p(out.ctypes.data), out.size, ctypes.byref(n),
                                      ctypes.byref(gx), ctypes.byref(gy), ctypes.byref(tb), ctypes.byref(al)))
    return out[:n.value], gx.value, gy.value, tb.value, bool(al.value)


def vccl_moe_pack(x, expert_ids, P: int, tokens: int, topk: int, row_bytes: int, num_experts: int,
                  packed, counts_dev, counts_host=None, bad_ids_dev=None, stream=None) -> None:
    """counts_dev / bad_ids_dev: device tensors (uint64 [P, E] as int64 storage, uint32 [1]);
    counts_host: pinned host tensor of the same shape, or None."""
    if len(x) != P or len(expert_ids) != P or len(packed) != P:
        raise ValueError("per-rank arrays must have P entries")
    _check(load().vccl_moe_pack(_ptrs(x), _ptrs(expert_ids), P, tokens, topk, int(row_bytes),
                                num_experts, _ptrs(packed), ctypes.c_void_p(_addr(counts_dev)),
                                ctypes.c_void_p(_addr(counts_host)),
                                ctypes.c_void_p(_addr(bad_ids_dev)), _stream(stream)))


def vccl_moe_pack_noalloc(x, expert_ids, P: int, tokens: int, topk: int, row_bytes: int, num_experts: int,
                          packed, counts_dev, bad_ids_dev=None, stream=None) -> None:
    """vccl_moe_pack without any allocation (index data in the library's static device array)."""
    if len(x) != P or len(expert_ids) != P or len(packed) != P:
        raise ValueError("per-rank arrays must have P entries")
    _check(load().vccl_moe_pack_noalloc(_ptrs(x), _ptrs(expert_ids), P, tokens, topk, int(row_bytes),
                                        num_experts, _ptrs(packed), ctypes.c_void_p(_addr(counts_dev)),
                                        ctypes.c_void_p(_addr(bad_ids_dev)), _stream(stream)))


def vccl_moe_pack_per_rank(x, expert_ids, P: int, tokens: int, topk: int, row_bytes: int, num_experts: int,
                           experts_per_rank: int, packed, counts_dev, counts_host=None, slot_row=None,
                           bad_ids_dev=None, stream=None) -> None:
    """One row per (token, destination rank).  counts_dev: device uint64 [P, R] (int64 storage),
    R = num_experts // experts_per_rank; slot_row: None or P device tensors of tokens*topk uint32
    (int32 storage)."""
    if len(x) != P or len(expert_ids) != P or len(packed) != P or (slot_row is not None and len(slot_row) != P):
        raise ValueError("per-rank arrays must have P entries")
    _check(load().vccl_moe_pack_per_rank(_ptrs(x), _ptrs(expert_ids), P, tokens, topk, int(row_bytes),
                                         num_experts, experts_per_rank, _ptrs(packed),
                                         ctypes.c_void_p(_addr(counts_dev)), ctypes.c_void_p(_addr(counts_host)),
                                         _ptrs(slot_row) if slot_row is not None else None,
                                         ctypes.c_void_p(_addr(bad_ids_dev)), _stream(stream)))


def vccl_moe_dispatch_fused(x, expert_ids, P: int, tokens: int, topk: int, row_bytes: int, num_experts: int,
                            experts_per_rank: int, recv, recv_capacity_rows, counts_dev, layout_dev,
                            layout_host=None, status_dev=None, stream=None) -> None:
    """Pack and exchange in one pass.  recv_capacity_rows: P row counts (host); layout_dev /
    layout_host: uint64 [4, P, P] (int64 storage) device tensor / pinned host tensor;
    status_dev: device uint32 [2] (int32 storage), zeroed by the caller."""
    if len(x) != P or len(expert_ids) != P or len(recv) != P:
        raise ValueError("per-rank arrays must have P entries")
    cap = _u64(recv_capacity_rows, (P,))
    _check(load().vccl_moe_dispatch_fused(_ptrs(x), _ptrs(expert_ids), P, tokens, topk, int(row_bytes),
                                          num_experts, experts_per_rank, _ptrs(recv), _p64(cap),
                                          ctypes.c_void_p(_addr(counts_dev)), ctypes.c_void_p(_addr(layout_dev)),
                                          ctypes.c_void_p(_addr(layout_host)), ctypes.c_void_p(_addr(status_dev)),
                                          _stream(stream)))


def vccl_moe_combine_fused(back, back_capacity_rows, expert_ids, P: int, tokens: int, topk: int,
                           row_bytes: int, num_experts: int, experts_per_rank: int, out, stream=None) -> None:
    """Inverse exchange and un-permute in one pass: out[s] row t*topk+k from back[rank of the expert]."""
    if len(back) != P or len(expert_ids) != P or len(out) != P:
        raise ValueError("per-rank arrays must have P entries")
    cap = _u64(back_capacity_rows, (P,))
    _check(load().vccl_moe_combine_fused(_ptrs(back), _p64(cap), _ptrs(expert_ids), P, tokens, topk,
                                         int(row_bytes), num_experts, experts_per_rank, _ptrs(out),
                                         _stream(stream)))


def vccl_moe_unpack(packed, expert_ids, P: int, tokens: int, topk: int, row_bytes: int,
                    num_experts: int, out, stream=None) -> None:
    if len(packed) != P or len(expert_ids) != P or len(out) != P:
        raise ValueError("per-rank arrays must have P entries")
    _check(load().vccl_moe_unpack(_ptrs(packed), _ptrs(expert_ids), P, tokens, topk, int(row_bytes),
                                  num_experts, _ptrs(out), _stream(stream)))


def vccl_moe_exchange_layout(counts, P: int, num_experts: int, experts_per_rank: int, row_bytes: int):
    cnt = _u64(counts, (P, num_experts))
    out = [np.zeros((P, P), dtype=np.uint64) for _ in range(4)]
    _check(load().vccl_moe_exchange_layout(_p64(cnt), P, num_experts, experts_per_rank,
                                           int(row_bytes), *[_p64(o) for o in out]))
    return {"sendcounts": out[0], "sdispls": out[1], "recvcounts": out[2], "rdispls": out[3]}


class MonitorSample(ctypes.Structure):
    _fields_ = [("t_ns", ctypes.c_uint64), ("bw_message", ctypes.c_double), ("bw_window", ctypes.c_double),
                ("outstanding", ctypes.c_uint64), ("anomaly", ctypes.c_int)]

    def as_dict(self):
        return {"t_ns": self.t_ns, "bw_message": self.bw_message, "bw_window": self.bw_window,
                "outstanding": self.outstanding, "anomaly": bool(self.anomaly)}


def vccl_monitor_create(window: int = 8, history_ns: int = 10_000_000) -> int:
    h = load().vccl_monitor_create(window, history_ns)
    if not h:
        raise VcclError(-1, vccl_last_error())
    return h


def vccl_monitor_destroy(handle: int) -> None:
    load().vccl_monitor_destroy(handle)


def vccl_monitor_post(handle: int, msg_id: int, nbytes: int, t_post_ns: int) -> None:
    _check(load().vccl_monitor_post(handle, msg_id, nbytes, t_post_ns))


def vccl_monitor_complete(handle: int, msg_id: int, t_done_ns: int) -> dict:
    s = MonitorSample()
    _check(load().vccl_monitor_complete(handle, msg_id, t_done_ns, ctypes.byref(s)))
    return s.as_dict()


def vccl_monitor_totals(handle: int) -> dict:
    a, b, s = ctypes.c_uint64(), ctypes.c_uint64(), MonitorSample()
    _check(load().vccl_monitor_totals(handle, ctypes.byref(a), ctypes.byref(b), ctypes.byref(s)))
    return {"messages": a.value, "anomalies": b.value, "last": s.as_dict()}


def vccl_proxy_monitor(primitive: int) -> dict:
    a, b, s = ctypes.c_uint64(), ctypes.c_uint64(), MonitorSample()
    _check(load().vccl_proxy_monitor(primitive, ctypes.byref(a), ctypes.byref(b), ctypes.byref(s)))
    return {"messages": a.value, "anomalies": b.value, "last": s.as_dict()}


def vccl_hbm_probe(kind: int, src, dst, nbytes: int, threads: int, vecs_per_lane: int, row_index=None,
                   n_rows: int = 0, row_bytes: int = 0, stream=None) -> None:
    """kind 0 read, 1 write, 2 copy, 3 write n_rows rows of row_bytes at row_index[i] (device int32 tensor or None)."""
    _check(load().vccl_hbm_probe(kind, ctypes.c_void_p(_addr(src)), ctypes.c_void_p(_addr(dst)), int(nbytes),
                                 threads, vecs_per_lane, ctypes.c_void_p(_addr(row_index)), int(n_rows),
                                 int(row_bytes), _stream(stream)))


def vccl_fma_probe(out_dev, workgroups: int, threads: int, iters: int, stream=None) -> None:
    _check(load().vccl_fma_probe(ctypes.c_void_p(_addr(out_dev)), workgroups, threads, int(iters),
                                 _stream(stream)))


def vccl_fma_probe_clocks(out_dev, clocks_dev, workgroups: int, threads: int, iters: int, stream=None) -> None:
    """clocks_dev: device tensor of 2 * workgroups int64 (shader-clock ticks, real-time ticks per workgroup)."""
    _check(load().vccl_fma_probe_clocks(ctypes.c_void_p(_addr(out_dev)), ctypes.c_void_p(_addr(clocks_dev)),
                                        workgroups, threads, int(iters), _stream(stream)))


def vccl_device_wall_clock_khz() -> int:
    return _check(load().vccl_device_wall_clock_khz())


def vccl_proxy_stats():
    v = [ctypes.c_uint64() for _ in range(4)]
    _check(load().vccl_proxy_stats(*[ctypes.byref(x) for x in v]))
    return {"ops": v[0].value, "copies": v[1].value, "bytes": v[2].value, "issue_ns": v[3].value}


def vccl_proxy_cpu_time():
    """Processor time (ns) used so far by the sender and the receiver proxy thread."""
    a, b = ctypes.c_uint64(), ctypes.c_uint64()
    _check(load().vccl_proxy_cpu_time(ctypes.byref(a), ctypes.byref(b)))
    return {"sender_ns": a.value, "receiver_ns": b.value}
