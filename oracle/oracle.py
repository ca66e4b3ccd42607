"""ctypes front end of the plain-C oracle in ``vccl_oracle.c``.

TEST INFRASTRUCTURE ONLY: argument marshalling between NumPy arrays and the C
loops; no arithmetic of the method lives here.  Buffers are lists of
one-dimensional ``uint8`` arrays, one per virtual rank; counts and
displacements are ``uint64`` [P, P] arrays in bytes (send side indexed [s][r],
receive side [r][s]).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vccl_oracle.c")
_LIB = os.path.join(_HERE, "libvccl_oracle.so")
_lib: Optional[ctypes.CDLL] = None


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle returned {code}")
        self.code = code


def build(force: bool = False, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the oracle with gcc (-O2, OpenMP for the optional rank-loop split)."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-Wall", "-Wextra", "-o", out, src])
    return out


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _u8(a: np.ndarray) -> np.ndarray:
    if a.dtype != np.uint8 or a.ndim != 1 or not a.flags.c_contiguous:
        raise TypeError("rank buffers must be contiguous 1-D uint8 arrays")
    return a


def _ptr_array(bufs: Sequence[np.ndarray]):
    arr = (ctypes.c_void_p * len(bufs))()
    for i, b in enumerate(bufs):
        arr[i] = _u8(b).ctypes.data
    return arr


def _mat(a, P: int) -> np.ndarray:
    m = np.ascontiguousarray(a, dtype=np.uint64)
    if m.shape != (P, P):
        raise ValueError("count/displacement matrices must be [P, P]")
    return m


def _check_span(bufs, counts, displs, what: str) -> None:
    for a, b in enumerate(bufs):
        for p in range(counts.shape[1]):
            n = int(counts[a, p])
            if n and int(displs[a, p]) + n > b.size:
                raise ValueError(f"{what} segment [{a}][{p}] exceeds its buffer")


def _vp(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def alltoallv(send: List[np.ndarray], sendcounts, sdispls, recv: List[np.ndarray], recvcounts,
              rdispls, threads: int = 1) -> None:
    P = len(send)
    sc, sd, rc, rd = (_mat(m, P) for m in (sendcounts, sdispls, recvcounts, rdispls))
    _check_span(send, sc, sd, "send")
    _check_span(recv, rc, rd, "recv")
    rv = _load().oracle_alltoallv(_ptr_array(send), _vp(sc), _vp(sd), _ptr_array(recv), _vp(rc),
                                  _vp(rd), ctypes.c_int(P), ctypes.c_int(threads))
    if rv:
        raise OracleError(rv)


def alltoall(send: List[np.ndarray], recv: List[np.ndarray], bytes_per_peer: int,
             threads: int = 1) -> None:
    P = len(send)
    for b in list(send) + list(recv):
        if b.size < P * bytes_per_peer:
            raise ValueError("buffer smaller than P * bytes_per_peer")
    rv = _load().oracle_alltoall(_ptr_array(send), _ptr_array(recv), ctypes.c_uint64(bytes_per_peer),
                                 ctypes.c_int(P), ctypes.c_int(threads))
    if rv:
        raise OracleError(rv)


def sendrecv(send: List[np.ndarray], sendbytes, send_to, recv: List[np.ndarray], recvbytes,
             recv_from) -> None:
    P = len(send)
    sb = np.ascontiguousarray(sendbytes, dtype=np.uint64)
    rb = np.ascontiguousarray(recvbytes, dtype=np.uint64)
    st = np.ascontiguousarray(send_to, dtype=np.int32)
    rf = np.ascontiguousarray(recv_from, dtype=np.int32)
    for i in range(P):
        if int(sb[i]) > send[i].size or int(rb[i]) > recv[i].size:
            raise ValueError("byte count exceeds buffer")
    rv = _load().oracle_sendrecv(_ptr_array(send), _vp(sb), _vp(st), _ptr_array(recv), _vp(rb),
                                 _vp(rf), ctypes.c_int(P))
    if rv:
        raise OracleError(rv)


def sendrecv_staged(src: np.ndarray, dst: np.ndarray, nbytes: int, chunk_bytes: int, slots: int,
                    schedule: Optional[bytes] = None) -> int:
    """One connection through the chunk FIFO; returns the peak FIFO occupancy."""
    if nbytes > _u8(src).size or nbytes > _u8(dst).size:
        raise ValueError("byte count exceeds buffer")
    fifo = np.zeros(max(1, chunk_bytes * max(slots, 0)), dtype=np.uint8)
    peak = ctypes.c_uint64(0)
    sched = (ctypes.c_uint8 * len(schedule)).from_buffer_copy(schedule) if schedule else None
    rv = _load().oracle_sendrecv_staged(_vp(src), _vp(dst), ctypes.c_uint64(nbytes),
                                        ctypes.c_uint64(chunk_bytes), ctypes.c_int(slots), _vp(fifo),
                                        sched, ctypes.c_uint64(8 * len(schedule) if schedule else 0),
                                        ctypes.byref(peak))
    if rv:
        raise OracleError(rv)
    return int(peak.value)


def moe_pack(x: np.ndarray, ids: np.ndarray, row_bytes: int, num_experts: int):
    """Returns (packed uint8 [T*K*row_bytes], order int64 [T*K], cnt uint64 [E])."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    if _u8(x).size < T * row_bytes:
        raise ValueError("x smaller than T rows")
    packed = np.empty(T * K * row_bytes, dtype=np.uint8)
    order = np.empty(T * K, dtype=np.int64)
    cnt = np.zeros(num_experts, dtype=np.uint64)
    rv = _load().oracle_moe_pack(_vp(x), _vp(ids), ctypes.c_int64(T), ctypes.c_int(K),
                                 ctypes.c_uint64(row_bytes), ctypes.c_int(num_experts), _vp(packed),
                                 _vp(order), _vp(cnt))
    if rv:
        raise OracleError(rv)
    return packed, order, cnt


def moe_unpack(packed: np.ndarray, ids: np.ndarray, row_bytes: int, num_experts: int) -> np.ndarray:
    """Inverse row movement of moe_pack: returns uint8 [T*K*row_bytes] in (token, slot) order."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    if _u8(packed).size < T * K * row_bytes:
        raise ValueError("packed smaller than T*K rows")
    out = np.empty(T * K * row_bytes, dtype=np.uint8)
    rv = _load().oracle_moe_unpack(_vp(packed), _vp(ids), ctypes.c_int64(T), ctypes.c_int(K),
                                   ctypes.c_uint64(row_bytes), ctypes.c_int(num_experts), _vp(out))
    if rv:
        raise OracleError(rv)
    return out


def moe_pack_dedup(x: np.ndarray, ids: np.ndarray, row_bytes: int, num_experts: int, experts_per_rank: int):
    """One row per (token, destination rank).  Returns (packed uint8 [rows*row_bytes],
    row_token int64 [rows], cnt uint64 [R], slot_row int64 [T*K])."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, K = ids.shape
    if _u8(x).size < T * row_bytes:
        raise ValueError("x smaller than T rows")
    if experts_per_rank < 1 or num_experts % experts_per_rank:
        raise OracleError(-1)
    R = num_experts // experts_per_rank
    packed = np.empty(T * min(K, R) * row_bytes, dtype=np.uint8)
    row_token = np.empty(T * min(K, R), dtype=np.int64)
    cnt = np.zeros(R, dtype=np.uint64)
    slot_row = np.full(T * K, -1, dtype=np.int64)
    rows = ctypes.c_int64(0)
    rv = _load().oracle_moe_pack_dedup(_vp(x), _vp(ids), ctypes.c_int64(T), ctypes.c_int(K),
                                       ctypes.c_uint64(row_bytes), ctypes.c_int(num_experts),
                                       ctypes.c_int(experts_per_rank), _vp(packed), _vp(row_token),
                                       _vp(cnt), _vp(slot_row), ctypes.byref(rows))
    if rv:
        raise OracleError(rv)
    n = int(rows.value)
    return packed[:n * row_bytes], row_token[:n], cnt, slot_row


def moe_exchange_layout(cnt: np.ndarray, experts_per_rank: int, row_bytes: int):
    """cnt uint64 [P, E] -> dict of the four [P, P] byte matrices of the exchange."""
    cnt = np.ascontiguousarray(cnt, dtype=np.uint64)
    P, E = cnt.shape
    out = {k: np.zeros((P, P), dtype=np.uint64)
           for k in ("sendcounts", "sdispls", "recvcounts", "rdispls")}
    rv = _load().oracle_moe_exchange_layout(_vp(cnt), ctypes.c_int(P), ctypes.c_int(E),
                                            ctypes.c_int(experts_per_rank),
                                            ctypes.c_uint64(row_bytes), _vp(out["sendcounts"]),
                                            _vp(out["sdispls"]), _vp(out["recvcounts"]),
                                            _vp(out["rdispls"]))
    if rv:
        raise OracleError(rv)
    return out
