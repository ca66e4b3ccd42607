"""Pins of the CPU oracle: each function checks the oracle against something
fixed by the paper's statement of the primitives or by mathematics (hand-worked
fixtures, NumPy library routines for the special cases that reduce to them,
invariants, exhaustive tiny cases) and raises AssertionError on a mismatch.

They are plain functions so that the mutation test can run the same list
against deliberately broken copies of the oracle.
"""
from __future__ import annotations

import itertools
import json
import os

import numpy as np

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
SENTINEL = 0xA5


def _b(s: str) -> np.ndarray:
    return np.frombuffer(s.encode("ascii"), dtype=np.uint8).copy()


def _s(a: np.ndarray) -> str:
    return a.tobytes().decode("ascii")


def _load(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def _run_layout(lay, seed, threads=1):
    P = lay["sendcounts"].shape[0]
    send = [wl.payload_bytes(seed, s, int(lay["send_sizes"][s])) for s in range(P)]
    recv = [np.full(int(lay["recv_sizes"][r]), SENTINEL, dtype=np.uint8) for r in range(P)]
    oracle.alltoallv(send, lay["sendcounts"], lay["sdispls"], recv, lay["recvcounts"],
                     lay["rdispls"], threads=threads)
    return send, recv


# ---------------------------------------------------------------- exchange ---

def pin_alltoallv_handworked():
    g = _load("alltoallv_p3_handworked.json")
    send = [_b(x) for x in g["send"]]
    recv = [_b(g["recv_prefill"]) for _ in range(g["P"])]
    oracle.alltoallv(send, g["sendcounts"], g["sdispls"], recv, g["recvcounts"], g["rdispls"])
    assert [_s(r) for r in recv] == g["recv_expected"]
    assert [_s(x) for x in send] == g["send"]


def pin_p1_identity():
    for n in (0, 1, 17, 4096):
        x = wl.payload_bytes(7, 0, n)
        y = np.full(n, SENTINEL, dtype=np.uint8)
        oracle.alltoall([x], [y], n)
        assert np.array_equal(x, y)
        y[:] = SENTINEL
        oracle.alltoallv([x], [[n]], [[0]], [y], [[n]], [[0]])
        assert np.array_equal(x, y)
        y[:] = SENTINEL
        oracle.sendrecv([x], [n], [0], [y], [n], [0])
        assert np.array_equal(x, y)


def pin_alltoall_is_axis_swap():
    for P, c in ((2, 1), (3, 5), (4, 64), (8, 33)):
        send = [wl.payload_bytes(11, s, P * c) for s in range(P)]
        recv = [np.full(P * c, SENTINEL, dtype=np.uint8) for _ in range(P)]
        oracle.alltoall(send, recv, c, threads=2)
        cube = np.stack(send).reshape(P, P, c)
        want = np.transpose(cube, (1, 0, 2)).reshape(P, P * c)
        assert np.array_equal(np.stack(recv), want)
        # the v form with the equal layout is the same exchange
        lay = wl.equal_layout(P, c)
        recv2 = [np.full(P * c, SENTINEL, dtype=np.uint8) for _ in range(P)]
        oracle.alltoallv(send, lay["sendcounts"], lay["sdispls"], recv2, lay["recvcounts"],
                         lay["rdispls"])
        assert np.array_equal(np.stack(recv2), want)


def pin_alltoallv_involution():
    """Exchanging back with the receive description as the send description
    restores every covered send byte."""
    for seed in range(6):
        P = 1 + seed % 5
        lay = wl.random_layout(100 + seed, P, 300)
        send, recv = _run_layout(lay, seed)
        back = [np.full(b.size, SENTINEL, dtype=np.uint8) for b in send]
        oracle.alltoallv(recv, lay["recvcounts"], lay["rdispls"], back, lay["sendcounts"],
                         lay["sdispls"])
        for s in range(P):
            covered = np.zeros(send[s].size, dtype=bool)
            for r in range(P):
                d, n = int(lay["sdispls"][s, r]), int(lay["sendcounts"][s, r])
                covered[d:d + n] = True
            assert np.array_equal(back[s][covered], send[s][covered])
            assert (back[s][~covered] == SENTINEL).all()


def pin_alltoallv_conservation_and_gaps():
    for seed in range(6):
        P = 2 + seed % 4
        lay = wl.random_layout(200 + seed, P, 500)
        send, recv = _run_layout(lay, 50 + seed, threads=1 + seed % 3)
        assert lay["sendcounts"].sum() == lay["recvcounts"].sum()
        sent_hist = np.zeros(256, dtype=np.int64)
        got_hist = np.zeros(256, dtype=np.int64)
        for r in range(P):
            covered = np.zeros(recv[r].size, dtype=bool)
            for s in range(P):
                d, n = int(lay["rdispls"][r, s]), int(lay["recvcounts"][r, s])
                assert not covered[d:d + n].any()
                covered[d:d + n] = True
                sd = int(lay["sdispls"][s, r])
                sent_hist += np.bincount(send[s][sd:sd + n], minlength=256)
            # per-rank received bytes equal the column sum of the send counts
            assert covered.sum() == int(lay["sendcounts"][:, r].sum())
            assert (recv[r][~covered] == SENTINEL).all(), "gap bytes were written"
            got_hist += np.bincount(recv[r][covered], minlength=256)
        assert np.array_equal(sent_hist, got_hist)


def _push_model(P, send, sc, sd, rd, recv_sizes):
    """Sender-centric restatement in pure Python: walk every send byte and push it."""
    out = [bytearray([SENTINEL]) * n for n in recv_sizes]
    for s in range(P):
        for r in range(P):
            for i in range(sc[s][r]):
                out[r][rd[r][s] + i] = int(send[s][sd[s][r] + i])
    return out


def pin_alltoallv_tiny_exhaustive():
    """P in {1,2}: every count matrix over {0,1,2,17} and every segment order;
    P = 3: a seeded sample.  Payload bytes encode (rank, offset) so a wrong
    source or shift cannot cancel."""
    vals = (0, 1, 2, 17)
    rng = np.random.Generator(np.random.PCG64(3))
    cases = []
    for P in (1, 2):
        for flat in itertools.product(vals, repeat=P * P):
            cases.append((P, np.array(flat, dtype=np.uint64).reshape(P, P)))
    for _ in range(300):
        cases.append((3, rng.choice(vals, size=(3, 3)).astype(np.uint64)))
    for P, counts in cases:
        orders = list(itertools.permutations(range(P)))
        so = orders[int(rng.integers(len(orders)))] if P == 3 else None
        for order_s in ([so] if so else orders):
            for order_r in ([orders[int(rng.integers(len(orders)))]] if P == 3 else orders):
                gap = int(rng.integers(0, 3))
                sd = np.zeros((P, P), dtype=np.uint64)
                rd = np.zeros((P, P), dtype=np.uint64)
                ssz, rsz = [], []
                for a in range(P):
                    pos = gap
                    for b in order_s:
                        sd[a, b] = pos
                        pos += int(counts[a, b]) + gap
                    ssz.append(pos + 1)
                    pos = 1
                    for b in order_r:
                        rd[a, b] = pos
                        pos += int(counts[b, a]) + gap
                    rsz.append(pos + 2)
                send = [((np.arange(n) * 7 + 64 * s + 1) % 251).astype(np.uint8)
                        for s, n in enumerate(ssz)]
                recv = [np.full(n, SENTINEL, dtype=np.uint8) for n in rsz]
                oracle.alltoallv(send, counts, sd, recv, counts.T.copy(), rd)
                want = _push_model(P, send, counts.astype(int).tolist(), sd.astype(int).tolist(),
                                   rd.astype(int).tolist(), rsz)
                for r in range(P):
                    assert recv[r].tobytes() == bytes(want[r]), (P, counts, order_s, order_r)


def pin_count_mismatch_is_an_error():
    c = np.array([[1, 2], [3, 4]], dtype=np.uint64)
    d = np.array([[0, 4], [0, 4]], dtype=np.uint64)
    send = [np.zeros(16, np.uint8), np.zeros(16, np.uint8)]
    recv = [np.zeros(16, np.uint8), np.zeros(16, np.uint8)]
    try:
        oracle.alltoallv(send, c, d, recv, c, d)   # recvcounts must be the transpose
    except oracle.OracleError as e:
        assert e.code == -2
    else:
        raise AssertionError("count mismatch not detected")
    oracle.alltoallv(send, c, d, recv, c.T.copy(), d)


# ---------------------------------------------------------------- sendrecv ---

def pin_sendrecv_handworked():
    g = _load("sendrecv_ring_p3_handworked.json")
    send = [_b(x) for x in g["send"]]
    recv = [_b(g["recv_prefill"]) for _ in range(g["P"])]
    sb = [len(x) for x in g["send"]]
    rb = [sb[g["recv_from"][r]] for r in range(g["P"])]
    oracle.sendrecv(send, sb, g["send_to"], recv, rb, g["recv_from"])
    assert [_s(r) for r in recv] == g["recv_expected"]


def pin_sendrecv_ring_is_roll():
    for P, n in ((2, 9), (5, 64), (8, 1000)):
        to, frm = wl.ring_peers(P)
        send = [wl.payload_bytes(21, s, n) for s in range(P)]
        recv = [np.full(n, SENTINEL, dtype=np.uint8) for _ in range(P)]
        oracle.sendrecv(send, [n] * P, to, recv, [n] * P, frm)
        assert np.array_equal(np.stack(recv), np.roll(np.stack(send), 1, axis=0))
        # P applications of the ring are the identity
        cur = send
        for _ in range(P):
            nxt = [np.full(n, SENTINEL, dtype=np.uint8) for _ in range(P)]
            oracle.sendrecv(cur, [n] * P, to, nxt, [n] * P, frm)
            cur = nxt
        assert np.array_equal(np.stack(cur), np.stack(send))


def pin_sendrecv_rejects_non_permutation():
    x = [np.zeros(4, np.uint8) for _ in range(3)]
    y = [np.zeros(4, np.uint8) for _ in range(3)]
    for to, frm in (([1, 1, 0], [2, 0, 1]), ([1, 2, 0], [1, 0, 2]), ([1, 2, 3], [2, 0, 1])):
        try:
            oracle.sendrecv(x, [4] * 3, to, y, [4] * 3, frm)
        except oracle.OracleError as e:
            assert e.code == -1
        else:
            raise AssertionError("bad peer tables accepted")
    try:
        oracle.sendrecv(x, [4, 3, 4], [1, 2, 0], y, [4] * 3, [2, 0, 1])
    except oracle.OracleError as e:
        assert e.code == -2
    else:
        raise AssertionError("size mismatch accepted")


def pin_staged_equals_direct():
    """The chunk-FIFO path ends with the same bytes as the direct copy under any
    interleaving; occupancy stays within the slot count; a short last chunk works."""
    rng = np.random.Generator(np.random.PCG64(5))
    for n, chunk, slots in ((0, 8, 2), (1, 8, 1), (64, 8, 8), (100, 8, 3), (1000, 64, 8),
                            (513, 512, 8), (4096 + 5, 512, 8)):
        src = wl.payload_bytes(31, 0, n + 3)
        for sched in (None, b"\x00", b"\xff", bytes(rng.integers(0, 256, 16, dtype=np.uint8))):
            dst = np.full(n + 3, SENTINEL, dtype=np.uint8)
            peak = oracle.sendrecv_staged(src, dst, n, chunk, slots, sched)
            assert np.array_equal(dst[:n], src[:n])
            assert (dst[n:] == SENTINEL).all()
            nchunks = -(-n // chunk)
            assert peak <= min(slots, nchunks)
            if sched in (None, b"\xff"):          # sender-greedy fills the FIFO
                assert peak == min(slots, nchunks)
            if sched == b"\x00" and nchunks:      # receiver-greedy keeps it at one
                assert peak == 1


# --------------------------------------------------------------------- moe ---

def pin_moe_handworked():
    g = _load("moe_dispatch_p2_handworked.json")
    cnts = []
    packed_all = []
    for s in range(g["P"]):
        packed, order, cnt = oracle.moe_pack(_b(g["x"][s]), np.array(g["ids"][s], np.int32),
                                             g["row_bytes"], g["E"])
        assert order.tolist() == g["order"][s]
        assert cnt.tolist() == g["cnt"][s]
        assert _s(packed) == g["packed"][s]
        cnts.append(cnt)
        packed_all.append(packed)
    lay = oracle.moe_exchange_layout(np.stack(cnts), g["experts_per_rank"], g["row_bytes"])
    for k in ("sendcounts", "sdispls", "recvcounts", "rdispls"):
        assert lay[k].tolist() == g[k], k
    recv = [np.full(len(x), SENTINEL, np.uint8) for x in g["recv"]]
    oracle.alltoallv(packed_all, lay["sendcounts"], lay["sdispls"], recv, lay["recvcounts"],
                     lay["rdispls"])
    assert [_s(r) for r in recv] == g["recv"]


def pin_moe_pack_is_stable_argsort():
    for seed, (T, K, E, row) in enumerate(((1, 1, 1, 3), (16, 2, 4, 8), (257, 8, 256, 6),
                                           (1000, 4, 32, 16))):
        ids = wl.zipf_topk_expert_ids(40 + seed, 0, T, K, E)
        x = wl.payload_bytes(41 + seed, 0, T * row)
        packed, order, cnt = oracle.moe_pack(x, ids, row, E)
        keys = ids.reshape(-1)
        assert np.array_equal(order, np.argsort(keys, kind="stable"))
        assert np.array_equal(cnt, np.bincount(keys, minlength=E).astype(np.uint64))
        assert int(cnt.sum()) == T * K
        # every token appears exactly K times, and un-permuting gives K copies of each row
        tok = order // K
        assert np.array_equal(np.bincount(tok, minlength=T), np.full(T, K))
        rows = packed.reshape(T * K, row)
        unperm = np.empty_like(rows)
        unperm[order] = rows
        assert np.array_equal(unperm, np.repeat(x.reshape(T, row), K, axis=0))
        # keys are non-decreasing along the packed order
        assert (np.diff(keys[order]) >= 0).all()


def pin_moe_unpack_handworked():
    g = _load("moe_dispatch_p2_handworked.json")
    for s in range(g["P"]):
        out = oracle.moe_unpack(_b(g["unpack_in"][s]), np.array(g["ids"][s], np.int32), g["row_bytes"], g["E"])
        assert _s(out) == g["unpack_out"][s]


def pin_moe_unpack_inverts_pack():
    """unpack(pack(x)) gives every row K times (dispatch then its inverse replicates),
    and unpack is a permutation of rows: NumPy's scatter with the stable argsort."""
    for seed, (T, K, E, row) in enumerate(((1, 1, 1, 4), (33, 3, 7, 8), (500, 8, 256, 16))):
        ids = wl.zipf_topk_expert_ids(70 + seed, 0, T, K, E)
        x = wl.payload_bytes(71 + seed, 0, T * row)
        packed, order, _ = oracle.moe_pack(x, ids, row, E)
        back = oracle.moe_unpack(packed, ids, row, E)
        assert np.array_equal(back.reshape(T * K, row), np.repeat(x.reshape(T, row), K, axis=0))
        y = wl.payload_bytes(72 + seed, 1, T * K * row)          # arbitrary distinct rows
        got = oracle.moe_unpack(y, ids, row, E).reshape(T * K, row)
        want = np.empty_like(got)
        want[np.argsort(ids.reshape(-1), kind="stable")] = y.reshape(T * K, row)
        assert np.array_equal(got, want)


def pin_moe_dedup_handworked():
    g = _load("moe_dispatch_dedup_handworked.json")
    packed, row_token, cnt, slot_row = oracle.moe_pack_dedup(_b(g["x"]), np.array(g["ids"], np.int32),
                                                             g["row_bytes"], g["E"], g["experts_per_rank"])
    assert _s(packed) == g["packed"]
    assert row_token.tolist() == g["row_token"]
    assert cnt.tolist() == g["cnt"]
    assert slot_row.tolist() == g["slot_row"]


def pin_moe_dedup_is_unique_over_rank_token_keys():
    """Rows sorted by (destination rank, token) with duplicates removed is NumPy's
    unique over the keys rank*T + token; the slot map inverts it; a slot's row holds
    its token's bytes and lies in its rank's block."""
    for seed, (T, K, E, epr, row) in enumerate(((1, 1, 1, 1, 3), (7, 3, 6, 2, 4), (300, 8, 256, 32, 8),
                                                (129, 4, 12, 1, 16), (64, 5, 10, 10, 2))):
        ids = wl.zipf_topk_expert_ids(80 + seed, 0, T, K, E)
        x = wl.payload_bytes(81 + seed, 0, T * row)
        packed, row_token, cnt, slot_row = oracle.moe_pack_dedup(x, ids, row, E, epr)
        R = E // epr
        rank = (ids // epr).astype(np.int64)
        keys = (rank * T + np.arange(T, dtype=np.int64)[:, None]).reshape(-1)
        u, inv = np.unique(keys, return_inverse=True)
        assert np.array_equal(row_token, u % T)
        assert np.array_equal(cnt, np.bincount(u // T, minlength=R).astype(np.uint64))
        assert np.array_equal(slot_row, inv.reshape(-1))
        rows = packed.reshape(-1, row)
        assert rows.shape[0] == u.size == int(cnt.sum())
        assert np.array_equal(rows, x.reshape(T, row)[row_token])
        assert np.array_equal(rows[slot_row], np.repeat(x.reshape(T, row), K, axis=0))
        first = np.concatenate(([0], np.cumsum(cnt.astype(np.int64))))
        assert ((slot_row >= first[rank.reshape(-1)]) & (slot_row < first[rank.reshape(-1) + 1])).all()
        # every token appears once per distinct destination rank
        distinct = np.array([len(set(r)) for r in rank.tolist()])
        assert np.array_equal(np.bincount(row_token, minlength=T), distinct)


def pin_moe_dedup_special_cases():
    # (a) no two slots of a token share a rank: the per-expert pack with rank ids
    T, K, P, row = 200, 3, 8, 8
    rng = np.random.Generator(np.random.PCG64(5))
    ranks = np.stack([rng.permutation(P)[:K] for _ in range(T)]).astype(np.int32)
    epr = 4
    ids = (ranks * epr + rng.integers(0, epr, size=(T, K))).astype(np.int32)
    x = wl.payload_bytes(90, 0, T * row)
    packed, row_token, cnt, slot_row = oracle.moe_pack_dedup(x, ids, row, P * epr, epr)
    pk, order, c = oracle.moe_pack(x, ranks, row, P)
    assert np.array_equal(packed, pk) and np.array_equal(cnt, c)
    assert np.array_equal(row_token, order // K)
    inv = np.empty(T * K, dtype=np.int64)
    inv[order] = np.arange(T * K)
    assert np.array_equal(slot_row, inv)
    # (b) every expert on one rank: each token once, in order - the identity
    ids = wl.zipf_topk_expert_ids(91, 0, 50, 4, 16)
    x = wl.payload_bytes(92, 0, 50 * 6)
    packed, row_token, cnt, slot_row = oracle.moe_pack_dedup(x, ids, 6, 16, 16)
    assert np.array_equal(packed, x) and cnt.tolist() == [50]
    assert np.array_equal(slot_row, np.repeat(np.arange(50), 4))
    # (c) bad arguments
    for bad in (lambda: oracle.moe_pack_dedup(x, ids, 6, 16, 5),
                lambda: oracle.moe_pack_dedup(x, np.full((50, 4), 16, np.int32), 6, 16, 4)):
        try:
            bad()
        except oracle.OracleError:
            continue
        raise AssertionError("bad argument accepted")


def pin_moe_layout_properties():
    rng = np.random.Generator(np.random.PCG64(9))
    for P, epr, row in ((1, 4, 2), (2, 3, 10), (8, 32, 14336)):
        E = P * epr
        cnt = rng.integers(0, 50, size=(P, E)).astype(np.uint64)
        lay = oracle.moe_exchange_layout(cnt, epr, row)
        per_rank = cnt.reshape(P, P, epr).sum(axis=2) * np.uint64(row)
        assert np.array_equal(lay["sendcounts"], per_rank)
        assert np.array_equal(lay["recvcounts"], per_rank.T)
        ex = lambda m: np.cumsum(m, axis=1) - m
        assert np.array_equal(lay["sdispls"], ex(per_rank))
        assert np.array_equal(lay["rdispls"], ex(per_rank.T))


def pin_moe_rejects_bad_ids():
    x = np.zeros(8, np.uint8)
    for bad in (-1, 4):
        try:
            oracle.moe_pack(x, np.array([[0, bad]], np.int32), 4, 4)
        except oracle.OracleError as e:
            assert e.code == -1
        else:
            raise AssertionError("out-of-range expert id accepted")


# ------------------------------------------------------------------- sizes ---

def pin_pp_message_size():
    g = _load("pp_message_sizes.json")
    for c in g["cases"]:
        n = wl.pp_message_bytes(c["B"], c["L"], c["H"], c["p"])
        assert n == c["bytes"]
        if c["paper_says_MiB"]:
            assert n == c["paper_says_MiB"] * (1 << 20)


ALL_PINS = [
    pin_alltoallv_handworked,
    pin_p1_identity,
    pin_alltoall_is_axis_swap,
    pin_alltoallv_involution,
    pin_alltoallv_conservation_and_gaps,
    pin_alltoallv_tiny_exhaustive,
    pin_count_mismatch_is_an_error,
    pin_sendrecv_handworked,
    pin_sendrecv_ring_is_roll,
    pin_sendrecv_rejects_non_permutation,
    pin_staged_equals_direct,
    pin_moe_handworked,
    pin_moe_pack_is_stable_argsort,
    pin_moe_unpack_handworked,
    pin_moe_unpack_inverts_pack,
    pin_moe_dedup_handworked,
    pin_moe_dedup_is_unique_over_rank_token_keys,
    pin_moe_dedup_special_cases,
    pin_moe_layout_properties,
    pin_moe_rejects_bad_ids,
    pin_pp_message_size,
]
