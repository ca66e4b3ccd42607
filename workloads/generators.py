"""Counter-based, seeded generators for every synthetic input of the path.

Everything here is a pure function of (seed, rank, index): a buffer can be
regenerated piecewise anywhere, so multi-GiB expected values never have to be
held whole.  All routines are NumPy on the host.

Workload recipes (they stand in for the NCCL-Tests style message sweeps,
pipeline-parallel activations of size S_PP = B*L*H*p (Appendix C), and the MoE
dispatch AlltoAll mentioned in Section 6 of the paper):

* payload: 64-bit word ``w`` of rank ``s`` is ``splitmix64(seed ^ (s << 48) ^ w)``
  stored little-endian.  "bf16 as random 16-bit patterns" is the same stream
  viewed as uint16 (NaN/Inf/denormal encodings included on purpose).
* activations: N(0,1) by Box-Muller in float32, rounded to nearest-even bf16.
* routing: for each token, K distinct experts drawn one after another from a
  Zipf(s) pmf over E ids (weight of id e is (e+1)^-s), redrawing on a repeat.
"""
from __future__ import annotations

import numpy as np

MASTER_SEED = 251000991

_U64 = np.uint64
_MASK53 = (1 << 53) - 1


def config_seed(n: int) -> int:
    """Seed of workload configuration number ``n`` (1-based)."""
    return MASTER_SEED + int(n)


def splitmix64(x: np.ndarray) -> np.ndarray:
    """The splitmix64 output function applied element-wise to uint64 ``x``."""
    with np.errstate(over="ignore"):
        z = (np.asarray(x, dtype=_U64) + _U64(0x9E3779B97F4A7C15)).astype(_U64)
        z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
        return z ^ (z >> _U64(31))


def _key(seed: int, rank: int) -> np.uint64:
    return _U64((int(seed) ^ (int(rank) << 48)) & 0xFFFFFFFFFFFFFFFF)


def payload_words(seed: int, rank: int, first_word: int, nwords: int) -> np.ndarray:
    """Words ``first_word .. first_word+nwords-1`` of rank ``rank``'s send stream."""
    w = np.arange(first_word, first_word + nwords, dtype=_U64)
    return splitmix64(w ^ _key(seed, rank))


def payload_bytes(seed: int, rank: int, nbytes: int, first_byte: int = 0) -> np.ndarray:
    """Bytes ``first_byte .. first_byte+nbytes-1`` of rank ``rank``'s send stream (uint8)."""
    if nbytes == 0:
        return np.zeros(0, dtype=np.uint8)
    w0 = first_byte // 8
    w1 = (first_byte + nbytes + 7) // 8
    words = payload_words(seed, rank, w0, w1 - w0).astype("<u8")
    b = words.view(np.uint8)
    off = first_byte - 8 * w0
    return b[off:off + nbytes].copy()


def _uniform_open(bits: np.ndarray) -> np.ndarray:
    """Map uint64 bits to float64 uniforms in (0, 1]."""
    return ((bits >> _U64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)


def normal_bf16_bits(seed: int, rank: int, n: int, first: int = 0) -> np.ndarray:
    """``n`` N(0,1) samples as bf16 bit patterns (uint16), elements first..first+n-1."""
    idx = np.arange(first, first + n, dtype=_U64)
    k = _key(seed ^ 0x5bf0_3635, rank)
    u1 = _uniform_open(splitmix64((idx * _U64(2)) ^ k))
    u2 = _uniform_open(splitmix64((idx * _U64(2) + _U64(1)) ^ k))
    z = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    bits = z.view(np.uint32)
    rounded = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def zipf_topk_expert_ids(seed: int, rank: int, tokens: int, topk: int, num_experts: int,
                         s: float = 1.2) -> np.ndarray:
    """int32 [tokens, topk]: per token ``topk`` distinct expert ids, Zipf(s) weighted.

    Slot order is draw order.  Draw ``j`` of token ``t`` uses the uniform derived
    from ``splitmix64(key(seed, rank) ^ (t << 20) ^ j)``; a repeated id is skipped.
    """
    if topk > num_experts:
        raise ValueError("topk exceeds the number of experts")
    w = np.arange(1, num_experts + 1, dtype=np.float64) ** (-float(s))
    cdf = np.cumsum(w / w.sum())
    cdf[-1] = 1.0
    k = _key(seed ^ 0x1d5_7a11, rank)
    t = np.arange(tokens, dtype=_U64) << _U64(20)
    out = np.full((tokens, topk), -1, dtype=np.int32)
    filled = np.zeros(tokens, dtype=np.int64)
    j = 0
    while True:
        todo = filled < topk
        if not todo.any():
            break
        if j >= (1 << 20):
            raise RuntimeError("routing draw did not terminate")
        u = _uniform_open(splitmix64(t ^ _U64(j) ^ k))
        cand = np.minimum(np.searchsorted(cdf, u, side="left"), num_experts - 1).astype(np.int32)
        fresh = todo & ~(out == cand[:, None]).any(axis=1)
        rows = np.nonzero(fresh)[0]
        out[rows, filled[rows]] = cand[rows]
        filled[rows] += 1
        j += 1
    return out


def equal_layout(P: int, bytes_per_peer: int):
    """Count/displacement matrices of the equal-block AlltoAll (all uint64 [P, P])."""
    c = np.full((P, P), bytes_per_peer, dtype=np.uint64)
    d = (np.arange(P, dtype=np.uint64) * np.uint64(bytes_per_peer))[None, :].repeat(P, axis=0)
    return {"sendcounts": c, "sdispls": d.copy(), "recvcounts": c.copy(), "rdispls": d.copy(),
            "send_sizes": np.full(P, P * bytes_per_peer, dtype=np.uint64),
            "recv_sizes": np.full(P, P * bytes_per_peer, dtype=np.uint64)}


def random_layout(seed: int, P: int, max_count: int, align: int = 1, zero_fraction: float = 0.2,
                  max_gap: int = 33):
    """A random AlltoAllv layout: counts (some zero), shuffled segment order, gaps.

    ``sendcounts``/``sdispls`` are indexed [s][r], ``recvcounts``/``rdispls`` [r][s];
    segments inside one buffer never overlap; counts, displacements and gaps are
    multiples of ``align`` bytes.  Also returns the per-rank buffer sizes.
    """
    rng = np.random.Generator(np.random.PCG64(int(seed)))
    units = max(1, max_count // align)
    counts = rng.integers(0, units + 1, size=(P, P)).astype(np.uint64) * np.uint64(align)
    counts[rng.random((P, P)) < zero_fraction] = 0

    def place(cnt_rows):
        displs = np.zeros((P, P), dtype=np.uint64)
        sizes = np.zeros(P, dtype=np.uint64)
        for a in range(P):
            pos = int(rng.integers(0, max_gap)) * align
            for b in rng.permutation(P):
                displs[a, b] = pos
                pos += int(cnt_rows[a, b]) + int(rng.integers(0, max_gap)) * align
            sizes[a] = pos + align
        return displs, sizes

    sdispls, send_sizes = place(counts)
    recvcounts = counts.T.copy()
    rdispls, recv_sizes = place(recvcounts)
    return {"sendcounts": counts, "sdispls": sdispls, "recvcounts": recvcounts, "rdispls": rdispls,
            "send_sizes": send_sizes, "recv_sizes": recv_sizes}


def ring_peers(P: int):
    """Forward ring: stage s sends to (s+1) mod P and receives from (s-1) mod P."""
    s = np.arange(P, dtype=np.int32)
    return ((s + 1) % P).astype(np.int32), ((s - 1) % P).astype(np.int32)


def pp_message_bytes(micro_batch: int, seq_len: int, hidden: int, bytes_per_element: int) -> int:
    """Pipeline-parallel message size S_PP = B * L * H * p (Appendix C)."""
    return micro_batch * seq_len * hidden * bytes_per_element
