"""Do the pins bite?  Plant one plausible mistake at a time in a copy of the
oracle's C source (on the CPU, in a temporary file), load the broken build in
place of the real one and require that at least one pin fails."""
import os
import subprocess
import sys

import pytest

import oracle.oracle as om
from pins import ALL_PINS

SRC = os.path.join(os.path.dirname(om.__file__), "vccl_oracle.c")

# (name, text in the source, replacement, occurrence index)
MUTANTS = [
    ("v_sdispl_transposed", "send[s] + sdispls[(size_t)s * P + r]", "send[s] + sdispls[(size_t)r * P + s]", 0),
    ("v_rdispl_transposed", "recv[r] + rdispls[(size_t)r * P + s]", "recv[r] + rdispls[(size_t)s * P + r]", 0),
    ("v_wrong_source_rank", "send[s] + sdispls", "send[r] + sdispls", 0),
    ("v_count_from_wrong_cell", "const uint64_t n = recvcounts[(size_t)r * P + s];", "const uint64_t n = recvcounts[(size_t)s * P + r];", 0),
    ("v_drops_last_byte", "for (uint64_t i = 0; i < n; ++i) dst[i] = src[i];", "for (uint64_t i = 0; i + 1 < n; ++i) dst[i] = src[i];", 0),
    ("v_no_mismatch_check", "return ORACLE_ERR_COUNT_MISMATCH;\n    if (threads", "{}\n    if (threads", 0),
    ("a2a_not_transposed", "recv[r][(uint64_t)s * c + i] = send[s][(uint64_t)r * c + i]", "recv[r][(uint64_t)r * c + i] = send[s][(uint64_t)s * c + i]", 0),
    ("a2a_source_block_wrong", "send[s][(uint64_t)r * c + i]", "send[s][(uint64_t)s * c + i]", 0),
    ("sr_wrong_direction", "uint8_t *dst = recv[send_to[s]];", "uint8_t *dst = recv[recv_from[s]];", 0),
    ("sr_no_inverse_check", "if (recv_from[r] != s) return ORACLE_ERR_ARG;", "", 0),
    ("sr_no_size_check", "if (sendbytes[s] != recvbytes[r]) return ORACLE_ERR_COUNT_MISMATCH;", "", 0),
    ("fifo_sender_slot_shifted", "uint8_t *slot = fifo + (k % (uint64_t)slots) * chunk_bytes;\n            for (uint64_t i = 0; i < n; ++i) slot[i]", "uint8_t *slot = fifo + ((k + 1) % (uint64_t)slots) * chunk_bytes;\n            for (uint64_t i = 0; i < n; ++i) slot[i]", 0),
    ("fifo_overrun", "head - tail < (uint64_t)slots;", "head - tail <= (uint64_t)slots;", 0),
    ("fifo_short_chunk_ignored", "const uint64_t n = nbytes - off < chunk_bytes ? nbytes - off : chunk_bytes;\n            const uint8_t *slot", "const uint64_t n = chunk_bytes;\n            const uint8_t *slot", 0),
    ("moe_unstable_order", "for (int64_t p = 0; p < npairs; ++p) {\n            if (ids[p] == e)", "for (int64_t p = npairs - 1; p >= 0; --p) {\n            if (ids[p] == e)", 0),
    ("moe_row_of_slot_not_token", "(order[j] / K) * row_bytes", "(order[j] % K) * row_bytes", 0),
    ("moe_no_id_check", "if (ids[p] < 0 || ids[p] >= E) return ORACLE_ERR_ARG;", "if (ids[p] < 0 || ids[p] >= E) continue;", 0),
    ("unpack_runs_forward", "uint8_t *dst = out + (uint64_t)p * row_bytes;\n            for (uint64_t i = 0; i < row_bytes; ++i) dst[i] = row[i];", "uint8_t *dst = out + (uint64_t)j * row_bytes; const uint8_t *rr = packed + (uint64_t)p * row_bytes;\n            for (uint64_t i = 0; i < row_bytes; ++i) dst[i] = rr[i];", 0),
    ("unpack_unstable", "for (int64_t p = 0; p < npairs; ++p) {\n            if (ids[p] != e) continue;", "for (int64_t p = npairs - 1; p >= 0; --p) {\n            if (ids[p] != e) continue;", 0),
    ("dedup_rank_by_modulo", "if (ids[t * K + k] / experts_per_rank == r) {", "if (ids[t * K + k] % (E / experts_per_rank) == r) {", 0),
    ("dedup_row_for_every_token", "            if (!hit) continue;\n", "", 0),
    ("dedup_first_slot_only", "hit = 1;\n                    slot_row[t * K + k] = j;", "if (!hit) slot_row[t * K + k] = j;\n                    hit = 1;", 0),
    ("dedup_token_major", "row_token[j] = t;\n            ++cnt[r];", "row_token[j] = T - 1 - t;\n            ++cnt[r];", 0),
    ("dedup_slot_row_off_by_one", "slot_row[t * K + k] = j;", "slot_row[t * K + k] = j + 1;", 0),
    ("dedup_copies_wrong_row", "const uint8_t *row = x + (uint64_t)t * row_bytes;\n            uint8_t *out = packed + (uint64_t)j * row_bytes;", "const uint8_t *row = x + (uint64_t)j * row_bytes;\n            uint8_t *out = packed + (uint64_t)j * row_bytes;", 0),
    ("dedup_no_id_check", "if (ids[p] < 0 || ids[p] >= E) return ORACLE_ERR_ARG;\n    int64_t j = 0;\n    for (int r = 0; r < R; ++r) {", "if (ids[p] < 0) return ORACLE_ERR_ARG;\n    int64_t j = 0;\n    for (int r = 0; r < R; ++r) {", 0),
    ("layout_expert_block_shifted", "for (int e = r * experts_per_rank; e < (r + 1) * experts_per_rank; ++e)", "for (int e = r; e < E; e += P)", 0),
    ("layout_recv_not_transposed", "recvcounts[(size_t)r * P + s] = sendcounts[(size_t)s * P + r];", "recvcounts[(size_t)r * P + s] = sendcounts[(size_t)r * P + s];", 0),
    ("layout_sdispl_inclusive", "sdispls[(size_t)s * P + r] = acc;\n            acc += sendcounts[(size_t)s * P + r];", "acc += sendcounts[(size_t)s * P + r];\n            sdispls[(size_t)s * P + r] = acc;", 0),
]


RUNNER = """
import ctypes, sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import oracle.oracle as om
om._lib = ctypes.CDLL({so!r})
from pins import ALL_PINS
for pin in ALL_PINS:
    try:
        pin()
    except (AssertionError, om.OracleError, ValueError, IndexError) as e:
        print("caught by", pin.__name__, type(e).__name__)
        sys.exit(3)
sys.exit(0)
"""


@pytest.mark.parametrize("name,old,new,_k", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(name, old, new, _k, tmp_path):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site for {name} no longer in the source"
    broken = text.replace(old, new, 1)
    c = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    c.write_text(broken)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-w",
                           "-o", str(so), str(c)])
    tests = os.path.dirname(os.path.abspath(__file__))
    # A broken oracle may read or write out of bounds, so it runs in a child
    # process; any non-zero exit (a failed pin or a crash) counts as caught.
    rv = subprocess.run([sys.executable, "-c",
                         RUNNER.format(root=os.path.dirname(tests), tests=tests, so=str(so))],
                        capture_output=True, text=True, timeout=300)
    assert rv.returncode != 0, f"no pin noticed the planted mistake '{name}'"
    assert rv.returncode == 3 or rv.returncode < 0, rv.stderr[-2000:]
    print(name, rv.returncode, rv.stdout.strip())
