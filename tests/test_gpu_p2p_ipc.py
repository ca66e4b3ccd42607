"""The two-process form of the SM-free SendRecv (the paper's Section 3.2): a receiver
process registers its buffer and owns the handshake record in shared memory, a sender
process maps both and its proxy drives the copy engines into the receiver's buffer.  Both
processes are children of this test, each started fresh (tests/p2p_child.py); the receiver
checks every transfer against the oracle's SendRecv."""
import os
import subprocess
import sys

import pytest

from gpu_util import require_gpu

pytestmark = pytest.mark.gpu

CHILD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "p2p_child.py")


def _run_pair(name, n_transfers, nbytes, sync, scenario):
    require_gpu()
    try:
        os.unlink("/dev/shm" + name)          # a name left behind by a killed run
    except OSError:
        pass
    args = [str(n_transfers), str(nbytes), sync, scenario]
    procs = [subprocess.Popen([sys.executable, "-u", "-X", "faulthandler", CHILD, role, name] + args,
                              stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
             for role in ("receiver", "sender")]
    outs = []
    for p in procs:
        try:                                   # the children bound their own waits (40 s) and give up cleanly
            outs.append(p.communicate(timeout=170)[0])
        except subprocess.TimeoutExpired:
            p.kill()                           # never leave a child behind
            outs.append("(killed after 170 s) " + (p.communicate()[0] or ""))
    report = "\n".join(f"--- {role} (rc {p.returncode}):\n{out[-3000:]}"
                       for role, p, out in zip(("receiver", "sender"), procs, outs))
    for role, p, out in zip(("receiver", "sender"), procs, outs):
        assert p.returncode == 0 and f"P2P-OK {role}" in out, report
    assert not os.path.exists("/dev/shm" + name), "the receiver removes the record's name when it closes"


@pytest.mark.parametrize("sync", ["event", "memops", "host"])
def test_two_process_sendrecv_matches_the_oracle(sync):
    _run_pair(f"/vccl_test_{os.getpid()}_{sync}", 7, (3 << 20) + 4321, sync, "stream")


def test_two_process_sendrecv_64mib_activation():
    """The pipeline message of the SendRecv workload (1 x 4096 x 8192 bf16 = 64 MiB) between two processes."""
    _run_pair(f"/vccl_test_{os.getpid()}_big", 3, 64 << 20, "event", "stream")


def test_two_process_byte_count_mismatch_copies_nothing():
    _run_pair(f"/vccl_test_{os.getpid()}_mm", 1, 8192, "event", "mismatch")


def test_abort_releases_a_receive_whose_sender_never_comes():
    """Failure handling, forced from the host: a receive is posted on a connection nobody
    connects to, the stream waits; vccl_p2p_abort ends the transfer without a copy, the
    stream resumes, the failure is reported by the next copy-engine call, and the connection
    refuses further transfers.  No kernel waits for ever."""
    torch = require_gpu()
    import time
    import numpy as np
    import paper_2510_00991_amd as v
    v.vccl_init(0, 8)
    name = f"/vccl_test_{os.getpid()}_abort"
    try:
        buf = torch.full((1 << 16,), 0xA5, dtype=torch.uint8, device="cuda")
        conn = v.vccl_p2p_export(name, buf[256:], (1 << 16) - 256)
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            v.vccl_p2p_recv(conn, 128, 4096, int(stream.cuda_stream))
            after = buf.clone()
        time.sleep(0.05)
        assert not stream.query(), "the stream must wait for the transfer"
        assert v.vccl_p2p_record(conn)[:3] == (1, 0, 0)          # ready raised, nothing started
        v.vccl_p2p_abort(conn)
        stream.synchronize()
        assert bool((after == 0xA5).all())
        with pytest.raises(v.VcclError) as e:                     # the failed transfer is reported once
            v.vccl_alltoall([buf], [buf[32768:]], 16, 1, v.MODE_CE, int(stream.cuda_stream))
        assert e.value.code == -4
        with pytest.raises(v.VcclError) as e:
            v.vccl_p2p_recv(conn, 0, 16, int(stream.cuda_stream))
        assert e.value.code == -7
        v.vccl_alltoall([buf], [buf[32768:]], 16, 1, v.MODE_CE, int(stream.cuda_stream))   # the library works on
        stream.synchronize()
        assert np.array_equal(buf[32768:32784].cpu().numpy(), buf[:16].cpu().numpy())
        v.vccl_p2p_close(conn)
        assert not os.path.exists("/dev/shm" + name)
    finally:
        v.vccl_finalize()


def test_p2p_calls_reject_what_cannot_work():
    """Argument errors of the cross-process calls, none of which needs a peer: a bad name, a
    buffer that reaches past its allocation, a name that is taken, a connect that finds no
    export before its deadline, a receive beyond the registered bytes, a send on the
    receiving end.  Nothing is enqueued by a call that fails."""
    torch = require_gpu()
    import paper_2510_00991_amd as v
    v.vccl_init(0, 8)
    name = f"/vccl_test_{os.getpid()}_args"
    try:
        buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
        st = int(torch.cuda.current_stream().cuda_stream)
        for bad in ("no_slash", "/with/two", ""):
            with pytest.raises(v.VcclError) as e:
                v.vccl_p2p_export(bad, buf, 1 << 16)
            assert e.value.code == -1, bad
        with pytest.raises(v.VcclError) as e:          # torch's allocations are at least 512 B apart, never 1 TiB long
            v.vccl_p2p_export(name, buf, 1 << 40)
        assert e.value.code == -1
        assert not os.path.exists("/dev/shm" + name)
        conn = v.vccl_p2p_export(name, buf, 1 << 16)
        with pytest.raises(v.VcclError) as e:          # the name is taken
            v.vccl_p2p_export(name, buf, 1 << 16)
        assert e.value.code == -1
        with pytest.raises(v.VcclError) as e:
            v.vccl_p2p_connect(name + "_nobody", 0.05)
        assert e.value.code == -7
        with pytest.raises(v.VcclError) as e:          # beyond the registered bytes
            v.vccl_p2p_recv(conn, (1 << 16) - 8, 16, st)
        assert e.value.code == -1
        with pytest.raises(v.VcclError) as e:          # the exporting end receives, it does not send
            v.vccl_p2p_send(conn, buf, 16, st)
        assert e.value.code == -1
        assert v.vccl_p2p_record(conn)[:3] == (0, 0, 0)   # none of the failed calls left a transfer behind
        torch.cuda.synchronize()
        v.vccl_p2p_close(conn)
        assert not os.path.exists("/dev/shm" + name)
    finally:
        v.vccl_finalize()


def test_close_with_a_transfer_outstanding_aborts_it_after_its_deadline():
    """vccl_p2p_close must not wait for ever for a peer that never comes: after its deadline
    (shortened here) it aborts the connection, the stream is released with the buffer
    untouched, the name is removed, and the call says what it did."""
    torch = require_gpu()
    import paper_2510_00991_amd as v
    v.vccl_init(0, 8)
    name = f"/vccl_test_{os.getpid()}_close"
    try:
        v.vccl_set_option("p2p_close_wait_ms", 100)
        buf = torch.full((4096,), 0x3C, dtype=torch.uint8, device="cuda")
        conn = v.vccl_p2p_export(name, buf, 4096)
        stream = torch.cuda.Stream()
        v.vccl_p2p_recv(conn, 0, 4096, int(stream.cuda_stream))
        with pytest.raises(v.VcclError) as e:
            v.vccl_p2p_close(conn)
        assert e.value.code == -7
        stream.synchronize()                                   # released by the abort
        assert bool((buf == 0x3C).all())
        assert not os.path.exists("/dev/shm" + name)
        with pytest.raises(v.VcclError):                       # the aborted transfer is reported once
            v.vccl_alltoall([buf], [buf[2048:]], 16, 1, v.MODE_CE, int(stream.cuda_stream))
        v.vccl_alltoall([buf], [buf[2048:]], 16, 1, v.MODE_CE, int(stream.cuda_stream))
        stream.synchronize()
    finally:
        v.vccl_finalize()
