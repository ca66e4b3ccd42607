"""One end of a SendRecv connection between two processes on one GPU; started (twice, as
receiver and as sender) by tests/test_gpu_p2p_ipc.py.  The receiver compares what arrives
with the CPU oracle's SendRecv of the payload the sender is known to send (both sides
draw it from the seeded generator).  Prints "P2P-OK" on success."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import paper_2510_00991_amd as v   # noqa: E402  (first: it prepares the process for the copy-engine path)
import numpy as np                 # noqa: E402
import torch                       # noqa: E402

import workloads as wl             # noqa: E402

SENTINEL = 0xA5
SEED = 9100


def wait(stream, conn, what, seconds=40.0):
    """Bounded wait for the stream: if the peer never does its part, give the connection up
    (which releases the stream) instead of waiting for ever."""
    import time
    t0 = time.time()
    while not stream.query():
        if time.time() - t0 > seconds:
            rec = v.vccl_p2p_record(conn)
            v.vccl_p2p_abort(conn)
            stream.synchronize()
            raise RuntimeError(f"{what}: not complete after {seconds:.0f} s, record (ready, started, done, offset, "
                               f"mismatches) = {rec}; connection aborted")
        time.sleep(0.0005)


def sizes(n_transfers, nbytes):
    """(offset in the registered buffer, byte count) of every transfer: alternating halves of the
    buffer, odd offsets, shrinking odd sizes - and one empty transfer."""
    out = []
    for i in range(n_transfers):
        nb = 0 if i == 2 else nbytes - 1001 * i
        out.append(((i % 2) * nbytes + 16 * (i % 3) + (i % 5), nb))
    return out


def receiver(name, n_transfers, nbytes, sync, scenario):
    import oracle
    cap = 2 * nbytes + 4096
    buf = torch.full((cap,), SENTINEL, dtype=torch.uint8, device="cuda")
    conn = v.vccl_p2p_export(name, buf, cap)
    print("exported", flush=True)
    stream = torch.cuda.Stream()
    sh = int(stream.cuda_stream)
    if scenario == "mismatch":
        with torch.cuda.stream(stream):
            v.vccl_p2p_recv(conn, 0, 4096, sh)
            got = buf.clone()
        wait(stream, conn, "mismatched transfer")
        assert bool((got == SENTINEL).all()), "a mismatched transfer must not write anything"
        rec = v.vccl_p2p_record(conn)
        assert rec[0] == rec[1] == rec[2] == 1 and rec[4] == 1, rec
    else:
        for i, (off, nb) in enumerate(sizes(n_transfers, nbytes)):
            with torch.cuda.stream(stream):
                buf.fill_(SENTINEL)                    # earlier work on the stream writes the buffer: the transfer comes after it
                v.vccl_p2p_recv(conn, off, nb, sh)
                got = buf.clone()                      # later work on the stream sees the arrived bytes
            wait(stream, conn, f"receive {i}")
            print("received", i, flush=True)
            want = np.full(cap, SENTINEL, dtype=np.uint8)
            payload = wl.payload_bytes(SEED + i, 1, nb)
            none = np.zeros(0, np.uint8)
            # rank 1 (the sender process) sends nb bytes to rank 0 (this process)
            oracle.sendrecv([none, payload], [0, nb], [1, 0], [want[off:off + nb], none], [nb, 0], [1, 0])
            got = got.cpu().numpy()
            if not np.array_equal(got, want):
                bad = np.nonzero(got != want)[0]
                raise AssertionError(f"transfer {i}: {bad.size} bytes differ, first at {bad[0]}")
        rec = v.vccl_p2p_record(conn)
        assert rec[0] == rec[1] == rec[2] == n_transfers and rec[4] == 0, rec
    v.vccl_p2p_close(conn)


def sender(name, n_transfers, nbytes, sync, scenario):
    conn = v.vccl_p2p_connect(name, 60.0)
    print("connected", flush=True)
    stream = torch.cuda.Stream()
    sh = int(stream.cuda_stream)
    if scenario == "mismatch":
        src = torch.zeros(8192, dtype=torch.uint8, device="cuda")
        v.vccl_p2p_send(conn, src, 4096 + 16, sh)       # the receiver expects 4096
        wait(stream, conn, "mismatched send")
        try:
            v.vccl_alltoall([src], [src[4096:]], 16, 1, v.MODE_CE, sh)
        except v.VcclError as e:
            assert e.code == -4, e
        else:
            raise AssertionError("the call after a mismatched transfer must report it")
    else:
        src = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda")
        # every payload has a tensor of its own that lives until the end: the side stream reads
        # them long after this loop has run ahead
        payloads = [torch.from_numpy(wl.payload_bytes(SEED + i, 1, nb)).cuda()
                    for i, (off, nb) in enumerate(sizes(n_transfers, nbytes))]
        torch.cuda.synchronize()
        for i, (off, nb) in enumerate(sizes(n_transfers, nbytes)):
            with torch.cuda.stream(stream):
                src[3:3 + nb].copy_(payloads[i])        # a kernel produces the bytes right before the send
                v.vccl_p2p_send(conn, src[3:], nb, sh)
                src.zero_()                             # and the buffer is reused right behind it
            print("posted send", i, flush=True)
        wait(stream, conn, "sends")
        rec = v.vccl_p2p_record(conn)
        assert rec[2] == n_transfers and rec[4] == 0, rec
    v.vccl_p2p_close(conn)


def main():
    role, name, n_transfers, nbytes, sync, scenario = sys.argv[1:7]
    torch.cuda.set_device(0)
    v.vccl_init(0, 8)
    v.vccl_set_option("ce_sync", sync)
    try:
        (receiver if role == "receiver" else sender)(name, int(n_transfers), int(nbytes), sync, scenario)
    finally:
        v.vccl_finalize()
    print("P2P-OK", role, flush=True)


if __name__ == "__main__":
    main()
