"""Helpers for the GPU parity tests: device buffers via torch (memory and streams
only), whole-buffer comparison against the CPU oracle."""
from __future__ import annotations

import numpy as np
import pytest

SENTINEL = 0xA5


def require_gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    return torch


def to_dev(torch, a: np.ndarray, misalign: int = 0):
    """Upload a uint8 array; with misalign > 0 the device view starts that many
    bytes past a 256-byte aligned allocation."""
    t = torch.empty(a.size + misalign + 64, dtype=torch.uint8, device="cuda")
    v = t[misalign:misalign + a.size]
    if a.size:
        v.copy_(torch.from_numpy(a))
    return v


def to_host(t) -> np.ndarray:
    return t.cpu().numpy()


def stream_handle(torch, stream=None) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def assert_same(got, want, what=""):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.nonzero(got != want)[0]
        raise AssertionError(f"{what}: {bad.size} of {got.size} bytes differ, first at {bad[0]}: "
                             f"got {got[bad[0]]:#x}, want {want[bad[0]]:#x}")
