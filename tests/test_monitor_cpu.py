"""The library's window monitor against the oracle, sample by sample, on synthetic
timelines (host only: no device)."""
import math

import numpy as np
import pytest

import paper_2510_00991_amd as vccl
from oracle import monitor_oracle as mo
from test_monitor_oracle import _timeline


def _feed(msgs_ns, window, history_ns):
    """Replay posts and completions in time order (posts first on ties)."""
    h = vccl.vccl_monitor_create(window, history_ns)
    try:
        events = [(m[0], 0, i) for i, m in enumerate(msgs_ns)] + [(m[1], 1, i) for i, m in enumerate(msgs_ns)]
        out = []
        for t, kind, i in sorted(events):
            if kind == 0:
                vccl.vccl_monitor_post(h, i, msgs_ns[i][2], t)
            else:
                out.append(vccl.vccl_monitor_complete(h, i, t))
        return out, vccl.vccl_monitor_totals(h)
    finally:
        vccl.vccl_monitor_destroy(h)


def _to_ns(msgs):
    return [(int(round(a * 1e9)), int(round(b * 1e9)), int(c)) for a, b, c in msgs]


def _compare(msgs_ns, window, history_ns):
    got, totals = _feed(msgs_ns, window, history_ns)
    # the oracle is unit-agnostic: give it integer nanoseconds (exact span boundaries), bytes per ns out
    want = mo.evaluate(msgs_ns, window=window, history=history_ns)
    assert len(got) == len(want)
    for g, w in zip(got, want):
        assert math.isclose(g["bw_window"], w["bw_window"] * 1e9, rel_tol=1e-9), (g, w)
        assert math.isclose(g["bw_message"], w["bw_message"] * 1e9, rel_tol=1e-9)
        assert g["outstanding"] == w["outstanding"]
        assert g["anomaly"] == w["anomaly"], (g, w)
    assert totals["messages"] == len(want)
    assert totals["anomalies"] == sum(w["anomaly"] for w in want)
    return want


@pytest.mark.parametrize("case", [(0.3, 2, 8), (0.7, 2, 2), (0.3, 2, 2), (1.0, 2, 8), (0.1, 1, 16)])
@pytest.mark.parametrize("window", [1, 8, 32])
def test_synthetic_link_timelines(case, window):
    msgs, _ = _timeline(*case)
    want = _compare(_to_ns(msgs), window, 10_000_000)
    if case == (0.3, 2, 8) and window == 8:
        assert any(w["anomaly"] for w in want)


@pytest.mark.parametrize("seed", range(5))
def test_random_out_of_order_completions(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    n = 300
    post = np.cumsum(rng.integers(1, 4000, n))
    dur = rng.integers(500, 60000, n)
    msgs = [(int(post[i]), int(post[i] + dur[i]), int(rng.integers(1, 1 << 22))) for i in range(n)]
    _compare(msgs, int(rng.choice([1, 4, 8])), int(rng.choice([20_000, 200_000, 10_000_000])))


def test_argument_errors():
    with pytest.raises(vccl.VcclError):
        vccl.vccl_monitor_create(0, 10)
    h = vccl.vccl_monitor_create(8, 1000)
    try:
        vccl.vccl_monitor_post(h, 1, 10, 100)
        with pytest.raises(vccl.VcclError):
            vccl.vccl_monitor_post(h, 1, 10, 101)          # duplicate id
        with pytest.raises(vccl.VcclError):
            vccl.vccl_monitor_complete(h, 2, 200)           # never posted
        with pytest.raises(vccl.VcclError):
            vccl.vccl_monitor_complete(h, 1, 100)           # zero duration
    finally:
        vccl.vccl_monitor_destroy(h)
