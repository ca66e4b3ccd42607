"""Pins of the window-monitor oracle against closed forms and a hand-worked case
(paper Section 3.4: B = w(M)/(t2-t1); window estimate sum w(M_i)/(t2-t1); window 8;
dual-threshold anomaly rule)."""
import math

from oracle import monitor_oracle as mo


def test_back_to_back_messages_give_the_link_rate_for_any_window():
    S, d = 1 << 20, 25e-6                      # one message per 25 us, one at a time
    msgs = [(i * d, (i + 1) * d, S) for i in range(40)]
    for w in (1, 3, 8, 32):
        for e in mo.evaluate(msgs, window=w):
            assert math.isclose(e["bw_window"], S / d, rel_tol=1e-12)
            assert math.isclose(e["bw_message"], S / d, rel_tol=1e-12)
            assert not e["anomaly"]


def test_window_one_is_the_per_message_scheme():
    msgs = [(0.0, 3e-6, 100), (1e-6, 9e-6, 700), (2e-6, 10e-6, 50), (11e-6, 12e-6, 4096)]
    for e in mo.evaluate(msgs, window=1):
        assert math.isclose(e["bw_window"], e["bw_message"], rel_tol=1e-12)


def test_concurrent_messages_closed_form():
    """k messages in flight share the link: posts every d, each takes k*d.  The
    per-message estimate is S/(k d); a full window of w gives w S/((w-1+k) d)."""
    S, d, k = 4096.0, 10e-6, 4
    msgs = [(i * d, (i + k) * d, S) for i in range(64)]
    for w in (2, 8, 32):
        ev = mo.evaluate(msgs, window=w)
        for n, e in enumerate(ev):
            assert math.isclose(e["bw_message"], S / (k * d), rel_tol=1e-12)
            m = min(w, n + 1)
            assert math.isclose(e["bw_window"], m * S / ((m - 1 + k) * d), rel_tol=1e-9)
    # a larger window is closer to the true rate S/d, as the appendix on window sizes argues
    full = {w: mo.evaluate(msgs, window=w)[-1]["bw_window"] for w in (1, 8, 32)}
    assert full[1] < full[8] < full[32] < S / d


def test_hand_worked_window_of_three():
    # sizes 10, 20, 30, 40 bytes; posts 0,1,2,6; completions 2,4,5,8 (seconds)
    msgs = [(0.0, 2.0, 10), (1.0, 4.0, 20), (2.0, 5.0, 30), (6.0, 8.0, 40)]
    ev = mo.evaluate(msgs, window=3, history=100.0)
    assert [e["bw_window"] for e in ev] == [10 / 2.0, 30 / 4.0, 60 / 5.0, 90 / 7.0]
    assert [e["bw_message"] for e in ev] == [5.0, 20 / 3.0, 10.0, 20.0]
    # outstanding right after each completion: at t=2 messages 2 (posted 1) and 3 (posted 2) are in flight
    assert [e["outstanding"] for e in ev] == [50, 30, 0, 0]


def _timeline(rate_factor, k_before, k_after, n_before=600, n_after=60):
    """A sender that keeps k messages of 1 MiB in flight on a link that serves them
    one after another: k_before at 40 GB/s for n_before messages (about 15 ms), then
    the link rate is multiplied by rate_factor and the sender keeps k_after in flight.
    With k in flight a full window of w estimates rate * w / (w - 1 + k)."""
    S = 1 << 20
    done, msgs = [], []
    for i in range(n_before + n_after):
        slow = i >= n_before
        k = k_after if slow else k_before
        d = S / (40e9 * (rate_factor if slow else 1.0))
        post = done[i - k] if i >= k else 0.0
        if slow and i - k < n_before:
            post = done[n_before - 1] if n_before else 0.0     # the extra messages are posted at the change
        start = max(post, done[-1] if done else 0.0)
        done.append(start + d)
        msgs.append((post, start + d, S))
    return msgs, n_before


def test_anomaly_needs_both_conditions():
    # rate falls to 30 % and the in-flight data grows from 2 to 8 messages: flagged
    msgs, n0 = _timeline(0.3, 2, 8)
    ev = mo.evaluate(msgs)
    assert not any(e["anomaly"] for e in ev[:n0])
    assert any(e["anomaly"] for e in ev[n0:])
    # rate falls to 70 % only: condition (i) fails
    msgs, n0 = _timeline(0.7, 2, 2)
    assert not any(e["anomaly"] for e in mo.evaluate(msgs))
    # rate falls to 30 % but the outstanding data does not grow: condition (ii) fails
    msgs, n0 = _timeline(0.3, 2, 2)
    ev = mo.evaluate(msgs)
    assert min(e["bw_window"] for e in ev[n0 + 8:]) < 0.5 * ev[n0 - 1]["bw_window"]
    assert not any(e["anomaly"] for e in ev)
    # same rate, but four times as much is posted at once (overlapping communication): the
    # estimate sags by w-1+k only (8/15 against 8/9), which stays above one half: no flag
    msgs, n0 = _timeline(1.0, 2, 8)
    assert not any(e["anomaly"] for e in mo.evaluate(msgs))


def test_steady_pipelined_sender_matches_the_closed_form():
    msgs, _ = _timeline(1.0, 4, 4, n_before=100, n_after=0)
    ev = mo.evaluate(msgs, window=8)
    assert math.isclose(ev[-1]["bw_window"], 40e9 * 8 / (8 - 1 + 4), rel_tol=1e-9)
