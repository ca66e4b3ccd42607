"""Plain restatement of the paper's window-based bandwidth monitor (Section 3.4).

TEST INFRASTRUCTURE ONLY; shares no code with the library's monitor.

Per-message estimate:  B = w(M) / (t2 - t1), t1 the post time and t2 the completion
time of message M.  Window estimate over the window W of the last `window`
completed messages:  B = sum_{i in W} w(M_i) / (t2 - t1) with t1 the post time of
the first message of the window and t2 the completion time of its last message.
Anomaly rule: flag a completion when (i) its window estimate is below half of the
average of the estimates of the preceding `history` time span, and (ii) the data
still outstanding (posted, not completed) exceeds twice the largest outstanding
amount seen in that span.  Window size 8 and a 10 ms span are the paper's values.

Readings where the text leaves room: the window slides by one message per
completion and holds fewer messages until `window` have completed; with
completions out of post order t1 is the earliest post and t2 the latest completion
in the window; the "preceding" span is the `history` seconds that end where the
current window begins (its t1), so that the messages being judged do not vote on
their own baseline - taken literally up to the present, a backlog that has just
appeared would already be part of the historical maximum and condition (ii) could
hardly ever hold; at least one earlier estimate must lie inside the span.
"""
from __future__ import annotations


def evaluate(messages, window=8, history=10e-3):
    """messages: list of (t_post, t_done, nbytes), any order.  Returns one dict per
    message in completion order: t, bw_message, bw_window, outstanding, anomaly."""
    done_order = sorted(range(len(messages)), key=lambda i: (messages[i][1], i))
    out = []
    past = []                      # (t, bw_window, outstanding) of earlier evaluations
    for n, i in enumerate(done_order):
        t_post, t_done, size = messages[i]
        members = [messages[j] for j in done_order[max(0, n + 1 - window):n + 1]]
        t1 = min(m[0] for m in members)
        t2 = max(m[1] for m in members)
        bw_window = sum(m[2] for m in members) / (t2 - t1)
        bw_message = size / (t_done - t_post)
        outstanding = sum(m[2] for m in messages if m[0] <= t_done and m[1] > t_done)
        prev = [p for p in past if t1 - history <= p[0] < t1]
        anomaly = False
        if prev:
            avg = sum(p[1] for p in prev) / len(prev)
            peak = max(p[2] for p in prev)
            anomaly = bw_window < 0.5 * avg and outstanding > 2 * peak
        out.append({"t": t_done, "bw_message": bw_message, "bw_window": bw_window,
                    "outstanding": outstanding, "anomaly": anomaly})
        past.append((t_done, bw_window, outstanding))
    return out
