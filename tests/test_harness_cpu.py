"""Host logic of the measurement harness, on the CPU: the 1F1B step order."""
from paper_2510_00991_amd.harness import _schedule_1f1b


def test_1f1b_schedule_properties():
    for stages, micro in ((1, 1), (2, 8), (4, 8), (4, 2), (8, 3)):
        sched = _schedule_1f1b(stages, micro)
        assert len(sched) == stages
        for i, ops in enumerate(sched):
            # every microbatch once forward and once backward, backward after its forward
            assert sorted(ops) == sorted([("F", m) for m in range(micro)] + [("B", m) for m in range(micro)])
            for m in range(micro):
                assert ops.index(("F", m)) < ops.index(("B", m))
            # forwards in order, backwards in order
            assert [m for k, m in ops if k == "F"] == list(range(micro))
            assert [m for k, m in ops if k == "B"] == list(range(micro))
            # warm-up: stage i runs min(stages - 1 - i, micro) forwards before its first backward
            first_b = next(j for j, (k, _) in enumerate(ops) if k == "B")
            assert first_b == min(stages - 1 - i, micro) + (1 if micro > min(stages - 1 - i, micro) else 0)
            # never more forwards than backwards + (stages - i) in flight: the 1F1B memory bound
            live = 0
            for k, _ in ops:
                live += 1 if k == "F" else -1
                assert 0 <= live <= stages - i
        # the last stage strictly alternates
        assert sched[-1] == [x for m in range(micro) for x in (("F", m), ("B", m))]


def test_1f1b_schedule_is_deadlock_free():
    """Running the per-stage orders against the data dependencies (F needs F of the stage
    before, B needs B of the stage after) always makes progress."""
    for stages, micro in ((2, 8), (4, 8), (4, 2), (6, 5)):
        sched = _schedule_1f1b(stages, micro)
        pos = [0] * stages
        done = set()
        steps = 0
        while any(pos[i] < len(sched[i]) for i in range(stages)):
            progressed = False
            for i in range(stages):
                if pos[i] == len(sched[i]):
                    continue
                k, m = sched[i][pos[i]]
                dep = ("F", i - 1, m) if k == "F" and i > 0 else ("B", i + 1, m) if k == "B" and i < stages - 1 else None
                if dep is None or dep in done:
                    done.add((k, i, m))
                    pos[i] += 1
                    progressed = True
                    steps += 1
            assert progressed, (stages, micro, pos)
        assert steps == 2 * stages * micro
