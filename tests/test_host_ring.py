"""CPU tests of the host-only part of libtutti: get_iocb / reaping of completions (sec. 3.2 "Async I/O
Processing", steps 2 and 4) and the slack-table lookups (sec. 3.3).  No GPU call is made: the CQ is a numpy
array written by the test, playing the completion kernel's part."""
import numpy as np
import pytest

from paper_2605_03375_amd import binding as B


def make_cq(depth):
    cq = np.zeros(16 + depth, np.uint32)
    cq[1] = depth
    cq[16:] = 0xFFFFFFFF
    return cq


def complete(cq, slots):
    """What the completion kernel does: append the IOCB indices, then advance the tail."""
    depth = int(cq[1])
    t = int(cq[0])
    for s in slots:
        cq[16 + t % depth] = s
        t += 1
    cq[0] = t & 0xFFFFFFFF


class Model:
    """The same bookkeeping written the slow way: a list of held slots in hand-out order."""

    def __init__(self, depth):
        self.depth, self.next, self.held, self.done = depth, 0, [], set()

    def get(self, n):
        if n > self.depth - len(self.held):
            return None
        first = self.next
        for i in range(n):
            self.held.append((first + i) % self.depth)
        self.next = (first + n) % self.depth
        return first

    def reap(self, slots):
        self.done.update(slots)
        while self.held and self.held[0] in self.done:
            self.done.discard(self.held.pop(0))


def test_get_iocb_hands_out_ring_order_and_wraps():
    st = B.make_sq_state(5)
    cq = make_cq(5)
    assert B.tutti_sq_free_count(st) == 5
    assert B.tutti_get_iocb(st, 3) == 0
    assert B.tutti_get_iocb(st, 2) == 3
    with pytest.raises(B.TuttiError) as ei:
        B.tutti_get_iocb(st, 1)
    assert ei.value.code == B.EAGAIN and B.tutti_sq_free_count(st) == 0
    complete(cq, [0, 1, 2])
    assert B.tutti_reap_cqe(st, cq) == 3 and B.tutti_sq_free_count(st) == 3
    assert B.tutti_get_iocb(st, 3) == 0              # the run wraps: slots 0, 1, 2 again
    complete(cq, [3, 4])
    assert B.tutti_reap_cqe(st, cq) == 2
    assert B.tutti_get_iocb(st, 2) == 3
    for bad in (0, 6):
        with pytest.raises(B.TuttiError) as ei:
            B.tutti_get_iocb(st, bad)
        assert ei.value.code == B.EINVAL


def test_out_of_order_completions_wait_for_older_slots():
    st = B.make_sq_state(4)
    cq = make_cq(4)
    a = B.tutti_get_iocb(st, 1)      # a deferred write: issued last
    b = B.tutti_get_iocb(st, 2)      # a read: completes first
    complete(cq, [b, b + 1])
    assert B.tutti_reap_cqe(st, cq) == 2
    assert B.tutti_iocb_completed(st, b) and B.tutti_iocb_completed(st, b + 1) and not B.tutti_iocb_completed(st, a)
    assert B.tutti_sq_free_count(st) == 1           # the read's slots are not handed out before the write's
    with pytest.raises(B.TuttiError):
        B.tutti_get_iocb(st, 2)
    complete(cq, [a])
    assert B.tutti_reap_cqe(st, cq) == 1 and B.tutti_sq_free_count(st) == 4
    assert B.tutti_get_iocb(st, 4) == 3             # the ring continues where it stopped


def test_reap_marks_a_host_visible_sq_free_and_rejects_foreign_queues():
    depth = 3
    st = B.make_sq_state(depth)
    cq = make_cq(depth)
    sq = np.zeros(depth, B.IOCB_DTYPE)
    sq["hdr"]["state"] = B.IOCB_DONE
    s0 = B.tutti_get_iocb(st, 2)
    complete(cq, [s0 + 1])
    assert B.tutti_reap_cqe(st, cq, sq) == 1
    assert list(sq["hdr"]["state"]) == [B.IOCB_DONE, B.IOCB_FREE, B.IOCB_DONE]
    # a slot that is not held, an index out of range, the same slot twice, more completions than held slots
    for entries in ([2], [7], [s0, s0], [s0, 2, 1]):
        bad = cq.copy()
        complete(bad, entries)
        before = (st.head, st.held, st.cq_seen)
        with pytest.raises(B.TuttiError) as ei:
            B.tutti_reap_cqe(st, bad, sq)
        assert ei.value.code == B.EINVAL and (st.head, st.held, st.cq_seen) == before
    # a slot already reaped cannot complete again
    again = cq.copy()
    complete(again, [s0 + 1])
    with pytest.raises(B.TuttiError):
        B.tutti_reap_cqe(st, again)
    complete(cq, [s0])
    assert B.tutti_reap_cqe(st, cq, sq) == 1 and B.tutti_sq_free_count(st) == depth


def test_wait_cqe_host_is_bounded():
    st = B.make_sq_state(2)
    cq = make_cq(2)
    s = B.tutti_get_iocb(st, 1)
    assert B.tutti_wait_cqe_host(st, cq, None, s, 1000) is False     # nobody completes it: returns, does not spin on
    complete(cq, [s])
    assert B.tutti_wait_cqe_host(st, cq, None, s, 0) is True
    assert B.tutti_iocb_completed(st, 1)                             # never handed out: nothing to wait for


@pytest.mark.parametrize("depth", [1, 2, 7, 64])
def test_allocator_against_a_list_model(depth):
    rng = np.random.default_rng(depth)
    st = B.make_sq_state(depth)
    cq = make_cq(depth)
    m = Model(depth)
    in_flight = []                    # held slots whose completion has not been written yet
    for step in range(3000):
        if rng.random() < 0.55:
            n = int(rng.integers(1, depth + 1))
            want = m.get(n)
            if want is None:
                with pytest.raises(B.TuttiError) as ei:
                    B.tutti_get_iocb(st, n)
                assert ei.value.code == B.EAGAIN
            else:
                assert B.tutti_get_iocb(st, n) == want
                in_flight += [(want + i) % depth for i in range(n)]
        elif in_flight:
            k = int(rng.integers(1, len(in_flight) + 1))
            picks = [in_flight.pop(int(rng.integers(0, len(in_flight)))) for _ in range(k)]   # any order
            complete(cq, picks)
            assert B.tutti_reap_cqe(st, cq) == k
            m.reap(picks)
        assert B.tutti_sq_free_count(st) == depth - len(m.held)
        assert st.head == m.next
    assert int(cq[0]) > depth         # the CQ wrapped around


def test_cq_tail_wraps_around_32_bits():
    depth = 4                         # a power of two keeps tail % depth continuous across the wrap
    st = B.make_sq_state(depth)
    cq = make_cq(depth)
    cq[0] = 0xFFFFFFFE
    st.cq_seen = 0xFFFFFFFE
    s = B.tutti_get_iocb(st, 4)
    complete(cq, [s, s + 1, s + 2])
    assert int(cq[0]) == 1 and B.tutti_reap_cqe(st, cq) == 3 and B.tutti_sq_free_count(st) == 3


# ---- slack table

ROWS = [  # cu_budget, n_iocbs, read_us, write_us
    (8, 2, 540.0, 500.0), (8, 1, 280.0, 260.0), (16, 2, 290.0, 270.0), (16, 1, 150.0, 140.0), (16, 4, 560.0, 520.0),
    (32, 2, 160.0, 150.0), (0, 2, 51.0, 47.0), (64, 2, 95.0, -1.0),
]


def test_iocbs_for_slack():
    prof, n = B.make_io_profile(ROWS)
    assert B.tutti_iocbs_for_slack(prof, n, 16, B.OP_READ, 300.0) == 2
    assert B.tutti_iocbs_for_slack(prof, n, 16, B.OP_READ, 289.9) == 1
    assert B.tutti_iocbs_for_slack(prof, n, 16, B.OP_READ, 1e9) == 4
    assert B.tutti_iocbs_for_slack(prof, n, 16, B.OP_WRITE, 270.0) == 2        # exactly fits
    assert B.tutti_iocbs_for_slack(prof, n, 16, B.OP_READ, 100.0) == 0         # nothing fits
    assert B.tutti_iocbs_for_slack(prof, n, 24, B.OP_READ, 1e9) == 0           # budget never profiled
    assert B.tutti_iocbs_for_slack(prof, n, 64, B.OP_WRITE, 1e9) == 0          # not measured for writes
    assert B.tutti_iocbs_for_slack(prof, n, 0, B.OP_READ, 60.0) == 2           # whole GPU
    assert B.tutti_iocbs_for_slack(prof, 0, 8, B.OP_READ, 60.0) == 0           # empty table
    with pytest.raises(B.TuttiError):
        B.tutti_iocbs_for_slack(prof, n, 8, 3, 60.0)


def test_budget_for_slack():
    prof, n = B.make_io_profile(ROWS)
    assert B.tutti_budget_for_slack(prof, n, 2, B.OP_READ, 600.0, 256) == 8
    assert B.tutti_budget_for_slack(prof, n, 2, B.OP_READ, 539.0, 256) == 16
    assert B.tutti_budget_for_slack(prof, n, 2, B.OP_READ, 200.0, 256) == 32
    assert B.tutti_budget_for_slack(prof, n, 2, B.OP_READ, 100.0, 256) == 64
    assert B.tutti_budget_for_slack(prof, n, 2, B.OP_READ, 100.0, 32) is None  # 64 is beyond what may be given
    assert B.tutti_budget_for_slack(prof, n, 2, B.OP_READ, 90.0, 256) is None  # only the whole GPU would do
    assert B.tutti_budget_for_slack(prof, n, 2, B.OP_WRITE, 100.0, 256) is None  # budget 64 has no write figure
    # 3 IOCBs were never profiled: the next larger launch at the same budget stands for them
    assert B.tutti_budget_for_slack(prof, n, 3, B.OP_READ, 600.0, 256) == 16
    assert B.tutti_budget_for_slack(prof, n, 3, B.OP_READ, 500.0, 256) is None
    assert B.tutti_budget_for_slack(prof, n, 1, B.OP_READ, 200.0, 256) == 16   # 1 IOCB: the 1-IOCB rows, not the larger ones
    assert B.tutti_budget_for_slack(prof, n, 5, B.OP_READ, 1e9, 256) is None   # larger than anything profiled
    with pytest.raises(B.TuttiError):
        B.tutti_budget_for_slack(prof, n, 0, B.OP_READ, 1.0, 256)


def test_committed_slack_table_answers_lookups():
    """The table a profiling run wrote (profiles/slack_lut_*.json: bench.py --write-lut) loads into the C lookups,
    and what they answer agrees with reading the rows by eye: durations grow with the IOCB count and shrink with
    the budget, so the answers are monotone in the window."""
    import glob
    import json
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    paths = glob.glob(os.path.join(root, "profiles", "slack_lut_*.json"))
    assert paths, "no slack table committed under profiles/"
    for path in paths:
        lut = json.load(open(path))
        rows = [(r["cu_budget"], r["n_iocbs"], r["read_us"], r["write_us"]) for r in lut["rows"]]
        prof, n = B.make_io_profile(rows)
        budgets = sorted({r[0] for r in rows if r[0]})
        for b in budgets:
            mine = sorted((r[1], r[2]) for r in rows if r[0] == b)
            for n_io, us in mine:
                assert B.tutti_iocbs_for_slack(prof, n, b, B.OP_READ, us * 1.001) >= n_io   # durations are stored as float
                fit = [m for m, t in mine if t <= us * 0.999]
                assert B.tutti_iocbs_for_slack(prof, n, b, B.OP_READ, us * 0.999) == (max(fit) if fit else 0)
        prev = None
        for slack in (50.0, 100.0, 200.0, 400.0, 800.0, 1600.0):
            got = B.tutti_budget_for_slack(prof, n, 2, B.OP_READ, slack, max(budgets))
            if prev is not None and got is not None:
                assert got <= prev          # a longer window never needs a larger budget
            if got is not None:
                prev = got
                us = [r[2] for r in rows if r[0] == got and r[1] == 2][0]
                assert us <= slack * 1.001


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    """tests/host_selftest.cpp drives the host-only part of the library (IOCB allocator, slack lookups, pairing of
    placed planes) with random call sequences on exact-size heap buffers, checked against simple models, under
    AddressSanitizer and UndefinedBehaviorSanitizer."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = tmp_path / "host_selftest"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-Werror", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", f"-I{os.path.join(root, 'include')}",
           os.path.join(root, "tests", "host_selftest.cpp"),
           os.path.join(root, "paper_2605_03375_amd", "csrc", "tutti_host.cpp"), "-o", str(exe)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "asan" in build.stderr.lower() and "cannot find" in build.stderr.lower():
        pytest.skip("no static sanitizer runtime on this machine")
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([str(exe), "2000"], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, (run.stdout[-500:], run.stderr[-3000:])
    assert run.stdout.strip() == "ok 2000"
