"""Pins of the schedule oracle (oracle/schedule.py) against what Section 3.1-3.2 of the paper and the
structure of the problem fix.  No GPU."""
import itertools
import os

import pytest

from oracle import schedule as SCH

CASES = [(P, i, M, k) for P in (1, 2, 4, 8) for i in range(1, P + 1) for M in (1, 2, 3, 5, 9, 16) for k in (1, 2, 3, 4)]


def test_hand_worked_order(golden_dir):
    """The order worked by hand from the text of Section 3.2 (tests/golden/seq1f1b_order_small.txt)."""
    want = []
    for line in open(os.path.join(golden_dir, "seq1f1b_order_small.txt")):
        if line.startswith("#") or not line.strip():
            continue
        kind, m, j = line.split()
        want.append((kind, int(m), int(j)))
    assert SCH.stage_order(2, 2, 3, 2) == want


def test_eq4_reduces_to_eq1_without_segments():
    """Eq. 4 with k = 1 is Eq. 1: w_i = P - i when M > P, and M otherwise."""
    assert [SCH.warmup_count(4, i, 8, 1) for i in (1, 2, 3, 4)] == [3, 2, 1, 0]
    assert [SCH.warmup_count(4, i, 3, 1) for i in (1, 2, 3, 4)] == [3, 3, 3, 3]


def test_eq4_values():
    """Eq. 4: each device forwards one more sub-sequence than the next one; the last one k - 1."""
    assert [SCH.warmup_count(4, i, 16, 4) for i in (1, 2, 3, 4)] == [6, 5, 4, 3]
    assert [SCH.warmup_count(8, i, 32, 2) for i in range(1, 9)] == [8, 7, 6, 5, 4, 3, 2, 1]


def test_last_device_starts_backward_with_the_last_segment_of_the_first_micro_batch():
    """Section 3.2: entering the steady phase the last device runs the backward of the last sub-sequence of
    the first micro-batch, right after its forward."""
    for P, M, k in ((2, 3, 2), (4, 8, 4), (8, 16, 3)):
        order = SCH.stage_order(P, P, M, k)
        first_b = next(n for n, p in enumerate(order) if p[0] == "B")
        assert order[first_b] == ("B", 0, k - 1)
        assert order[first_b - 1] == ("F", 0, k - 1)


@pytest.mark.parametrize("P,i,M,k", CASES)
def test_order_invariants(P, i, M, k):
    order = SCH.stage_order(P, i, M, k)
    pos = {p: n for n, p in enumerate(order)}
    assert len(order) == 2 * M * k == len(pos)                      # every pass exactly once
    fwd = [p for p in order if p[0] == "F"]
    assert fwd == [("F", m, j) for m in range(M) for j in range(k)]  # tokens are forwarded in sequence order
    for m, j in itertools.product(range(M), range(k)):
        assert pos[("B", m, j)] > pos[("F", m, k - 1)]              # gradients of later tokens come first:
        if j + 1 < k:                                               # a segment's backward needs the whole
            assert pos[("B", m, j)] > pos[("B", m, j + 1)]          # micro-batch forwarded and segment j+1 done
    bwd_mb = [p[1] for p in order if p[0] == "B"]
    assert bwd_mb == sorted(bwd_mb)                                 # first-in-first-out over micro-batches
    w = SCH.warmup_count(P, i, M, k)
    assert [p[0] for p in order[:w]] == ["F"] * w
    if w < M * k:
        assert order[w][0] == "F" and order[w + 1][0] == "B"       # 1F1B steps follow the warm-up
        steady = order[w:w + 2 * (M * k - w)]
        assert [p[0] for p in steady] == ["F", "B"] * (M * k - w)
    assert [p[0] for p in order[len(order) - w:]] == ["B"] * w      # cooling-down mirrors the warm-up
    assert SCH.peak_live_states(order) == min(w + 1, M * k)         # what the queue holds does not grow with M


def test_without_segments_the_order_is_plain_1f1b():
    """k = 1: backward passes leave in the order the micro-batches entered (the FIFO queue of Section 3.1)."""
    order = SCH.stage_order(4, 2, 10, 1)
    assert [p[1] for p in order if p[0] == "B"] == list(range(10))
    assert [p[0] for p in order[:6]] == ["F", "F", "F", "B", "F", "B"]


def test_memory_shares_sum_to_one_and_fall_with_the_device_index():
    shares = [SCH.peak_memory_fraction(8, i, 32, 4) for i in range(1, 9)]
    assert abs(sum(shares) - 1.0) < 1e-12
    assert shares == sorted(shares, reverse=True)
    assert shares[0] == pytest.approx(10 / sum(range(3, 11)))
