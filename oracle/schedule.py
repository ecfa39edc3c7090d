"""Oracle for the Seq1F1B order of passes on one pipeline stage (test infrastructure, not the product).

Written from Section 3.1 (1F1B: warm-up, steady, cooling-down phases; FIFO queue of intermediate states) and
Section 3.2 (sequence-level 1F1B: warm-up count of Eq. 4; the partially ordered queue whose pop returns the
tail sub-sequence of the earliest enqueued micro-batch).  Plain Python, one explicit queue, no closed forms.

Readings of the paper taken here:
  * Eq. 4 counts sub-sequences.  Its second case (M <= P) prints "M", the count of micro-batches of Eq. 1; with
    k segments per micro-batch every forward pass is then run before the first backward pass (the GPipe
    behaviour the text describes), i.e. M * k sub-sequences.
  * The warm-up count never exceeds the number of forward passes, M * k.
  * In the steady phase a step is one forward pass followed by one backward pass (Section 3.1).
"""
from __future__ import annotations

from typing import List, Tuple

Pass = Tuple[str, int, int]   # ("F" | "B", micro-batch (0-based), segment (0-based))


def warmup_count(P: int, i: int, M: int, k: int) -> int:
    """Sub-sequences forwarded by device i (1-based) before its first backward pass (Eq. 4)."""
    if not (P >= 1 and 1 <= i <= P and M >= 1 and k >= 1):
        raise ValueError("need P >= 1, 1 <= i <= P, M >= 1, k >= 1")
    total = M * k
    w = P - i - 1 + k if M > P else total
    return min(w, total)


class PartiallyOrderedQueue:
    """Q_s of Section 3.2: first-in-first-out over micro-batches, first-in-last-out over the segments of one."""

    def __init__(self):
        self.items: List[Tuple[int, int]] = []   # (micro-batch, segment) in the order they were enqueued

    def push(self, m: int, j: int) -> None:
        self.items.append((m, j))

    def pop(self) -> Tuple[int, int]:
        earliest = self.items[0][0]                      # the micro-batch enqueued first
        tail = max(j for m, j in self.items if m == earliest)
        self.items.remove((earliest, tail))
        return earliest, tail

    def __len__(self) -> int:
        return len(self.items)


def stage_order(P: int, i: int, M: int, k: int) -> List[Pass]:
    """Passes of device i in execution order."""
    w = warmup_count(P, i, M, k)
    forwards = [(m, j) for m in range(M) for j in range(k)]
    q = PartiallyOrderedQueue()
    order: List[Pass] = []
    nxt = 0
    for _ in range(w):                                   # warm-up phase
        m, j = forwards[nxt]; nxt += 1
        q.push(m, j)
        order.append(("F", m, j))
    while nxt < len(forwards):                           # steady phase: one forward, one backward
        m, j = forwards[nxt]; nxt += 1
        q.push(m, j)
        order.append(("F", m, j))
        bm, bj = q.pop()
        order.append(("B", bm, bj))
    while len(q):                                        # cooling-down phase
        bm, bj = q.pop()
        order.append(("B", bm, bj))
    return order


def peak_live_states(order: List[Pass]) -> int:
    """Largest number of sub-sequences whose intermediate states are held at once."""
    live = peak = 0
    for kind, _, _ in order:
        live += 1 if kind == "F" else -1
        peak = max(peak, live)
    return peak


def peak_memory_fraction(P: int, i: int, M: int, k: int) -> float:
    """Share of all intermediate states held by device i at its peak: w_i / sum_j w_j (Section 3.1)."""
    ws = [warmup_count(P, j, M, k) for j in range(1, P + 1)]
    return ws[i - 1] / sum(ws)
