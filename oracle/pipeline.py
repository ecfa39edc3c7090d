"""Oracle for the pipeline calculators: interleaved warm-up counts and order (Section 3.3, Eq. 5-6), a timeline
of all devices (Sections 3.1-3.3: phases, bubbles, intermediate states held), and the variant whose backward
pass is split into an input-gradient pass and a deferrable weight-gradient pass (Appendix A.1).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain Python, explicit lists and dictionaries.

What the paper fixes: the warm-up counts (Eq. 1, 4, 5, 6); that a device switches to its next stage after P
passes (Section 3.3); that backward passes pop the partially ordered queue (Section 3.2); that a device holds
w_i intermediate states at the end of its warm-up (Section 3.1).  Readings taken where it is silent:

  * Interleaved order.  The M*k sub-sequences of a batch, in forward order (micro-batch, then segment), are cut
    into groups of P.  A device forwards group g through its first stage, then through its second, ... (n
    stages), then group g+1.  Backward passes take the groups in the same order, the device's stages from last
    to first, and inside a group the order the partially ordered queue gives (tail segment of the earliest
    micro-batch first).  A group must hold whole micro-batches (k divides P) or the backward of a micro-batch's
    tail segment would have to precede that of an earlier group; M*k must be a multiple of P.
  * Warm-up counts are capped at the number of forward passes.
  * Timeline.  A pass starts when the device is free and its input has arrived: a forward pass needs the same
    sub-sequence forwarded by the previous stage, a backward pass needs it back-propagated by the next stage
    (the last stage needs its own forward pass), plus t_comm when that stage lives on another device.
    Devices never reorder their passes.
  * Split backward (the zero-bubble integration of Appendix A.1, described there only by a figure): the F/B order
    stays the sequence-level one; each B leaves a weight-gradient pass W pending.  A device runs its oldest
    pending W whenever its next F or B has not yet received its input, or when more than `max_pending`
    are waiting; what is left runs at the end.  The intermediate states of a sub-sequence are held until its W
    is done.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

from oracle.schedule import PartiallyOrderedQueue, stage_order

StagePass = Tuple[str, int, int, int]   # ("F" | "B", micro-batch, segment, chunk = which of the device's stages)


def interleaved_warmup(P: int, i: int, M: int, k: int, n: int) -> int:
    """Eq. 6 (Eq. 5 when k = 1): sub-sequences device i (1-based) forwards before its first backward pass."""
    if not (P >= 1 and 1 <= i <= P and M >= 1 and k >= 1 and n >= 1):
        raise ValueError("need P >= 1, 1 <= i <= P, M >= 1, k >= 1, n >= 1")
    return min((P - i) * 2 + (n - 1) * P + k - 1, M * k * n)


def interleaved_order(P: int, i: int, M: int, k: int, n: int, warmup: Optional[int] = None) -> List[StagePass]:
    """Passes of device i, which owns stages i, i+P, ..., i+(n-1)P (chunks 0..n-1), in execution order."""
    w = interleaved_warmup(P, i, M, k, n) if warmup is None else warmup
    if (M * k) % P != 0 or P % k != 0:
        raise ValueError("groups of P sub-sequences must hold whole micro-batches")
    units = [(m, j) for m in range(M) for j in range(k)]
    groups = [units[g:g + P] for g in range(0, len(units), P)]
    forwards: List[Tuple[int, int, int]] = []
    backwards: List[Tuple[int, int, int]] = []
    for grp in groups:
        for c in range(n):
            forwards += [(m, j, c) for m, j in grp]
        q = PartiallyOrderedQueue()
        for m, j in grp:
            q.push(m, j)
        popped = [q.pop() for _ in grp]
        for c in reversed(range(n)):
            backwards += [(m, j, c) for m, j in popped]
    order: List[StagePass] = [("F", *f) for f in forwards[:w]]
    fi, bi = w, 0
    while fi < len(forwards):                      # steady phase: one forward, one backward
        order.append(("F", *forwards[fi])); fi += 1
        order.append(("B", *backwards[bi])); bi += 1
    while bi < len(backwards):                     # cooling-down phase
        order.append(("B", *backwards[bi])); bi += 1
    return order


def device_orders(P: int, M: int, k: int, n: int) -> List[List[StagePass]]:
    """Orders of all P devices: the sequence-level 1F1B order for n = 1, the interleaved one for n >= 2."""
    if n == 1:
        return [[(kind, m, j, 0) for kind, m, j in stage_order(P, d + 1, M, k)] for d in range(P)]
    return [interleaved_order(P, d + 1, M, k, n) for d in range(P)]


def order_is_consistent(order: Sequence[StagePass], k: int) -> bool:
    """Every pass once; a segment is forwarded after its predecessor on the same stage, and back-propagated
    after its own forward pass and after its successor's backward pass (the prefix K/V and their gradients)."""
    seen = set()
    for kind, m, j, c in order:
        if (kind, m, j, c) in seen:
            return False
        if kind == "F" and j > 0 and ("F", m, j - 1, c) not in seen:
            return False
        if kind == "B" and (("F", m, j, c) not in seen or (j < k - 1 and ("B", m, j + 1, c) not in seen)):
            return False
        seen.add((kind, m, j, c))
    return True


def simulate(P: int, n: int, orders: Sequence[Sequence[StagePass]], t_fwd: Sequence[int], t_bwd: Sequence[int],
             t_wgrad: Optional[Sequence[int]] = None, t_comm: int = 0, max_pending: int = 0,
             seg_tokens: Optional[Sequence[int]] = None):
    """Timeline of the P devices.  Returns a dict with `makespan`, and per device `busy`, `peak_live` (largest
    total of seg_tokens over sub-sequences whose intermediate states are held; counts when seg_tokens is None)
    and `peak_pending` (most weight-gradient passes waiting).  None if the orders dead-lock."""
    V = n * P
    k = len(t_fwd)
    tokens = [1] * k if seg_tokens is None else list(seg_tokens)
    finish: Dict[Tuple[str, int, int, int], int] = {}    # (kind, micro-batch, segment, stage) -> end time
    nxt = [0] * P
    free = [0] * P
    busy = [0] * P
    live = [0] * P
    peak_live = [0] * P
    pending: List[List[int]] = [[] for _ in range(P)]    # segments of the waiting weight-gradient passes
    peak_pending = [0] * P

    def run_wgrad(d):
        j = pending[d].pop(0)
        free[d] += t_wgrad[j]
        busy[d] += t_wgrad[j]
        live[d] -= tokens[j]

    remaining = sum(len(o) for o in orders)
    while remaining:
        moved = False
        for d in range(P):
            while nxt[d] < len(orders[d]):
                kind, m, j, c = orders[d][nxt[d]]
                s = c * P + d
                if kind == "F":
                    need = None if s == 0 else ("F", m, j, s - 1)
                else:
                    need = ("F", m, j, s) if s == V - 1 else ("B", m, j, s + 1)
                if need is not None and need not in finish:
                    break
                ready = 0
                if need is not None:
                    ready = finish[need] + (t_comm if need[3] % P != d else 0)
                if t_wgrad is not None:
                    while pending[d] and (ready > free[d] or len(pending[d]) > max_pending):
                        run_wgrad(d)
                start = max(free[d], ready)
                dur = t_fwd[j] if kind == "F" else t_bwd[j]
                free[d] = start + dur
                busy[d] += dur
                finish[(kind, m, j, s)] = free[d]
                if kind == "F":
                    live[d] += tokens[j]
                    peak_live[d] = max(peak_live[d], live[d])
                elif t_wgrad is None:
                    live[d] -= tokens[j]
                else:
                    pending[d].append(j)
                    peak_pending[d] = max(peak_pending[d], len(pending[d]))
                nxt[d] += 1
                remaining -= 1
                moved = True
        if not moved:
            return None
    if t_wgrad is not None:
        for d in range(P):
            while pending[d]:
                run_wgrad(d)
    return {"makespan": max(free), "busy": busy, "peak_live": peak_live, "peak_pending": peak_pending}


def bubble_ratio(result, P: int) -> float:
    """Idle share of the device-time rectangle P x makespan."""
    return 1.0 - sum(result["busy"]) / (P * result["makespan"])
