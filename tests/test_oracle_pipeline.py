"""Pins of the pipeline calculators' oracle (oracle/pipeline.py): hand-worked warm-up counts and timelines,
closed forms of the 1F1B family, invariants, and the necessity of the printed warm-up counts
(Section 3.1, Section 3.2 Eq. 4, Section 3.3 Eq. 5-6, Appendix A.1)."""
import itertools

import pytest

from oracle import pipeline as PL
from oracle import schedule as S


def _cases(golden_dir, what):
    for line in open(f"{golden_dir}/pipeline_tiny.txt"):
        if line.startswith(what + " "):
            args, want = line[len(what):].split(":")
            yield [int(x) for x in args.split()], [int(x) for x in want.split()]


def test_hand_worked_warmup_counts(golden_dir):
    n_cases = 0
    for (P, i, M, k, n), (w,) in _cases(golden_dir, "warmup"):
        assert PL.interleaved_warmup(P, i, M, k, n) == w
        n_cases += 1
    assert n_cases >= 8


def test_hand_worked_timelines(golden_dir):
    n_cases = 0
    for (P, M, k, n, tf, tb, comm), want in _cases(golden_dir, "timeline"):
        r = PL.simulate(P, n, PL.device_orders(P, M, k, n), [tf] * k, [tb] * k, t_comm=comm)
        assert [r["makespan"], *r["busy"]] == want
        n_cases += 1
    assert n_cases >= 2


def test_eq6_reduces_to_eq5_and_orders_devices():
    for P, n in ((4, 2), (8, 2), (8, 4)):
        for i in range(1, P + 1):
            assert PL.interleaved_warmup(P, i, 10**6, 1, n) == (P - i) * 2 + (n - 1) * P          # Eq. 5
            for k in (2, 4):
                assert (PL.interleaved_warmup(P, i, 10**6, k, n)
                        == PL.interleaved_warmup(P, i, 10**6, 1, n) + k - 1)                       # Eq. 6
        ws = [PL.interleaved_warmup(P, i, 10**6, 4, n) for i in range(1, P + 1)]
        assert all(a - b == 2 for a, b in zip(ws[:-1], ws[1:]))      # an earlier device warms up two passes longer


@pytest.mark.parametrize("P,M,k,n", [(2, 2, 1, 2), (2, 4, 2, 2), (4, 8, 1, 2), (4, 8, 2, 2), (4, 8, 4, 2), (4, 6, 2, 3),
                                      (8, 4, 4, 2), (8, 8, 8, 2), (4, 1, 4, 2), (1, 3, 1, 2), (4, 4, 1, 4)])
def test_interleaved_order_is_complete_and_consistent(P, M, k, n):
    for i in range(1, P + 1):
        order = PL.interleaved_order(P, i, M, k, n)
        assert len(order) == 2 * M * k * n and len(set(order)) == len(order)
        assert PL.order_is_consistent(order, k)
        w = PL.interleaved_warmup(P, i, M, k, n)
        assert all(p[0] == "F" for p in order[:w])
        if w < M * k * n:
            assert order[w][0] == "F" and order[w + 1][0] == "B"       # steady phase: one forward, one backward
        # a device switches to its next stage after P passes (Section 3.3)
        chunks = [c for kind, _, _, c in order if kind == "F"]
        assert chunks[:P * n] == [c for c in range(n) for _ in range(min(P, M * k))][:len(chunks[:P * n])]
    r = PL.simulate(P, n, PL.device_orders(P, M, k, n), [3] * k, [5] * k)
    assert r is not None                                               # no dead-lock


def test_interleaved_order_rejects_groups_that_split_a_micro_batch():
    for P, M, k, n in ((4, 8, 8, 2), (4, 4, 3, 2), (4, 3, 2, 2), (8, 3, 4, 2)):
        with pytest.raises(ValueError):
            PL.interleaved_order(P, 1, M, k, n)


@pytest.mark.parametrize("P,M", [(2, 3), (4, 8), (4, 5), (8, 16), (3, 7)])
def test_1f1b_closed_forms(P, M):
    tf, tb = 7, 13
    r = PL.simulate(P, 1, PL.device_orders(P, M, 1, 1), [tf], [tb])
    assert r["makespan"] == (M + P - 1) * (tf + tb)
    assert r["busy"] == [M * (tf + tb)] * P
    assert abs(PL.bubble_ratio(r, P) - (P - 1) / (M + P - 1)) < 1e-12
    # a device holds its warm-up count of states at the end of the warm-up, one more during a steady step
    for i in range(1, P + 1):
        assert r["peak_live"][i - 1] == min(S.warmup_count(P, i, M, 1) + 1, M)


@pytest.mark.parametrize("P,M,k", [(4, 8, 2), (4, 8, 4), (8, 16, 4), (4, 5, 3), (2, 3, 8)])
def test_seq1f1b_equal_segments_closed_form(P, M, k):
    tf, tb = 6, 10                                   # per segment
    r = PL.simulate(P, 1, PL.device_orders(P, M, k, 1), [tf] * k, [tb] * k)
    assert r["makespan"] == (M * k + P - 1) * (tf + tb)          # a 1F1B pipeline over M*k units
    whole = PL.simulate(P, 1, PL.device_orders(P, M, 1, 1), [tf * k], [tb * k])
    assert r["makespan"] < whole["makespan"]                      # fewer bubbles than 1F1B (Section 3.2)
    assert PL.bubble_ratio(r, P) < PL.bubble_ratio(whole, P)
    # memory in tokens: sub-sequences are 1/k of a micro-batch, so the peak falls (Section 3.2)
    for d in range(P):
        assert r["peak_live"][d] == min(S.warmup_count(P, d + 1, M, k) + 1, M * k)
        assert r["peak_live"][d] < k * whole["peak_live"][d] or P - d - 1 == 0


@pytest.mark.parametrize("P,M,k,n", [(4, 8, 1, 2), (4, 8, 2, 2), (4, 8, 4, 2), (8, 16, 4, 2), (4, 8, 2, 4), (4, 6, 2, 2)])
def test_interleaved_closed_form_and_necessity_of_eq6(P, M, k, n):
    tf, tb = 4, 8                                    # per segment and stage
    orders = PL.device_orders(P, M, k, n)
    r = PL.simulate(P, n, orders, [tf] * k, [tb] * k)
    assert r["makespan"] == (M * k * n + P - 1) * (tf + tb)
    flat = PL.simulate(P, 1, PL.device_orders(P, M, k, 1), [tf * n] * k, [tb * n] * k)
    assert r["makespan"] < flat["makespan"]          # interleaving removes bubbles (Section 3.3) ...
    assert all(a >= b for a, b in zip(r["peak_live"], [x * 1 for x in flat["peak_live"]]))   # ... and holds more states
    # with one forward pass fewer in every warm-up the pipeline dead-locks: the printed counts are the least ones
    short = [PL.interleaved_order(P, d + 1, M, k, n, warmup=PL.interleaved_warmup(P, d + 1, M, k, n) - 1)
             for d in range(P)]
    assert PL.simulate(P, n, short, [tf] * k, [tb] * k) is None


def test_timeline_invariants_with_unequal_segments():
    P, M, k = 4, 6, 3
    tf, tb, tok = [5, 4, 3], [11, 9, 8], [50, 30, 20]
    for n in (1, 2):
        if n == 2 and P % k:
            continue
        orders = PL.device_orders(P, M, k, n)
        r = PL.simulate(P, n, orders, tf, tb, t_comm=2, seg_tokens=tok)
        assert r["busy"] == [M * n * (sum(tf) + sum(tb))] * P
        assert r["makespan"] >= max(r["busy"]) + (P - 1) * 2
        assert 0 < PL.bubble_ratio(r, P) < 1
        assert all(0 < x <= M * sum(tok) for x in r["peak_live"])
        slower = PL.simulate(P, n, orders, tf, tb, t_comm=5, seg_tokens=tok)
        assert slower["makespan"] >= r["makespan"]


@pytest.mark.parametrize("P,M,k", [(4, 8, 1), (4, 8, 2), (8, 16, 1), (8, 16, 4), (4, 12, 4)])
def test_split_backward_fills_bubbles(P, M, k):
    T = 6
    orders = PL.device_orders(P, M, k, 1)
    fused = PL.simulate(P, 1, orders, [T] * k, [2 * T] * k)
    free = PL.simulate(P, 1, orders, [T] * k, [T] * k, [T] * k, max_pending=10**9)
    # with nothing limiting the deferral the bubble falls from (P-1)(tf+tb+tw) to (P-1)(tf+tb-tw)
    assert fused["makespan"] == (M * k + P - 1) * 3 * T
    assert free["makespan"] == M * k * 3 * T + (P - 1) * T
    assert free["busy"] == fused["busy"]
    capped = [PL.simulate(P, 1, orders, [T] * k, [T] * k, [T] * k, max_pending=c) for c in (0, 1, 2, 4, 10**9)]
    spans = [c["makespan"] for c in capped]
    assert spans[0] <= fused["makespan"] and spans[-1] == free["makespan"]
    assert all(a >= b for a, b in zip(spans[:-1], spans[1:]))           # more deferral, fewer bubbles ...
    held = [max(c["peak_live"]) for c in capped]
    assert all(a <= b for a, b in zip(held[:-1], held[1:]))             # ... and more states held
    assert max(capped[1]["peak_pending"]) <= 2 and max(capped[0]["peak_pending"]) <= 1


def test_validation():
    with pytest.raises(ValueError):
        PL.interleaved_warmup(4, 0, 8, 1, 2)
    with pytest.raises(ValueError):
        PL.interleaved_warmup(4, 5, 8, 1, 2)
    with pytest.raises(ValueError):
        PL.interleaved_warmup(4, 1, 8, 1, 0)
