"""Computation-wise partition of a sequence into segments of equal FLOPs (Section 3.4, Eq. 7-8).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Eq. 8 gives the cost of a whole sequence of n tokens as 2 n P + 2 L n^2 d (P parameters, L layers,
d model width) and asks (Eq. 7) that every segment cost 1/k of it.  The per-segment line of Eq. 8 does
not sum to the whole-sequence line (its key count starts at an undefined n_0 and counts a segment's
own keys for every one of its rows), so Eq. 7 cannot hold literally.  The reading taken here:

  * the cost is additive over tokens, and token t (1-based) costs what a causal kernel executes for it:
    the linear layers plus attention over its t visible keys;
  * with P/L = 12 d^2 (4 d^2 attention projections + 8 d^2 MLP, which reproduces the model sizes of
    Table 1) and the common factor 4 L d divided out, token t costs w(t) = 6 d + t, and the first x
    tokens cost W(x) = 6 d x + x (x + 1) / 2;
  * boundary b_i (i = 1..k-1) is the x whose prefix cost is nearest to i/k of the total,
    i.e. it minimises |k W(x) - i W(n)| over integers x, the smaller x on a tie;
  * every segment keeps at least one token: b_i is clamped into [b_{i-1} + 1, n - (k - i)].

`heads` does not enter the cost (attention FLOPs depend on heads * head_dim = hidden only); it is
validated and otherwise unused.  Everything is exact integer arithmetic, found by linear scan.

Variants of the same section, each with its own function below:

  * `align`: interior boundaries restricted to multiples of `align` tokens (the paper is silent on
    alignment; exact boundaries, align = 1, are the default);
  * `partition_literal`: the per-segment line of Eq. 8 taken as printed, cost_i = n_i (12 d + c_i) with c_i
    the keys up to and including segment i (common factor 2 L d removed).  It is not additive over tokens, so
    "equal" becomes: the composition that minimises the largest cost, the lexicographically smallest
    boundaries among those;
  * `rebalance`: the same nearest-prefix rule applied to MEASURED segment costs: each token of segment i is
    taken to cost seg_cost[i] / n_i, and new boundaries are placed where the measured prefix cost is nearest
    to i/k of the measured total.
"""
from __future__ import annotations

import itertools
from fractions import Fraction


def token_cost(t: int, hidden: int) -> int:
    """w(t): cost of token t (1-based) in units of 4 * L * hidden FLOPs."""
    return 6 * hidden + t


def prefix_cost(x: int, hidden: int) -> int:
    """W(x): cost of the first x tokens, by summing token costs one by one."""
    total = 0
    for t in range(1, x + 1):
        total += token_cost(t, hidden)
    return total


def _check(seq_len, n_seg, hidden, heads, align):
    if n_seg < 1 or seq_len < n_seg or hidden < 1 or heads < 1 or hidden % heads != 0 or align < 1:
        raise ValueError("invalid partition arguments")
    if (seq_len - 1) // align < n_seg - 1:
        raise ValueError("too few aligned positions for the segment count")


def partition(seq_len: int, n_seg: int, hidden: int, heads: int, align: int = 1):
    """Boundaries [b_0=0, b_1, ..., b_k=seq_len] of the computation-wise partition; interior boundaries are
    multiples of `align`."""
    _check(seq_len, n_seg, hidden, heads, align)
    n, k = seq_len, n_seg
    # W[x] for x = 0..n, accumulated token by token.
    W = [0] + list(itertools.accumulate(token_cost(t, hidden) for t in range(1, n + 1)))
    total = W[n]
    last = (n - 1) // align * align          # largest aligned position that leaves the last segment a token
    b = [0]
    for i in range(1, k):
        best_x, best_err = None, None
        for x in range(0, n + 1, align):
            err = abs(k * W[x] - i * total)
            if best_err is None or err < best_err:      # strict: the smaller x wins a tie
                best_x, best_err = x, err
        x = min(max(best_x, b[-1] + align), last - (k - 1 - i) * align)
        b.append(x)
    b.append(n)
    return b


def literal_cost(a: int, b: int, hidden: int) -> int:
    """Eq. 8's per-segment line as printed for the segment of tokens a+1..b: n_i (12 d + c_i) with n_i = b - a
    and c_i = b (units of 2 * L * hidden FLOPs)."""
    return (b - a) * (12 * hidden + b)


def partition_literal(seq_len: int, n_seg: int, hidden: int, heads: int, align: int = 1):
    """Min-max composition under `literal_cost`, lexicographically smallest boundaries among the optima.
    Dynamic programme over (segments used, aligned position); quadratic in the number of positions."""
    _check(seq_len, n_seg, hidden, heads, align)
    n, k = seq_len, n_seg
    pos = list(range(0, n, align)) + [n]          # candidate boundaries: aligned ones below n, and n itself
    idx = {x: j for j, x in enumerate(pos)}
    INF = float("inf")
    # best[i][j]: smallest possible largest cost when tokens 1..pos[j] form exactly i segments
    best = [[INF] * len(pos) for _ in range(k + 1)]
    best[0][0] = 0
    for i in range(1, k + 1):
        for j in range(1, len(pos)):
            for a in range(j):
                if best[i - 1][a] is INF:
                    continue
                c = max(best[i - 1][a], literal_cost(pos[a], pos[j], hidden))
                if c < best[i][j]:
                    best[i][j] = c
    T = best[k][idx[n]]
    # ok[i][j]: tokens pos[j]+1..n can form exactly k - i segments, none costing more than T
    ok = [[False] * len(pos) for _ in range(k + 1)]
    ok[k][idx[n]] = True
    for i in range(k - 1, -1, -1):
        for j in range(len(pos) - 1):
            ok[i][j] = any(ok[i + 1][y] and literal_cost(pos[j], pos[y], hidden) <= T
                           for y in range(j + 1, len(pos)))
    b = [0]
    for i in range(1, k):
        for y in range(idx[b[-1]] + 1, len(pos)):
            if literal_cost(b[-1], pos[y], hidden) <= T and ok[i][y]:
                b.append(pos[y])
                break
    b.append(n)
    return b


def rebalance(boundaries, seg_cost, align: int = 1):
    """New boundaries from measured segment costs (non-negative integers, positive sum).  Inside segment i
    every token costs seg_cost[i] / n_i; boundary j is the aligned x whose measured prefix cost is nearest to
    j/k of the total (the smaller x on a tie), clamped like `partition`."""
    k = len(boundaries) - 1
    n = boundaries[-1]
    if k < 1 or len(seg_cost) != k or boundaries[0] != 0 or align < 1:
        raise ValueError("invalid rebalance arguments")
    if any(y <= x for x, y in zip(boundaries[:-1], boundaries[1:])) or any(c < 0 for c in seg_cost):
        raise ValueError("invalid rebalance arguments")
    total = sum(seg_cost)
    if total <= 0 or (n - 1) // align < k - 1:
        raise ValueError("invalid rebalance arguments")
    # prefix cost at every token position, as exact fractions
    C = [Fraction(0)]
    for (a, b), c in zip(zip(boundaries[:-1], boundaries[1:]), seg_cost):
        for _ in range(a, b):
            C.append(C[-1] + Fraction(c, b - a))
    last = (n - 1) // align * align
    out = [0]
    for j in range(1, k):
        best_x, best_err = None, None
        for x in range(0, n + 1, align):
            err = abs(k * C[x] - j * total)
            if best_err is None or err < best_err:
                best_x, best_err = x, err
        out.append(min(max(best_x, out[-1] + align), last - (k - 1 - j) * align))
    out.append(n)
    return out


def segment_costs(boundaries, hidden: int):
    """Cost of each segment, summing its tokens' costs one by one."""
    return [sum(token_cost(t, hidden) for t in range(a + 1, b + 1))
            for a, b in zip(boundaries[:-1], boundaries[1:])]
