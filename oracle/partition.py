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
"""
from __future__ import annotations

import itertools


def token_cost(t: int, hidden: int) -> int:
    """w(t): cost of token t (1-based) in units of 4 * L * hidden FLOPs."""
    return 6 * hidden + t


def prefix_cost(x: int, hidden: int) -> int:
    """W(x): cost of the first x tokens, by summing token costs one by one."""
    total = 0
    for t in range(1, x + 1):
        total += token_cost(t, hidden)
    return total


def partition(seq_len: int, n_seg: int, hidden: int, heads: int):
    """Boundaries [b_0=0, b_1, ..., b_k=seq_len] of the computation-wise partition."""
    if n_seg < 1 or seq_len < n_seg or hidden < 1 or heads < 1 or hidden % heads != 0:
        raise ValueError("invalid partition arguments")
    n, k = seq_len, n_seg
    # W[x] for x = 0..n, accumulated token by token.
    W = [0] + list(itertools.accumulate(token_cost(t, hidden) for t in range(1, n + 1)))
    total = W[n]
    b = [0]
    for i in range(1, k):
        best_x, best_err = None, None
        for x in range(0, n + 1):
            err = abs(k * W[x] - i * total)
            if best_err is None or err < best_err:      # strict: the smaller x wins a tie
                best_x, best_err = x, err
        x = min(max(best_x, b[-1] + 1), n - (k - i))
        b.append(x)
    b.append(n)
    return b


def segment_costs(boundaries, hidden: int):
    """Cost of each segment, summing its tokens' costs one by one."""
    return [sum(token_cost(t, hidden) for t in range(a + 1, b + 1))
            for a, b in zip(boundaries[:-1], boundaries[1:])]
