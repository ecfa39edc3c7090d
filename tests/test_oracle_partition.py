"""Pins of the partition oracle (oracle/partition.py) against a hand-worked example, limits with a
closed form, structural invariants and brute force (Section 3.4, Eq. 7-8)."""
import itertools
import math

import pytest

from oracle import partition as P


def test_hand_worked_examples(golden_dir):
    for line in open(f"{golden_dir}/partition_tiny.txt"):
        if line.startswith("#") or not line.strip():
            continue
        args, want = line.split(":")
        n, k, hidden, heads = (int(x) for x in args.split())
        assert P.partition(n, k, hidden, heads) == [int(x) for x in want.split()]


def test_prefix_cost_closed_form():
    for hidden in (1, 7, 64):
        for x in (0, 1, 2, 17, 100):
            assert P.prefix_cost(x, hidden) == 6 * hidden * x + x * (x + 1) // 2


@pytest.mark.parametrize("n,k,hidden", [(100, 4, 8), (1000, 7, 64), (4096, 8, 512), (999, 3, 1)])
def test_structure_and_within_one_token(n, k, hidden):
    b = P.partition(n, k, hidden, 1)
    assert b[0] == 0 and b[-1] == n and len(b) == k + 1
    assert all(x < y for x, y in zip(b[:-1], b[1:]))
    costs = P.segment_costs(b, hidden)
    total = P.prefix_cost(n, hidden)
    assert sum(costs) == total
    # each boundary is nearest in prefix cost, hence every segment is within one (largest) token of total/k
    for c in costs:
        assert abs(k * c - total) <= k * P.token_cost(n, hidden)
    for i in range(1, k):
        err = abs(k * P.prefix_cost(b[i], hidden) - i * total)
        assert 2 * err <= k * P.token_cost(b[i] + 1, hidden)


def test_linear_limit_is_uniform():
    # when the linear term dwarfs attention (6*hidden >> n) the split is the even one
    assert P.partition(64, 4, 10**6, 1) == [0, 16, 32, 48, 64]
    assert P.partition(120, 5, 10**7, 1) == [0, 24, 48, 72, 96, 120]


def test_attention_limit_is_square_root_law():
    # with a negligible linear term prefix cost ~ x^2/2, so b_i ~ n sqrt(i/k)
    n, k = 10000, 5
    hidden = 1   # 6*hidden = 6 << n
    b = P.partition(n, k, hidden, 1)
    for i in range(1, k):
        # solve 6x + x(x+1)/2 = i/k * W(n) exactly in floating point
        tgt = i / k * (6 * n + n * (n + 1) / 2)
        x = -6.5 + math.sqrt(6.5 ** 2 + 2 * tgt)
        assert abs(b[i] - x) <= 1.0
        assert abs(b[i] - n * math.sqrt(i / k)) < 10


def test_degenerate_counts():
    assert P.partition(37, 1, 16, 4) == [0, 37]
    assert P.partition(9, 9, 16, 4) == list(range(10))
    for bad in ((8, 0, 4, 1), (3, 4, 4, 1), (8, 2, 0, 1), (8, 2, 4, 0), (8, 2, 6, 4)):
        with pytest.raises(ValueError):
            P.partition(*bad)


@pytest.mark.parametrize("n,k,hidden", [(12, 2, 1), (16, 3, 2), (20, 4, 1), (24, 4, 3), (24, 3, 40), (10, 4, 1)])
def test_brute_force_over_all_compositions(n, k, hidden):
    b = P.partition(n, k, hidden, 1)
    total = P.prefix_cost(n, hidden)
    # (i) every boundary is individually the nearest prefix (smaller x on ties), found by exhaustive search
    for i in range(1, k):
        errs = [abs(k * P.prefix_cost(x, hidden) - i * total) for x in range(n + 1)]
        best = min(range(n + 1), key=lambda x: (errs[x], x))
        clamped = min(max(best, b[i - 1] + 1), n - (k - i))
        assert b[i] == clamped
    # (ii) the worst segment is within one token of the min-max optimum over all C(n-1, k-1) compositions
    opt = min(max(P.segment_costs([0, *cuts, n], hidden))
              for cuts in itertools.combinations(range(1, n), k - 1))
    assert max(P.segment_costs(b, hidden)) <= opt + P.token_cost(n, hidden)


def test_contract_workloads_are_balanced():
    for n, k, hidden, heads in ((8192, 4, 2560, 32), (32768, 8, 4096, 32)):
        b = P.partition(n, k, hidden, heads)
        costs = [6 * hidden * (y - x) + (y * (y + 1) - x * (x + 1)) // 2 for x, y in zip(b[:-1], b[1:])]
        assert max(costs) / (sum(costs) / k) < 1.002
        # and clearly better than the even split
        u = [i * n // k for i in range(k + 1)]
        ucosts = [6 * hidden * (y - x) + (y * (y + 1) - x * (x + 1)) // 2 for x, y in zip(u[:-1], u[1:])]
        assert max(ucosts) / (sum(ucosts) / k) > 1.1
