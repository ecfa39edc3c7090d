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


# ---------------------------------------------------------------------------------------------------
# Variants: aligned boundaries, Eq. 8's per-segment line taken literally, re-balancing on measured costs.

def _variant_cases(golden_dir):
    for line in open(f"{golden_dir}/partition_variants_tiny.txt"):
        if line.startswith("#") or not line.strip():
            continue
        kind, args, want = (f.strip() for f in line.split(":"))
        yield kind, args, [int(x) for x in want.split()]


def test_variant_hand_worked_examples(golden_dir):
    seen = set()
    for kind, args, want in _variant_cases(golden_dir):
        seen.add(kind)
        if kind == "literal":
            n, k, hidden, heads, align = (int(x) for x in args.split())
            assert P.partition_literal(n, k, hidden, heads, align) == want
        elif kind == "additive":
            n, k, hidden, heads, align = (int(x) for x in args.split())
            assert P.partition(n, k, hidden, heads, align) == want
        else:
            align, old, cost = args.split(";")
            assert P.rebalance([int(x) for x in old.split()], [int(x) for x in cost.split()], int(align)) == want
    assert seen == {"literal", "additive", "rebalance"}


def test_literal_cost_is_the_printed_line():
    # n_i * (12 d + c_i): 2 n_i P + 2 L n_i c_i d with P = 12 L d^2, divided by 2 L d
    L, d = 3, 5
    for a, b in ((0, 4), (4, 9), (2, 3)):
        n_i, c_i, Pm = b - a, b, 12 * L * d * d
        assert (2 * n_i * Pm + 2 * L * n_i * c_i * d) == 2 * L * d * P.literal_cost(a, b, d)


@pytest.mark.parametrize("n,k,hidden,align", [(10, 3, 1, 1), (12, 4, 2, 1), (14, 3, 5, 1), (9, 9, 1, 1), (16, 3, 1, 2),
                                              (18, 4, 1, 3), (13, 1, 2, 1), (21, 3, 30, 4)])
def test_literal_brute_force(n, k, hidden, align):
    pos = [x for x in range(align, n, align)]
    best = None
    for cuts in itertools.combinations(pos, k - 1):
        b = [0, *cuts, n]
        key = (max(P.literal_cost(x, y, hidden) for x, y in zip(b[:-1], b[1:])), b)
        if best is None or key < best:
            best = key
    assert P.partition_literal(n, k, hidden, 1, align) == best[1]


def test_literal_later_segments_are_shorter():
    # the printed cost grows with the prefix, so equalising it makes segment lengths fall (Section 3.4's intent)
    b = P.partition_literal(400, 5, 8, 1)
    lens = [y - x for x, y in zip(b[:-1], b[1:])]
    assert all(x >= y for x, y in zip(lens[:-1], lens[1:])) and lens[0] > lens[-1]


@pytest.mark.parametrize("n,k,hidden,align", [(64, 4, 1, 4), (100, 3, 2, 8), (257, 5, 4, 16), (50, 2, 1, 7)])
def test_aligned_additive_is_nearest_among_multiples(n, k, hidden, align):
    b = P.partition(n, k, hidden, 1, align)
    assert b[0] == 0 and b[-1] == n and all(x % align == 0 for x in b[1:-1])
    assert all(x < y for x, y in zip(b[:-1], b[1:]))
    total = P.prefix_cost(n, hidden)
    last = (n - 1) // align * align
    for i in range(1, k):
        cands = range(0, n + 1, align)
        best = min(cands, key=lambda x: (abs(k * P.prefix_cost(x, hidden) - i * total), x))
        assert b[i] == min(max(best, b[i - 1] + align), last - (k - 1 - i) * align)


def test_alignment_that_divides_the_exact_boundaries_changes_nothing():
    b = P.partition(240, 4, 3, 1)
    g = 0
    for x in b[1:-1]:
        g = math.gcd(g, x)
    assert P.partition(240, 4, 3, 1, g) == b
    assert P.partition(240, 4, 3, 1, 1) == b


def test_rebalance_fixed_point_and_uniform_density():
    b = [0, 13, 30, 41, 64]
    assert P.rebalance(b, [5, 5, 5, 5]) == b                      # already equal: nothing moves
    assert P.rebalance(b, [7 * (y - x) for x, y in zip(b[:-1], b[1:])]) == [0, 16, 32, 48, 64]   # flat density
    assert P.rebalance([0, 64], [9]) == [0, 64]


def test_rebalance_on_additive_costs_recovers_the_partition():
    # feed the exact additive segment costs of a fine uniform split: the prefix cost is then known every 8
    # tokens and linear in between, so the result is within a token or two of the exact partition
    n, k, hidden = 512, 4, 16
    fine = list(range(0, n + 1, 8))
    got = P.rebalance(fine, P.segment_costs(fine, hidden))          # k = 64 segments in, 64 out: identity-like
    assert len(got) == len(fine)
    coarse = P.partition(n, k, hidden, 1)
    u = [i * n // k for i in range(k + 1)]
    for _ in range(6):                                              # iterate from the even split
        u = P.rebalance(u, P.segment_costs(u, hidden))
    assert max(abs(x - y) for x, y in zip(u, coarse)) <= 2


def test_rebalance_rejects_bad_input():
    for b, c, a in (([0, 4, 4, 8], [1, 1, 1], 1), ([1, 4, 8], [1, 1], 1), ([0, 4, 8], [1], 1), ([0, 4, 8], [0, 0], 1),
                    ([0, 4, 8], [1, -1], 1), ([0, 4, 8], [1, 1], 0), ([0, 1, 2, 3], [1, 1, 1], 2)):
        with pytest.raises(ValueError):
            P.rebalance(b, c, a)


def test_variant_validation():
    for bad in ((8, 3, 1, 1, 4), (8, 2, 1, 1, 0), (15, 4, 1, 1, 5)):
        with pytest.raises(ValueError):
            P.partition(*bad)
        with pytest.raises(ValueError):
            P.partition_literal(*bad)
