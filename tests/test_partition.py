"""Pins of the partitioner oracle (oracle/partition.py): worked textbook examples, brute force on
tiny inputs, the known worst-case ratios, conservation and the equal-count property; then the
library's host-side partitioner against that oracle."""
import itertools
import random

import pytest

from oracle import partition as P


def _sums(values, bin_of, bins):
    return sorted(P.bin_costs(values, bin_of, bins, lin=1.0, quad=0.0))


def test_two_way_differencing_worked_example():
    # {8,7,6,5,4}: 8-7 -> 1, 6-5 -> 1, 4-1 -> 3, 3-1 -> 2: the two sets differ by 2 (16 and 14),
    # although a perfect split {8,7} / {6,5,4} exists: the classic example of the method's gap
    b = P.karmarkar_karp([8, 7, 6, 5, 4], 2, lin=1.0, quad=0.0)
    assert _sums([8, 7, 6, 5, 4], b, 2) == [14.0, 16.0]


def test_three_way_differencing_worked_example():
    # by hand: (8,7,0) -> (8,7,6); (5,4,0); (5+6, 4+7, 0+8) = (11,11,8): bins {8}, {7,4}, {6,5}
    vals = [8, 7, 6, 5, 4]
    b = P.karmarkar_karp(vals, 3, lin=1.0, quad=0.0)
    groups = sorted(sorted(v for v, bb in zip(vals, b) if bb == k) for k in range(3))
    assert groups == [[4, 7], [5, 6], [8]]
    assert b[0] == 2  # bins are numbered by decreasing cost: the lone 8 is the cheapest bin


def test_lpt_worked_example():
    # Graham's list scheduling on sorted jobs 7,7,6,6,5,5,4,4,4 with 4 machines... kept small:
    # {5,5,4,4,3,3,3} on 3 bins: 5|5|4, 5|5|4+4, 5+3|5|8, 8|5+3|8, 8|8|8+3 -> 8, 8, 11
    b = P.lpt([5, 5, 4, 4, 3, 3, 3], 3, lin=1.0, quad=0.0)
    assert _sums([5, 5, 4, 4, 3, 3, 3], b, 3) == [8.0, 8.0, 11.0]
    assert P.optimum_max_cost([5, 5, 4, 4, 3, 3, 3], 3, lin=1.0, quad=0.0) == 9.0  # {5,4},{5,4},{3,3,3}


@pytest.mark.parametrize("bins", [2, 3, 4])
def test_against_brute_force_and_worst_case_ratios(bins):
    rng = random.Random(100 + bins)
    for trial in range(60):
        n = rng.randint(1, 9)
        vals = [rng.randint(1, 40) for _ in range(n)]
        opt = P.optimum_max_cost(vals, bins, lin=1.0, quad=0.0)
        for method, bound in ((P.karmarkar_karp, 4.0 / 3.0), (P.lpt, 4.0 / 3.0 - 1.0 / (3.0 * bins))):
            b = method(vals, bins, lin=1.0, quad=0.0)
            assert len(b) == n and all(0 <= x < bins for x in b)
            sums = P.bin_costs(vals, b, bins, lin=1.0, quad=0.0)
            assert abs(sum(sums) - sum(vals)) < 1e-9          # every sample in exactly one bin
            assert opt - 1e-9 <= max(sums) <= bound * opt + 1e-9, (method.__name__, vals, sums, opt)


def test_quadratic_cost_is_what_gets_balanced():
    # one long sample against many short ones: by token count 1 x 1000 = 10 x 100, by attention cost
    # the long one alone outweighs all the short ones together
    lengths = [1000] + [100] * 10
    b = P.karmarkar_karp(lengths, 2, lin=0.0, quad=1.0)
    assert [x for x in b[1:]] == [b[1]] * 10 and b[0] != b[1]
    b = P.karmarkar_karp(lengths, 2, lin=1.0, quad=0.0)
    assert _sums(lengths, b, 2) == [1000.0, 1000.0]


@pytest.mark.parametrize("method", [P.karmarkar_karp, P.lpt])
def test_equal_counts(method):
    rng = random.Random(7)
    for n, bins in ((16, 4), (17, 4), (5, 8), (64, 8)):
        vals = [rng.randint(1, 1000) for _ in range(n)]
        b = method(vals, bins, lin=1.0, quad=0.0, equal_counts=True)
        counts = [b.count(k) for k in range(bins)]
        assert max(counts) - min(counts) <= 1 and sum(counts) == n


def test_equal_counts_differencing_worked_examples():
    # By hand, 2 bins, cost = length.  {10,9,7,6,4,2}: the start is one partial solution per group of 2
    # consecutive values of the sorted order: A = (10|9), B = (7|6), C = (4|2), spreads 1, 1, 2.
    # The first merge step merges the two of largest spread, C (2) and the earlier of the 1s, A, largest slot with
    # smallest: (4+9 | 2+10) = (13|12).  The second merges B and that: (7+12 | 6+13) = (19|19), and the
    # stable sort keeps the order: bin 0 = {7,2,10}, bin 1 = {6,4,9}.
    assert P.karmarkar_karp([10, 9, 7, 6, 4, 2], 2, lin=1.0, quad=0.0, equal_counts=True) == [0, 1, 0, 1, 1, 0]
    # {10,1,1,1}: A = (10|1) from indices 0, 1 and B = (1|1) from indices 2, 3 merge to
    # (10 + 1[index 3] | 1[index 1] + 1[index 2]) = (11|2): two samples each, where the unconstrained
    # method leaves the 10 alone (10 | 1+1+1)
    assert P.karmarkar_karp([10, 1, 1, 1], 2, lin=1.0, quad=0.0, equal_counts=True) == [0, 1, 1, 0]
    assert P.karmarkar_karp([10, 1, 1, 1], 2, lin=1.0, quad=0.0) in ([0, 1, 1, 1], [1, 0, 0, 0])
    # 3 bins, {9,8,7,6,5,4}: A = (9|8|7), B = (6|5|4); merged (9+4 | 8+5 | 7+6) = (13|13|13)
    b = P.karmarkar_karp([9, 8, 7, 6, 5, 4], 3, lin=1.0, quad=0.0, equal_counts=True)
    assert b == [0, 1, 2, 2, 1, 0]


def test_equal_counts_lpt_worked_examples():
    # By hand, 2 bins, cost = length.  {9,8,7,3,2,1}, 3 samples per bin: 9 -> bin 0 (tie: lower bin),
    # 8 -> 1, 7 -> 1 (9 vs 8), 3 -> 0 (9 vs 15), 2 -> 0 (12 vs 15), and the 1 would go to bin 0 (14 vs 15)
    # but bin 0 already holds its 3 samples: it goes to bin 1.  Totals 14 | 16 where the unconstrained
    # greedy gets 15 | 15.
    assert P.lpt([9, 8, 7, 3, 2, 1], 2, lin=1.0, quad=0.0, equal_counts=True) == [0, 1, 1, 0, 0, 1]
    assert P.lpt([9, 8, 7, 3, 2, 1], 2, lin=1.0, quad=0.0) == [0, 1, 1, 0, 0, 0]
    # 5 samples in 2 bins: sizes 3 and 2, and only ONE bin may take a third sample.  {10,1,1,1,1}:
    # 10 -> 0, then 1 -> 1 three times (the third is the one allowed extra), the last 1 would again go to
    # bin 1 (3 vs 10) but no bin may grow to 4 and no second bin to 3 ... bin 0 takes it as its 2nd.
    assert P.lpt([10, 1, 1, 1, 1], 2, lin=1.0, quad=0.0, equal_counts=True) == [0, 1, 1, 1, 0]


def test_result_does_not_depend_on_input_order_when_costs_are_distinct():
    vals = [3, 17, 29, 41, 58, 66, 71, 89, 97, 104, 120]
    ref = _sums(vals, P.karmarkar_karp(vals, 3, lin=1.0, quad=0.0), 3)
    rng = random.Random(3)
    for _ in range(10):
        perm = vals[:]
        rng.shuffle(perm)
        assert _sums(perm, P.karmarkar_karp(perm, 3, lin=1.0, quad=0.0), 3) == ref


def test_differencing_beats_or_matches_greedy_on_average():
    # the reason the paper picks it: on random inputs its largest bin is (on average) smaller
    rng = random.Random(11)
    kk = lp = 0.0
    for _ in range(200):
        vals = [rng.randint(1, 10_000) for _ in range(24)]
        kk += max(P.bin_costs(vals, P.karmarkar_karp(vals, 4, lin=1.0, quad=0.0), 4, lin=1.0, quad=0.0))
        lp += max(P.bin_costs(vals, P.lpt(vals, 4, lin=1.0, quad=0.0), 4, lin=1.0, quad=0.0))
    assert kk <= lp


# --- the library's host-side partitioner against the oracle (no GPU involved) ---

def _groups(bin_of, bins):
    return [sorted(i for i, b in enumerate(bin_of) if b == k) for k in range(bins)]


@pytest.mark.parametrize("equal_counts", [False, True])
@pytest.mark.parametrize("method", ["kk", "lpt"])
def test_library_matches_oracle_exactly(method, equal_counts):
    from paper_2605_08962_amd import binding, workloads as W
    rng = random.Random(5)
    cases = [[], [7], [5, 5, 5, 5], [8, 7, 6, 5, 4]]
    cases += [[rng.randint(1, 9216) for _ in range(rng.randint(2, 70))] for _ in range(25)]
    cases += [list(W.make(2, lengths_only=True).lengths), list(W.make(3, lengths_only=True).lengths),
              list(W.make(4, lengths_only=True).lengths)]
    for lengths in cases:
        for bins in (1, 2, 3, 8):
            for lin, quad in ((0.0, 1.0), (1.0, 0.0), (4096.0, 1.0)):
                ref = (P.karmarkar_karp if method == "kk" else P.lpt)(lengths, bins, lin, quad, equal_counts)
                got, cost = binding.balance_partition(
                    lengths, bins, binding.PARTITION_KARMARKAR_KARP if method == "kk" else binding.PARTITION_LPT,
                    equal_counts, lin, quad)
                assert list(got) == ref, (lengths, bins, lin, quad)
                assert list(cost) == P.bin_costs(lengths, ref, bins, lin, quad) or \
                    max(abs(a - b) for a, b in zip(cost, P.bin_costs(lengths, ref, bins, lin, quad))) <= 1e-6 * max(cost)


def test_library_partition_rejects_bad_arguments():
    from paper_2605_08962_amd import binding
    for kwargs in (dict(bins=0), dict(bins=2, method=5), dict(bins=2, quad_cost=-1.0), dict(bins=2, lin_cost=float("nan"))):
        with pytest.raises(binding.VarlenAttnError):
            binding.balance_partition([3, 4, 5], **kwargs)
    with pytest.raises(binding.VarlenAttnError):
        binding.balance_partition([3, -4, 5], 2)


def test_library_partition_large_input_is_valid_and_balanced():
    # 20000 samples in 64 bins: far beyond what the oracle's quadratic loops finish quickly; check
    # what must hold at any size
    import numpy as np
    from paper_2605_08962_amd import binding
    rng = np.random.default_rng(1)
    lengths = np.floor(np.exp(rng.uniform(np.log(64), np.log(16384), 20000))).astype(np.int32)
    c = lengths.astype(np.float64) ** 2
    for method in (binding.PARTITION_KARMARKAR_KARP, binding.PARTITION_LPT):
        b, cost = binding.balance_partition(lengths, 64, method)
        assert b.min() >= 0 and b.max() < 64
        assert np.allclose(np.bincount(b, weights=c, minlength=64), cost)
        assert cost.max() / cost.mean() < 1.001
