"""Load balancing (paper Section 4, Appendix C): pins for the Python oracle, then parity of
the native implementation against it.  CPU only."""
import heapq
import itertools
import os
import re

import numpy as np
import pytest

from oracle import packing_oracle as po
from paper_2601_19362_amd import packing

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def sums(costs, parts):
    return [sum(costs[i] for i in p) for p in parts]


def assert_partition(parts, n, k):
    assert len(parts) == k
    flat = sorted(i for p in parts for i in p)
    assert flat == list(range(n))


def lengths(n, seed):
    rng = np.random.default_rng(seed)
    return [int(v) for v in np.clip(np.rint(np.exp(7.0 + rng.standard_normal(n))), 128, 32768)]


# ----------------------------------------------------------------------------- oracle pins
def test_kk_two_way_worked_example():
    """{8, 7, 6, 5, 4}: 8-7 -> 1, 6-5 -> 1, 4-1 -> 3, 3-1 -> 2: the differencing method ends with
    difference 2 (the optimum would be 0), e.g. {8, 6} against {7, 5, 4}."""
    costs = [8, 7, 6, 5, 4]
    parts = po.karmarkar_karp(costs, 2, False)
    assert_partition(parts, 5, 2)
    s = sums(costs, parts)
    assert abs(s[0] - s[1]) == 2 and sorted(s) == [14, 16]


def test_kk_three_way_worked_example():
    """{8, 7, 6, 5, 4}, k = 3, worked by hand with tuples (largest first), always merging the two
    tuples of largest spread, largest subset with smallest:
    (8,0,0)+(7,0,0) -> (8,7,0) [spread 8]; (8,7,0)+(6,0,0) -> (8,7,6) [spread 2];
    (5,0,0)+(4,0,0) -> (5,4,0) [spread 5]; (5,4,0)+(8,7,6) -> (5+6, 4+7, 0+8) = (11, 11, 8).
    So the parts are {5, 6}, {4, 7}, {8}."""
    costs = [8, 7, 6, 5, 4]
    parts = po.karmarkar_karp(costs, 3, False)
    assert_partition(parts, 5, 3)
    assert sums(costs, parts) == [11, 11, 8]
    assert sorted(map(sorted, parts)) == [[0], [1, 4], [2, 3]]


def test_kk_equal_size_worked_example():
    """equal_size with n = 6, k = 3, worked by hand.  Costs 9, 8, 7, 4, 3, 1 sorted descending are
    grouped three at a time into tuples of singletons: A = (9, 8, 7), spread 2, and B = (4, 3, 1),
    spread 3.  The larger spread is taken first, so B's i-th largest subset meets A's i-th
    smallest: 4 + 7, 3 + 8, 1 + 9 = (11, 11, 10): parts {2, 3}, {1, 4}, {0, 5}, two items each.
    The same with k = 2: pairs (10, 9), (7, 6), (3, 1) with spreads 1, 1, 2.  (3, 1) goes first
    and meets the earlier of the two spread-1 pairs, (10, 9): 3 + 9, 1 + 10 = (12, 11); then (7, 6),
    created before (12, 11), meets it: 7 + 11, 6 + 12 = (18, 18): parts {0, 2, 5} and {1, 3, 4}."""
    for kk in (po.karmarkar_karp, packing.kk_partition):
        costs = [9, 8, 7, 4, 3, 1]
        parts = kk(costs, 3, True)
        assert sums(costs, parts) == [11, 11, 10]
        assert parts == [[1, 4], [2, 3], [0, 5]]          # equal sums: the part with the smaller first index first
        costs = [10, 9, 7, 6, 3, 1]
        parts = kk(costs, 2, True)
        assert sums(costs, parts) == [18, 18]
        assert parts == [[0, 2, 5], [1, 3, 4]]


def test_kk_result_depends_on_the_stated_tie_break():
    """Costs 5, 4, 3, 3, 2, 2, 2 into k = 3, by hand with the stated rules (larger spread first, among
    equal spreads the tuple created earlier; subsets by sum, then by smallest index):
      (5)+(4) -> (5, 4, 0) [spread 5];  it meets the earlier (3): (5, 4, 3) [2];
      the other (3) meets the earliest (2): (3, 2, 0) [3];  it meets the next (2): (3, 2, 2) [1];
      the last (2), created before (5, 4, 3), meets it: 2 + 3, 0 + 4, 0 + 5 = (5, 5, 4) [1];
      (3, 2, 2), created before (5, 5, 4), meets it: 3 + 4, 2 + 5, 2 + 5 = (7, 7, 7).
    Taking the LATER tuple among equal spreads instead ends in (8, 7, 6), so this instance tells
    the two rules apart; both implementations must give the perfect split."""
    costs = [5, 4, 3, 3, 2, 2, 2]
    for kk in (po.karmarkar_karp, packing.kk_partition):
        parts = kk(costs, 3, False)
        assert sums(costs, parts) == [7, 7, 7]
        assert parts == [[0, 5], [1, 3], [2, 4, 6]]


def best_makespan_and_spread(costs, k):
    """Exhaustive search over all k^n assignments: the smallest possible largest part and the
    smallest possible spread (largest minus smallest part)."""
    best_max, best_spread = None, None
    for assign in itertools.product(range(k), repeat=len(costs)):
        s = [0] * k
        for c, a in zip(costs, assign):
            s[a] += c
        m, sp = max(s), max(s) - min(s)
        best_max = m if best_max is None else min(best_max, m)
        best_spread = sp if best_spread is None else min(best_spread, sp)
    return best_max, best_spread


@pytest.mark.parametrize("seed", range(10))
def test_kk_against_exhaustive_search_on_small_inputs(seed):
    """n <= 8 items, k in {2, 3, 4}: the differencing result can be no better than the optimum found
    by exhaustive search, its spread is at most the largest item (merging largest with smallest
    never widens a tuple beyond the wider of the two), and its largest part is within the factor
    4/3 - 1/(3k) of the optimal one that is proven for the largest differencing method."""
    rng = np.random.default_rng(100 + seed)
    k = int(rng.choice([2, 3, 4]))
    n = int(rng.integers(k + 1, 9))
    costs = [int(v) for v in rng.integers(1, 60, size=n)]
    opt_max, opt_spread = best_makespan_and_spread(costs, k)
    for kk in (po.karmarkar_karp, packing.kk_partition):
        parts = kk(costs, k, False)
        assert_partition(parts, n, k)
        s = sums(costs, parts)
        assert max(s) >= opt_max and max(s) - min(s) >= opt_spread
        assert max(s) - min(s) <= max(costs)
        assert 3 * k * max(s) <= (4 * k - 1) * opt_max


def scalar_differencing(costs):
    """Textbook two-way differencing on bare numbers: replace the two largest by their
    difference until one number is left.  Independent of the tuple-based oracle."""
    h = [-c for c in costs]
    heapq.heapify(h)
    while len(h) > 1:
        a, b = -heapq.heappop(h), -heapq.heappop(h)
        heapq.heappush(h, -(a - b))
    return -h[0] if h else 0


@pytest.mark.parametrize("seed", range(8))
def test_kk_two_way_equals_scalar_differencing(seed):
    rng = np.random.default_rng(seed)
    costs = [int(v) for v in rng.integers(1, 10_000, size=int(rng.integers(2, 60)))]
    parts = po.karmarkar_karp(costs, 2, False)
    s = sums(costs, parts)
    assert abs(s[0] - s[1]) == scalar_differencing(costs)
    assert abs(s[0] - s[1]) <= max(costs)


@pytest.mark.parametrize("n,k,equal", [(1, 1, False), (7, 1, False), (3, 5, False), (12, 4, True),
                                       (12, 4, False), (64, 8, True), (100, 7, False)])
def test_kk_invariants(n, k, equal):
    rng = np.random.default_rng(n * 31 + k)
    costs = [int(v) for v in rng.integers(0, 1_000_000, size=n)]
    parts = po.karmarkar_karp(costs, k, equal)
    assert_partition(parts, n, k)
    s = sums(costs, parts)
    assert sum(s) == sum(costs)
    assert s == sorted(s, reverse=True)                       # parts come largest first
    if equal:
        assert {len(p) for p in parts} == {n // k}
    if k == 1:
        assert parts == [list(range(n))]
    if n <= k:
        assert sorted(len(p) for p in parts) == [0] * (k - n) + [1] * n
    if n > k:
        # never worse than putting everything in one part; spread at most the largest item for k = 2
        assert s[0] - s[-1] <= sum(costs)
    with pytest.raises(ValueError):
        po.karmarkar_karp(costs, 0, False)
    if n % 3:
        with pytest.raises(ValueError):
            po.karmarkar_karp(costs, 3, True)


def test_kk_balance_quality():
    """On moderately varied costs the k-way differencing spread is tiny next to dealing the
    samples out in order; on a long-tailed sample whose largest item exceeds a fair share, that
    item ends up alone in the largest part (nothing can be balanced against it)."""
    rng = np.random.default_rng(3)
    seq = [int(v) for v in rng.integers(128, 4096, size=256)]
    costs = [po.compute_cost(s) for s in seq]
    s = sums(costs, po.karmarkar_karp(costs, 8, False))
    rr = [sum(costs[i] for i in range(d, 256, 8)) for d in range(8)]
    assert s[0] - s[-1] < 0.01 * (max(rr) - min(rr))
    seq = lengths(256, 3)
    costs = [po.compute_cost(v) for v in seq]
    assert max(costs) > sum(costs) / 8
    parts = po.karmarkar_karp(costs, 8, False)
    assert parts[0] == [costs.index(max(costs))]


def test_cost_model_and_plans_by_hand():
    assert po.compute_cost(10) == 100 and po.compute_cost(10, hidden=2) == 10 * (10 + 12)
    # 4 samples, 2 devices, cap 10 tokens.  costs 64, 36, 16, 4 -> KK: {8} | {6, 4, 2} (64 vs 56)
    seq = [8, 6, 4, 2]
    plan = po.lb_mini(seq, 2, max_tokens=10)
    assert sorted(map(sorted, [sorted(i for mb in dev for i in mb) for dev in plan])) == [[0], [1, 2, 3]]
    dev_b = next(dev for dev in plan if len([i for mb in dev for i in mb]) == 3)
    # device with {6, 4, 2}: one microbatch has 12 tokens > 10, so k = 2: costs 36 | 16 + 4
    assert sorted(map(sorted, dev_b)) == [[1], [2, 3]]
    t_coll, t_odc, busy = po.runtimes(seq, plan)
    assert sorted(busy) == [56, 64]
    assert t_odc == 64                      # ODC: slowest device's total
    assert t_coll == 64 + 20                # step 0: max(64, 36) ; step 1: max(0, 20)
    assert po.bubble_rate(t_odc, busy) == pytest.approx(1 - 120 / 128)
    assert po.bubble_rate(t_coll, busy) == pytest.approx(1 - 120 / 168)
    # LB-Micro: equal counts (2 + 2) and a common k
    plan_m = po.lb_micro(seq, 2, max_tokens=10)
    assert [sum(len(mb) for mb in dev) for dev in plan_m] == [2, 2]
    assert len({len(dev) for dev in plan_m}) == 1
    for dev in plan_m:
        for mb in dev:
            assert sum(seq[i] for i in mb) <= 10


def test_local_sort_by_hand():
    """LocalSort: dealt in order, sorted inside the device, one sample per microbatch.
    2 devices: device 0 gets lengths (3, 9, 5) -> 9, 5, 3; device 1 gets (4, 4, 10) -> 10, 4, 4."""
    seq = [3, 9, 5, 4, 4, 10]
    plan = po.local_sort(seq, 2)
    assert plan == [[[1], [2], [0]], [[5], [3], [4]]]
    t_coll, t_odc, busy = po.runtimes(seq, plan)
    assert busy == [81 + 25 + 9, 100 + 16 + 16]
    assert t_coll == 100 + 25 + 16                    # per step the longer of the two
    assert t_odc == 132
    with pytest.raises(ValueError):
        po.local_sort(seq, 4)


@pytest.mark.parametrize("seed", range(4))
def test_balancing_beats_local_sort(seed):
    """On long-tailed lengths both balanced plans finish a minibatch sooner than LocalSort under
    the scheme they are meant for (collectives for LB-Micro, ODC for LB-Mini)."""
    seq = lengths(64, 50 + seed)
    ls = po.runtimes(seq, po.local_sort(seq, 8), 3584)
    micro = po.runtimes(seq, po.lb_micro(seq, 8, 32768, 3584), 3584)
    mini = po.runtimes(seq, po.lb_mini(seq, 8, 32768, 3584), 3584)
    assert micro[0] <= ls[0]
    assert mini[1] <= ls[1]


@pytest.mark.parametrize("seed", range(4))
def test_lb_mini_never_slower_than_lb_micro_under_odc(seed):
    """What Section 4 claims for LB-Mini: balancing whole minibatches is at least as good as
    balancing with equal sample counts, and every microbatch respects the memory cap."""
    seq = lengths(64, seed)
    mini = po.lb_mini(seq, 8, max_tokens=16384)
    micro = po.lb_micro(seq, 8, max_tokens=16384)
    for plan in (mini, micro):
        assert sorted(i for dev in plan for mb in dev for i in mb) == list(range(64))
        for dev in plan:
            for mb in dev:
                assert sum(seq[i] for i in mb) <= 16384 or len(mb) == 1
    _, t_odc_mini, busy_mini = po.runtimes(seq, mini)
    t_coll_micro, t_odc_micro, busy_micro = po.runtimes(seq, micro)
    assert t_odc_mini <= t_odc_micro <= t_coll_micro
    assert po.bubble_rate(t_odc_mini, busy_mini) <= po.bubble_rate(t_coll_micro, busy_micro)
    assert len({len(dev) for dev in micro}) == 1              # LB-Micro: same count everywhere


# ----------------------------------------------------------------------------- native vs oracle
def test_library_exports_every_declared_packing_symbol():
    header = open(os.path.join(ROOT, "include", "odc_packing.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(odc_[a-z_0-9]+)\s*\(", header))
    assert declared == set(packing.EXPORTS)
    from paper_2601_19362_amd import binding
    for name in declared:
        assert hasattr(binding.lib(), name)


@pytest.mark.parametrize("n,k,equal", [(0, 3, False), (1, 1, False), (5, 2, False), (5, 3, False), (3, 5, False),
                                       (12, 4, True), (64, 8, True), (64, 8, False), (257, 16, False),
                                       (1000, 32, False), (960, 32, True)])
def test_native_kk_equals_oracle(n, k, equal):
    rng = np.random.default_rng(n + 7 * k)
    for trial in range(3):
        costs = [int(v) for v in rng.integers(0, 50 if trial == 0 else 10 ** 9, size=n)]   # trial 0: many ties
        assert packing.kk_partition(costs, k, equal) == po.karmarkar_karp(costs, k, equal)


@pytest.mark.parametrize("n,world,cap,hidden", [(4, 2, 10, 0), (16, 4, 16384, 0), (64, 8, 16384, 3584),
                                                (128, 16, 16384, 3584), (256, 32, 32768, 5120), (64, 8, 1000, 0)])
def test_native_plans_and_runtime_equal_oracle(n, world, cap, hidden):
    seq = [8, 6, 4, 2] if n == 4 else lengths(n, n + world)
    for mode, fn in ((packing.LB_MINI, po.lb_mini), (packing.LB_MICRO, po.lb_micro),
                     (packing.LOCAL_SORT, lambda s, w, c, h: po.local_sort(s, w))):
        plan, counts = packing.plan_minibatch(seq, world, cap, hidden, mode)
        want = fn(seq, world, cap, hidden)
        assert plan == want
        assert counts == [len(dev) for dev in want]
        tc, to, busy, bc, bo = packing.plan_runtime(seq, plan, hidden)
        wtc, wto, wbusy = po.runtimes(seq, want, hidden)
        assert (tc, to, busy) == (wtc, wto, wbusy)
        assert bc == pytest.approx(po.bubble_rate(wtc, wbusy), abs=1e-15)
        assert bo == pytest.approx(po.bubble_rate(wto, wbusy), abs=1e-15)


def test_native_argument_errors():
    from paper_2601_19362_amd import binding as odc
    import ctypes
    lib = odc.lib()
    packing.compute_cost(1)
    assert packing.compute_cost(-1) == -1 and packing.compute_cost(2 ** 40) == -1 and packing.compute_cost(5, -1) == -1
    assert packing.compute_cost(2 ** 31, 0) == 2 ** 62
    arr = (ctypes.c_int64 * 4)(1, 2, 3, -4)
    out = (ctypes.c_int * 4)()
    assert lib.odc_kk_partition(arr, 4, 2, 0, out) == odc.ODC_ERR_INVALID_ARG          # negative cost
    arr = (ctypes.c_int64 * 4)(1, 2, 3, 4)
    assert lib.odc_kk_partition(arr, 4, 0, 0, out) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_kk_partition(arr, 4, 3, 1, out) == odc.ODC_ERR_INVALID_ARG          # 4 % 3 != 0
    assert lib.odc_kk_partition(None, 4, 2, 0, out) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_kk_partition(arr, 4, 2, 0, None) == odc.ODC_ERR_INVALID_ARG
    big = (ctypes.c_int64 * 2)(2 ** 62, 2 ** 62)
    assert lib.odc_kk_partition(big, 2, 2, 0, out) == odc.ODC_ERR_OVERFLOW
    cnt = (ctypes.c_int * 2)()
    assert lib.odc_plan_minibatch(arr, 4, 2, 0, 0, 0, out, out, cnt) == odc.ODC_ERR_INVALID_ARG   # cap < 1
    assert lib.odc_plan_minibatch(arr, 4, 3, 10, 0, 1, out, out, cnt) == odc.ODC_ERR_INVALID_ARG  # LB-Micro 4 % 3
    assert lib.odc_plan_minibatch(arr, 4, 3, 10, 0, 2, out, out, cnt) == odc.ODC_ERR_INVALID_ARG  # LocalSort 4 % 3
    assert lib.odc_plan_minibatch(arr, 4, 2, 10, 0, 3, out, out, cnt) == odc.ODC_ERR_INVALID_ARG  # bad mode


def test_bubble_table_estimates():
    """The bubble-rate table: ODC is never slower than collectives for the same plan (a maximum
    of sums against a sum of maxima), Collective + LocalSort is the unit, LB-Mini exists only
    under ODC, and every figure equals what the oracle gives for the same minibatches."""
    from paper_2601_19362_amd import bubble_table as bt
    table = bt.estimate(world=4, samples_per_device=4, minibatches=6, max_tokens=16384, hidden=1536, seed=3)
    assert set(table) == {("Collective", "LocalSort"), ("Collective", "LB-Micro"), ("ODC", "LocalSort"),
                          ("ODC", "LB-Micro"), ("ODC", "LB-Mini")}
    assert table[("Collective", "LocalSort")][0] == pytest.approx(1.0)
    for name in ("LocalSort", "LB-Micro"):
        assert table[("ODC", name)][0] <= table[("Collective", name)][0] + 1e-12
        assert table[("ODC", name)][1] <= table[("Collective", name)][1] + 1e-12
    for t, bub in table.values():
        assert t > 0 and 0.0 <= bub < 1.0
    # the same six minibatches through the oracle
    rel, bubbles = [], []
    for b in range(6):
        seq = bt.synthetic_lengths(16, 3 * 100003 + b, 7.0, 1.0, 128, 32768)
        base = po.runtimes(seq, po.local_sort(seq, 4), 1536)[0]
        t_coll, t_odc, busy = po.runtimes(seq, po.lb_mini(seq, 4, 16384, 1536), 1536)
        rel.append(t_odc / base)
        bubbles.append(po.bubble_rate(t_odc, busy))
    assert table[("ODC", "LB-Mini")][0] == pytest.approx(np.mean(rel), rel=1e-12)
    assert table[("ODC", "LB-Mini")][1] == pytest.approx(np.mean(bubbles), rel=1e-12)
