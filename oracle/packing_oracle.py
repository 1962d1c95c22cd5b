"""CPU oracle for the load-balancing side of ODC (paper Section 4 and Appendix C).

TEST INFRASTRUCTURE ONLY; shares no code with the native implementation.

What the paper fixes: the interface of the helpers (Appendix C, helper-function listing) --
a Karmarkar-Karp partition of compute costs into k parts with an `equal_size` switch, a
minibatch partition over the devices (equal_size for LB-Micro, not for LB-Mini), and a
microbatch partition that raises k until every microbatch is memory-feasible (all devices in
lockstep for LB-Micro, each device on its own for LB-Mini) -- plus Eq. 1 for the runtime under
per-layer synchronisation and the definition of the bubble rate (Appendix F: idle time over
total time, as estimated by the packing algorithm).  The bodies of karmarkar_karp,
get_compute_costs and check_oom are not printed; the readings taken here:

  * karmarkar_karp: the k-way largest differencing method of the cited 1982 paper.  Every
    item starts as a k-tuple of subsets (itself and k-1 empty ones).  Repeatedly the two
    tuples with the largest spread (largest minus smallest subset sum) are merged, pairing the
    i-th largest subset of one with the i-th smallest of the other, until one tuple is left.
    equal_size: items sorted by cost (descending) are first grouped k at a time into tuples of
    k singletons, so every merge keeps the subset sizes equal (n must be a multiple of k).
    Ties are broken deterministically: larger spread first, then the tuple created earlier;
    inside a tuple subsets are ordered by sum (descending), then by their smallest item index.
    The returned partition lists, for each of the k parts in final order (largest sum first),
    the item indices in ascending order.
  * get_compute_costs: cost(s) = s * (s + 6 * hidden) -- the attention term grows with s^2 and
    the dense term with s (Section 4: runtime O(s^2), activation memory O(s)); hidden = 0
    gives the pure quadratic model.  parity unpinned (the paper prints no body).
  * check_oom: a microbatch is infeasible when it holds more than one sample and its token
    count exceeds `max_tokens` (a single sample longer than the cap cannot be split, so it is
    accepted alone).  parity unpinned.

  * LocalSort (Section 5.1 says only: sorted by length within each device's minibatch, not
    packed): samples dealt in order, n / world per device, longest first, one per microbatch.
    The sort direction does not change either runtime estimate.

All arithmetic is exact Python integer arithmetic.
"""
from __future__ import annotations

import heapq
from typing import List, Sequence, Tuple


def compute_cost(seqlen: int, hidden: int = 0) -> int:
    return int(seqlen) * (int(seqlen) + 6 * int(hidden))


def karmarkar_karp(costs: Sequence[int], k: int, equal_size: bool) -> List[List[int]]:
    n = len(costs)
    if k < 1:
        raise ValueError("k must be >= 1")
    if equal_size and n % k != 0:
        raise ValueError("equal_size needs len(costs) to be a multiple of k")
    if n == 0:
        return [[] for _ in range(k)]

    def make_state(subsets):
        # subsets: list of (sum, items tuple); ordered by sum descending, then smallest index
        subsets = sorted(subsets, key=lambda s: (-s[0], s[1][0] if s[1] else n))
        return subsets

    states = []
    serial = 0
    if equal_size:
        order = sorted(range(n), key=lambda i: (-costs[i], i))
        for g in range(0, n, k):
            subs = [(int(costs[i]), (i,)) for i in order[g:g + k]]
            st = make_state(subs)
            states.append((-(st[0][0] - st[-1][0]), serial, st))
            serial += 1
    else:
        for i in range(n):
            subs = [(int(costs[i]), (i,))] + [(0, ())] * (k - 1)
            st = make_state(subs)
            states.append((-(st[0][0] - st[-1][0]), serial, st))
            serial += 1
    heapq.heapify(states)
    while len(states) > 1:
        _, _, a = heapq.heappop(states)
        _, _, b = heapq.heappop(states)
        merged = []
        for i in range(k):
            sa, ia = a[i]
            sb, ib = b[k - 1 - i]
            merged.append((sa + sb, tuple(sorted(ia + ib))))
        st = make_state(merged)
        heapq.heappush(states, (-(st[0][0] - st[-1][0]), serial, st))
        serial += 1
    final = states[0][2]
    return [list(items) for _, items in final]


def minibatch_partition(seqlens: Sequence[int], world: int, equal_size: bool, hidden: int = 0) -> List[List[int]]:
    costs = [compute_cost(s, hidden) for s in seqlens]
    return karmarkar_karp(costs, world, equal_size)


def _micro_parts(seqlens: Sequence[int], k: int, hidden: int) -> List[List[int]]:
    costs = [compute_cost(s, hidden) for s in seqlens]
    parts = karmarkar_karp(costs, k, False)
    return parts


def _oom(seqlens: Sequence[int], parts: List[List[int]], max_tokens: int) -> bool:
    return any(len(p) > 1 and sum(seqlens[i] for i in p) > max_tokens for p in parts)


def microbatch_partition(seqlens: Sequence[int], max_tokens: int, hidden: int = 0, k_start: int = 1) -> List[List[int]]:
    """One device, LB-Mini: raise k until every microbatch fits (a sample longer than
    max_tokens counts as fitting when it is alone).  Empty microbatches are kept out of the
    result."""
    n = len(seqlens)
    if n == 0:
        return []
    k = max(1, k_start)
    while True:
        parts = _micro_parts(seqlens, k, hidden)
        if not _oom(seqlens, parts, max_tokens) or k >= n:
            return [p for p in parts if p]
        k += 1


def lb_mini(seqlens: Sequence[int], world: int, max_tokens: int, hidden: int = 0):
    """LB-Mini (Section 4): balance the minibatch over devices by compute cost alone
    (equal_size = False), then every device packs its own samples, with its own k."""
    device_parts = minibatch_partition(seqlens, world, False, hidden)
    out = []
    for part in device_parts:
        local = [seqlens[i] for i in part]
        micro = microbatch_partition(local, max_tokens, hidden)
        out.append([[part[j] for j in mb] for mb in micro])
    return out


def lb_micro(seqlens: Sequence[int], world: int, max_tokens: int, hidden: int = 0):
    """LB-Micro: equal sample counts per device (equal_size = True) and the same number of
    microbatches on every device: k grows until no device reports an infeasible microbatch
    (the all-reduce of is_oom in the listing)."""
    device_parts = minibatch_partition(seqlens, world, True, hidden)
    n_max = max(len(p) for p in device_parts)
    k = 1
    while True:
        per_device = [_micro_parts([seqlens[i] for i in part], k, hidden) for part in device_parts]
        bad = any(_oom([seqlens[i] for i in part], parts, max_tokens)
                  for part, parts in zip(device_parts, per_device))
        if not bad or k >= n_max:
            return [[[part[j] for j in mb] for mb in parts] for part, parts in zip(device_parts, per_device)]
        k += 1


def local_sort(seqlens: Sequence[int], world: int):
    """LocalSort (Section 5.1): no balancing and no packing -- the minibatch is dealt to the
    devices in the order given, each device sorts its samples by length (longest first, ties by
    index) and runs one sample per microbatch."""
    n = len(seqlens)
    if n % world != 0:
        raise ValueError("LocalSort needs len(seqlens) to be a multiple of world")
    per = n // world
    plan = []
    for d in range(world):
        ids = sorted(range(d * per, (d + 1) * per), key=lambda i: (-seqlens[i], i))
        plan.append([[i] for i in ids])
    return plan


def runtimes(seqlens: Sequence[int], plan, hidden: int = 0) -> Tuple[int, int, List[int]]:
    """(T_collective, T_odc, busy per device) in cost units.

    Eq. 1: with per-layer collectives every device waits for the slowest one in every
    microbatch step, T = sum_m max_d cost(d, m) (the per-layer factor is common and dropped; a
    device that has run out of microbatches contributes 0).  With ODC the only barrier is at
    the minibatch end, T = max_d sum_m cost(d, m)."""
    cost = [[sum(compute_cost(seqlens[i], hidden) for i in mb) for mb in dev] for dev in plan]
    steps = max((len(c) for c in cost), default=0)
    t_coll = sum(max((c[m] if m < len(c) else 0) for c in cost) for m in range(steps))
    busy = [sum(c) for c in cost]
    t_odc = max(busy, default=0)
    return t_coll, t_odc, busy


def bubble_rate(total_time: int, busy: Sequence[int]) -> float:
    """Idle time over total device time (Appendix F)."""
    d = len(busy)
    if total_time == 0 or d == 0:
        return 0.0
    return 1.0 - sum(busy) / (d * total_time)
