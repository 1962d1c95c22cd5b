"""ctypes binding of the host-side load-balancing entry points (include/odc_packing.h):
Karmarkar-Karp partitioning, the LB-Mini / LB-Micro minibatch plans of paper Section 4 and
Appendix C, and the runtime / bubble-rate estimate (Eq. 1, Appendix F).  Argument marshalling
only; the algorithms run in the native library."""
from __future__ import annotations

import ctypes
from typing import List, Sequence, Tuple

from . import binding

LB_MINI = 0
LB_MICRO = 1
LOCAL_SORT = 2
EXPORTS = ("odc_compute_cost", "odc_kk_partition", "odc_plan_minibatch", "odc_plan_runtime")

_i64 = ctypes.c_int64
_int = ctypes.c_int
_ready = False


def _lib():
    global _ready
    L = binding.lib()
    if not _ready:
        L.odc_compute_cost.restype = _i64
        L.odc_compute_cost.argtypes = [_i64, _i64]
        L.odc_kk_partition.restype = _int
        L.odc_kk_partition.argtypes = [ctypes.POINTER(_i64), _int, _int, _int, ctypes.POINTER(_int)]
        L.odc_plan_minibatch.restype = _int
        L.odc_plan_minibatch.argtypes = [ctypes.POINTER(_i64), _int, _int, _i64, _i64, _int,
                                         ctypes.POINTER(_int), ctypes.POINTER(_int), ctypes.POINTER(_int)]
        L.odc_plan_runtime.restype = _int
        L.odc_plan_runtime.argtypes = [ctypes.POINTER(_i64), _int, _int, _i64, ctypes.POINTER(_int),
                                       ctypes.POINTER(_int), ctypes.POINTER(_i64), ctypes.POINTER(_i64),
                                       ctypes.POINTER(_i64), ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_double)]
        _ready = True
    return L


def _check(rc: int, where: str) -> None:
    if rc != binding.ODC_OK:
        raise binding.OdcError(rc, where)


def compute_cost(seqlen: int, hidden: int = 0) -> int:
    return int(_lib().odc_compute_cost(int(seqlen), int(hidden)))


def kk_partition(costs: Sequence[int], k: int, equal_size: bool) -> List[List[int]]:
    """Parts in the library's order (largest sum first), item indices ascending."""
    n = len(costs)
    arr = (_i64 * max(n, 1))(*[int(c) for c in costs])
    out = (_int * max(n, 1))()
    _check(_lib().odc_kk_partition(arr, n, int(k), 1 if equal_size else 0, out), "odc_kk_partition")
    parts: List[List[int]] = [[] for _ in range(k)]
    for i in range(n):
        parts[out[i]].append(i)
    return parts


def plan_minibatch(seqlens: Sequence[int], world: int, max_tokens: int, hidden: int = 0,
                   mode: int = LB_MINI) -> Tuple[List[List[List[int]]], List[int]]:
    """(plan, micro_count): plan[d][m] lists the sample indices of device d's microbatch m."""
    n = len(seqlens)
    arr = (_i64 * max(n, 1))(*[int(s) for s in seqlens])
    dev = (_int * max(n, 1))()
    mic = (_int * max(n, 1))()
    cnt = (_int * max(world, 1))()
    _check(_lib().odc_plan_minibatch(arr, n, int(world), int(max_tokens), int(hidden), int(mode), dev, mic, cnt),
           "odc_plan_minibatch")
    counts = [cnt[d] for d in range(world)]
    plan = [[[] for _ in range(counts[d])] for d in range(world)]
    for i in range(n):
        plan[dev[i]][mic[i]].append(i)
    return plan, counts


def plan_runtime(seqlens: Sequence[int], plan, hidden: int = 0):
    """(t_collective, t_odc, busy per device, bubble_collective, bubble_odc) of a plan."""
    n = len(seqlens)
    world = len(plan)
    dev = (_int * max(n, 1))()
    mic = (_int * max(n, 1))()
    for d, micros in enumerate(plan):
        for m, mb in enumerate(micros):
            for i in mb:
                dev[i], mic[i] = d, m
    arr = (_i64 * max(n, 1))(*[int(s) for s in seqlens])
    tc, to = _i64(), _i64()
    busy = (_i64 * world)()
    bc, bo = ctypes.c_double(), ctypes.c_double()
    _check(_lib().odc_plan_runtime(arr, n, world, int(hidden), dev, mic, ctypes.byref(tc), ctypes.byref(to), busy,
                                   ctypes.byref(bc), ctypes.byref(bo)), "odc_plan_runtime")
    return tc.value, to.value, [busy[d] for d in range(world)], bc.value, bo.value
