"""CPU oracle for the ODC gather / scatter-accumulate path: Python face of odc_oracle.c.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this module;
it is used by the tests, by the smoke check and by the benchmark's CPU-baseline leg.
It shares no code with the HIP library.

All bf16 data are numpy uint16 arrays holding the raw bit patterns; accumulators
are numpy float32 arrays.  The arithmetic lives in odc_oracle.c (plain loops, one
binary32 add per element and contribution); this file only marshals arrays and, for
timing, splits the flat element range over host threads, which leaves every element's
sequence of operations unchanged.

Paper passages followed: Section 3 (gather and scatter-accumulate as the point-to-point
decomposition of all-gather and reduce-scatter), Section 3.1 (even partition),
Section 2.1 (accumulated gradient = sum of the contributions, w_m = 1), Appendix B
(owner accumulates on receipt), Section 3.2 (accumulators are per minibatch), Section 6.1
(hybrid sharding: the groups' gradient shards are summed at the minibatch end).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "odc_oracle.c")
_BUILD_DIR = os.path.join(_HERE, "_build")
_LIB_PATH = os.path.join(_BUILD_DIR, "libodc_oracle.so")
_CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared", "-fPIC"]
_LDLIBS = ["-lm"]

_lib = None
_lock = threading.Lock()

_i64 = ctypes.c_int64
_vp = ctypes.c_void_p
_vpp = ctypes.POINTER(ctypes.c_void_p)


def build(force: bool = False) -> str:
    """Compile odc_oracle.c with gcc into oracle/_build/ (skipped when up to date)."""
    os.makedirs(_BUILD_DIR, exist_ok=True)
    stale = (not os.path.exists(_LIB_PATH)
             or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC))
    if force or stale:
        tmp = _LIB_PATH + f".tmp{os.getpid()}"
        subprocess.run(["gcc", *_CFLAGS, _SRC, "-o", tmp, *_LDLIBS], check=True)
        os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            lib.odc_oracle_shard_elems.restype = _i64
            lib.odc_oracle_shard_elems.argtypes = [_i64, _i64]
            lib.odc_oracle_valid_elems.restype = _i64
            lib.odc_oracle_valid_elems.argtypes = [_i64, _i64, _i64]
            lib.odc_oracle_make_shard.restype = None
            lib.odc_oracle_make_shard.argtypes = [_vp, _i64, _i64, _i64, _vp]
            lib.odc_oracle_gather.restype = None
            lib.odc_oracle_gather.argtypes = [_vpp, _i64, _i64, _vp, _i64, _i64]
            lib.odc_oracle_reset.restype = None
            lib.odc_oracle_reset.argtypes = [_vpp, _i64, _i64, _i64, _i64]
            lib.odc_oracle_accumulate.restype = None
            lib.odc_oracle_accumulate.argtypes = [_vp, _vpp, _i64, _i64, _i64, _i64]
            lib.odc_oracle_gather_batched.restype = ctypes.c_int
            lib.odc_oracle_gather_batched.argtypes = [_vpp, _i64, _vp, _vp, _vp, _i64, _vp]
            lib.odc_oracle_reset_batched.restype = ctypes.c_int
            lib.odc_oracle_reset_batched.argtypes = [_vpp, _i64, _vp, _vp, _i64]
            lib.odc_oracle_accumulate_batched.restype = ctypes.c_int
            lib.odc_oracle_accumulate_batched.argtypes = [_vp, _vpp, _i64, _vp, _vp, _vp, _i64]
            _f32 = ctypes.c_float
            lib.odc_oracle_accumulate_weighted.restype = None
            lib.odc_oracle_accumulate_weighted.argtypes = [_vp, _vpp, _i64, _i64, _f32, _i64, _i64]
            lib.odc_oracle_retrieve_f32.restype = None
            lib.odc_oracle_retrieve_f32.argtypes = [_vpp, _vpp, _i64, _i64, _f32, _i64, _i64]
            lib.odc_oracle_retrieve_bf16.restype = None
            lib.odc_oracle_retrieve_bf16.argtypes = [_vpp, _vpp, _i64, _i64, _f32, _i64, _i64]
            lib.odc_oracle_accumulate_weighted_batched.restype = ctypes.c_int
            lib.odc_oracle_accumulate_weighted_batched.argtypes = [_vp, _vpp, _i64, _vp, _vp, _vp, _i64, _f32]
            lib.odc_oracle_retrieve_batched.restype = ctypes.c_int
            lib.odc_oracle_retrieve_batched.argtypes = [_vpp, _vpp, _i64, _vp, _vp, _i64, _f32, ctypes.c_int]
            _f64pp = _vpp
            lib.odc_oracle_accumulate_wide.restype = None
            lib.odc_oracle_accumulate_wide.argtypes = [_vp, _f64pp, _i64, _i64, _i64, _i64]
            lib.odc_oracle_reset_wide.restype = None
            lib.odc_oracle_reset_wide.argtypes = [_f64pp, _i64, _i64, _i64, _i64]
            lib.odc_oracle_retrieve_wide.restype = None
            lib.odc_oracle_retrieve_wide.argtypes = [_f64pp, _vpp, _i64, _i64, ctypes.c_float, ctypes.c_int, _i64, _i64]
            lib.odc_oracle_reduce_groups.restype = None
            lib.odc_oracle_reduce_groups.argtypes = [_vpp, _i64, _vpp, _i64, _i64, _i64, _i64]
            lib.odc_oracle_reduce_groups_batched.restype = ctypes.c_int
            lib.odc_oracle_reduce_groups_batched.argtypes = [_vpp, _i64, _vpp, _i64, _vp, _vp, _i64]
            _lib = lib
    return _lib


# ----------------------------------------------------------------------------- helpers
def _check(a: np.ndarray, dtype, min_len: int, what: str) -> None:
    if not isinstance(a, np.ndarray) or a.dtype != dtype or a.ndim != 1:
        raise TypeError(f"{what}: expected 1-D numpy {np.dtype(dtype).name} array")
    if not a.flags.c_contiguous:
        raise ValueError(f"{what}: array must be contiguous")
    if a.shape[0] < min_len:
        raise ValueError(f"{what}: needs at least {min_len} elements, has {a.shape[0]}")


def _ptr_array(arrays):
    arr = (ctypes.c_void_p * len(arrays))()
    for k, a in enumerate(arrays):
        arr[k] = a.ctypes.data
    return arr


def _i64_array(xs) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(xs, dtype=np.int64))


def _split(N: int, nthreads: int):
    nthreads = max(1, min(int(nthreads), N))
    edges = [N * k // nthreads for k in range(nthreads + 1)]
    return [(edges[k], edges[k + 1]) for k in range(nthreads) if edges[k + 1] > edges[k]]


def _run_ranges(fn, N: int, nthreads: int, ranges=None) -> None:
    """Call fn(j_begin, j_end) over a partition of [0, N) (or over the given flat-index
    ranges only, for sampled checks of very large tensors); ctypes drops the GIL."""
    if ranges is not None:
        end = 0
        for a, b in sorted(ranges):
            if not 0 <= a <= b <= N:
                raise ValueError(f"range ({a}, {b}) outside [0, {N}]")
            if a < end:
                raise ValueError("ranges overlap: an element would be processed twice")
            end = b
        for a, b in ranges:
            fn(a, b)
        return
    ranges = _split(N, nthreads)
    if len(ranges) <= 1:
        fn(0, N)
        return
    with ThreadPoolExecutor(max_workers=len(ranges)) as ex:
        for f in [ex.submit(fn, a, b) for a, b in ranges]:
            f.result()


# ----------------------------------------------------------------------------- layout
def shard_elems(N: int, R: int) -> int:
    """S = ceil(N / R): slots in every owner's shard (Section 3.1, even partition)."""
    if N < 1 or R < 1:
        raise ValueError("N and R must be >= 1")
    return int(_load().odc_oracle_shard_elems(N, R))


def valid_elems(N: int, R: int, r: int) -> int:
    """Non-padding elements held by owner r."""
    if N < 1 or R < 1 or not 0 <= r < R:
        raise ValueError("bad (N, R, r)")
    return int(_load().odc_oracle_valid_elems(N, R, r))


def make_shards(flat: np.ndarray, R: int, pad_bits: int = 0xDEAD) -> list:
    """Cut a flat bf16 parameter (uint16 bits) into R owner shards of S slots each.

    Padding slots hold pad_bits so that a test can see whether anything reads them
    into the result or overwrites them.
    """
    _check(flat, np.uint16, 1, "flat")
    N = flat.shape[0]
    S = shard_elems(N, R)
    lib = _load()
    out = []
    for r in range(R):
        sh = np.full(S, pad_bits, dtype=np.uint16)
        lib.odc_oracle_make_shard(flat.ctypes.data, N, R, r, sh.ctypes.data)
        out.append(sh)
    return out


# ----------------------------------------------------------------------------- primitives
def gather(shards, N: int, full: np.ndarray, nthreads: int = 1, ranges=None) -> np.ndarray:
    """full[r*S + i] = shard_r[i] for valid i; full[N:] is left untouched.  Returns full.
    With `ranges` only the flat indices inside those [a, b) intervals are produced."""
    R = len(shards)
    S = shard_elems(N, R)
    for r, sh in enumerate(shards):
        _check(sh, np.uint16, S, f"shards[{r}]")
    _check(full, np.uint16, N, "full")
    lib = _load()
    ptrs = _ptr_array(shards)
    _run_ranges(lambda a, b: lib.odc_oracle_gather(ptrs, N, R, full.ctypes.data, a, b), N, nthreads, ranges)
    return full


def reset(acc, N: int, nthreads: int = 1, ranges=None) -> None:
    """Valid accumulator elements become +0.0f; padding slots keep their content."""
    R = len(acc)
    S = shard_elems(N, R)
    for r, a in enumerate(acc):
        _check(a, np.float32, S, f"acc[{r}]")
    lib = _load()
    ptrs = _ptr_array(acc)
    _run_ranges(lambda a, b: lib.odc_oracle_reset(ptrs, N, R, a, b), N, nthreads, ranges)


def accumulate(g: np.ndarray, acc, N: int, nthreads: int = 1, ranges=None) -> None:
    """Apply ONE contribution: acc_r[i] = fl32(acc_r[i] + widen(g[r*S+i])) for valid i."""
    R = len(acc)
    S = shard_elems(N, R)
    _check(g, np.uint16, N, "g")
    for r, a in enumerate(acc):
        _check(a, np.float32, S, f"acc[{r}]")
    lib = _load()
    ptrs = _ptr_array(acc)
    _run_ranges(lambda a, b: lib.odc_oracle_accumulate(g.ctypes.data, ptrs, N, R, a, b), N, nthreads, ranges)


def accumulate_weighted(g: np.ndarray, acc, N: int, weight: float, nthreads: int = 1, ranges=None) -> None:
    """ONE weighted contribution: acc_r[i] = fma32(weight, widen(g[r*S+i]), acc_r[i]) (Section 2.1,
    w_m != 1; one rounding per element)."""
    R = len(acc)
    S = shard_elems(N, R)
    _check(g, np.uint16, N, "g")
    for r, a in enumerate(acc):
        _check(a, np.float32, S, f"acc[{r}]")
    lib = _load()
    ptrs = _ptr_array(acc)
    w = float(np.float32(weight))
    _run_ranges(lambda a, b: lib.odc_oracle_accumulate_weighted(g.ctypes.data, ptrs, N, R, w, a, b),
                N, nthreads, ranges)


def retrieve(acc, out, N: int, scale: float = 1.0, nthreads: int = 1, ranges=None) -> None:
    """Minibatch-end retrieval (Section 3.2): out_r[i] = cast(fl32(scale * acc_r[i])) for valid i.
    `out` arrays are float32 (no further rounding) or uint16 (bf16 bits, round-to-nearest-even)."""
    R = len(acc)
    S = shard_elems(N, R)
    to_bf16 = out[0].dtype == np.uint16
    for r in range(R):
        _check(acc[r], np.float32, S, f"acc[{r}]")
        _check(out[r], np.uint16 if to_bf16 else np.float32, S, f"out[{r}]")
    lib = _load()
    pa, po = _ptr_array(acc), _ptr_array(out)
    sc = float(np.float32(scale))
    fn = lib.odc_oracle_retrieve_bf16 if to_bf16 else lib.odc_oracle_retrieve_f32
    _run_ranges(lambda a, b: fn(pa, po, N, R, sc, a, b), N, nthreads, ranges)


def accumulate_wide(g: np.ndarray, acc64, N: int, nthreads: int = 1, ranges=None) -> None:
    """ONE contribution into binary64 accumulators: acc64_r[i] = fl64(acc64_r[i] + widen(g[r*S+i]))."""
    R = len(acc64)
    S = shard_elems(N, R)
    _check(g, np.uint16, N, "g")
    for r, a in enumerate(acc64):
        _check(a, np.float64, S, f"acc64[{r}]")
    lib = _load()
    ptrs = _ptr_array(acc64)
    _run_ranges(lambda a, b: lib.odc_oracle_accumulate_wide(g.ctypes.data, ptrs, N, R, a, b), N, nthreads, ranges)


def reset_wide(acc64, N: int, nthreads: int = 1, ranges=None) -> None:
    R = len(acc64)
    S = shard_elems(N, R)
    for r, a in enumerate(acc64):
        _check(a, np.float64, S, f"acc64[{r}]")
    lib = _load()
    ptrs = _ptr_array(acc64)
    _run_ranges(lambda a, b: lib.odc_oracle_reset_wide(ptrs, N, R, a, b), N, nthreads, ranges)


def retrieve_wide(acc64, out, N: int, scale: float = 1.0, nthreads: int = 1, ranges=None) -> None:
    """out_r[i] = cast(fl32(scale * fl32(acc64_r[i]))): one rounding to binary32, then as `retrieve`."""
    R = len(acc64)
    S = shard_elems(N, R)
    to_bf16 = out[0].dtype == np.uint16
    for r in range(R):
        _check(acc64[r], np.float64, S, f"acc64[{r}]")
        _check(out[r], np.uint16 if to_bf16 else np.float32, S, f"out[{r}]")
    lib = _load()
    pa, po = _ptr_array(acc64), _ptr_array(out)
    sc = float(np.float32(scale))
    _run_ranges(lambda a, b: lib.odc_oracle_retrieve_wide(pa, po, N, R, sc, 1 if to_bf16 else 0, a, b),
                N, nthreads, ranges)


def wide_views(arenas, numel, shard_off, t: int, R: int):
    """Views of tensor t's shard slots inside R arenas (for the multi-tensor forms of the wide
    routines, which handle one tensor after the other with the single-tensor routine)."""
    S = -(-int(numel[t]) // R)
    return [a[int(shard_off[t]):int(shard_off[t]) + S] for a in arenas]


def reduce_groups(group_acc, out, N: int, nthreads: int = 1, ranges=None) -> None:
    """Hybrid sharding (Section 6.1): out_r = ((a_0r + a_1r) + ...) over the K groups' shard r, in
    ascending group order, one binary32 add each.  group_acc[k][r] is group k's accumulator
    shard of owner r; out[r] may be group_acc[0][r]."""
    K, R = len(group_acc), len(out)
    S = shard_elems(N, R)
    flat = []
    for k, grp in enumerate(group_acc):
        if len(grp) != R:
            raise ValueError("every group needs R shards")
        for r, a in enumerate(grp):
            _check(a, np.float32, S, f"group_acc[{k}][{r}]")
            flat.append(a)
    for r, a in enumerate(out):
        _check(a, np.float32, S, f"out[{r}]")
    lib = _load()
    pg, po = _ptr_array(flat), _ptr_array(out)
    _run_ranges(lambda a, b: lib.odc_oracle_reduce_groups(pg, K, po, N, R, a, b), N, nthreads, ranges)


def reduce_groups_batched(group_arenas, out_arenas, numel, shard_off) -> None:
    K, R = len(group_arenas), len(out_arenas)
    numel, shard_off = _i64_array(numel), _i64_array(shard_off)
    flat = []
    for grp in group_arenas:
        _bounds_batched(grp, np.float32, numel, shard_off, R, "group_arenas")
        flat.extend(grp)
    _bounds_batched(out_arenas, np.float32, numel, shard_off, R, "out_arenas")
    rc = _load().odc_oracle_reduce_groups_batched(_ptr_array(flat), K, _ptr_array(out_arenas), numel.shape[0],
                                                  numel.ctypes.data, shard_off.ctypes.data, R)
    if rc != 0:
        raise MemoryError("oracle scratch allocation failed")


def scatter_accumulate_ordered(grads, acc, N: int, nthreads: int = 1) -> int:
    """Ordered scatter-accumulate of a whole minibatch.

    grads[w][m] is worker w's bf16 gradient for its m-th microbatch (len(grads) = R
    workers, len(grads[w]) = M_w, which may differ per worker).  Contributions are applied
    worker ascending, then microbatch ascending, one at a time.  Returns their count.
    """
    count = 0
    for w in range(len(grads)):
        for m in range(len(grads[w])):
            accumulate(grads[w][m], acc, N, nthreads)
            count += 1
    return count


def widen(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> the float32 values they denote (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def fp64_add(g: np.ndarray, tot: np.ndarray, mag: np.ndarray, nthreads: int = 1, ranges=None) -> None:
    """One contribution added to a float64 reference: tot[j] += widen(g[j]), mag[j] += |widen(g[j])|
    for every j (or only inside the given [a, b) intervals).  tot and mag are float64 arrays as
    long as g; the element range may be split over threads."""
    n = g.shape[0]
    _check(g, np.uint16, n, "g")
    _check(tot, np.float64, n, "tot")
    _check(mag, np.float64, n, "mag")

    def part(a, b):
        step = 1 << 22                                   # bounded temporaries
        for lo in range(a, b, step):
            hi = min(b, lo + step)
            v = widen(g[lo:hi]).astype(np.float64)
            tot[lo:hi] += v
            mag[lo:hi] += np.abs(v)

    _run_ranges(part, n, nthreads, ranges)


def fp64_sum_shards(grads, N: int, R: int, nthreads: int = 1):
    """Reference for the unordered mode: per owner, the float64 sum of all contributions.

    Returns (sum64, abs64): lists of R float64 arrays of S slots (padding = 0) holding
    the sum of the widened values and the sum of their magnitudes (the scale of the
    forward error bound).
    """
    S = shard_elems(N, R)
    tot = np.zeros(R * S, dtype=np.float64)
    mag = np.zeros(R * S, dtype=np.float64)
    for per_worker in grads:
        for g in per_worker:
            fp64_add(np.ascontiguousarray(g[:N]), tot[:N], mag[:N], nthreads)
    return ([tot[r * S:(r + 1) * S] for r in range(R)],
            [mag[r * S:(r + 1) * S] for r in range(R)])


# ----------------------------------------------------------------------------- batched
def gather_batched(arenas, numel, shard_off, full_off, full: np.ndarray) -> np.ndarray:
    """Gather T tensors; tensor t's shard sits at arenas[r][shard_off[t]:] for every owner
    r and its full copy goes to full[full_off[t]:full_off[t]+numel[t]]."""
    R = len(arenas)
    numel, shard_off, full_off = _i64_array(numel), _i64_array(shard_off), _i64_array(full_off)
    T = numel.shape[0]
    _bounds_batched(arenas, np.uint16, numel, shard_off, R, "arenas")
    _check(full, np.uint16, int((full_off + numel).max()), "full")
    rc = _load().odc_oracle_gather_batched(_ptr_array(arenas), T, numel.ctypes.data,
                                           shard_off.ctypes.data, full_off.ctypes.data, R,
                                           full.ctypes.data)
    if rc != 0:
        raise MemoryError("oracle scratch allocation failed")
    return full


def reset_batched(acc_arenas, numel, shard_off) -> None:
    R = len(acc_arenas)
    numel, shard_off = _i64_array(numel), _i64_array(shard_off)
    _bounds_batched(acc_arenas, np.float32, numel, shard_off, R, "acc_arenas")
    rc = _load().odc_oracle_reset_batched(_ptr_array(acc_arenas), numel.shape[0],
                                          numel.ctypes.data, shard_off.ctypes.data, R)
    if rc != 0:
        raise MemoryError("oracle scratch allocation failed")


def accumulate_batched(g_full: np.ndarray, acc_arenas, numel, shard_off, full_off) -> None:
    R = len(acc_arenas)
    numel, shard_off, full_off = _i64_array(numel), _i64_array(shard_off), _i64_array(full_off)
    _bounds_batched(acc_arenas, np.float32, numel, shard_off, R, "acc_arenas")
    _check(g_full, np.uint16, int((full_off + numel).max()), "g_full")
    rc = _load().odc_oracle_accumulate_batched(g_full.ctypes.data, _ptr_array(acc_arenas),
                                               numel.shape[0], numel.ctypes.data,
                                               shard_off.ctypes.data, full_off.ctypes.data, R)
    if rc != 0:
        raise MemoryError("oracle scratch allocation failed")


def _bounds_batched(arenas, dtype, numel, shard_off, R, what) -> None:
    if numel.shape != shard_off.shape or numel.ndim != 1 or numel.shape[0] < 1:
        raise ValueError("numel / shard_off must be 1-D and equally long")
    if (numel < 1).any() or (shard_off < 0).any():
        raise ValueError("numel must be >= 1 and offsets >= 0")
    S = -(-numel // R)
    need = int((shard_off + S).max())
    for r, a in enumerate(arenas):
        _check(a, dtype, need, f"{what}[{r}]")


def accumulate_weighted_batched(g_full: np.ndarray, acc_arenas, numel, shard_off, full_off, weight: float) -> None:
    R = len(acc_arenas)
    numel, shard_off, full_off = _i64_array(numel), _i64_array(shard_off), _i64_array(full_off)
    _bounds_batched(acc_arenas, np.float32, numel, shard_off, R, "acc_arenas")
    _check(g_full, np.uint16, int((full_off + numel).max()), "g_full")
    rc = _load().odc_oracle_accumulate_weighted_batched(
        g_full.ctypes.data, _ptr_array(acc_arenas), numel.shape[0], numel.ctypes.data,
        shard_off.ctypes.data, full_off.ctypes.data, R, float(np.float32(weight)))
    if rc != 0:
        raise MemoryError("oracle scratch allocation failed")


def retrieve_batched(acc_arenas, out_arenas, numel, shard_off, scale: float = 1.0) -> None:
    R = len(acc_arenas)
    numel, shard_off = _i64_array(numel), _i64_array(shard_off)
    to_bf16 = out_arenas[0].dtype == np.uint16
    _bounds_batched(acc_arenas, np.float32, numel, shard_off, R, "acc_arenas")
    _bounds_batched(out_arenas, np.uint16 if to_bf16 else np.float32, numel, shard_off, R, "out_arenas")
    rc = _load().odc_oracle_retrieve_batched(_ptr_array(acc_arenas), _ptr_array(out_arenas), numel.shape[0],
                                             numel.ctypes.data, shard_off.ctypes.data, R,
                                             float(np.float32(scale)), 1 if to_bf16 else 0)
    if rc != 0:
        raise MemoryError("oracle scratch allocation failed")


class Staging:
    """Server-side staging of Appendix B, as plain bookkeeping around `accumulate`.

    Every owner has one receive slot per client, which is empty, being written, or full.
    A push by client w is decided once per owner, when it begins: an owner whose slot for w
    is empty keeps slice r of g there (the slot is being written until the push ends, then
    full); an owner whose slot is not empty refuses (counted) -- a client has one buffer per
    owner, and its requests are serialised.  A drain first notes which slots are full, adds
    those to the accumulators in ascending client order, one contribution after the other,
    and then empties exactly those.  push() and drain() are the undivided forms; the phase
    methods let a test interleave a push with a drain the way two streams can.
    """

    EMPTY, WRITING, FULL = 0, 2, 1

    def __init__(self, numel, R: int, shard_off=None, full_off=None):
        self.numel = [int(n) for n in numel]
        self.R = R
        self.shard_off = list(shard_off) if shard_off is not None else [0] * len(self.numel)
        self.full_off = list(full_off) if full_off is not None else [0] * len(self.numel)
        self.slot = {}
        self.state = [[self.EMPTY] * R for _ in range(R)]
        self.refused = 0
        self.noted = []

    @property
    def full(self):
        return [[s == self.FULL for s in row] for row in self.state]

    # -- push, in two phases
    def begin_push(self, g_full: np.ndarray, worker: int) -> None:
        for r in range(self.R):
            if self.state[r][worker] != self.EMPTY:
                self.refused += 1
            else:
                self.slot[(r, worker)] = g_full.copy()
                self.state[r][worker] = self.WRITING

    def end_push(self, worker: int) -> None:
        for r in range(self.R):
            if self.state[r][worker] == self.WRITING:
                self.state[r][worker] = self.FULL

    def push(self, g_full: np.ndarray, worker: int) -> None:
        self.begin_push(g_full, worker)
        self.end_push(worker)

    # -- drain, in three phases
    def begin_drain(self) -> None:
        self.noted = [(r, w) for r in range(self.R) for w in range(self.R) if self.state[r][w] == self.FULL]

    def add_noted(self, acc_arenas) -> int:
        for (r, w) in self.noted:
            g = self.slot[(r, w)]
            for t, n in enumerate(self.numel):
                S = shard_elems(n, self.R)
                lo, hi = r * S, min((r + 1) * S, n)
                if hi <= lo:
                    continue
                views = [a[self.shard_off[t]:self.shard_off[t] + S] for a in acc_arenas]
                accumulate(np.ascontiguousarray(g[self.full_off[t]:self.full_off[t] + n]), views, n,
                           ranges=[(lo, hi)])
        return len(self.noted)

    def end_drain(self) -> None:
        for (r, w) in self.noted:
            del self.slot[(r, w)]
            self.state[r][w] = self.EMPTY
        self.noted = []

    def drain(self, acc_arenas) -> int:
        self.begin_drain()
        done = self.add_noted(acc_arenas)
        self.end_drain()
        return done
