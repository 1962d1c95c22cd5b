"""The unordered mode at the contribution counts of the workload configurations.

Tolerance checked, per element: |x - ref64| <= 1e-6 * sum_c |g_c|, where ref64 is the float64
sum of the widened bf16 contributions built by the oracle (a forward-error form: relative to
|ref64| alone the error of any summation is unbounded under cancellation).  The normwise figure
max|x - ref64| / max|ref64| is printed beside it.  One float atomic per element and contribution
is a sequential binary32 sum in arrival order, whose worst case over ALL inputs is
(C - 1) * 2^-24 * sum|g|, above 1e-6 for C > 17; what is asserted here is the error on the
configurations' own data (Normal gradients), where it stays far below the tolerance, and
`test_compensated_*` covers inputs built to hit the worst case."""
import os

import numpy as np
import pytest
import torch

from paper_2601_19362_amd import binding as odc
from paper_2601_19362_amd import inputs

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)
TOL = 1e-6


def contributions(M):
    return [(w, m) for w in range(len(M)) for m in range(M[w])]


def check_against_fp64(acc, tot, mag, N, S, what, ranges=None):
    """acc: R device accumulator shards; tot/mag: float64 reference over the flat index space."""
    worst, err_max, ref_max = 0.0, 0.0, 0.0
    for r, a in enumerate(acc):
        lo, hi = r * S, min((r + 1) * S, N)
        if hi <= lo:
            continue
        spans = [(lo, hi)] if ranges is None else [(max(a0, lo), min(b0, hi)) for a0, b0 in ranges if min(b0, hi) > max(a0, lo)]
        for a0, b0 in spans:
            x = a[a0 - lo:b0 - lo].cpu().numpy().astype(np.float64)
            err = np.abs(x - tot[a0:b0])
            assert (err <= TOL * mag[a0:b0]).all(), f"{what}: owner {r}: error above 1e-6 * sum|g|"
            worst = max(worst, float((err / np.maximum(mag[a0:b0], 1e-300)).max()))
            err_max = max(err_max, float(err.max()))
            ref_max = max(ref_max, float(np.abs(tot[a0:b0]).max()))
    print(f"{what}: worst |err| / sum|g| = {worst:.3e} (tolerance {TOL:.0e}); normwise max|err| / max|ref| = "
          f"{err_max / ref_max:.3e}", flush=True)
    return worst


@pytest.mark.parametrize("name", ["1.5b", "7b"])
def test_unordered_at_config_contribution_count(oracle, name):
    """All contributions of the configuration (7B: C = 37), unordered, in a scrambled order on
    three streams; every element checked against the float64 reference."""
    wl = inputs.workload(name)
    N, R = wl.numel[0], wl.R
    seq = contributions(inputs.microbatch_counts(wl))
    np.random.default_rng(3).shuffle(seq)
    print(f"unordered {name}: N={N} R={R} C={len(seq)}", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    acc = [torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    L.reset_accum(acc)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(3)]
    pinned = torch.empty(N, dtype=torch.int16, pin_memory=True)
    g_h = pinned.numpy().view(np.uint16)
    tot, mag = np.zeros(N), np.zeros(N)
    pool = []
    for k, (w, m) in enumerate(seq):
        g = inputs.device_normal_bf16(N, wl.grad_sigma, 9000 + 64 * w + m, dev)
        torch.cuda.current_stream().synchronize()            # g is complete before another stream reads it
        L.scatter_accumulate(g, acc, w, m, odc.ODC_UNORDERED, stream=streams[k % 3])
        pinned.copy_(g.view(torch.int16))
        oracle.fp64_add(g_h, tot, mag, nthreads=THREADS)
        pool.append(g)                                       # keep alive until the streams are done
        if len(pool) > 6:
            torch.cuda.synchronize()
            pool.clear()
    torch.cuda.synchronize()
    check_against_fp64(acc, tot, mag, N, S, f"unordered {name} C={len(seq)}")
    L.close()


def test_unordered_at_32b_contribution_count(oracle):
    """The 32B-shaped layer with all its contributions (C in the hundreds); the float64 reference
    is built on sampled windows: tensor ends, every shard boundary, windows inside shards."""
    wl = inputs.workload("32b")
    N, R = wl.numel[0], wl.R
    seq = contributions(inputs.microbatch_counts(wl))
    np.random.default_rng(4).shuffle(seq)
    print(f"unordered 32b: N={N} R={R} C={len(seq)}", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    acc = [torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    L.reset_accum(acc)
    win = 4096
    ranges = [(0, win), (N - win, N)] + [(r * S - win // 2, r * S + win // 2) for r in range(1, R)]
    rng = np.random.default_rng(8)
    for r in rng.integers(0, R, size=32):
        a = int(r) * S + int(rng.integers(2 * win, S - 3 * win))
        if all(b <= a or a + win <= x for x, b in ranges):
            ranges.append((a, a + win))
    ranges.sort()
    idx = torch.cat([torch.arange(a, b, device=dev) for a, b in ranges])
    idx_h = idx.cpu().numpy()
    g_h = np.zeros(N, dtype=np.uint16)
    tot, mag = np.zeros(N), np.zeros(N)
    for k, (w, m) in enumerate(seq):
        g = inputs.device_normal_bf16(N, wl.grad_sigma, 9500 + 64 * w + m, dev)
        L.scatter_accumulate(g, acc, w, m, odc.ODC_UNORDERED)
        g_h[idx_h] = g[idx].view(torch.int16).cpu().numpy().view(np.uint16)
        oracle.fp64_add(g_h, tot, mag, ranges=ranges)
        del g
    torch.cuda.synchronize()
    check_against_fp64(acc, tot, mag, N, S, f"unordered 32b C={len(seq)} (sampled)", ranges=ranges)
    L.close()


def test_unordered_at_stress_contribution_count(oracle):
    """10,000 tensors, R = 64, all contributions of the configuration through the batched
    unordered kernel; every valid element checked (the reference lives in the full-buffer index
    space, tensor by tensor)."""
    wl = inputs.workload("stress")
    numel, R = list(wl.numel), wl.R
    seq = contributions(inputs.microbatch_counts(wl))
    np.random.default_rng(5).shuffle(seq)
    print(f"unordered stress: T={len(numel)} R={R} C={len(seq)}", flush=True)
    L = odc.Layout(R, numel)
    T = len(numel)
    so = [L.shard_offset(t) for t in range(T)]
    fo = [L.full_offset(t) for t in range(T)]
    arena, full_n = L.rank_arena_elems(), L.full_elems()
    dev = torch.device("cuda")
    acc = [torch.full((arena,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    L.reset_accum(acc)
    pinned = torch.empty(full_n, dtype=torch.int16, pin_memory=True)
    g_h = pinned.numpy().view(np.uint16)
    tot, mag = np.zeros(full_n), np.zeros(full_n)
    for k, (w, m) in enumerate(seq):
        g = inputs.device_normal_bf16(full_n, wl.grad_sigma, 9800 + 8 * w + m, dev)
        L.scatter_accumulate(g, acc, w, m, odc.ODC_UNORDERED)
        pinned.copy_(g.view(torch.int16))
        oracle.fp64_add(g_h, tot, mag, nthreads=THREADS)
    torch.cuda.synchronize()
    acc_h = [a.cpu().numpy() for a in acc]
    worst, err_max, ref_max = 0.0, 0.0, 0.0
    for t, n in enumerate(numel):
        S = -(-n // R)
        got = np.concatenate([a[so[t]:so[t] + S] for a in acc_h])[:n].astype(np.float64)
        err = np.abs(got - tot[fo[t]:fo[t] + n])
        m_t = mag[fo[t]:fo[t] + n]
        assert (err <= TOL * m_t).all(), f"tensor {t}: error above 1e-6 * sum|g|"
        worst = max(worst, float((err / np.maximum(m_t, 1e-300)).max()))
        err_max, ref_max = max(err_max, float(err.max())), max(ref_max, float(np.abs(tot[fo[t]:fo[t] + n]).max()))
    print(f"unordered stress C={len(seq)}: worst |err| / sum|g| = {worst:.3e} (tolerance {TOL:.0e}); normwise "
          f"{err_max / ref_max:.3e}", flush=True)
    L.close()
