"""The unordered mode at the contribution counts of the workload configurations.

Tolerance checked, per element: |x - ref64| <= 1e-6 * sum_c |g_c|, where ref64 is the float64
sum of the widened bf16 contributions built by the oracle (a forward-error form: relative to
|ref64| alone the error of any summation is unbounded under cancellation).  The normwise figure
max|x - ref64| / max|ref64| is printed beside it.  One float atomic per element and contribution
is a sequential binary32 sum in arrival order, whose worst case over ALL inputs is
(C - 1) * 2^-24 * sum|g|, above 1e-6 for C > 17; what is asserted here is the error on the
configurations' own data (Normal gradients), where it stays far below the tolerance.  The wide
(binary64) accumulators in the second half of this file hold the tolerance for any inputs, and
`test_wide_keeps_the_tolerance_where_binary32_atomics_cannot` runs an input built to hit the
worst case through both."""
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


def test_concurrent_streams_with_private_accumulators(oracle):
    """The other way to take contributions that arrive concurrently: every stream adds into an
    accumulator set of its own with the ordered kernel (no atomics, full rate) and the sets are
    summed at the minibatch end by the group reduction of Section 6.1.  Whatever the streams'
    interleaving, the result is one fixed sequence of binary32 additions, so it is compared
    with the oracle bit for bit, and with the float64 reference under the bound that follows
    from the counts: (most contributions in one set - 1) + (sets - 1) roundings."""
    wl = inputs.workload("1.5b")
    N, R, K = wl.numel[0], wl.R, 4
    seq = contributions(inputs.microbatch_counts(wl))
    print(f"private accumulators 1.5b: N={N} R={R} C={len(seq)} sets={K}", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    accs = [torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(K * R)]
    accs_h = [[np.full(S, 3.25, dtype=np.float32) for _ in range(R)] for _ in range(K)]
    streams = [torch.cuda.Stream() for _ in range(K)]
    for k in range(K):
        L.reset_accum(accs[k * R:(k + 1) * R])
        oracle.reset(accs_h[k], N, nthreads=THREADS)
    torch.cuda.synchronize()
    pinned = torch.empty(N, dtype=torch.int16, pin_memory=True)
    g_h = pinned.numpy().view(np.uint16)
    tot, mag = np.zeros(N), np.zeros(N)
    pool, per_set = [], [0] * K
    for i, (w, m) in enumerate(seq):
        k = i % K
        g = inputs.device_normal_bf16(N, wl.grad_sigma, 9700 + 64 * w + m, dev)
        torch.cuda.current_stream().synchronize()            # g is complete before another stream reads it
        L.scatter_accumulate(g, accs[k * R:(k + 1) * R], w, m, stream=streams[k])
        per_set[k] += 1
        pinned.copy_(g.view(torch.int16))
        oracle.accumulate(g_h, accs_h[k], N, nthreads=THREADS)
        oracle.fp64_add(g_h, tot, mag, nthreads=THREADS)
        pool.append(g)                                       # keep alive until the streams are done
        if len(pool) > 6:
            torch.cuda.synchronize()
            pool.clear()
    torch.cuda.synchronize()
    out = [torch.full((S,), -1.0, dtype=torch.float32, device=dev) for _ in range(R)]
    out_h = [np.full(S, -1.0, dtype=np.float32) for _ in range(R)]
    L.reduce_groups(K, accs, out)
    oracle.reduce_groups(accs_h, out_h, N, nthreads=THREADS)
    torch.cuda.synchronize()
    for r in range(R):
        assert np.array_equal(out[r].cpu().numpy().view(np.uint32), out_h[r].view(np.uint32)), f"reduced shard of owner {r}"
    worst = check_against_fp64(out, tot, mag, N, S, f"private accumulators 1.5b C={len(seq)} sets={K}")
    roundings = max(per_set) - 1 + K - 1
    assert roundings * 2.0 ** -24 < TOL and worst <= roundings * 2.0 ** -24 * (1 + 1e-6)
    L.close()


# ----------------------------------------------------------------------------- wide accumulators
def wide_case(oracle, numel, R, C, seed, streams=3):
    """reset, C contributions in scrambled order on several streams, both retrievals; the binary64
    sums of these inputs are exact (no rounding at this magnitude), so every order gives the same
    bits and the GPU must equal the oracle bit for bit, accumulators and outputs."""
    print(f"wide case R={R} T={len(numel)} total={sum(numel)} C={C}", flush=True)
    L = odc.Layout(R, numel)
    T = len(numel)
    so = [L.shard_offset(t) for t in range(T)]
    fo = [L.full_offset(t) for t in range(T)]
    arena, full_n = L.rank_arena_elems(), L.full_elems()
    dev = torch.device("cuda")
    PAD = -9876.5
    acc = [torch.full((arena,), PAD, dtype=torch.float64, device=dev) for _ in range(R)]
    acc_h = [np.full(arena, PAD, dtype=np.float64) for _ in range(R)]
    L.reset_accum_wide(acc)
    gs = [inputs.normal_bf16(full_n, 1e-2, seed=(seed, k)) for k in range(C)]
    dev_g = [torch.from_numpy(g.view(np.int16)).cuda() for g in gs]
    torch.cuda.synchronize()
    ss = [torch.cuda.Stream() for _ in range(streams)]
    order = list(range(C))
    np.random.default_rng(seed).shuffle(order)
    for i, k in enumerate(order):
        L.scatter_accumulate_wide(dev_g[k], acc, stream=ss[i % streams])
    torch.cuda.synchronize()
    out32 = [torch.full((arena,), 77.0, dtype=torch.float32, device=dev) for _ in range(R)]
    out16 = [torch.full((arena,), 0x1234, dtype=torch.int16, device=dev) for _ in range(R)]
    scale = 1.0 / C
    L.retrieve_grads_wide(acc, out32, scale, odc.ODC_OUT_F32)
    L.retrieve_grads_wide(acc, out16, scale, odc.ODC_OUT_BF16)
    torch.cuda.synchronize()
    o32_h = [np.full(arena, 77.0, dtype=np.float32) for _ in range(R)]
    o16_h = [np.full(arena, 0x1234, dtype=np.uint16) for _ in range(R)]
    for t, n in enumerate(numel):
        va = oracle.wide_views(acc_h, numel, so, t, R)
        oracle.reset_wide(va, n)
        for g in gs:
            oracle.accumulate_wide(np.ascontiguousarray(g[fo[t]:fo[t] + n]), va, n)
        oracle.retrieve_wide(va, oracle.wide_views(o32_h, numel, so, t, R), n, scale=scale)
        oracle.retrieve_wide(va, oracle.wide_views(o16_h, numel, so, t, R), n, scale=scale)
    for r in range(R):
        assert np.array_equal(acc[r].cpu().numpy().view(np.uint64), acc_h[r].view(np.uint64)), f"wide accumulator of owner {r}"
        assert np.array_equal(out32[r].cpu().numpy().view(np.uint32), o32_h[r].view(np.uint32)), f"binary32 retrieval, owner {r}"
        assert np.array_equal(out16[r].cpu().numpy().view(np.uint16), o16_h[r]), f"bf16 retrieval, owner {r}"
    L.close()


@pytest.mark.parametrize("numel,R,C", [([1_048_589], 4, 9), ([1], 64, 3), ([3_000_001], 16, 20), ([350], 70, 4),
                                       ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8, 7),
                                       ([30000, 17, 2048, 2049, 1_000_001], 5, 12), ([5] * 70 + [100_000], 70, 5)])
def test_wide_accumulators_equal_the_oracle_in_any_order(oracle, numel, R, C):
    wide_case(oracle, numel, R, C, seed=sum(numel) % 991 + C)


def test_wide_accumulators_on_the_stress_config(oracle):
    wl = inputs.workload("stress")
    wide_case(oracle, list(wl.numel), wl.R, 6, seed=17)


def test_wide_keeps_the_tolerance_where_binary32_atomics_cannot(oracle):
    """An input built to hit the worst case of a binary32 running sum: 1.0 first, then 271
    contributions of 2^-17 + 2^-24 (exact in bf16), all on one stream so that they arrive in that
    order.  Every binary32 addition is a tie that rounds the 2^-24 away: the plain unordered mode
    ends 1.6e-5 * sum|g| off, 16 times the tolerance, while the wide accumulators stay within
    2^-24 * sum|g| after their single rounding at retrieval."""
    N, R, C = 1_000_003, 8, 272
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    big = torch.full((N,), 1.0, dtype=torch.bfloat16, device=dev)
    small = torch.full((N,), 2.0 ** -17 + 2.0 ** -24, dtype=torch.bfloat16, device=dev)
    assert float(small[0]) == 2.0 ** -17 + 2.0 ** -24
    exact = 1.0 + (C - 1) * (2.0 ** -17 + 2.0 ** -24)            # exact in binary64; all terms positive
    acc32 = [torch.zeros(S, dtype=torch.float32, device=dev) for _ in range(R)]
    acc64 = [torch.zeros(S, dtype=torch.float64, device=dev) for _ in range(R)]
    L.reset_accum(acc32)
    L.reset_accum_wide(acc64)
    for k in range(C):
        g = big if k == 0 else small
        L.scatter_accumulate(g, acc32, 0, 0, odc.ODC_UNORDERED)
        L.scatter_accumulate_wide(g, acc64)
    out = [torch.zeros(S, dtype=torch.float32, device=dev) for _ in range(R)]
    L.retrieve_grads_wide(acc64, out, 1.0, odc.ODC_OUT_F32)
    torch.cuda.synchronize()
    worst32 = worst64 = 0.0
    for r in range(R):
        v = L.valid_elems(0, r)
        worst32 = max(worst32, float((acc32[r][:v].double() - exact).abs().max()) / exact)
        worst64 = max(worst64, float((out[r][:v].double() - exact).abs().max()) / exact)
        assert bool((acc64[r][:v] == exact).all())
    print(f"adversarial C={C}: binary32 atomics |err|/sum|g| = {worst32:.3e}; wide accumulators {worst64:.3e}", flush=True)
    assert worst32 > 10 * TOL            # the sequence does what it was built for
    assert worst64 <= 2.0 ** -24
    L.close()


def test_wide_at_the_7b_contribution_count(oracle):
    """The 7B-shaped layer with all 37 contributions through the wide accumulators on three streams,
    retrieved to binary32 and checked against the float64 reference at every element."""
    wl = inputs.workload("7b")
    N, R = wl.numel[0], wl.R
    seq = contributions(inputs.microbatch_counts(wl))
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    acc = [torch.empty(S, dtype=torch.float64, device=dev) for _ in range(R)]
    L.reset_accum_wide(acc)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(3)]
    pinned = torch.empty(N, dtype=torch.int16, pin_memory=True)
    g_h = pinned.numpy().view(np.uint16)
    tot, mag = np.zeros(N), np.zeros(N)
    pool = []
    for k, (w, m) in enumerate(seq):
        g = inputs.device_normal_bf16(N, wl.grad_sigma, 9900 + 64 * w + m, dev)
        torch.cuda.current_stream().synchronize()
        L.scatter_accumulate_wide(g, acc, stream=streams[k % 3])
        pinned.copy_(g.view(torch.int16))
        oracle.fp64_add(g_h, tot, mag, nthreads=THREADS)
        pool.append(g)
        if len(pool) > 6:
            torch.cuda.synchronize()
            pool.clear()
    torch.cuda.synchronize()
    out = [torch.zeros(S, dtype=torch.float32, device=dev) for _ in range(R)]
    L.retrieve_grads_wide(acc, out, 1.0, odc.ODC_OUT_F32)
    torch.cuda.synchronize()
    worst = check_against_fp64(out, tot, mag, N, S, f"wide 7b C={len(seq)}")
    assert worst <= 2.0 ** -24 * 1.01
    L.close()


def test_wide_argument_errors():
    L = odc.Layout(4, [1000])
    S = L.shard_elems(0)
    acc = [torch.zeros(S, dtype=torch.float64, device="cuda") for _ in range(4)]
    out = [torch.zeros(S, dtype=torch.float32, device="cuda") for _ in range(4)]
    g = torch.zeros(1000, dtype=torch.bfloat16, device="cuda")
    lib = odc.lib()
    import ctypes
    arr = lambda ts: (ctypes.c_void_p * 4)(*[t.data_ptr() for t in ts])
    assert lib.odc_scatter_accumulate_wide(L.handle, None, arr(acc), None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_scatter_accumulate_wide(L.handle, g.data_ptr(), None, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_scatter_accumulate_wide(L.handle, g.data_ptr() + 2, arr(acc), None) == odc.ODC_ERR_ALIGNMENT
    assert lib.odc_retrieve_grads_wide(L.handle, arr(acc), arr(out), ctypes.c_float(1.0), 9, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_retrieve_grads_wide(L.handle, arr(acc), None, ctypes.c_float(1.0), 0, None) == odc.ODC_ERR_INVALID_ARG
    bad = [acc[0], acc[1][1:], acc[2], acc[3]]
    assert lib.odc_reset_accum_wide(L.handle, arr(bad), None) == odc.ODC_ERR_ALIGNMENT
    assert lib.odc_reset_accum_wide(L.handle, arr(acc), None) == 0
    torch.cuda.synchronize()
    L.close()
