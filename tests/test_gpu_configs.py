"""GPU parity of every workload configuration at its OWN contribution sequence: the per-rank
microbatch counts M_w of the configuration (imbalanced, Section 4), every (worker, microbatch)
contribution with a gradient of its own, applied in worker-then-microbatch order through the
C ABI with the default launch knobs, and every accumulator element compared bit for bit with
the CPU oracle (the 32B-shaped configuration on sampled flat-index windows, because its
accumulators do not fit a host pass per contribution in reasonable time).

Inputs are drawn on the device with a seeded generator and copied to the host through a
pinned buffer, so both sides consume the same bits.
"""
import os

import numpy as np
import pytest
import torch

from paper_2601_19362_amd import binding as odc
from paper_2601_19362_amd import inputs

from gpu_util import assert_bits_equal

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


def contributions(M):
    return [(w, m) for w in range(len(M)) for m in range(M[w])]


class HostMirror:
    """A pinned host buffer of n 16-bit words that device tensors are copied into."""

    def __init__(self, n):
        self.t = torch.empty(n, dtype=torch.int16, pin_memory=True)
        self.np = self.t.numpy().view(np.uint16)

    def load(self, dev_tensor):
        self.t[:dev_tensor.numel()].copy_(dev_tensor.view(torch.int16))
        return self.np[:dev_tensor.numel()]


def grad_seed(seed, layer, w, m):
    return ((seed * 131 + layer) * 4099 + w) * 257 + m


def layer_full_sequence(oracle, name, check_gather=True):
    """One layer of workload `name`: gather, reset, all C contributions; everything compared."""
    wl = inputs.workload(name)
    N, R = wl.numel[0], wl.R
    M = inputs.microbatch_counts(wl)
    seq = contributions(M)
    print(f"config {name}: N={N} R={R} M={M} C={len(seq)}", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    mirror = HostMirror(N)

    if check_gather:
        flat = inputs.device_uniform_bf16(N, wl.param_range[0], wl.param_range[1], wl.seed, dev)
        shards = []
        for r in range(R):
            sh = torch.full((S,), -1.0, dtype=torch.bfloat16, device=dev)
            v = L.valid_elems(0, r)
            if v:
                sh[:v] = flat[r * S:r * S + v]
            shards.append(sh)
        full = torch.full((N,), 7.0, dtype=torch.bfloat16, device=dev)
        L.gather(shards, full)
        torch.cuda.synchronize()
        flat_h = mirror.load(flat).copy()
        shards_h = [s.view(torch.int16).cpu().numpy().view(np.uint16) for s in shards]
        want = np.empty(N, dtype=np.uint16)
        oracle.gather(shards_h, N, want, nthreads=THREADS)
        assert_bits_equal(mirror.load(full), want, "gather")
        assert np.array_equal(want, flat_h)
        del flat, shards, full, flat_h, shards_h, want

    acc = [torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    acc_h = [np.full(S, 3.25, dtype=np.float32) for _ in range(R)]
    L.reset_accum(acc)
    oracle.reset(acc_h, N, nthreads=THREADS)
    for k, (w, m) in enumerate(seq):
        g = inputs.device_normal_bf16(N, wl.grad_sigma, grad_seed(wl.seed, 0, w, m), dev)
        L.scatter_accumulate(g, acc, w, m)
        oracle.accumulate(mirror.load(g), acc_h, N, nthreads=THREADS)
        del g
        if k % 8 == 7:
            print(f"  {k + 1}/{len(seq)} contributions", flush=True)
    torch.cuda.synchronize()
    for r in range(R):
        assert_bits_equal(acc[r].cpu().numpy(), acc_h[r], f"{name}: accumulator of owner {r} after {len(seq)} contributions")
    L.close()


def test_config_1p5b_full_contribution_sequence(oracle):
    layer_full_sequence(oracle, "1.5b")


def test_config_7b_full_contribution_sequence(oracle):
    """The configuration the throughput target is stated on: 37 contributions with the
    long-tailed per-rank microbatch counts."""
    layer_full_sequence(oracle, "7b")


def test_config_stress_full_contribution_sequence(oracle):
    """10,000 tensors, R = 64: gather, reset and every contribution of the configuration through
    the batched kernels, one launch per call; all arenas compared in full."""
    wl = inputs.workload("stress")
    numel, R = list(wl.numel), wl.R
    M = inputs.microbatch_counts(wl)
    seq = contributions(M)
    print(f"config stress: T={len(numel)} R={R} total={sum(numel)} C={len(seq)}", flush=True)
    L = odc.Layout(R, numel)
    T = len(numel)
    so = [L.shard_offset(t) for t in range(T)]
    fo = [L.full_offset(t) for t in range(T)]
    arena, full_n = L.rank_arena_elems(), L.full_elems()
    dev = torch.device("cuda")
    mirror = HostMirror(full_n)

    params = [inputs.device_uniform_bf16(arena, wl.param_range[0], wl.param_range[1], 600 + r, dev) for r in range(R)]
    full = torch.full((full_n,), 7.0, dtype=torch.bfloat16, device=dev)
    L.gather(params, full)
    torch.cuda.synchronize()
    arenas_h = [p.view(torch.int16).cpu().numpy().view(np.uint16) for p in params]
    want = np.full(full_n, 0x40E0, dtype=np.uint16)            # bf16(7.0) where nothing is written
    oracle.gather_batched(arenas_h, numel, so, fo, want)
    assert_bits_equal(mirror.load(full), want, "gather")
    del params, arenas_h, full, want

    acc = [torch.full((arena,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    acc_h = [np.full(arena, 3.25, dtype=np.float32) for _ in range(R)]
    L.reset_accum(acc)
    oracle.reset_batched(acc_h, numel, so)
    for k, (w, m) in enumerate(seq):
        g = inputs.device_normal_bf16(full_n, wl.grad_sigma, grad_seed(wl.seed, 0, w, m), dev)
        L.scatter_accumulate(g, acc, w, m)
        oracle.accumulate_batched(mirror.load(g), acc_h, numel, so, fo)
        if k % 16 == 15:
            print(f"  {k + 1}/{len(seq)} contributions", flush=True)
    torch.cuda.synchronize()
    for r in range(R):
        assert_bits_equal(acc[r].cpu().numpy(), acc_h[r], f"stress: arena of owner {r} after {len(seq)} contributions")
    L.close()


def sample_windows(N, R, S, win, extra, seed):
    """Flat-index windows: both ends of the tensor, every shard boundary, `extra` inside shards."""
    ranges = [(0, win), (N - win, N)]
    for r in range(1, R):
        ranges.append((r * S - win // 2, r * S + win // 2))
    rng = np.random.default_rng(seed)
    for r in rng.integers(0, R, size=extra):
        a = int(r) * S + int(rng.integers(2 * win, S - 3 * win))
        if all(b <= a or a + win <= x for x, b in ranges):
            ranges.append((a, a + win))
    return sorted(ranges)


def test_config_32b_window_full_contribution_sequence(oracle):
    """The 32B-shaped configuration: 4 resident buffer sets, layer l in set l mod 4, each layer
    with the configuration's own per-rank microbatch counts (a few hundred contributions).  Five
    layers, so that one set is reused.  Compared with the oracle on sampled windows (tensor ends,
    every shard boundary, windows inside shards): only those elements are copied to the host."""
    wl = inputs.workload("32b")
    N, R = wl.numel[0], wl.R
    M = inputs.microbatch_counts(wl)
    seq = contributions(M)
    print(f"config 32b: N={N} R={R} M={M} C={len(seq)}", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    nset = wl.resident_layers
    sets = [([torch.empty(S, dtype=torch.bfloat16, device=dev) for _ in range(R)],
             [torch.empty(S, dtype=torch.float32, device=dev) for _ in range(R)]) for _ in range(nset)]
    full = torch.empty(N, dtype=torch.bfloat16, device=dev)
    ranges = sample_windows(N, R, S, 2048, 24, seed=7)
    idx = torch.cat([torch.arange(a, b, device=dev) for a, b in ranges])
    idx_h = idx.cpu().numpy()
    g_h = np.zeros(N, dtype=np.uint16)          # only the sampled positions are ever filled or read
    for layer in range(nset + 1):
        params, acc = sets[layer % nset]
        flat = inputs.device_uniform_bf16(N, wl.param_range[0], wl.param_range[1], 100 + layer, dev)
        for r in range(R):
            params[r].copy_(flat[r * S:(r + 1) * S])
        L.gather(params, full)
        L.reset_accum(acc)
        acc_h = [np.full(S, 123.0, dtype=np.float32) for _ in range(R)]
        oracle.reset(acc_h, N, ranges=ranges)
        for k, (w, m) in enumerate(seq):
            g = inputs.device_normal_bf16(N, wl.grad_sigma, grad_seed(wl.seed, layer, w, m), dev)
            L.scatter_accumulate(g, acc, w, m)
            g_h[idx_h] = g[idx].view(torch.int16).cpu().numpy().view(np.uint16)
            oracle.accumulate(g_h, acc_h, N, ranges=ranges)
            del g
        torch.cuda.synchronize()
        print(f"  layer {layer} (buffer set {layer % nset}): {len(seq)} contributions issued", flush=True)
        got_full = full[idx].view(torch.int16).cpu().numpy().view(np.uint16)
        want_flat = flat[idx].view(torch.int16).cpu().numpy().view(np.uint16)
        assert_bits_equal(got_full, want_flat, f"layer {layer} gather (sampled)")
        for a, b in ranges:
            for r in range(R):
                lo, hi = max(a, r * S), min(b, (r + 1) * S)
                if hi > lo:
                    assert_bits_equal(acc[r][lo - r * S:hi - r * S].cpu().numpy(), acc_h[r][lo - r * S:hi - r * S],
                                      f"layer {layer} accumulator of owner {r} [{lo},{hi})")
        del flat
    L.close()


def test_two_layer_interleaved_step(oracle):
    """Two layers with a buffer set each, calls issued in the interleaved order of a training
    step: reset both; then per (worker, microbatch) gather layer 0, gather layer 1 (forward), and
    backwards gather + contribution for layer 1, then for layer 0.  The 1.5B-shaped layer with its
    own microbatch counts.  The gathered buffer is checked after chosen gathers, both accumulator
    sets in full at the end."""
    wl = inputs.workload("1.5b")
    N, R = wl.numel[0], wl.R
    M = inputs.microbatch_counts(wl)
    seq = contributions(M)
    print(f"interleaved step: N={N} R={R} M={M} C={len(seq)} x 2 layers", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    mirror = HostMirror(N)
    layers = 2
    flats = [inputs.device_uniform_bf16(N, wl.param_range[0], wl.param_range[1], 40 + l, dev) for l in range(layers)]
    params = [[flats[l][r * S:(r + 1) * S].clone() for r in range(R)] for l in range(layers)]
    accs = [[torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)] for _ in range(layers)]
    accs_h = [[np.full(S, 3.25, dtype=np.float32) for _ in range(R)] for _ in range(layers)]
    full = torch.zeros(N, dtype=torch.bfloat16, device=dev)
    for l in range(layers):
        L.reset_accum(accs[l])
        oracle.reset(accs_h[l], N, nthreads=THREADS)
    for k, (w, m) in enumerate(seq):
        for l in range(layers):
            L.gather(params[l], full)
        if k % 12 == 0:      # the forward pass ends with the last layer in the buffer
            assert torch.equal(full, flats[layers - 1])
        for l in reversed(range(layers)):
            L.gather(params[l], full)
            g = inputs.device_normal_bf16(N, wl.grad_sigma, grad_seed(wl.seed, l, w, m), dev)
            L.scatter_accumulate(g, accs[l], w, m)
            oracle.accumulate(mirror.load(g), accs_h[l], N, nthreads=THREADS)
            del g
        if k % 12 == 0:
            assert torch.equal(full, flats[0])
    torch.cuda.synchronize()
    for l in range(layers):
        for r in range(R):
            assert_bits_equal(accs[l][r].cpu().numpy(), accs_h[l][r], f"layer {l} accumulator of owner {r}")
    L.close()
