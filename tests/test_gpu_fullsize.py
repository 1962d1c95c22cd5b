"""GPU parity at the full layer shapes of the model-shaped workloads, in the launch
configuration the benchmark times (default knobs, one call per primitive).  Inputs are drawn
on the device with a seeded generator and copied to the host, so both sides consume the same
bits; the oracle runs element-range-parallel on the host cores (same per-element sequence)."""
import os

import numpy as np
import pytest
import torch

from paper_2601_19362_amd import binding as odc
from paper_2601_19362_amd import inputs

from gpu_util import assert_bits_equal

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


def full_layer_case(oracle, N, R, contribs, seed, prange=(-0.05, 0.05), sigma=1e-3):
    print(f"full-size case N={N} R={R} C={len(contribs)} seed={seed}", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    assert L.rank_arena_elems() == S and L.full_elems() == N
    dev = torch.device("cuda")
    # owner shards: S slots each; the valid ones hold the flat parameter, padding a sentinel
    flat = inputs.device_uniform_bf16(N, prange[0], prange[1], seed, dev)
    shards = []
    for r in range(R):
        sh = torch.full((S,), -1.0, dtype=torch.bfloat16, device=dev)
        valid = L.valid_elems(0, r)
        if valid:
            sh[:valid] = flat[r * S:r * S + valid]
        shards.append(sh)
    full = torch.full((N + 64,), 7.0, dtype=torch.bfloat16, device=dev)
    L.gather(shards, full)
    torch.cuda.synchronize()
    flat_h = flat.view(torch.int16).cpu().numpy().view(np.uint16)
    shards_h = [s.view(torch.int16).cpu().numpy().view(np.uint16) for s in shards]
    want = np.empty(N, dtype=np.uint16)
    oracle.gather(shards_h, N, want, nthreads=THREADS)
    got = full.view(torch.int16).cpu().numpy().view(np.uint16)
    assert_bits_equal(got[:N], want, "gather")
    assert np.array_equal(want, flat_h)                       # round trip
    assert (got[N:] == 0x40E0).all()                          # bf16(7.0): tail untouched
    del full, flat, shards

    acc = [torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    acc_h = [np.full(S, 3.25, dtype=np.float32) for _ in range(R)]
    L.reset_accum(acc)
    oracle.reset(acc_h, N, nthreads=THREADS)
    for k, (w, m) in enumerate(contribs):
        g = inputs.device_normal_bf16(N, sigma, seed * 1000 + k, dev)
        L.scatter_accumulate(g, acc, w, m)
        g_h = g.view(torch.int16).cpu().numpy().view(np.uint16)
        oracle.accumulate(g_h, acc_h, N, nthreads=THREADS)
    torch.cuda.synchronize()
    for r in range(R):
        assert_bits_equal(acc[r].cpu().numpy(), acc_h[r], f"accumulate rank {r}")
    L.close()


def test_7b_layer_weighted_and_retrieve(oracle):
    """Weighted contributions and both retrieval forms at the 7B layer shape."""
    w = inputs.workload("7b")
    N, R = w.numel[0], w.R
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    acc = [torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    acc_h = [np.full(S, 3.25, dtype=np.float32) for _ in range(R)]
    L.reset_accum(acc)
    oracle.reset(acc_h, N, nthreads=THREADS)
    for k, wt in enumerate((0.37, 1.0 / 3.0)):
        g = inputs.device_normal_bf16(N, 1e-3, 900 + k, dev)
        L.scatter_accumulate_weighted(g, acc, 2, k, wt)
        oracle.accumulate_weighted(g.view(torch.int16).cpu().numpy().view(np.uint16), acc_h, N, wt, nthreads=THREADS)
    for r in range(R):
        assert_bits_equal(acc[r].cpu().numpy(), acc_h[r], f"weighted accumulate rank {r}")
    scale = 1.0 / 4096.0 * 3.0
    out32 = [torch.zeros(S, dtype=torch.float32, device=dev) for _ in range(R)]
    out16 = [torch.zeros(S, dtype=torch.int16, device=dev) for _ in range(R)]
    L.retrieve_grads(acc, out32, scale, odc.ODC_OUT_F32)
    L.retrieve_grads(acc, out16, scale, odc.ODC_OUT_BF16)
    w32 = [np.zeros(S, dtype=np.float32) for _ in range(R)]
    w16 = [np.zeros(S, dtype=np.uint16) for _ in range(R)]
    oracle.retrieve(acc_h, w32, N, scale=scale, nthreads=THREADS)
    oracle.retrieve(acc_h, w16, N, scale=scale, nthreads=THREADS)
    for r in range(R):
        assert_bits_equal(out32[r].cpu().numpy(), w32[r], f"retrieve f32 rank {r}")
        assert_bits_equal(out16[r].cpu().numpy().view(np.uint16), w16[r], f"retrieve bf16 rank {r}")
    L.close()


def test_1p5b_layer(oracle):
    w = inputs.workload("1.5b")
    full_layer_case(oracle, w.numel[0], w.R, [(0, 0), (0, 1), (3, 0), (7, 2)], seed=w.seed)


@pytest.mark.parametrize("delta", [1, -5])
def test_1p5b_layer_off_size(oracle, delta):
    """Same shape with N not divisible by R: padding and misaligned boundaries at scale."""
    w = inputs.workload("1.5b")
    full_layer_case(oracle, w.numel[0] + delta, w.R, [(1, 0), (2, 0)], seed=20 + delta)


def test_7b_layer(oracle):
    w = inputs.workload("7b")
    full_layer_case(oracle, w.numel[0], w.R, [(0, 0), (0, 1), (15, 0)], seed=w.seed)


def test_32b_layer(oracle):
    w = inputs.workload("32b")
    full_layer_case(oracle, w.numel[0], w.R, [(0, 0), (31, 3)], seed=w.seed)


def test_32b_rotating_window(oracle):
    """The 32B-shaped workload keeps only 4 layers' buffers resident and reuses buffer set
    l mod 4 for layer l.  Eight layers go through the four sets (each set is reused once, so
    stale contents from its previous layer would show); every layer is gathered and receives
    three contributions.  Checked against the oracle on sampled flat-index windows of every
    layer -- the start and end of the tensor, every shard boundary and windows in between --
    which the oracle computes one by one."""
    w = inputs.workload("32b")
    N, R = w.numel[0], w.R
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    nset = w.resident_layers
    sets = [([torch.empty(S, dtype=torch.bfloat16, device=dev) for _ in range(R)],
             [torch.empty(S, dtype=torch.float32, device=dev) for _ in range(R)]) for _ in range(nset)]
    full = torch.empty(N, dtype=torch.bfloat16, device=dev)
    win = 2048
    ranges = [(0, win), (N - win, N)]
    for r in range(1, R):
        ranges.append((r * S - win // 2, r * S + win // 2))
    rng = np.random.default_rng(7)
    for r in rng.integers(0, R, size=16):   # windows strictly inside a shard, away from its edges
        a = int(r) * S + int(rng.integers(2 * win, S - 3 * win))
        if all(b <= a or a + win <= x for x, b in ranges):
            ranges.append((a, a + win))
    contribs = [(0, 0), (5, 1), (31, 0)]
    for layer in range(2 * nset):
        print(f"32b window: layer {layer} -> buffer set {layer % nset}", flush=True)
        params, acc = sets[layer % nset]
        flat = inputs.device_uniform_bf16(N, -0.05, 0.05, 100 + layer, dev)
        for r in range(R):
            params[r].copy_(flat[r * S:(r + 1) * S])
        L.gather(params, full)
        L.reset_accum(acc)
        grads = []
        for k, (wk, m) in enumerate(contribs):
            g = inputs.device_normal_bf16(N, 1e-3, 1000 * layer + k, dev)
            L.scatter_accumulate(g, acc, wk, m)
            grads.append(g)
        torch.cuda.synchronize()
        # host side: only the sampled windows are copied and computed
        flat_h = np.zeros(N, dtype=np.uint16)
        full_h = np.zeros(N, dtype=np.uint16)
        shards_h = [np.zeros(S, dtype=np.uint16) for _ in range(R)]
        acc_h = [np.full(S, 123.0, dtype=np.float32) for _ in range(R)]
        grads_h = [np.zeros(N, dtype=np.uint16) for _ in contribs]
        for a, b in ranges:
            flat_h[a:b] = flat[a:b].view(torch.int16).cpu().numpy().view(np.uint16)
            for gh, g in zip(grads_h, grads):
                gh[a:b] = g[a:b].view(torch.int16).cpu().numpy().view(np.uint16)
            for r in range(R):
                lo, hi = max(a, r * S), min(b, (r + 1) * S)
                if hi > lo:
                    shards_h[r][lo - r * S:hi - r * S] = params[r][lo - r * S:hi - r * S].view(torch.int16).cpu().numpy().view(np.uint16)
        oracle.gather(shards_h, N, full_h, ranges=ranges)
        oracle.reset(acc_h, N, ranges=ranges)
        for gh in grads_h:
            oracle.accumulate(gh, acc_h, N, ranges=ranges)
        for a, b in ranges:
            got = full[a:b].view(torch.int16).cpu().numpy().view(np.uint16)
            assert_bits_equal(got, full_h[a:b], f"layer {layer} gather [{a},{b})")
            assert np.array_equal(got, flat_h[a:b])
            for r in range(R):
                lo, hi = max(a, r * S), min(b, (r + 1) * S)
                if hi > lo:
                    assert_bits_equal(acc[r][lo - r * S:hi - r * S].cpu().numpy(), acc_h[r][lo - r * S:hi - r * S],
                                      f"layer {layer} accumulate rank {r} [{lo},{hi})")
        del flat, grads
    L.close()


def test_multi_tensor_layout_with_a_2p30_element_tensor(oracle):
    """A multi-tensor layout whose first tensor has more than 2^30 elements: the batched gather
    kernel leaves its 32-bit tile-relative arithmetic for such a tensor, and every batched
    kernel has to carry 64-bit offsets.  Gather, reset and two ordered contributions, compared
    in full with the oracle."""
    numel = [(1 << 30) + 5, 1000, 7, 70_001]
    R = 8
    print(f"huge-tensor case numel={numel} R={R}", flush=True)
    L = odc.Layout(R, numel)
    T = len(numel)
    S = [L.shard_elems(t) for t in range(T)]
    so = [L.shard_offset(t) for t in range(T)]
    fo = [L.full_offset(t) for t in range(T)]
    arena, full_n = L.rank_arena_elems(), L.full_elems()
    dev = torch.device("cuda")
    params = [torch.full((arena,), -1.0, dtype=torch.bfloat16, device=dev) for _ in range(R)]
    for t, n in enumerate(numel):
        flat = inputs.device_uniform_bf16(n, -0.05, 0.05, 300 + t, dev)
        for r in range(R):
            v = L.valid_elems(t, r)
            if v:
                params[r][so[t]:so[t] + v] = flat[r * S[t]:r * S[t] + v]
        del flat
    full = torch.full((full_n,), 7.0, dtype=torch.bfloat16, device=dev)
    L.gather(params, full)
    torch.cuda.synchronize()
    arenas_h = [p.view(torch.int16).cpu().numpy().view(np.uint16) for p in params]
    want = np.full(full_n, 0x40E0, dtype=np.uint16)   # bf16(7.0) where nothing is written
    oracle.gather_batched(arenas_h, numel, so, fo, want)
    got = full.view(torch.int16).cpu().numpy().view(np.uint16)
    assert_bits_equal(got, want, "gather")
    del params, arenas_h, full, got, want

    acc = [torch.full((arena,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    acc_h = [np.full(arena, 3.25, dtype=np.float32) for _ in range(R)]
    L.reset_accum(acc)
    oracle.reset_batched(acc_h, numel, so)
    for k in range(2):
        g = inputs.device_normal_bf16(full_n, 1e-3, 400 + k, dev)
        L.scatter_accumulate(g, acc, k, 0)
        oracle.accumulate_batched(g.view(torch.int16).cpu().numpy().view(np.uint16), acc_h, numel, so, fo)
        del g
    torch.cuda.synchronize()
    for r in range(R):
        assert_bits_equal(acc[r].cpu().numpy(), acc_h[r], f"accumulate rank {r}")
    L.close()


def test_7b_layer_staging_and_fused(oracle):
    """Server-side staging and the fused contribution at the 7B layer shape (7.5 GB of staging
    slots): three clients push, the owners drain in client order; two more push and are drained;
    then three contributions go through the fused entry point.  All compared with the oracle's
    single ordered contributions in the same order."""
    w = inputs.workload("7b")
    N, R = w.numel[0], w.R
    print(f"7b staging case N={N} R={R}", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    slot = L.stage_slot_elems()
    bufs = [torch.empty(R * slot, dtype=torch.bfloat16, device=dev) for _ in range(R)]
    flags = torch.full((L.stage_flag_count(),), 5, dtype=torch.int32, device=dev)
    snap = torch.zeros(L.stage_snapshot_count(), dtype=torch.int32, device=dev)
    L.stage_init(flags)
    acc = [torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    acc_h = [np.full(S, 3.25, dtype=np.float32) for _ in range(R)]
    L.reset_accum(acc)
    oracle.reset(acc_h, N, nthreads=THREADS)

    def host(g):
        return g.view(torch.int16).cpu().numpy().view(np.uint16)

    seed = [700]

    def fresh():
        seed[0] += 1
        return inputs.device_normal_bf16(N, 1e-3, seed[0], dev)

    for clients in ([3, 0, 9], [15, 0]):
        staged = {}
        for c in clients:
            g = fresh()
            L.stage_push(g, bufs, flags, c)
            staged[c] = host(g)
            del g
        L.stage_drain(bufs, flags, snap, acc)
        for c in sorted(staged):                      # the drain adds in ascending client order
            oracle.accumulate(staged[c], acc_h, N, nthreads=THREADS)
    torch.cuda.synchronize()
    assert not flags.cpu().numpy().any()
    grads = [fresh() for _ in range(3)]
    L.scatter_accumulate_multi(grads, acc, [1, 1, 2], [0, 1, 0])
    for g in grads:
        oracle.accumulate(host(g), acc_h, N, nthreads=THREADS)
    torch.cuda.synchronize()
    for r in range(R):
        assert_bits_equal(acc[r].cpu().numpy(), acc_h[r], f"staged + fused accumulate rank {r}")
    L.close()


def test_single_tensor_beyond_32_bit_indices(oracle):
    """N = 2^31 + 5 elements, R = 8: flat indices, byte offsets and work-item counts all pass
    2^31 / 2^32; an index computed in 32 bits anywhere in the flat kernels would show here."""
    full_layer_case(oracle, (1 << 31) + 5, 8, [(0, 0), (7, 1)], seed=77)


def test_beyond_32_bit_indices_fused_unordered_and_retrieve(oracle):
    """The same size through the fused entry point (ordered), one unordered contribution and
    both retrievals.  Gradients are small integers, so every sum is exact and the unordered
    result must equal the ordered oracle bit for bit."""
    N, R = (1 << 31) + 5, 8
    print(f"beyond-32-bit fused/retrieve case N={N} R={R}", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    acc = [torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    acc_h = [np.full(S, 3.25, dtype=np.float32) for _ in range(R)]
    L.reset_accum(acc)
    oracle.reset(acc_h, N, nthreads=THREADS)
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    grads = [torch.randint(-200, 201, (N,), generator=gen, device=dev, dtype=torch.int16).to(torch.bfloat16)
             for _ in range(3)]
    L.scatter_accumulate_multi(grads[:2], acc, [0, 0], [0, 1])
    L.scatter_accumulate(grads[2], acc, 0, 0, odc.ODC_UNORDERED)
    for g in grads:
        oracle.accumulate(g.view(torch.int16).cpu().numpy().view(np.uint16), acc_h, N, nthreads=THREADS)
    torch.cuda.synchronize()
    del grads
    for r in range(R):
        assert_bits_equal(acc[r].cpu().numpy(), acc_h[r], f"fused + unordered accumulate rank {r}")
    scale = 1.0 / 3.0
    for bf16 in (False, True):
        out = [torch.zeros(S, dtype=torch.int16 if bf16 else torch.float32, device=dev) for _ in range(R)]
        want = [np.zeros(S, dtype=np.uint16 if bf16 else np.float32) for _ in range(R)]
        L.retrieve_grads(acc, out, scale, odc.ODC_OUT_BF16 if bf16 else odc.ODC_OUT_F32)
        oracle.retrieve(acc_h, want, N, scale=scale, nthreads=THREADS)
        for r in range(R):
            got = out[r].cpu().numpy()
            assert_bits_equal(got.view(np.uint16) if bf16 else got, want[r], f"retrieve bf16={bf16} rank {r}")
        del out
    L.close()


def test_7b_layer_as_nine_tensors(oracle):
    """The 7B decoder layer kept as nine separate tensors (q, k, v, o, gate, up, down and two
    norm vectors) in one multi-tensor layout: the lean uniform-tile paths of the batched kernels
    carry almost all of it.  Gather, reset, two contributions and a retrieval, compared in full."""
    h, ffn, q, kv = 3584, 18944, 28, 4
    numel = [h * q * 128, h * kv * 128, h * kv * 128, h * q * 128, h * ffn, h * ffn, h * ffn, h, h]
    R = 16
    assert sum(numel) == inputs.workload("7b").numel[0]
    print(f"nine-tensor 7b layer R={R}", flush=True)
    L = odc.Layout(R, numel)
    T = len(numel)
    S = [L.shard_elems(t) for t in range(T)]
    so = [L.shard_offset(t) for t in range(T)]
    fo = [L.full_offset(t) for t in range(T)]
    arena, full_n = L.rank_arena_elems(), L.full_elems()
    dev = torch.device("cuda")
    params = [inputs.device_uniform_bf16(arena, -0.05, 0.05, 600 + r, dev) for r in range(R)]
    full = torch.full((full_n,), 7.0, dtype=torch.bfloat16, device=dev)
    L.gather(params, full)
    torch.cuda.synchronize()
    arenas_h = [p.view(torch.int16).cpu().numpy().view(np.uint16) for p in params]
    want = np.full(full_n, 0x40E0, dtype=np.uint16)
    oracle.gather_batched(arenas_h, numel, so, fo, want)
    assert_bits_equal(full.view(torch.int16).cpu().numpy().view(np.uint16), want, "gather")
    del params, arenas_h, full, want

    acc = [torch.full((arena,), 3.25, dtype=torch.float32, device=dev) for _ in range(R)]
    acc_h = [np.full(arena, 3.25, dtype=np.float32) for _ in range(R)]
    L.reset_accum(acc)
    oracle.reset_batched(acc_h, numel, so)
    for k in range(2):
        g = inputs.device_normal_bf16(full_n, 1e-3, 650 + k, dev)
        if k == 0:
            L.scatter_accumulate(g, acc, 3, 0)
            oracle.accumulate_batched(g.view(torch.int16).cpu().numpy().view(np.uint16), acc_h, numel, so, fo)
        else:
            L.scatter_accumulate_weighted(g, acc, 3, 1, 0.37)
            oracle.accumulate_weighted_batched(g.view(torch.int16).cpu().numpy().view(np.uint16), acc_h, numel, so, fo,
                                               0.37)
        del g
    out = [torch.full((arena,), -1.0, dtype=torch.float32, device=dev) for _ in range(R)]
    out_h = [np.full(arena, -1.0, dtype=np.float32) for _ in range(R)]
    L.retrieve_grads(acc, out, 1.0 / 3.0, odc.ODC_OUT_F32)
    oracle.retrieve_batched(acc_h, out_h, numel, so, scale=1.0 / 3.0)
    torch.cuda.synchronize()
    for r in range(R):
        assert_bits_equal(acc[r].cpu().numpy(), acc_h[r], f"accumulate rank {r}")
        assert_bits_equal(out[r].cpu().numpy(), out_h[r], f"retrieve rank {r}")
    L.close()
