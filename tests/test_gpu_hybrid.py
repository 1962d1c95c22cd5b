"""GPU parity of hybrid sharding (Section 6.1, Appendix E): K groups of R owners, every world
worker gathers from and contributes to its own group, and the groups' gradient shards are
summed at the minibatch end.  Compared with the CPU oracle bit for bit (ordered contributions
inside a group, ascending group order across groups)."""
import os

import numpy as np
import pytest
import torch

from paper_2601_19362_amd import binding as odc
from paper_2601_19362_amd import inputs

from gpu_util import PAD32, DeviceCase, Guarded, assert_bits_equal, host_arenas_from_flats, to_dev_u16, to_host_u16

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


def hybrid_case(oracle, numel, R, K, M_world, seed, inplace):
    """A whole minibatch under hybrid sharding on a small layout, everything compared."""
    print(f"hybrid case R={R} K={K} T={len(numel)} total={sum(numel)} M={M_world} inplace={inplace}", flush=True)
    assert len(M_world) == R * K
    case = DeviceCase(R, numel)          # group 0's buffers (guarded); the other groups get plain tensors
    L = case.layout
    flats = [inputs.uniform_bf16(n, -0.05, 0.05, seed=(seed, 1, t)) for t, n in enumerate(numel)]
    arenas = host_arenas_from_flats(oracle, flats, R, case.S, case.shard_off, case.arena)
    case.load_params(arenas)
    params = [[p.t for p in case.params]] + [[to_dev_u16(a) for a in arenas] for _ in range(1, K)]
    accs = [[a.t for a in case.acc]] + [[torch.full((case.arena,), float(PAD32), dtype=torch.float32, device="cuda")
                                         for _ in range(R)] for _ in range(1, K)]
    flat_params = [p for grp in params for p in grp]
    flat_accs = [a for grp in accs for a in grp]
    accs_h = [[np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)] for _ in range(K)]
    for k in range(K):
        L.reset_accum(accs[k])
        oracle.reset_batched(accs_h[k], numel, case.shard_off)

    want_full = np.full(case.full_n, 0xBEEF, dtype=np.uint16)
    oracle.gather_batched(arenas, numel, case.shard_off, case.full_off, want_full)
    for w in (0, R * K - 1, R):                                   # a worker of the first, last and second group
        case.full.t.fill_(-16657)                                 # 0xBEEF
        L.gather_hybrid(K, flat_params, w % (R * K), case.full.t)
        assert_bits_equal(to_host_u16(case.full.t), want_full, f"gather by world worker {w}")

    for w, mw in enumerate(M_world):
        assert L.hybrid_group_of(K, w) == w // R
        for m in range(mw):
            g = inputs.normal_bf16(case.full_n, 1e-3, seed=(seed, 2, w, m))
            case.grad.t.copy_(to_dev_u16(g))
            L.scatter_accumulate_hybrid(K, case.grad.t, flat_accs, w, m)
            oracle.accumulate_batched(g, accs_h[w // R], numel, case.shard_off, case.full_off)
    for k in range(K):
        for r in range(R):
            assert_bits_equal(accs[k][r].cpu().numpy(), accs_h[k][r], f"group {k} accumulator of owner {r}")

    if inplace:
        out, out_h = accs[0], accs_h[0]
    else:
        out_g = [Guarded(case.arena, torch.float32, float(PAD32)) for _ in range(R)]
        out, out_h = [o.t for o in out_g], [np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)]
    L.reduce_groups(K, flat_accs, out)
    oracle.reduce_groups_batched(accs_h, out_h, numel, case.shard_off)
    for r in range(R):
        assert_bits_equal(out[r].cpu().numpy(), out_h[r], f"reduced shard of owner {r}")
    if not inplace:
        for o in out_g:
            o.check()
        for k in range(K):                                        # the groups' own accumulators are untouched
            for r in range(R):
                assert_bits_equal(accs[k][r].cpu().numpy(), accs_h[k][r], f"group {k} accumulator of owner {r} after reduce")
    ret = [torch.full((case.arena,), float(PAD32), dtype=torch.float32, device="cuda") for _ in range(R)]
    ret_h = [np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)]
    scale = 1.0 / sum(M_world)
    L.retrieve_grads(out, ret, scale, odc.ODC_OUT_F32)
    oracle.retrieve_batched(out_h, ret_h, numel, case.shard_off, scale=scale)
    for r in range(R):
        assert_bits_equal(ret[r].cpu().numpy(), ret_h[r], f"retrieved shard of owner {r}")
    case.check_guards()
    case.close()


@pytest.mark.parametrize("numel,R,K,inplace", [
    ([3_000_001], 4, 3, False),
    ([1_048_589], 8, 2, True),
    ([4099], 20, 9, False),                      # two launches of owners, two passes of groups
    ([1], 64, 2, True),
    ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8, 3, True),
    ([30000, 17, 2048, 2049, 1_000_001], 5, 17, False),
    ([5] * 34 + [100_000], 34, 2, False),
])
def test_hybrid_minibatch(oracle, numel, R, K, inplace):
    rng = np.random.default_rng(R * 31 + K)
    M = [int(v) for v in rng.integers(0, 3, size=R * K)]
    M[0] = max(M[0], 1)
    hybrid_case(oracle, numel, R, K, M, seed=R + K, inplace=inplace)


def test_hybrid_equals_full_sharding_on_integer_gradients(oracle):
    """The same 12 workers under full sharding (R = 12) and under hybrid sharding (3 groups of 4),
    both on the GPU, with integer-valued gradients (every sum exact): the gradient at every flat
    index is the same, which is the section's claim that only the placement changes."""
    N, G, K = 2_000_003, 4, 3
    W = G * K
    rng = np.random.default_rng(11)
    grads = [to_dev_u16(inputs.f32_to_bf16_bits(rng.integers(-200, 201, size=N).astype(np.float32))) for _ in range(W)]
    full_case = DeviceCase(W, [N], with_params=False)
    full_case.layout.reset_accum(full_case.acc_ptrs)
    for w in range(W):
        full_case.layout.scatter_accumulate(grads[w], full_case.acc_ptrs, w, 0)
    hyb = DeviceCase(G, [N], with_params=False)
    accs = [a.t for a in hyb.acc] + [torch.zeros(hyb.arena, dtype=torch.float32, device="cuda") for _ in range(G * (K - 1))]
    for k in range(K):
        hyb.layout.reset_accum(accs[k * G:(k + 1) * G])
    for w in range(W):
        hyb.layout.scatter_accumulate_hybrid(K, grads[w], accs, w, 0)
    hyb.layout.reduce_groups(K, accs, accs[:G])
    torch.cuda.synchronize()
    flat_full = np.concatenate([a[:full_case.S[0]] for a in full_case.acc_host()])[:N]
    flat_hyb = np.concatenate([a[:hyb.S[0]] for a in hyb.acc_host()])[:N]
    assert np.array_equal(flat_full.view(np.uint32), flat_hyb.view(np.uint32))
    full_case.close()
    hyb.close()


def test_hybrid_7b_layer_two_groups_of_eight(oracle):
    """The 7B-shaped layer with its 16 workers as 2 groups of 8 owners: every contribution of the
    configuration's microbatch counts, then the group reduction, compared in full."""
    wl = inputs.workload("7b")
    N, W = wl.numel[0], wl.R
    K, R = 2, W // 2
    M = inputs.microbatch_counts(wl)
    print(f"hybrid 7b: N={N} groups={K} R={R} M={M}", flush=True)
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    dev = torch.device("cuda")
    accs = [torch.full((S,), 3.25, dtype=torch.float32, device=dev) for _ in range(K * R)]
    accs_h = [[np.full(S, 3.25, dtype=np.float32) for _ in range(R)] for _ in range(K)]
    pinned = torch.empty(N, dtype=torch.int16, pin_memory=True)
    for k in range(K):
        L.reset_accum(accs[k * R:(k + 1) * R])
        oracle.reset(accs_h[k], N, nthreads=THREADS)
    for w, mw in enumerate(M):
        for m in range(mw):
            g = inputs.device_normal_bf16(N, wl.grad_sigma, 5000 + 16 * w + m, dev)
            L.scatter_accumulate_hybrid(K, g, accs, w, m)
            pinned.copy_(g.view(torch.int16))
            oracle.accumulate(pinned.numpy().view(np.uint16), accs_h[w // R], N, nthreads=THREADS)
            del g
    out = [torch.full((S,), -1.0, dtype=torch.float32, device=dev) for _ in range(R)]
    out_h = [np.full(S, -1.0, dtype=np.float32) for _ in range(R)]
    L.reduce_groups(K, accs, out)
    oracle.reduce_groups(accs_h, out_h, N, nthreads=THREADS)
    torch.cuda.synchronize()
    for r in range(R):
        assert_bits_equal(out[r].cpu().numpy(), out_h[r], f"reduced shard of owner {r}")
    L.close()


def test_hybrid_argument_errors():
    case = DeviceCase(4, [1000], with_params=False)
    L = case.layout
    accs = [a.t for a in case.acc] + [torch.zeros(case.arena, dtype=torch.float32, device="cuda") for _ in range(4)]
    out = [torch.zeros(case.arena, dtype=torch.float32, device="cuda") for _ in range(4)]
    assert L.hybrid_group_of(2, 7) == 1 and L.hybrid_group_of(2, 8) == -1 and L.hybrid_group_of(0, 0) == -1
    assert odc.reduce_groups_rc(L, 0, [], out) == odc.ODC_ERR_INVALID_ARG
    assert odc.reduce_groups_rc(L, 2, accs, None) == odc.ODC_ERR_INVALID_ARG
    assert odc.reduce_groups_rc(L, 2, accs, accs[4:]) == odc.ODC_ERR_INVALID_ARG      # output = a later group
    bad = list(accs)
    bad[5] = accs[5][1:]
    assert odc.reduce_groups_rc(L, 2, bad, out) == odc.ODC_ERR_ALIGNMENT
    assert odc.scatter_accumulate_hybrid_rc(L, 2, case.grad.t, accs, 8, 0) == odc.ODC_ERR_INVALID_ARG
    assert odc.scatter_accumulate_hybrid_rc(L, 2, case.grad.t, accs, 5, 0) == 0
    assert odc.scatter_accumulate_hybrid_rc(L, 2, case.grad.t, accs, 4, 0) == odc.ODC_ERR_ORDER   # group 1: local rank 0 after 1
    assert odc.scatter_accumulate_hybrid_rc(L, 2, case.grad.t, accs, 1, 0) == 0                    # group 0 has its own history
    assert odc.reduce_groups_rc(L, 2, accs, accs[:4]) == 0
    torch.cuda.synchronize()
    case.close()
