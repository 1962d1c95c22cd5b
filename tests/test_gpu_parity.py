"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by
element on the same seeded inputs.  Gather and ordered scatter-accumulate must be bit-exact;
reset must give +0.0f; nothing outside the valid elements may change."""
import numpy as np
import pytest
import torch

from paper_2601_19362_amd import binding as odc
from paper_2601_19362_amd import inputs

from gpu_util import (FULL16, PAD16, PAD32, DeviceCase, assert_bits_equal, host_arenas_from_flats,
                      to_dev_u16, to_host_u16)

pytestmark = pytest.mark.gpu


def run_case(oracle, numel, R, contribs, seed, grad_sigma=1e-3, prange=(-0.05, 0.05)):
    """Gather once, reset, then apply `contribs` = [(worker, microbatch)] in order; compare all
    buffers (including padding, gaps and guards) with the oracle."""
    print(f"case R={R} T={len(numel)} total={sum(numel)} C={len(contribs)} seed={seed}", flush=True)
    case = DeviceCase(R, numel)
    flats = [inputs.uniform_bf16(n, prange[0], prange[1], seed=(seed, 1, t)) for t, n in enumerate(numel)]
    arenas = host_arenas_from_flats(oracle, flats, R, case.S, case.shard_off, case.arena)
    case.load_params(arenas)

    # gather
    case.layout.gather(case.param_ptrs, case.full.t)
    got_full = to_host_u16(case.full.t)
    want_full = np.full(case.full_n, FULL16, dtype=np.uint16)
    oracle.gather_batched(arenas, numel, case.shard_off, case.full_off, want_full)
    assert_bits_equal(got_full, want_full, "gather")
    for t, n in enumerate(numel):  # round trip: the flat parameter comes back bit for bit
        assert np.array_equal(got_full[case.full_off[t]:case.full_off[t] + n], flats[t])
    for p, a in zip(case.params, arenas):  # sources untouched
        assert np.array_equal(to_host_u16(p.t), a)

    # reset + ordered accumulate
    acc_host = [np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)]
    case.layout.reset_accum(case.acc_ptrs)
    oracle.reset_batched(acc_host, numel, case.shard_off)
    for r, a in enumerate(case.acc_host()):
        assert_bits_equal(a, acc_host[r], f"reset rank {r}")
    for (w, m) in contribs:
        g = inputs.normal_bf16(case.full_n, grad_sigma, seed=(seed, 2, w, m))
        case.grad.t.copy_(to_dev_u16(g))
        case.layout.scatter_accumulate(case.grad.t, case.acc_ptrs, w, m)
        oracle.accumulate_batched(g, acc_host, numel, case.shard_off, case.full_off)
    for r, a in enumerate(case.acc_host()):
        assert_bits_equal(a, acc_host[r], f"accumulate rank {r}")
    torch.cuda.synchronize()
    case.check_guards()
    case.close()


def contributions(M):
    return [(w, m) for w in range(len(M)) for m in range(M[w])]


def test_tiny_config(oracle):
    """Config 1: R = 4, N = 1,048,589 (tail padding, 8-byte-misaligned shard boundaries)."""
    w = inputs.workload("tiny")
    run_case(oracle, list(w.numel), w.R, contributions(inputs.microbatch_counts(w)), seed=w.seed)


@pytest.mark.parametrize("N,R", [(1, 1), (1, 64), (7, 3), (64, 64), (65, 64), (1000, 7), (4099, 8),
                                 (8 * 1024 * 3 + 5, 4), (524_309, 2), (1_000_003, 33),
                                 (4 * 1024 * 1024, 8), (3_000_001, 16), (350, 70),
                                 (8 * 1_000_001 - 3, 8)])   # S = 1,000,001: owner r's source shifted by 16 - 2r bytes
def test_single_tensor_shapes(oracle, N, R):
    M = [1 + (w % 3 == 0) for w in range(R)]
    run_case(oracle, [N], R, contributions(M)[:6], seed=N % 1000 + R)


@pytest.mark.parametrize("numel,R", [
    ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8),
    ([3, 1, 1, 2, 70, 5000, 2, 2, 129, 1], 64),
    ([30000, 17, 2048, 2049, 1_000_001], 5),
    ([5] * 70 + [100_000], 70),
])
def test_batched_shapes(oracle, numel, R):
    run_case(oracle, numel, R, [(0, 0), (0, 1), (R - 1, 0)], seed=len(numel) + R, grad_sigma=1e-2,
             prange=(-1, 1))


def test_stress_config(oracle):
    """Config 5: 10,000 flat params, R = 64, one batched launch per call."""
    w = inputs.workload("stress")
    M = inputs.microbatch_counts(w)
    run_case(oracle, list(w.numel), w.R, contributions(M)[:5], seed=w.seed, grad_sigma=w.grad_sigma,
             prange=w.param_range)


@pytest.mark.parametrize("knobs", [
    dict(gather_threads=64, accum_threads=64, reset_threads=64, gather_unroll=1, accum_unroll=1, reset_unroll=1),
    dict(gather_threads=128, accum_threads=128, reset_threads=128, gather_unroll=2, accum_unroll=2, reset_unroll=2,
         nontemporal=0),
    dict(gather_threads=256, accum_threads=256, reset_threads=256, gather_unroll=4, accum_unroll=4, reset_unroll=4,
         max_grid_x=7),
    dict(gather_threads=64, accum_threads=64, reset_threads=256, gather_unroll=1, accum_unroll=1, reset_unroll=1,
         tile_remap=1),
    dict(gather_threads=256, accum_threads=128, reset_threads=64, gather_unroll=2, accum_unroll=4, reset_unroll=4,
         tile_remap=1, nontemporal=0),
    dict(gather_threads=64, gather_unroll=1, gather_store_sc1=0),
    dict(gather_threads=128, gather_unroll=4, gather_store_sc1=1, tile_remap=1),
])
def test_results_do_not_depend_on_launch_knobs(oracle, knobs):
    """Every launch configuration gives the same bits."""
    neutral = dict(nontemporal=1, max_grid_x=0, tile_remap=0, gather_store_sc1=1)
    try:
        for k, v in {**neutral, **knobs}.items():
            odc.tune(k, v)
        run_case(oracle, [2_000_003], 4, [(0, 0), (1, 0), (1, 1)], seed=77)
        run_case(oracle, [1_000_000], 8, [(0, 0)], seed=79)
        run_case(oracle, [30000, 17, 2048, 2049, 100_001], 5, [(0, 0), (4, 2)], seed=78)
        weighted_retrieve_case(oracle, [1_500_007], 4, seed=80, weights=[0.37, None], scale=1.0 / 3.0)
        staging_case(oracle, [1_000_003], 4)
    finally:
        odc.reset_tuning()


@pytest.mark.parametrize("rg", [2, 4, 8])
def test_owner_groups_forced(oracle, rg):
    """The multi-tensor kernels with 2, 4 and 8 owners per workgroup forced (the built-in choice
    takes more than one only on large launches, which the small parity layouts never are): the
    accumulate, reset and retrieve variants, and the two-owner staging push."""
    try:
        odc.tune("batch_rank_group", rg)
        run_case(oracle, [30000, 17, 2048, 2049, 100_001], 5, [(0, 0), (4, 2)], seed=81)
        run_case(oracle, [3, 1, 1, 2, 70, 5000, 2, 2, 129, 1], 64, [(0, 0), (63, 1)], seed=82)
        weighted_retrieve_case(oracle, [30000, 17, 2048, 2049, 100_001], 5, seed=83, weights=[0.37, None], scale=0.25)
        staging_case(oracle, [30000, 17, 2048, 2049, 1_000_001], 5)
        staging_case(oracle, [5] * 70 + [100_000], 70)
    finally:
        odc.reset_tuning()


def test_special_values(oracle):
    """Subnormals are kept, signed zeros and infinities follow IEEE-754, NaN stays NaN."""
    specials = np.array([0x0001, 0x0003, 0x8001, 0x007F, 0x0080, 0x8000, 0x0000, 0x7F80, 0xFF80,
                         0x7FC0, 0x3F80, 0xBF80, 0x7F7F, 0xFF7F], dtype=np.uint16)
    N, R = 4096 + 11, 4
    rng = np.random.default_rng(3)
    gs = [specials[rng.integers(0, specials.size, size=N)] for _ in range(4)]
    case = DeviceCase(R, [N], with_params=False)
    acc_host = [np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)]
    case.layout.reset_accum(case.acc_ptrs)
    oracle.reset(acc_host, N)
    for k, g in enumerate(gs):
        case.grad.t.copy_(to_dev_u16(g))
        case.layout.scatter_accumulate(case.grad.t, case.acc_ptrs, 0, k)
        oracle.accumulate(g, acc_host, N)
    saw_sub = saw_nan = False
    for r, a in enumerate(case.acc_host()):
        want = acc_host[r]
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(a), nan)            # NaN-ness; payloads are not pinned
        assert_bits_equal(a[~nan], want[~nan], f"specials rank {r}")
        valid = want != PAD32
        saw_sub |= bool(((np.abs(want[valid & ~nan]) < 1.17549435e-38) & (want[valid & ~nan] != 0)).any())
        saw_nan |= bool(nan.any())
    assert saw_sub and saw_nan
    case.check_guards()
    case.close()


def test_ordered_mode_history_and_reset(oracle):
    case = DeviceCase(4, [1000], with_params=False)
    L = case.layout
    L.reset_accum(case.acc_ptrs)
    g = to_dev_u16(inputs.normal_bf16(1000, 1e-3, seed=5))
    case.grad.t.copy_(g)
    sa = lambda w, m, flags=odc.ODC_ORDERED: odc.scatter_accumulate_rc(L, case.grad.t, case.acc_ptrs, w, m, flags)
    assert sa(0, 0) == 0
    assert sa(0, 0) == odc.ODC_ERR_ORDER          # same slot twice
    assert sa(0, 2) == 0                           # gaps are fine
    assert sa(0, 1) == odc.ODC_ERR_ORDER          # microbatch going back
    assert sa(2, 0) == 0
    assert sa(1, 5) == odc.ODC_ERR_ORDER          # worker going back
    assert sa(1, 5, odc.ODC_UNORDERED) == 0        # unordered calls are not checked
    before = [a.copy() for a in case.acc_host()]
    assert sa(1, 0) == odc.ODC_ERR_ORDER
    for a, b in zip(case.acc_host(), before):      # a refused call enqueues nothing
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    # a second accumulator set has its own history
    other = [torch.zeros(case.arena, dtype=torch.float32, device="cuda") for _ in range(4)]
    assert odc.scatter_accumulate_rc(L, case.grad.t, other, 0, 0) == 0
    L.reset_accum(case.acc_ptrs)
    assert sa(0, 0) == 0                           # reset forgets the history
    torch.cuda.synchronize()
    case.close()


def test_ordered_history_is_bounded_and_can_be_forgotten():
    """The ordered-mode table keeps at most 1024 accumulator sets per layout (least recently used
    out first), and odc_forget_accum drops one set's history without touching the accumulators."""
    R, N = 2, 64
    L = odc.Layout(R, [N])
    S = L.shard_elems(0)
    g = torch.zeros(N, dtype=torch.bfloat16, device="cuda")
    pool = torch.zeros(1100 * R * S, dtype=torch.float32, device="cuda")
    sets = [[pool[(2 * k + r) * S:(2 * k + r + 1) * S] for r in range(R)] for k in range(1100)]
    sa = lambda k, w, m: odc.scatter_accumulate_rc(L, g, sets[k], w, m)
    assert sa(0, 1, 5) == 0
    assert sa(0, 1, 5) == odc.ODC_ERR_ORDER            # remembered
    L.forget_accum(sets[0])
    assert sa(0, 0, 0) == 0                             # forgotten: any (worker, microbatch) is fine again
    assert sa(1, 1, 0) == 0
    for k in range(2, 1100):                            # 1098 more sets: sets 0 and 1 are the oldest and go
        assert sa(k, 1, 0) == 0
    assert sa(1099, 1, 0) == odc.ODC_ERR_ORDER         # a recent set is still remembered
    assert sa(0, 0, 0) == 0                             # the oldest was dropped and starts afresh
    torch.cuda.synchronize()
    L.close()


def test_unordered_mode_within_tolerance(oracle):
    """Unordered mode: |x - ref64| <= 1e-6 * sum|g| per element against a float64 sum, with
    contributions issued in a scrambled order from two streams."""
    N, R = 1_000_003, 8
    M = [2, 1, 3, 1, 2, 2, 1, 2]
    grads = [[inputs.normal_bf16(N, 1e-3, seed=(91, w, m)) for m in range(M[w])] for w in range(R)]
    case = DeviceCase(R, [N], with_params=False)
    case.layout.reset_accum(case.acc_ptrs)
    torch.cuda.synchronize()
    order = contributions(M)
    rng = np.random.default_rng(1)
    rng.shuffle(order)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    dev = {(w, m): to_dev_u16(grads[w][m]) for (w, m) in order}
    torch.cuda.synchronize()
    for k, (w, m) in enumerate(order):
        case.layout.scatter_accumulate(dev[(w, m)], case.acc_ptrs, w, m, odc.ODC_UNORDERED,
                                       stream=streams[k % 2])
    torch.cuda.synchronize()
    sum64, abs64 = oracle.fp64_sum_shards(grads, N, R)
    worst = 0.0
    for r, a in enumerate(case.acc_host()):
        valid = max(0, min(case.S[0], N - r * case.S[0]))
        err = np.abs(a[:valid].astype(np.float64) - sum64[r][:valid])
        bound = 1e-6 * abs64[r][:valid]
        assert (err <= bound).all()
        worst = max(worst, float((err / np.maximum(abs64[r][:valid], 1e-300)).max()))
        assert (a[valid:] == PAD32).all()
    print(f"unordered worst |err|/sum|g| = {worst:.3e}", flush=True)
    case.check_guards()
    case.close()


def test_non_default_stream_and_probe_copy():
    s = torch.cuda.Stream()
    n = 1 << 20
    src = torch.arange(n, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    torch.cuda.synchronize()
    odc.probe_copy(dst, src, n * 4, stream=s)
    s.synchronize()
    assert torch.equal(src, dst)


# ----------------------------------------------------------------------------- weighted, retrieve
def weighted_retrieve_case(oracle, numel, R, seed, weights, scale):
    """reset, weighted contributions in order, then retrieval as binary32 and as bf16."""
    print(f"weighted/retrieve case R={R} T={len(numel)} total={sum(numel)} weights={weights} scale={scale}", flush=True)
    case = DeviceCase(R, numel, with_params=False)
    acc_host = [np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)]
    case.layout.reset_accum(case.acc_ptrs)
    oracle.reset_batched(acc_host, numel, case.shard_off)
    for k, w in enumerate(weights):
        g = inputs.normal_bf16(case.full_n, 1e-2, seed=(seed, 3, k))
        case.grad.t.copy_(to_dev_u16(g))
        if w is None:
            case.layout.scatter_accumulate(case.grad.t, case.acc_ptrs, 0, k)
            oracle.accumulate_batched(g, acc_host, numel, case.shard_off, case.full_off)
        else:
            case.layout.scatter_accumulate_weighted(case.grad.t, case.acc_ptrs, 0, k, w)
            oracle.accumulate_weighted_batched(g, acc_host, numel, case.shard_off, case.full_off, w)
    for r, a in enumerate(case.acc_host()):
        assert_bits_equal(a, acc_host[r], f"weighted accumulate rank {r}")
    from gpu_util import Guarded, i16
    for out_dtype, np_dtype, t_dtype, fill in ((odc.ODC_OUT_F32, np.float32, torch.float32, float(PAD32)),
                                               (odc.ODC_OUT_BF16, np.uint16, torch.int16, i16(PAD16))):
        outs = [Guarded(case.arena, t_dtype, fill) for _ in range(R)]
        case.layout.retrieve_grads(case.acc_ptrs, [o.t for o in outs], scale, out_dtype)
        want = [np.full(case.arena, PAD32 if np_dtype == np.float32 else PAD16, dtype=np_dtype) for _ in range(R)]
        oracle.retrieve_batched(acc_host, want, numel, case.shard_off, scale=scale)
        for r in range(R):
            got = outs[r].t.cpu().numpy()
            got = got.view(np.uint16) if np_dtype == np.uint16 else got
            assert_bits_equal(got, want[r], f"retrieve dtype {out_dtype} rank {r}")
            outs[r].check()
    for r, a in enumerate(case.acc_host()):            # retrieval leaves the accumulators alone
        assert_bits_equal(a, acc_host[r], f"accumulator after retrieve rank {r}")
    case.check_guards()
    case.close()


@pytest.mark.parametrize("numel,R", [([1_048_589], 4), ([1], 64), ([4099], 8), ([3_000_001], 16), ([350], 70),
                                     ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8),
                                     ([30000, 17, 2048, 2049, 1_000_001], 5), ([5] * 70 + [100_000], 70)])
def test_weighted_accumulate_and_retrieve(oracle, numel, R):
    weighted_retrieve_case(oracle, numel, R, seed=sum(numel) % 997, weights=[0.37, None, -1.5, 1.0 / 3.0],
                           scale=1.0 / 7.0)


def test_weighted_and_retrieve_on_stress_config(oracle):
    w = inputs.workload("stress")
    weighted_retrieve_case(oracle, list(w.numel), w.R, seed=w.seed, weights=[0.25, 1.7], scale=0.5)


def test_weight_one_equals_unweighted_and_scale_one_is_a_copy(oracle):
    N, R = 2_000_003, 4
    case = DeviceCase(R, [N], with_params=False)
    other = [torch.full((case.arena,), float(PAD32), dtype=torch.float32, device="cuda") for _ in range(R)]
    case.layout.reset_accum(case.acc_ptrs)
    case.layout.reset_accum(other)
    for k in range(3):
        case.grad.t.copy_(to_dev_u16(inputs.normal_bf16(N, 1e-3, seed=(44, k))))
        case.layout.scatter_accumulate(case.grad.t, case.acc_ptrs, 1, k)
        case.layout.scatter_accumulate_weighted(case.grad.t, other, 1, k, 1.0)
    out = [torch.zeros(case.arena, dtype=torch.float32, device="cuda") for _ in range(R)]
    case.layout.retrieve_grads(other, out, 1.0, odc.ODC_OUT_F32)
    for r in range(R):
        valid = case.layout.valid_elems(0, r)
        a = case.acc[r].t.cpu().numpy()
        assert_bits_equal(other[r].cpu().numpy(), a, f"weight 1 rank {r}")
        assert_bits_equal(out[r].cpu().numpy()[:valid], a[:valid], f"scale 1 rank {r}")
        assert (out[r].cpu().numpy()[valid:] == 0).all()
    case.close()


def test_weighted_unordered_within_tolerance(oracle):
    """Unordered weighted contributions: |x - ref64| <= 1e-6 * sum |w g| against a float64 sum."""
    N, R = 500_009, 8
    ws = [0.3, 1.0, 2.5, 0.7, 1.1, 0.05, 3.0, 1.9]
    case = DeviceCase(R, [N], with_params=False)
    case.layout.reset_accum(case.acc_ptrs)
    ref = np.zeros(N)
    mag = np.zeros(N)
    for k, w in enumerate(ws):
        g = inputs.normal_bf16(N, 1e-3, seed=(45, k))
        case.grad.t.copy_(to_dev_u16(g))
        case.layout.scatter_accumulate_weighted(case.grad.t, case.acc_ptrs, k % R, k, w, odc.ODC_UNORDERED)
        v = np.float64(np.float32(w)) * inputs.bf16_bits_to_f32(g).astype(np.float64)
        ref += v
        mag += np.abs(v)
    S = case.S[0]
    got = np.concatenate([a[:S] for a in case.acc_host()])[:N].astype(np.float64)
    assert (np.abs(got - ref) <= 1e-6 * mag).all()
    case.close()


def test_retrieve_argument_errors():
    case = DeviceCase(4, [1000], with_params=False)
    out = [torch.zeros(case.arena, dtype=torch.float32, device="cuda") for _ in range(4)]
    assert odc.retrieve_grads_rc(case.layout, case.acc_ptrs, out, 1.0, 7) == odc.ODC_ERR_INVALID_ARG
    assert odc.retrieve_grads_rc(case.layout, case.acc_ptrs, None, 1.0, 0) == odc.ODC_ERR_INVALID_ARG
    bad = [out[0], out[1][1:], out[2], out[3]]
    assert odc.retrieve_grads_rc(case.layout, case.acc_ptrs, bad, 1.0, 0) == odc.ODC_ERR_ALIGNMENT
    assert odc.retrieve_grads_rc(case.layout, case.acc_ptrs, out, 1.0, 0) == 0
    torch.cuda.synchronize()
    case.close()


# ----------------------------------------------------------------------------- fused contributions
@pytest.mark.parametrize("numel,R", [([1_048_589], 4), ([4099], 8), ([3_000_001], 16), ([350], 70),
                                     ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8),
                                     ([30000, 17, 2048, 2049, 1_000_001], 5)])
@pytest.mark.parametrize("count", [2, 3, 8])
def test_fused_contributions_equal_single_calls(oracle, numel, R, count):
    case = DeviceCase(R, numel, with_params=False)
    acc_host = [np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)]
    case.layout.reset_accum(case.acc_ptrs)
    oracle.reset_batched(acc_host, numel, case.shard_off)
    g0 = inputs.normal_bf16(case.full_n, 1e-2, seed=(80, 0))
    case.grad.t.copy_(to_dev_u16(g0))
    case.layout.scatter_accumulate(case.grad.t, case.acc_ptrs, 0, 0)
    oracle.accumulate_batched(g0, acc_host, numel, case.shard_off, case.full_off)
    gs = [inputs.normal_bf16(case.full_n, 1e-2, seed=(80, 1 + k)) for k in range(count)]
    dev = [to_dev_u16(g) for g in gs]
    case.layout.scatter_accumulate_multi(dev, case.acc_ptrs, [0] * count, list(range(1, count + 1)))
    for g in gs:
        oracle.accumulate_batched(g, acc_host, numel, case.shard_off, case.full_off)
    for r, a in enumerate(case.acc_host()):
        assert_bits_equal(a, acc_host[r], f"fused x{count} rank {r}")
    case.check_guards()
    case.close()


def test_fused_order_rules_and_unordered():
    N, R = 100_003, 4
    case = DeviceCase(R, [N], with_params=False)
    L = case.layout
    L.reset_accum(case.acc_ptrs)
    gs = [to_dev_u16(inputs.normal_bf16(N, 1e-3, seed=(81, k))) for k in range(3)]
    rc = lambda w, m, flags=odc.ODC_ORDERED, g=gs: odc.scatter_accumulate_multi_rc(L, g, case.acc_ptrs, w, m, flags)
    assert rc([0, 0, 1], [0, 1, 0]) == 0
    assert rc([1, 1, 1], [0, 1, 2]) == odc.ODC_ERR_ORDER         # first pair not after the history (1, 0)
    assert rc([1, 1, 1], [1, 3, 2]) == odc.ODC_ERR_ORDER         # not ascending inside the call
    assert rc([1, 2, 3], [1, 0, 0]) == 0
    assert odc.scatter_accumulate_multi_rc(L, gs + gs + gs, case.acc_ptrs, [3] * 9, list(range(1, 10))) == odc.ODC_ERR_INVALID_ARG
    assert odc.scatter_accumulate_multi_rc(L, [], case.acc_ptrs, [], []) == odc.ODC_ERR_INVALID_ARG
    assert rc([9, 9, 9], [0, 1, 2]) == odc.ODC_ERR_INVALID_ARG   # worker out of range
    assert odc.scatter_accumulate_multi_rc(L, gs[:1], case.acc_ptrs, [3], [5]) == 0   # count 1 = the single call
    assert rc([0, 0, 0], [0, 0, 0], odc.ODC_UNORDERED) == 0      # unordered: no order rules
    torch.cuda.synchronize()
    case.close()


def test_fused_unordered_within_tolerance(oracle):
    N, R = 500_009, 8
    case = DeviceCase(R, [N], with_params=False)
    case.layout.reset_accum(case.acc_ptrs)
    gs = [inputs.normal_bf16(N, 1e-3, seed=(82, k)) for k in range(8)]
    dev = [to_dev_u16(g) for g in gs]
    case.layout.scatter_accumulate_multi(dev[:5], case.acc_ptrs, [0] * 5, [0] * 5, odc.ODC_UNORDERED)
    case.layout.scatter_accumulate_multi(dev[5:], case.acc_ptrs, [0] * 3, [0] * 3, odc.ODC_UNORDERED)
    ref = sum(inputs.bf16_bits_to_f32(g).astype(np.float64) for g in gs)
    mag = sum(np.abs(inputs.bf16_bits_to_f32(g).astype(np.float64)) for g in gs)
    S = case.S[0]
    got = np.concatenate([a[:S] for a in case.acc_host()])[:N].astype(np.float64)
    assert (np.abs(got - ref) <= 1e-6 * mag).all()
    case.close()


# ----------------------------------------------------------------------------- staging
class DeviceStaging:
    def __init__(self, case):
        L = case.layout
        self.slot = L.stage_slot_elems()
        self.bufs = [torch.full((case.R * self.slot,), -3.0, dtype=torch.bfloat16, device="cuda") for _ in range(case.R)]
        self.flags = torch.full((L.stage_flag_count(),), 77, dtype=torch.int32, device="cuda")
        self.snap = torch.zeros(L.stage_snapshot_count(), dtype=torch.int32, device="cuda")
        L.stage_init(self.flags)


@pytest.mark.parametrize("numel,R", [([1_048_589], 4), ([1], 64), ([4099], 8), ([3_000_001], 16), ([350], 70),
                                     ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8),
                                     ([30000, 17, 2048, 2049, 1_000_001], 5), ([5] * 70 + [100_000], 70)])
def test_staging_push_and_drain(oracle, numel, R):
    staging_case(oracle, numel, R)


def staging_case(oracle, numel, R):
    case = DeviceCase(R, numel, with_params=False)
    st = DeviceStaging(case)
    model = oracle.Staging(numel, R, case.shard_off, case.full_off)
    acc_host = [np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)]
    case.layout.reset_accum(case.acc_ptrs)
    oracle.reset_batched(acc_host, numel, case.shard_off)
    hi = R - 1
    steps = [("p", hi), ("p", 0), ("d", None), ("p", 0), ("p", 0), ("p", min(1, hi)), ("p", min(2, hi)), ("d", None),
             ("d", None), ("p", hi)]
    for k, (kind, w) in enumerate(steps):
        if kind == "p":
            g = inputs.normal_bf16(case.full_n, 1e-2, seed=(90, k))
            case.grad.t.copy_(to_dev_u16(g))
            case.layout.stage_push(case.grad.t, st.bufs, st.flags, w)
            model.push(g, w)
        else:
            case.layout.stage_drain(st.bufs, st.flags, st.snap, case.acc_ptrs)
            model.drain(acc_host)
    for r, a in enumerate(case.acc_host()):
        assert_bits_equal(a, acc_host[r], f"staged accumulate rank {r}")
    flags = st.flags.cpu().numpy()
    assert flags[:R * R].reshape(R, R).astype(bool).tolist() == model.full
    assert flags[R * R] == model.refused
    case.check_guards()
    case.close()


def test_staging_concurrent_push_and_drain_loses_nothing():
    """Pushes on one stream, drains on another, no ordering between them: whichever drain
    picks a contribution up, each is added exactly once.  Integer-valued gradients make every
    sum exact, so the final result does not depend on the grouping."""
    N, R = 3_000_001, 8
    case = DeviceCase(R, [N], with_params=False)
    st = DeviceStaging(case)
    other_snap = torch.zeros_like(st.snap)
    case.layout.reset_accum(case.acc_ptrs)
    rng = np.random.default_rng(5)
    ints = [rng.integers(-100, 101, size=N) for _ in range(R)]
    grads = [to_dev_u16(inputs.f32_to_bf16_bits(v.astype(np.float32))) for v in ints]
    torch.cuda.synchronize()
    s_push, s_drain = torch.cuda.Stream(), torch.cuda.Stream()
    for w in range(R):
        case.layout.stage_push(grads[w], st.bufs, st.flags, w, stream=s_push)
        if w % 2 == 1:
            case.layout.stage_drain(st.bufs, st.flags, st.snap, case.acc_ptrs, stream=s_drain)
    torch.cuda.synchronize()
    case.layout.stage_drain(st.bufs, st.flags, other_snap, case.acc_ptrs)      # whatever is left
    torch.cuda.synchronize()
    total = sum(ints).astype(np.float32)
    S = case.S[0]
    got = np.concatenate([a[:S] for a in case.acc_host()])[:N]
    assert np.array_equal(got, total)
    flags = st.flags.cpu().numpy()
    assert not flags.any()
    case.close()


def test_staging_repeated_pushes_race_drains_on_another_stream():
    """Two clients push five times each, back to back on a stream of their own, without waiting
    for the owners; drains run meanwhile on a third stream.  Whether an owner takes a given push
    depends on timing -- its slot may still be full -- but each owner decides once per push: a
    push is added exactly once in full or refused in full and counted.  Push i of client w
    carries 4^(5w+i) * (1 + j mod 3) at flat index j (exact in bf16, every partial sum exact in
    binary32), so an accumulator element divided by (1 + j mod 3) spells in base 4 how often
    each push was added: every digit must be 0 or 1, the same over the whole shard of an owner,
    and the zeros must add up to the refused counter."""
    N, R, K, clients = 48_000_005, 8, 5, (0, 5)
    case = DeviceCase(R, [N], with_params=False)
    st = DeviceStaging(case)
    case.layout.reset_accum(case.acc_ptrs)
    pos = (torch.arange(N, device="cuda") % 3 + 1).to(torch.float32)
    grads = {(w, i): (pos * float(4 ** (K * c + i))).to(torch.bfloat16) for c, w in enumerate(clients) for i in range(K)}
    for g in grads.values():
        assert torch.equal(g.to(torch.float32) / pos, torch.full_like(pos, float(g[0])))   # exact in bf16
    torch.cuda.synchronize()
    s_client = {w: torch.cuda.Stream() for w in clients}
    s_drain = torch.cuda.Stream()
    for i in range(K):
        for w in clients:
            case.layout.stage_push(grads[(w, i)], st.bufs, st.flags, w, stream=s_client[w])
        case.layout.stage_drain(st.bufs, st.flags, st.snap, case.acc_ptrs, stream=s_drain)
        case.layout.stage_drain(st.bufs, st.flags, st.snap, case.acc_ptrs, stream=s_drain)
    torch.cuda.synchronize()
    case.layout.stage_drain(st.bufs, st.flags, st.snap, case.acc_ptrs)      # whatever is left
    torch.cuda.synchronize()
    flags = st.flags.cpu().numpy()
    assert not flags[:R * R].any()
    S = case.S[0]
    taken = 0
    pos_h = (np.arange(N) % 3 + 1).astype(np.float64)
    for r, a in enumerate(case.acc_host()):
        valid = max(0, min(S, N - r * S))
        code = a[:valid].astype(np.float64) / pos_h[r * S:r * S + valid]
        assert (code == code[0]).all(), f"owner {r}: pushes added to part of the shard only"
        digits = [int(code[0]) // 4 ** d % 4 for d in range(K * len(clients))]
        assert int(code[0]) == code[0] and all(d in (0, 1) for d in digits), f"owner {r}: base-4 digits {digits}"
        taken += sum(digits)
    refused = int(flags[R * R])
    print(f"staging race: {taken} pushes taken, {refused} refused of {R * K * len(clients)}", flush=True)
    assert taken + refused == R * K * len(clients)
    case.check_guards()
    case.close()


def test_host_daemon_polls_the_flags_and_accumulates_on_receipt():
    """The server side as Appendix B runs it: a daemon on the HOST polls for notifications (it
    occupies no compute unit) and accumulates what has arrived, and a client pushes again only
    once its previous push has been consumed.  Here the daemon is a host thread that copies the
    slot states to the host and calls the drain when a slot is full; the clients are the main
    thread, one stream each, which poll their own column of the states before pushing.  No
    kernel ever waits.  Gradients are small integers (every sum exact), so the result does not
    depend on which drain took which push: nothing may be refused, lost or added twice."""
    import threading
    import time

    N, R, K = 6_000_005, 4, 6
    case = DeviceCase(R, [N], with_params=False)
    L = case.layout
    st = DeviceStaging(case)
    L.reset_accum(case.acc_ptrs)
    pos = (torch.arange(N, device="cuda") % 5 + 1).to(torch.float32)
    grads = {(w, i): (pos * float(w * K + i + 1)).to(torch.bfloat16) for w in range(R) for i in range(K)}   # <= 120: exact
    torch.cuda.synchronize()
    nflag = R * R
    stop, failed, drains = threading.Event(), [], [0]

    def daemon():
        try:
            stream = torch.cuda.Stream()
            seen = torch.empty(nflag + 1, dtype=torch.int32, pin_memory=True)
            with torch.cuda.stream(stream):
                while True:
                    seen.copy_(st.flags, non_blocking=True)
                    stream.synchronize()
                    if bool((seen[:nflag] == 1).any()):
                        L.stage_drain(st.bufs, st.flags, st.snap, case.acc_ptrs, stream=stream)
                        drains[0] += 1
                    elif stop.is_set():
                        return
                    else:
                        time.sleep(0.0002)
        except BaseException as e:          # reported by the main thread
            failed.append(repr(e))

    server = threading.Thread(target=daemon)
    server.start()
    try:
        streams = [torch.cuda.Stream() for _ in range(R)]
        mine = torch.empty(nflag + 1, dtype=torch.int32, pin_memory=True)
        poll = torch.cuda.Stream()

        def wait_until(ready, what):
            deadline = time.time() + 60
            while True:
                with torch.cuda.stream(poll):
                    mine.copy_(st.flags, non_blocking=True)
                poll.synchronize()
                if ready(mine[:nflag].view(R, R)):
                    return
                assert time.time() < deadline and not failed, f"{what}: {failed or 'timed out'}"
                time.sleep(0.0002)

        for i in range(K):
            for w in range(R):
                wait_until(lambda states: bool((states[:, w] == 0).all()), f"client {w} waiting for its slots")
                L.stage_push(grads[(w, i)], st.bufs, st.flags, w, stream=streams[w])
        for s in streams:
            s.synchronize()
        wait_until(lambda states: bool((states == 0).all()), "waiting for the daemon to consume everything")
    finally:
        stop.set()
        server.join(timeout=60)
    assert not failed and not server.is_alive(), failed
    torch.cuda.synchronize()
    flags = st.flags.cpu().numpy()
    assert not flags[:nflag].any() and flags[nflag] == 0                      # nothing staged, nothing refused
    total = float(sum(range(1, R * K + 1)))
    S = case.S[0]
    pos_h = (np.arange(N) % 5 + 1).astype(np.float32)
    for r, a in enumerate(case.acc_host()):
        valid = max(0, min(S, N - r * S))
        assert np.array_equal(a[:valid], pos_h[r * S:r * S + valid] * np.float32(total)), f"owner {r}"
    print(f"host daemon: {R * K} pushes consumed by {drains[0]} drains", flush=True)
    case.check_guards()
    case.close()


def test_staging_argument_errors():
    case = DeviceCase(4, [1000], with_params=False)
    st = DeviceStaging(case)
    L = case.layout
    assert odc.stage_push_rc(L, case.grad.t, st.bufs, st.flags, 4) == odc.ODC_ERR_INVALID_ARG
    assert odc.stage_push_rc(L, case.grad.t, st.bufs, None, 0) == odc.ODC_ERR_INVALID_ARG
    assert odc.stage_push_rc(L, case.grad.t, st.bufs, st.flags[1:], 0) == odc.ODC_ERR_ALIGNMENT
    assert odc.stage_drain_rc(L, st.bufs, st.flags, None, case.acc_ptrs) == odc.ODC_ERR_INVALID_ARG
    assert odc.stage_drain_rc(L, st.bufs, st.flags, st.snap, None) == odc.ODC_ERR_INVALID_ARG
    assert L.stage_slot_elems() == 256 and L.stage_flag_count() == 17 and L.stage_snapshot_count() == 20
    assert odc.stage_push_rc(L, case.grad.t, st.bufs, st.flags, 0) == 0
    assert odc.stage_drain_rc(L, st.bufs, st.flags, st.snap, case.acc_ptrs) == 0
    torch.cuda.synchronize()
    case.close()


@pytest.mark.parametrize("numel,R", [([1_048_589], 4), ([4099, 1, 70_001, 12_345, 8], 8)])
def test_hip_graph_replay_matches_oracle(oracle, numel, R):
    """The entry points only enqueue kernels (no allocation, memset or synchronisation), so a
    step -- gather, reset, three ordered contributions, retrieval -- can be captured into a HIP
    graph.  Every replay reads the buffers as they are at replay time: the inputs change between
    replays, with eager launches and synchronisations in between, and each replay is checked
    against the oracle."""
    print(f"graph case R={R} numel={numel}", flush=True)
    case = DeviceCase(R, numel)
    L = case.layout
    grads = [torch.zeros(case.full_n, dtype=torch.int16, device="cuda") for _ in range(3)]
    out = [torch.zeros(case.arena, dtype=torch.float32, device="cuda") for _ in range(R)]
    out_ptrs = odc.PtrArray(out)
    scale = 0.25

    def step():
        L.gather(case.param_ptrs, case.full.t)
        L.reset_accum(case.acc_ptrs)
        for k, g in enumerate(grads):
            L.scatter_accumulate(g, case.acc_ptrs, k, 0)
        L.retrieve_grads(case.acc_ptrs, out_ptrs, scale, odc.ODC_OUT_F32)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    for replay in range(4):
        flats = [inputs.uniform_bf16(n, -0.05, 0.05, seed=(77, replay, t)) for t, n in enumerate(numel)]
        arenas = host_arenas_from_flats(oracle, flats, R, case.S, case.shard_off, case.arena)
        case.load_params(arenas)
        g_host = [inputs.normal_bf16(case.full_n, 1e-3, seed=(78, replay, k)) for k in range(3)]
        for g, h in zip(grads, g_host):
            g.copy_(to_dev_u16(h))
        # eager work between replays: dirty the outputs the replay has to rewrite
        case.full.t[:case.full_n].fill_(0x1234)
        L.scatter_accumulate(grads[0], case.acc_ptrs, 0, 0, odc.ODC_UNORDERED)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()

        want_full = np.full(case.full_n, FULL16, dtype=np.uint16)
        got_full = to_host_u16(case.full.t)
        oracle.gather_batched(arenas, numel, case.shard_off, case.full_off, want_full)
        for t, n in enumerate(numel):
            a = case.full_off[t]
            assert_bits_equal(got_full[a:a + n], want_full[a:a + n], f"replay {replay} gather tensor {t}")
        acc_host = [np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)]
        oracle.reset_batched(acc_host, numel, case.shard_off)
        for h in g_host:
            oracle.accumulate_batched(h, acc_host, numel, case.shard_off, case.full_off)
        for r, a in enumerate(case.acc_host()):
            assert_bits_equal(a, acc_host[r], f"replay {replay} accumulate rank {r}")
        want_out = [np.zeros(case.arena, dtype=np.float32) for _ in range(R)]
        oracle.retrieve_batched(acc_host, want_out, numel, case.shard_off, scale=scale)
        for r in range(R):
            got = out[r].cpu().numpy()
            for t in range(len(numel)):
                a, v = case.shard_off[t], L.valid_elems(t, r)
                assert_bits_equal(got[a:a + v], want_out[r][a:a + v], f"replay {replay} retrieve rank {r} tensor {t}")
    case.check_guards()
    case.close()


@pytest.mark.parametrize("numel,R", [([3_000_001], 16), ([4099, 1, 70_001, 12_345, 8, 300_000], 8)])
def test_unordered_concurrent_streams_lose_no_update(oracle, numel, R):
    """Small-integer gradients (exact in bf16, every partial sum exact in binary32) make the
    result independent of the order, so the unordered mode must reproduce the ordered oracle bit
    for bit even when 12 contributions race on three streams: a lost or doubled atomic update
    would show as a wrong integer."""
    print(f"unordered concurrency case R={R} numel={numel}", flush=True)
    case = DeviceCase(R, numel, with_params=False)
    rng = np.random.default_rng(5)
    C = 12
    ints = [rng.integers(-256, 257, size=case.full_n).astype(np.float32) for _ in range(C)]
    grads = [inputs.f32_to_bf16_bits(x) for x in ints]
    for g, x in zip(grads, ints):
        assert np.array_equal(inputs.bf16_bits_to_f32(g), x)     # exactly representable
    dev = [to_dev_u16(g) for g in grads]
    case.layout.reset_accum(case.acc_ptrs)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(3)]
    for k in range(C):
        if k % 4 == 3:   # every fourth through the weighted entry point with weight 1
            case.layout.scatter_accumulate_weighted(dev[k], case.acc_ptrs, 0, 0, 1.0, odc.ODC_UNORDERED,
                                                    stream=streams[k % 3])
        else:
            case.layout.scatter_accumulate(dev[k], case.acc_ptrs, 0, 0, odc.ODC_UNORDERED, stream=streams[k % 3])
    torch.cuda.synchronize()
    acc_host = [np.full(case.arena, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reset_batched(acc_host, numel, case.shard_off)
    for g in grads:
        oracle.accumulate_batched(g, acc_host, numel, case.shard_off, case.full_off)
    for r, a in enumerate(case.acc_host()):
        assert_bits_equal(a, acc_host[r], f"unordered concurrent rank {r}")
    case.check_guards()
    case.close()


def random_layout(seed):
    """Seeded random multi-tensor layout, up to about 6 M elements, with single- and
    multi-launch rank counts."""
    rng = np.random.default_rng(seed)
    R = int(rng.choice([1, 2, 3, 7, 8, 16, 33, 64, 65, 100, 130]))
    T = int(rng.integers(2, 120))
    sizes = []
    for _ in range(T):
        kind = rng.choice(5, p=[0.3, 0.3, 0.2, 0.15, 0.05])
        lo, hi = [(1, 16), (17, 600), (601, 20_000), (20_001, 200_000), (200_001, 2_000_000)][kind]
        sizes.append(int(rng.integers(lo, hi + 1)))
    while sum(sizes) > 6_000_000:
        sizes.remove(max(sizes))
    if len(sizes) < 2:
        sizes.append(5)
    return sizes, R


@pytest.mark.parametrize("seed", range(12))
def test_random_layouts(oracle, seed):
    numel, R = random_layout(500 + seed)
    print(f"random layout seed={seed} R={R} T={len(numel)} total={sum(numel)}", flush=True)
    run_case(oracle, numel, R, [(0, 0), (0, 1), (R - 1, 0)], seed=300 + seed, grad_sigma=1e-2, prange=(-1, 1))
    weighted_retrieve_case(oracle, numel, R, seed=400 + seed, weights=[0.37, 1.0 / 3.0], scale=1.0 / 7.0)
