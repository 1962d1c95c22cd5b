"""Pins for the CPU oracle: every check here compares the oracle with something that is
not the oracle -- a closed form, a brute-force index map, a numpy library routine, exact
integer arithmetic, or a hand-computed rounding case -- chosen so that a dropped term,
a wrong index or a wrong order fails at least one of them.  No GPU needed.
"""
import os

import numpy as np
import pytest

from paper_2601_19362_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
PAD16 = 0xDEAD
PAD32 = np.float32(-12345.678)


def bits32(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def f32_from_bits(u):
    return np.array([u], dtype=np.uint32).view(np.float32)[0]


def new_acc(S, R):
    return [np.full(S, PAD32, dtype=np.float32) for _ in range(R)]


# ----------------------------------------------------------------------------- layout
@pytest.mark.parametrize("R", [1, 2, 3, 4, 7, 8, 16, 33, 64, 70])
def test_layout_closed_forms_and_owner_map(oracle, R):
    """Section 3.1 even partition: S is the least integer with R*S >= N; the valid counts
    tile [0, N) exactly; brute-force owner map owner(j) = floor(j / S)."""
    for N in list(range(1, 201)) + [1000, 1023, 1024, 1025]:
        S = oracle.shard_elems(N, R)
        assert R * (S - 1) < N <= R * S
        valid = [oracle.valid_elems(N, R, r) for r in range(R)]
        assert sum(valid) == N
        assert all(0 <= v <= S for v in valid)
        assert all(valid[r] >= valid[r + 1] for r in range(R - 1))
        assert sum(1 for v in valid if 0 < v < S) <= 1
        owners = np.arange(N) // S
        counts = np.bincount(owners, minlength=R)
        assert counts.tolist() == valid


def test_layout_golden_table(oracle):
    """Hand-computed shard sizes for the five workload shapes."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "layout_table.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for name, h, ffn, q, kv, R, N, S, pad, vlast in rows:
        R, N, S, pad, vlast = int(R), int(N), int(S), int(pad), int(vlast)
        assert oracle.shard_elems(N, R) == S
        assert R * S - N == pad
        assert oracle.valid_elems(N, R, R - 1) == vlast
        w = inputs.workload(name)
        assert w.R == R and w.numel == (N,)
        if h != "-":
            assert inputs.decoder_layer_numel(int(h), int(ffn), int(q), int(kv)) == N


def test_layout_many_ranks_only_padding(oracle):
    """N < R: S = 1, the first N owners hold one element, the rest hold only padding."""
    assert oracle.shard_elems(1, 64) == 1
    assert [oracle.valid_elems(1, 64, r) for r in range(64)] == [1] + [0] * 63
    assert oracle.shard_elems(5, 64) == 1
    assert sum(oracle.valid_elems(5, 64, r) for r in range(64)) == 5
    # several wholly-padding owners also occur with S > 1
    assert oracle.shard_elems(9, 8) == 2
    assert [oracle.valid_elems(9, 8, r) for r in range(8)] == [2, 2, 2, 2, 1, 0, 0, 0]


# ----------------------------------------------------------------------------- gather
@pytest.mark.parametrize("N,R", [(1, 1), (1, 64), (7, 3), (64, 64), (65, 64), (1000, 7),
                                 (4099, 8), (1_048_589, 4), (100_003, 33)])
def test_gather_round_trip_concatenate_and_sentinel(oracle, N, R):
    """(i) shard then gather reproduces the flat parameter bit for bit (gather is the
    decomposed all-gather, Section 3); (ii) equals np.concatenate(shards)[:N] built from
    slices taken here, not by the oracle; (iii) slots >= N of the output keep a sentinel."""
    flat = inputs.uniform_bf16(N, -0.05, 0.05, seed=(1, N, R))
    S = -(-N // R)
    # shards built independently of the oracle: pad the flat array and reshape
    padded = np.full(R * S, PAD16, dtype=np.uint16)
    padded[:N] = flat
    mine = [np.ascontiguousarray(padded[r * S:(r + 1) * S]) for r in range(R)]
    theirs = oracle.make_shards(flat, R, pad_bits=PAD16)
    for a, b in zip(mine, theirs):
        assert np.array_equal(a, b)
    cap = R * S + 5
    full = np.full(cap, 0xBEEF, dtype=np.uint16)
    oracle.gather(theirs, N, full)
    assert np.array_equal(full[:N], flat)
    assert np.array_equal(full[:N], np.concatenate(mine)[:N])
    assert (full[N:] == 0xBEEF).all()


def test_gather_brute_force_index_map(oracle):
    """full[j] = shard_{j // S}[j % S], element by element in Python, distinct values."""
    for N, R in [(1, 1), (5, 2), (17, 4), (23, 5), (64, 8), (97, 64)]:
        S = -(-N // R)
        shards = [np.arange(r * 1000, r * 1000 + S, dtype=np.uint16) for r in range(R)]
        full = np.full(N + 3, 0xFFFF, dtype=np.uint16)
        oracle.gather(shards, N, full)
        for j in range(N):
            assert full[j] == shards[j // S][j % S]
        assert (full[N:] == 0xFFFF).all()


def test_gather_does_not_read_padding_into_result(oracle):
    """Padding slots of the owners' shards never reach the output."""
    N, R = 10, 4  # S = 3, last owner has 1 valid + 2 padding slots
    shards = [np.full(3, 0x1111 * (r + 1), dtype=np.uint16) for r in range(R)]
    shards[3][1:] = 0x9999
    full = np.zeros(12, dtype=np.uint16)
    oracle.gather(shards, N, full)
    assert full.tolist() == [0x1111] * 3 + [0x2222] * 3 + [0x3333] * 3 + [0x4444, 0, 0]


@pytest.mark.parametrize("D,K", [(4, 5), (8, 16), (16, 3)])
def test_gather_remote_volume_closed_form(oracle, D, K):
    """Appendix D (communication volume table): a client's gather moves (D-1)*K elements
    from other owners, K = per-device shard size, when the partition is exact."""
    N = D * K
    S = oracle.shard_elems(N, D)
    assert S == K
    owners = np.arange(N) // S
    for w in range(D):
        assert int((owners != w).sum()) == (D - 1) * K == N - oracle.valid_elems(N, D, w)


# ----------------------------------------------------------------------------- reset
def test_reset_zero_bits_and_padding_untouched(oracle):
    for N, R in [(10, 4), (1, 8), (1027, 4)]:
        S = -(-N // R)
        acc = new_acc(S, R)
        oracle.reset(acc, N)
        flat = np.concatenate(acc)
        assert (bits32(flat[:N]) == 0).all()          # +0.0f exactly
        assert (flat[N:] == PAD32).all()               # padding slots never written


# ----------------------------------------------------------------------------- accumulate
def brute_force_ordered(grads, N, R):
    """Sequential binary32 sum per element, worker then microbatch order, in Python."""
    S = -(-N // R)
    out = [[np.float32(0.0)] * S for _ in range(R)]
    for w in range(len(grads)):
        for g in grads[w]:
            for j in range(N):
                r, i = divmod(j, S)
                v = f32_from_bits(np.uint32(int(g[j]) << 16))
                out[r][i] = np.float32(out[r][i] + v)
    return out


@pytest.mark.parametrize("N,R,M", [(13, 4, [2, 1, 3, 2]), (64, 8, [1] * 8), (7, 3, [3, 0, 2]),
                                   (50, 64, [1] * 64)])
def test_accumulate_equals_brute_force_sequential_sum(oracle, N, R, M):
    S = -(-N // R)
    grads = [[inputs.normal_bf16(N, 1e-3, seed=(9, N, w, m)) for m in range(M[w])]
             for w in range(R)]
    acc = new_acc(S, R)
    oracle.reset(acc, N)
    assert oracle.scatter_accumulate_ordered(grads, acc, N) == sum(M)
    ref = brute_force_ordered(grads, N, R)
    for r in range(R):
        valid = max(0, min(S, N - r * S))
        want = np.array(ref[r][:valid], dtype=np.float32)
        assert np.array_equal(bits32(acc[r][:valid]), bits32(want))
        assert (acc[r][valid:] == PAD32).all()


def test_accumulate_single_contribution_is_exact_widening(oracle):
    """C = 1 from +0: the accumulator holds the bf16 bits shifted into the high half."""
    N, R = 1003, 4
    S = -(-N // R)
    g = inputs.normal_bf16(N, 1e-3, seed=77)
    g[g == 0x8000] = 0  # -0 + +0 = +0 loses the sign; covered by its own test below
    acc = new_acc(S, R)
    oracle.reset(acc, N)
    oracle.accumulate(g, acc, N)
    got = np.concatenate(acc)[:N]
    assert np.array_equal(bits32(got), g.astype(np.uint32) << 16)


def test_accumulate_small_integers_exact(oracle):
    """Integer-valued contributions (|k| <= 256 is exact in bf16) with C*256 < 2^24: every
    partial sum is exact, so the result equals the integer sum whatever the order."""
    N, R = 999, 8
    S = -(-N // R)
    rng = np.random.default_rng(5)
    M = [3, 1, 2, 4, 1, 1, 2, 3]
    ints = [[rng.integers(-256, 257, size=N) for _ in range(M[w])] for w in range(R)]
    grads = [[inputs.f32_to_bf16_bits(k.astype(np.float32)) for k in per] for per in ints]
    for per_i, per_g in zip(ints, grads):
        for k, g in zip(per_i, per_g):
            assert np.array_equal(inputs.bf16_bits_to_f32(g), k.astype(np.float32))
    acc = new_acc(S, R)
    oracle.reset(acc, N)
    oracle.scatter_accumulate_ordered(grads, acc, N)
    total = sum(k for per in ints for k in per)
    got = np.concatenate(acc)[:N]
    assert np.array_equal(got, total.astype(np.float32))
    sum64, _ = oracle.fp64_sum_shards(grads, N, R)
    assert np.array_equal(np.concatenate(sum64)[:N], total.astype(np.float64))


def test_accumulate_order_is_worker_then_microbatch(oracle):
    """1.0, 2^-24, 2^-24 in that order stay 1.0 (each add is a tie, rounds to even); with
    1.0 last the result is 1 + 2^-23.  Placing the three values at chosen (w, m) slots
    shows the oracle walks worker ascending, then microbatch ascending."""
    one = inputs.f32_to_bf16_bits(np.array([1.0], dtype=np.float32))[0]
    tiny = inputs.f32_to_bf16_bits(np.array([2.0 ** -24], dtype=np.float32))[0]
    zero = np.uint16(0)
    N, R = 6, 3  # S = 2
    S = 2

    def run(slots):
        # slots: {(w, m): bits}; every worker has 2 microbatches
        grads = [[np.full(N, slots.get((w, m), zero), dtype=np.uint16) for m in range(2)]
                 for w in range(R)]
        acc = new_acc(S, R)
        oracle.reset(acc, N)
        oracle.scatter_accumulate_ordered(grads, acc, N)
        out = np.concatenate(acc)
        assert (out == out[0]).all()
        return out[0]

    assert run({(0, 0): one, (0, 1): tiny, (1, 0): tiny}) == np.float32(1.0)
    assert run({(0, 0): one, (1, 1): tiny, (2, 0): tiny}) == np.float32(1.0)
    big = np.float32(1.0) + np.float32(2.0 ** -23)
    assert run({(0, 0): tiny, (0, 1): tiny, (1, 0): one}) == big
    assert run({(0, 1): tiny, (1, 0): tiny, (2, 1): one}) == big
    # microbatch order inside a worker: (w, 0) before (w, 1)
    assert run({(0, 0): tiny, (1, 0): tiny, (1, 1): one}) == big
    # (tiny + 1.0) ties to 1.0, then + tiny ties to 1.0 again
    assert run({(0, 0): tiny, (1, 0): one, (1, 1): tiny}) == np.float32(1.0)
    # worker order dominates microbatch order: (1, 0) is applied after (0, 1)
    assert run({(0, 1): one, (1, 0): tiny, (2, 0): tiny}) == np.float32(1.0)
    assert run({(1, 0): one, (0, 1): tiny, (0, 0): tiny}) == big


def test_accumulate_within_fp32_bound_of_fp64_sum(oracle):
    """Reduce-scatter semantics (Section 3): shard r of the sum of all contributions,
    within the sequential binary32 bound (C-1) * 2^-24 * sum|g| of a float64 sum."""
    N, R = 20011, 8
    S = -(-N // R)
    M = [2, 3, 1, 4, 2, 2, 1, 3]
    C = sum(M)
    grads = [[inputs.normal_bf16(N, 1e-3, seed=(3, w, m)) for m in range(M[w])] for w in range(R)]
    acc = new_acc(S, R)
    oracle.reset(acc, N)
    oracle.scatter_accumulate_ordered(grads, acc, N)
    sum64, abs64 = oracle.fp64_sum_shards(grads, N, R)
    # independent fp64 reference built here
    ref = np.zeros(N)
    mag = np.zeros(N)
    for per in grads:
        for g in per:
            v = inputs.bf16_bits_to_f32(g).astype(np.float64)
            ref += v
            mag += np.abs(v)
    assert np.array_equal(np.concatenate(sum64)[:N], ref)
    assert np.array_equal(np.concatenate(abs64)[:N], mag)
    got = np.concatenate(acc)[:N].astype(np.float64)
    assert (np.abs(got - ref) <= (C - 1) * 2.0 ** -24 * mag + 1e-300).all()
    assert np.abs(got - ref).max() > 0  # binary32 rounding really happens


def test_accumulate_subnormals_signed_zero_inf_nan(oracle):
    """IEEE-754 binary32 semantics without flush-to-zero."""
    sub_a, sub_b = np.uint16(0x0001), np.uint16(0x0003)       # bf16 subnormals
    minus_zero, plus_inf, minus_inf = np.uint16(0x8000), np.uint16(0x7F80), np.uint16(0xFF80)
    qnan = np.uint16(0x7FC0)
    one = np.uint16(0x3F80)
    g1 = np.array([sub_a, minus_zero, plus_inf, plus_inf, qnan, one, sub_a], dtype=np.uint16)
    g2 = np.array([sub_b, minus_zero, minus_inf, one, one, qnan, np.uint16(0x8001)], dtype=np.uint16)
    N, R = g1.size, 2
    S = -(-N // R)
    acc = new_acc(S, R)
    oracle.reset(acc, N)
    oracle.accumulate(g1, acc, N)
    oracle.accumulate(g2, acc, N)
    got = np.concatenate(acc)[:N]
    b = bits32(got)
    assert b[0] == 0x00040000            # 1*2^-133 + 3*2^-133 = 4*2^-133, still subnormal
    assert b[1] == 0x00000000            # (+0 + -0) + -0 = +0 under round-to-nearest
    assert np.isnan(got[2])              # inf - inf
    assert b[3] == 0x7F800000            # inf + 1
    assert np.isnan(got[4]) and np.isnan(got[5])
    assert b[6] == 0x00000000            # x + (-x) = +0
    # an accumulator that already holds -0 keeps it when -0 is added (no reset in between)
    acc2 = [np.array([-0.0, -0.0], dtype=np.float32)]
    oracle.accumulate(np.array([0x8000, 0x0000], dtype=np.uint16), acc2, 2)
    assert bits32(acc2[0]).tolist() == [0x80000000, 0x00000000]


def test_accumulate_starts_from_stored_value(oracle):
    """The add starts from what the accumulator holds, not from zero."""
    N, R = 5, 2
    acc = [np.array([1.5, 2.5, 3.5], dtype=np.float32), np.array([4.5, 5.5, 99.0], dtype=np.float32)]
    g = inputs.f32_to_bf16_bits(np.array([1, 2, 3, 4, 5], dtype=np.float32))
    oracle.accumulate(g, acc, N)
    assert acc[0].tolist() == [2.5, 4.5, 6.5]
    assert acc[1].tolist() == [8.5, 10.5, 99.0]


# ----------------------------------------------------------------------------- threads, batched
def test_element_range_threads_do_not_change_bits(oracle):
    N, R = 300_007, 8
    S = -(-N // R)
    flat = inputs.uniform_bf16(N, -0.05, 0.05, seed=21)
    shards = oracle.make_shards(flat, R)
    f1 = np.zeros(N, dtype=np.uint16)
    f8 = np.zeros(N, dtype=np.uint16)
    oracle.gather(shards, N, f1, nthreads=1)
    oracle.gather(shards, N, f8, nthreads=8)
    assert np.array_equal(f1, f8) and np.array_equal(f1, flat)
    grads = [[inputs.normal_bf16(N, 1e-3, seed=(22, w, m)) for m in range(2)] for w in range(R)]
    a1, a8 = new_acc(S, R), new_acc(S, R)
    oracle.reset(a1, N, nthreads=1)
    oracle.reset(a8, N, nthreads=5)
    oracle.scatter_accumulate_ordered(grads, a1, N, nthreads=1)
    oracle.scatter_accumulate_ordered(grads, a8, N, nthreads=7)
    for x, y in zip(a1, a8):
        assert np.array_equal(bits32(x), bits32(y))


def test_sampled_ranges_touch_only_their_elements(oracle):
    """The flat-index range arguments (used for sampled checks at the largest shapes): inside
    the ranges the result equals the full computation, outside nothing is touched."""
    N, R = 10_007, 4
    S = -(-N // R)
    ranges = [(0, 5), (1200, 1210), (S - 3, S + 4), (N - 2, N)]
    inside = np.zeros(N, dtype=bool)
    for a, b in ranges:
        inside[a:b] = True
    flat = inputs.uniform_bf16(N, -1, 1, seed=51)
    shards = oracle.make_shards(flat, R)
    full = np.full(N, 0xBEEF, dtype=np.uint16)
    oracle.gather(shards, N, full, ranges=ranges)
    assert np.array_equal(full[inside], flat[inside]) and (full[~inside] == 0xBEEF).all()
    g = inputs.normal_bf16(N, 1e-3, seed=52)
    a_full, a_part = new_acc(S, R), new_acc(S, R)
    oracle.reset(a_full, N)
    oracle.accumulate(g, a_full, N)
    oracle.reset(a_part, N, ranges=ranges)
    oracle.accumulate(g, a_part, N, ranges=ranges)
    f, p = np.concatenate(a_full)[:N], np.concatenate(a_part)[:N]
    assert np.array_equal(bits32(f[inside]), bits32(p[inside]))
    assert (p[~inside] == PAD32).all()
    with pytest.raises(ValueError):
        oracle.gather(shards, N, full, ranges=[(5, N + 1)])
    with pytest.raises(ValueError):
        oracle.accumulate(g, a_part, N, ranges=[(0, 10), (9, 20)])


def test_batched_equals_per_tensor_numpy(oracle):
    """Batched forms against numpy slicing done here: tensor t of owner r sits at
    arena_r[off_t : off_t + S_t]; gaps between tensors and padding keep their sentinels."""
    R = 8
    numel = [1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63]
    T = len(numel)
    S = [-(-n // R) for n in numel]
    rng = np.random.default_rng(0)
    shard_off, full_off, a, f = [], [], 3, 1
    for t in range(T):          # arbitrary placement with gaps
        shard_off.append(a)
        full_off.append(f)
        a += S[t] + int(rng.integers(0, 5))
        f += numel[t] + int(rng.integers(0, 5))
    arena_len, full_len = a + 2, f + 2
    flats = [inputs.uniform_bf16(n, -1, 1, seed=(31, t)) for t, n in enumerate(numel)]
    arenas = [np.full(arena_len, PAD16, dtype=np.uint16) for _ in range(R)]
    for t, n in enumerate(numel):
        for r in range(R):
            lo, hi = r * S[t], min((r + 1) * S[t], n)
            if hi > lo:
                arenas[r][shard_off[t]:shard_off[t] + hi - lo] = flats[t][lo:hi]
    full = np.full(full_len, 0xBEEF, dtype=np.uint16)
    oracle.gather_batched(arenas, numel, shard_off, full_off, full)
    want = np.full(full_len, 0xBEEF, dtype=np.uint16)
    for t, n in enumerate(numel):
        want[full_off[t]:full_off[t] + n] = flats[t]
    assert np.array_equal(full, want)

    g1 = inputs.normal_bf16(full_len, 1e-2, seed=41)
    g2 = inputs.normal_bf16(full_len, 1e-2, seed=42)
    acc = [np.full(arena_len, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reset_batched(acc, numel, shard_off)
    oracle.accumulate_batched(g1, acc, numel, shard_off, full_off)
    oracle.accumulate_batched(g2, acc, numel, shard_off, full_off)
    want_acc = [np.full(arena_len, PAD32, dtype=np.float32) for _ in range(R)]
    for t, n in enumerate(numel):
        v1 = inputs.bf16_bits_to_f32(g1[full_off[t]:full_off[t] + n])
        v2 = inputs.bf16_bits_to_f32(g2[full_off[t]:full_off[t] + n])
        s = (np.float32(0) + v1) + v2         # numpy float32 adds, same order
        for r in range(R):
            lo, hi = r * S[t], min((r + 1) * S[t], n)
            if hi > lo:
                want_acc[r][shard_off[t]:shard_off[t] + hi - lo] = s[lo:hi]
    for r in range(R):
        assert np.array_equal(bits32(acc[r]), bits32(want_acc[r]))


def test_planted_mistakes_are_caught():
    """The pins must be able to tell a wrong oracle from a right one: three plausible
    mistakes, written here in numpy, each differ from the definition on these inputs."""
    N, R = 10, 4
    S = 3
    flat = np.arange(100, 100 + N, dtype=np.uint16)
    padded = np.zeros(R * S, dtype=np.uint16)
    padded[:N] = flat
    shards = [padded[r * S:(r + 1) * S] for r in range(R)]
    floor_S = N // R  # wrong partition rule (floor instead of ceil)
    wrong_partition = np.concatenate([s[:floor_S] for s in shards])
    assert not np.array_equal(wrong_partition[:N - 2], flat[:N - 2])
    transposed = np.stack(shards).T.reshape(-1)[:N]  # owner index fastest instead of slowest
    assert not np.array_equal(transposed, flat)
    # accumulating in microbatch-then-worker order changes a rounding-sensitive sum
    vals = {(0, 0): 2.0 ** -24, (0, 1): 1.0, (1, 0): 2.0 ** -24}
    wm = np.float32(0)
    for w in range(2):
        for m in range(2):
            wm = np.float32(wm + np.float32(vals.get((w, m), 0.0)))
    mw = np.float32(0)
    for m in range(2):
        for w in range(2):
            mw = np.float32(mw + np.float32(vals.get((w, m), 0.0)))
    assert wm != mw


def test_staging_model_is_ordered_accumulation_by_client(oracle):
    """The staging bookkeeping (Appendix B: one receive slot per client and owner) against
    plain ordered accumulation written out here: a drain adds the staged gradients in
    ascending client order; a push into a slot that is still full is refused."""
    N, R = 1001, 4
    S = -(-N // R)
    gs = {k: inputs.normal_bf16(N, 1e-3, seed=(70, k)) for k in range(5)}
    st = oracle.Staging([N], R)
    acc = new_acc(S, R)
    ref = new_acc(S, R)
    oracle.reset(acc, N)
    oracle.reset(ref, N)
    st.push(gs[0], 3)
    st.push(gs[1], 1)
    st.push(gs[2], 3)            # refused by every owner: slot (r, 3) is still full
    assert st.refused == R
    assert st.drain(acc) == 2 * R
    oracle.accumulate(gs[1], ref, N)   # client 1 before client 3
    oracle.accumulate(gs[0], ref, N)
    for a, b in zip(acc, ref):
        assert np.array_equal(bits32(a), bits32(b))
    assert st.drain(acc) == 0          # nothing staged: nothing changes
    st.push(gs[3], 3)
    st.push(gs[4], 0)
    st.drain(acc)
    oracle.accumulate(gs[4], ref, N)
    oracle.accumulate(gs[3], ref, N)
    for a, b in zip(acc, ref):
        assert np.array_equal(bits32(a), bits32(b))
    assert not any(any(row) for row in st.full)


def test_staging_model_phases(oracle):
    """The phased form of the staging bookkeeping, against outcomes written out by hand: the
    fate of a push is fixed when it begins (a slot that is full or being written refuses it as a
    whole, even if a drain empties the slot before the push ends), and a drain takes exactly
    the slots that were full when it began."""
    N, R = 1001, 4
    S = -(-N // R)
    gs = {k: inputs.normal_bf16(N, 1e-3, seed=(71, k)) for k in range(4)}

    def fresh():
        acc, ref = new_acc(S, R), new_acc(S, R)
        oracle.reset(acc, N)
        oracle.reset(ref, N)
        return oracle.Staging([N], R), acc, ref

    def same(acc, ref):
        return all(np.array_equal(bits32(a), bits32(b)) for a, b in zip(acc, ref))

    # a second push of one client begins while its slot is full; a drain runs before it ends
    st, acc, ref = fresh()
    st.push(gs[0], 0)
    st.begin_push(gs[1], 0)
    assert st.refused == R
    assert st.drain(acc) == R
    st.end_push(0)                       # ends a push that no owner took: nothing becomes full
    assert not any(any(row) for row in st.full)
    assert st.drain(acc) == 0
    oracle.accumulate(gs[0], ref, N)
    assert same(acc, ref)

    # a drain that begins while a push is being written leaves it for the next drain
    st, acc, ref = fresh()
    st.begin_push(gs[0], 2)
    st.begin_drain()
    st.end_push(2)
    assert st.add_noted(acc) == 0
    st.end_drain()
    assert same(acc, ref) and all(row[2] for row in st.full)
    assert st.drain(acc) == R
    oracle.accumulate(gs[0], ref, N)
    assert same(acc, ref)

    # a push that lands between a drain's beginning and its end is not emptied by that drain;
    # a client whose slot the drain has noted but not yet emptied is still refused
    st, acc, ref = fresh()
    st.push(gs[0], 0)
    st.begin_drain()
    st.push(gs[1], 1)
    st.begin_push(gs[2], 0)
    assert st.refused == R
    assert st.add_noted(acc) == R
    st.end_drain()
    st.end_push(0)
    assert [row[:2] for row in st.full] == [[False, True]] * R
    st.push(gs[3], 0)
    assert st.refused == R
    assert st.drain(acc) == 2 * R
    for k in (0, 3, 1):                  # first drain: client 0; second: client 0 before client 1
        oracle.accumulate(gs[k], ref, N)
    assert same(acc, ref)


def test_fp64_reference_is_the_exact_rational_sum_on_small_cases(oracle):
    """The float64 reference of the unordered mode against exact rational arithmetic: bf16 values
    of similar magnitude add without rounding in float64, so tot must equal the exact sum and mag
    the exact sum of magnitudes; elements outside the given ranges stay untouched."""
    from fractions import Fraction

    n, C = 64, 7
    gs = [inputs.normal_bf16(n, 1e-3, seed=(72, k)) for k in range(C)]
    tot, mag = np.zeros(n), np.zeros(n)
    for g in gs:
        oracle.fp64_add(g, tot, mag, nthreads=3)
    for j in range(n):
        vals = [Fraction(float(oracle.widen(g[j:j + 1])[0])) for g in gs]
        assert Fraction(float(tot[j])) == sum(vals)
        assert Fraction(float(mag[j])) == sum(abs(v) for v in vals)
    tot2, mag2 = np.zeros(n), np.zeros(n)
    oracle.fp64_add(gs[0], tot2, mag2, ranges=[(3, 9), (40, 41)])
    keep = np.zeros(n, dtype=bool)
    keep[3:9] = keep[40:41] = True
    assert (tot2[~keep] == 0).all() and np.array_equal(tot2[keep], oracle.widen(gs[0]).astype(np.float64)[keep])
