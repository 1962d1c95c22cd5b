"""Pins of the oracle's hybrid-sharding step (Section 6.1, Appendix E): the sum of the groups'
gradient shards at the minibatch end.  None of them retypes the oracle's loop: exact integer
sums, an order-sensitive rounding case worked by hand, the K = 1 copy, the equivalence with
full sharding that the section claims (same training semantics), a float64 bound, sentinels."""
import numpy as np

from paper_2601_19362_amd import inputs

PAD32 = np.float32(-12345.678)


def bits32(a):
    return a.view(np.uint32)


def shards_of(values, R, S, N):
    """Cut a flat float32 vector into R shards of S slots; padding holds a sentinel."""
    out = []
    for r in range(R):
        sh = np.full(S, PAD32, dtype=np.float32)
        v = max(0, min(S, N - r * S))
        sh[:v] = values[r * S:r * S + v]
        out.append(sh)
    return out


def test_reduce_groups_exact_integers_and_padding(oracle):
    N, R, K = 1003, 4, 5
    S = oracle.shard_elems(N, R)
    rng = np.random.default_rng(0)
    ints = [rng.integers(-1000, 1001, size=N) for _ in range(K)]
    groups = [shards_of(v.astype(np.float32), R, S, N) for v in ints]
    out = [np.full(S, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reduce_groups(groups, out, N)
    total = sum(ints)
    for r in range(R):
        v = oracle.valid_elems(N, R, r)
        assert np.array_equal(out[r][:v], total[r * S:r * S + v].astype(np.float32))
        assert (out[r][v:] == PAD32).all()                  # padding never written
    for k in range(K):                                       # sources untouched
        for r in range(R):
            assert np.array_equal(bits32(groups[k][r]), bits32(shards_of(ints[k].astype(np.float32), R, S, N)[r]))


def test_reduce_groups_order_is_ascending_group_order(oracle):
    """1 + 2^-24 is a tie that rounds to even (1.0), so (1, 2^-24, 2^-24) summed left to right
    stays 1.0, while any order that meets the two small terms first gives 1 + 2^-23."""
    N, R = 8, 2
    S = 4
    tiny = np.float32(2.0 ** -24)
    one = np.float32(1.0)
    mk = lambda x: shards_of(np.full(N, x, dtype=np.float32), R, S, N)
    out = [np.zeros(S, dtype=np.float32) for _ in range(R)]
    oracle.reduce_groups([mk(one), mk(tiny), mk(tiny)], out, N)
    assert all((o == one).all() for o in out)
    oracle.reduce_groups([mk(tiny), mk(tiny), mk(one)], out, N)
    assert all((o == np.float32(1.0 + 2.0 ** -23)).all() for o in out)
    # a pairwise tree over four groups would differ from the sequential sum here
    oracle.reduce_groups([mk(one), mk(tiny), mk(tiny), mk(tiny)], out, N)
    assert all((o == one).all() for o in out)


def test_reduce_groups_single_group_is_a_copy_and_in_place_sum(oracle):
    N, R = 37, 3
    S = oracle.shard_elems(N, R)
    special = np.array([0x80000000, 0x00000001, 0x7F800000, 0xFF800000, 0x3F800000, 0x00000000], dtype=np.uint32)
    vals = special[np.arange(N) % special.size].view(np.float32)
    g0 = shards_of(vals, R, S, N)
    out = [np.full(S, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reduce_groups([g0], out, N)
    for r in range(R):
        v = oracle.valid_elems(N, R, r)
        assert np.array_equal(bits32(out[r][:v]), bits32(g0[r][:v]))     # bits, including -0 and subnormals
    # in place: the output is group 0's shards
    a = shards_of(np.arange(N, dtype=np.float32), R, S, N)
    b = shards_of(np.full(N, 0.5, dtype=np.float32), R, S, N)
    oracle.reduce_groups([a, b], a, N)
    for r in range(R):
        v = oracle.valid_elems(N, R, r)
        assert np.array_equal(a[r][:v], np.arange(r * S, r * S + v, dtype=np.float32) + np.float32(0.5))
        assert (a[r][v:] == PAD32).all()


def test_hybrid_sharding_equals_full_sharding_on_integer_gradients(oracle):
    """Section 6.1 changes where shards live, not what is computed: with gradients whose sums
    are exact, W = K*G workers under full sharding (R = W owners) and the same workers under
    hybrid sharding (K groups of G owners, worker w in group w // G, then the groups reduced)
    give the same gradient at every flat index."""
    N, G, K = 1001, 4, 3
    W = G * K
    rng = np.random.default_rng(1)
    grads = [inputs.f32_to_bf16_bits(rng.integers(-200, 201, size=N).astype(np.float32)) for _ in range(W)]
    S_full = oracle.shard_elems(N, W)
    full = [np.full(S_full, PAD32, dtype=np.float32) for _ in range(W)]
    oracle.reset(full, N)
    for w in range(W):
        oracle.accumulate(grads[w], full, N)
    S = oracle.shard_elems(N, G)
    groups = []
    for k in range(K):
        acc = [np.full(S, PAD32, dtype=np.float32) for _ in range(G)]
        oracle.reset(acc, N)
        for w in range(k * G, (k + 1) * G):
            oracle.accumulate(grads[w], acc, N)
        groups.append(acc)
    oracle.reduce_groups(groups, groups[0], N)
    flat_full = np.concatenate(full)[:N]
    flat_hybrid = np.concatenate(groups[0])[:N]
    assert np.array_equal(flat_full, flat_hybrid)
    assert np.array_equal(flat_full, sum(inputs.bf16_bits_to_f32(g).astype(np.float64) for g in grads).astype(np.float32))


def test_reduce_groups_within_the_sequential_bound_of_a_float64_sum(oracle):
    N, R, K = 4099, 8, 16
    S = oracle.shard_elems(N, R)
    rng = np.random.default_rng(2)
    vals = [rng.standard_normal(N).astype(np.float32) * np.float32(1e-3) for _ in range(K)]
    groups = [shards_of(v, R, S, N) for v in vals]
    out = [np.zeros(S, dtype=np.float32) for _ in range(R)]
    oracle.reduce_groups(groups, out, N, nthreads=3)
    got = np.concatenate(out)[:N].astype(np.float64)
    ref = sum(v.astype(np.float64) for v in vals)
    mag = sum(np.abs(v.astype(np.float64)) for v in vals)
    assert (np.abs(got - ref) <= (K - 1) * 2.0 ** -24 * mag).all()
    assert np.abs(got - ref).max() > 0                      # it is a binary32 sum, not the float64 one


def test_reduce_groups_batched_is_per_tensor_slicing(oracle):
    numel, R, K = [5, 1000, 1, 77], 4, 3
    S = [-(-n // R) for n in numel]
    so = [0, 8, 264, 272]
    arena = so[-1] + S[-1]
    rng = np.random.default_rng(3)
    groups = [[rng.standard_normal(arena).astype(np.float32) for _ in range(R)] for _ in range(K)]
    out = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reduce_groups_batched(groups, out, numel, so)
    want = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    for t, n in enumerate(numel):
        views_g = [[a[so[t]:so[t] + S[t]] for a in grp] for grp in groups]
        views_o = [a[so[t]:so[t] + S[t]] for a in want]
        oracle.reduce_groups(views_g, views_o, n)
    for r in range(R):
        assert np.array_equal(bits32(out[r]), bits32(want[r]))
        touched = np.zeros(arena, dtype=bool)
        for t, n in enumerate(numel):
            v = max(0, min(S[t], n - r * S[t]))
            touched[so[t]:so[t] + v] = True
        assert (out[r][~touched] == PAD32).all() and (out[r][touched] != PAD32).all()
