"""Pins of the oracle's wide (binary64) accumulators for the unordered mode: exact rational
arithmetic on small cases, the adversarial sequence on which a binary32 accumulator misses the
1e-6 tolerance and the wide one does not, numpy's own float64 -> float32 rounding, sentinels."""
from fractions import Fraction

import numpy as np

from paper_2601_19362_amd import inputs

PAD64 = -9876.5


def test_wide_accumulate_is_the_exact_sum_on_small_cases(oracle):
    N, R, C = 37, 4, 9
    S = oracle.shard_elems(N, R)
    gs = [inputs.normal_bf16(N, 1e-3, seed=(73, k)) for k in range(C)]
    acc = [np.full(S, PAD64, dtype=np.float64) for _ in range(R)]
    oracle.reset_wide(acc, N)
    for g in gs:
        oracle.accumulate_wide(g, acc, N)
    for j in range(N):
        exact = sum(Fraction(float(oracle.widen(g[j:j + 1])[0])) for g in gs)
        assert Fraction(float(acc[j // S][j % S])) == exact      # no rounding happens at this magnitude
    for r in range(R):
        v = oracle.valid_elems(N, R, r)
        assert (acc[r][v:] == PAD64).all()                       # padding never written


def adversarial(N, C):
    """1.0 first, then C - 1 contributions of 2^-17 + 2^-24 (exact in bf16): every binary32 addition
    is a tie that rounds the 2^-24 away."""
    big = inputs.f32_to_bf16_bits(np.full(N, 1.0, dtype=np.float32))
    small = inputs.f32_to_bf16_bits(np.full(N, 2.0 ** -17 + 2.0 ** -24, dtype=np.float32))
    assert inputs.bf16_bits_to_f32(small)[0] == np.float32(2.0 ** -17 + 2.0 ** -24)
    return [big] + [small] * (C - 1)


def test_wide_accumulator_keeps_the_tolerance_where_binary32_cannot(oracle):
    N, R, C = 64, 2, 272
    S = oracle.shard_elems(N, R)
    seq = adversarial(N, C)
    exact = Fraction(1) + (C - 1) * (Fraction(1, 2 ** 17) + Fraction(1, 2 ** 24))
    mag = float(exact)                                           # all terms positive: sum|g| = the sum
    acc32 = [np.zeros(S, dtype=np.float32) for _ in range(R)]
    acc64 = [np.zeros(S, dtype=np.float64) for _ in range(R)]
    for g in seq:
        oracle.accumulate(g, acc32, N)
        oracle.accumulate_wide(g, acc64, N)
    err32 = abs(Fraction(float(acc32[0][0])) - exact)
    assert float(err32) > 1e-6 * mag                             # (C - 1) * 2^-24 lost: 1.6e-5
    assert Fraction(float(acc64[0][0])) == exact                 # binary64 holds it exactly
    out = [np.zeros(S, dtype=np.float32) for _ in range(R)]
    oracle.retrieve_wide(acc64, out, N)
    err = abs(Fraction(float(out[0][0])) - exact)
    assert float(err) <= 2.0 ** -24 * mag                        # one rounding to binary32


def test_retrieve_wide_rounds_once_to_binary32_then_as_the_binary32_retrieval(oracle):
    N, R = 1001, 3
    S = oracle.shard_elems(N, R)
    rng = np.random.default_rng(4)
    vals = rng.standard_normal(R * S) * 1e-3
    vals[:6] = [0.0, -0.0, 1.0 + 2.0 ** -24, 1.0 + 2.0 ** -24 + 2.0 ** -40, 3.0e-39, -1.0e300]   # tie, above tie, subnormal, overflow
    acc64 = [vals[r * S:(r + 1) * S].copy() for r in range(R)]
    scale = float(np.float32(1.0 / 3.0))
    out32 = [np.full(S, 77.0, dtype=np.float32) for _ in range(R)]
    out16 = [np.full(S, 0xDEAD, dtype=np.uint16) for _ in range(R)]
    oracle.retrieve_wide(acc64, out32, N, scale=scale)
    oracle.retrieve_wide(acc64, out16, N, scale=scale)
    with np.errstate(over="ignore"):
        narrow = [a.astype(np.float32) for a in acc64]           # numpy rounds to nearest even
    assert narrow[0][2] == np.float32(1.0) and narrow[0][3] == np.float32(1.0 + 2.0 ** -23)
    want32 = [np.full(S, 77.0, dtype=np.float32) for _ in range(R)]
    want16 = [np.full(S, 0xDEAD, dtype=np.uint16) for _ in range(R)]
    oracle.retrieve(narrow, want32, N, scale=scale)              # the binary32 retrieval, pinned elsewhere
    oracle.retrieve(narrow, want16, N, scale=scale)
    for r in range(R):
        assert np.array_equal(out32[r].view(np.uint32), want32[r].view(np.uint32))
        assert np.array_equal(out16[r], want16[r])
        v = oracle.valid_elems(N, R, r)
        assert (out32[r][v:] == 77.0).all() and (out16[r][v:] == 0xDEAD).all()
    assert np.isinf(out32[0][5]) and out32[0][5] < 0


def test_wide_accumulate_equals_the_float64_reference_and_splits_over_threads(oracle):
    N, R, C = 50_003, 8, 12
    S = oracle.shard_elems(N, R)
    gs = [inputs.normal_bf16(N, 1e-3, seed=(74, k)) for k in range(C)]
    a1 = [np.zeros(S, dtype=np.float64) for _ in range(R)]
    a2 = [np.zeros(S, dtype=np.float64) for _ in range(R)]
    tot, mag = np.zeros(N), np.zeros(N)
    for g in gs:
        oracle.accumulate_wide(g, a1, N)
        oracle.accumulate_wide(g, a2, N, nthreads=5)
        oracle.fp64_add(g, tot, mag)
    flat = np.concatenate(a1)[:N]
    assert np.array_equal(flat, tot) and np.array_equal(np.concatenate(a2)[:N], tot)
