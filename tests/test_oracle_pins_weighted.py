"""Pins for the oracle's weighted contribution (Section 2.1, w_m != 1) and minibatch-end
retrieval (Section 3.2).  As in test_oracle_pins.py nothing here retypes the oracle: the
references are exact rational arithmetic, special cases that reduce to the unweighted path,
and torch's own float32 -> bfloat16 conversion."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2601_19362_amd import inputs

PAD32 = np.float32(-12345.678)


def bits32(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def new_acc(S, R, fill=PAD32):
    return [np.full(S, fill, dtype=np.float32) for _ in range(R)]


def round_to_f32(x: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) binary32 value of an exact rational, found by
    comparing the two neighbouring float32 values exactly."""
    c = np.float32(float(x))                      # close; may be off by one ulp (double rounding)
    cands = {c, np.nextafter(c, np.float32(np.inf)), np.nextafter(c, np.float32(-np.inf))}
    best = None
    for f in cands:
        d = abs(Fraction(float(f)) - x)
        even = (int(np.array([f], dtype=np.float32).view(np.uint32)[0]) & 1) == 0
        key = (d, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, f)
    return best[1]


def test_weighted_equals_exact_rational_fma(oracle):
    """acc' = round32(w * g + acc) with a single rounding, checked with exact fractions."""
    rng = np.random.default_rng(11)
    N, R = 37, 4
    S = -(-N // R)
    g = inputs.normal_bf16(N, 1.0, seed=5)
    start = rng.standard_normal(R * S).astype(np.float32)
    for w in (np.float32(0.3), np.float32(-1.7), np.float32(1.0) + np.float32(2.0 ** -23), np.float32(1 / 3)):
        acc = [start[r * S:(r + 1) * S].copy() for r in range(R)]
        oracle.accumulate_weighted(g, acc, N, w)
        got = np.concatenate(acc)
        gv = inputs.bf16_bits_to_f32(g)
        for j in range(N):
            exact = Fraction(float(w)) * Fraction(float(gv[j])) + Fraction(float(start[j]))
            want = round_to_f32(exact)
            assert bits32(got[j:j + 1])[0] == bits32(np.array([want]))[0], (j, w)
        assert np.array_equal(bits32(got[N:]), bits32(start[N:]))   # padding slots untouched


def test_weighted_is_fused_not_multiply_then_add(oracle):
    """w = 1 + 2^-23, g = 1 + 2^-7, acc = -(1 + 2^-7 + 2^-23): the exact w*g + acc is 2^-30;
    rounding the product first would lose that term and give 0."""
    w = np.float32(1.0) + np.float32(2.0 ** -23)
    g = inputs.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -7], dtype=np.float32))
    assert inputs.bf16_bits_to_f32(g)[0] == np.float32(1.0 + 2.0 ** -7)
    acc = [np.array([-(1.0 + 2.0 ** -7 + 2.0 ** -23)], dtype=np.float32)]
    oracle.accumulate_weighted(g, acc, 1, w)
    assert acc[0][0] == np.float32(2.0 ** -30)
    assert np.float32(np.float32(w * inputs.bf16_bits_to_f32(g)[0]) + np.float32(-(1.0 + 2.0 ** -7 + 2.0 ** -23))) == 0


def test_weight_one_is_the_unweighted_contribution(oracle):
    N, R = 5003, 8
    S = -(-N // R)
    a1, a2 = new_acc(S, R), new_acc(S, R)
    oracle.reset(a1, N)
    oracle.reset(a2, N)
    for k in range(3):
        g = inputs.normal_bf16(N, 1e-3, seed=(8, k))
        oracle.accumulate(g, a1, N)
        oracle.accumulate_weighted(g, a2, N, 1.0)
    for x, y in zip(a1, a2):
        assert np.array_equal(bits32(x), bits32(y))


def test_power_of_two_weight_scales_exactly(oracle):
    """w = 2^k: w*g is exact, so the result is the unweighted sum of the scaled gradient."""
    N, R = 1001, 4
    S = -(-N // R)
    g = inputs.normal_bf16(N, 1e-3, seed=9)
    for w in (0.5, 4.0, 2.0 ** -6):
        a1, a2 = new_acc(S, R), new_acc(S, R)
        oracle.reset(a1, N)
        oracle.reset(a2, N)
        oracle.accumulate(inputs.normal_bf16(N, 1e-3, seed=10), a1, N)
        oracle.accumulate(inputs.normal_bf16(N, 1e-3, seed=10), a2, N)
        oracle.accumulate_weighted(g, a1, N, w)
        scaled = inputs.f32_to_bf16_bits(inputs.bf16_bits_to_f32(g) * np.float32(w))
        assert np.array_equal(inputs.bf16_bits_to_f32(scaled), inputs.bf16_bits_to_f32(g) * np.float32(w))
        oracle.accumulate(scaled, a2, N)
        for x, y in zip(a1, a2):
            assert np.array_equal(bits32(x), bits32(y))


def test_retrieve_f32(oracle):
    N, R = 1003, 4
    S = -(-N // R)
    rng = np.random.default_rng(3)
    acc = [rng.standard_normal(S).astype(np.float32) for _ in range(R)]
    before = [a.copy() for a in acc]
    out = new_acc(S, R)
    oracle.retrieve(acc, out, N, scale=1.0)
    flat_acc, flat_out = np.concatenate(acc), np.concatenate(out)
    assert np.array_equal(bits32(flat_out[:N]), bits32(flat_acc[:N]))       # scale 1: a bit copy
    assert (flat_out[N:] == PAD32).all()                                    # output padding untouched
    for a, b in zip(acc, before):
        assert np.array_equal(bits32(a), bits32(b))                         # accumulators unchanged
    out = new_acc(S, R)
    oracle.retrieve(acc, out, N, scale=1.0 / 3.0)
    want = flat_acc[:N] * np.float32(1.0 / 3.0)                             # numpy float32 multiply
    assert np.array_equal(bits32(np.concatenate(out)[:N]), bits32(want))


def test_retrieve_bf16_matches_torch_rounding_and_hand_ties(oracle):
    import torch

    N, R = 4099, 4
    S = -(-N // R)
    rng = np.random.default_rng(4)
    vals = (rng.standard_normal(R * S) * 1e-2).astype(np.float32)
    vals[:6] = [1.00390625, 1.01171875, -1.00390625, 0.0, -0.0, 3.0e38]   # two ties, zeros, near-overflow
    acc = [vals[r * S:(r + 1) * S].copy() for r in range(R)]
    out = [np.full(S, 0xDEAD, dtype=np.uint16) for _ in range(R)]
    oracle.retrieve(acc, out, N, scale=1.0)
    got = np.concatenate(out)
    want = torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got[:N], want[:N])
    assert got[:5].tolist() == [0x3F80, 0x3F82, 0xBF80, 0x0000, 0x8000]
    assert (got[N:] == 0xDEAD).all()
    # scaled: one binary32 multiply, then one rounding to bf16
    out = [np.full(S, 0xDEAD, dtype=np.uint16) for _ in range(R)]
    oracle.retrieve(acc, out, N, scale=0.125)
    want = torch.from_numpy(vals * np.float32(0.125)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(np.concatenate(out)[:N], want[:N])
    # NaN stays NaN, infinities keep their sign
    acc = [np.array([np.nan, np.inf, -np.inf, 1.0], dtype=np.float32)]
    out = [np.zeros(4, dtype=np.uint16)]
    oracle.retrieve(acc, out, 4, scale=1.0)
    back = inputs.bf16_bits_to_f32(out[0])
    assert np.isnan(back[0]) and back[1] == np.inf and back[2] == -np.inf and back[3] == 1.0


def test_weighted_and_retrieve_batched_match_numpy(oracle):
    R = 8
    numel = [1, 5, 8, 9, 64, 100, 777, 3, 4096, 63]
    S = [-(-n // R) for n in numel]
    so, fo, a, f = [], [], 0, 0
    for n, s in zip(numel, S):
        so.append(a)
        fo.append(f)
        a += (s + 7) // 8 * 8
        f += (n + 7) // 8 * 8
    arena, full_n = so[-1] + S[-1], fo[-1] + numel[-1]
    g = inputs.normal_bf16(full_n, 1e-2, seed=61)
    w = np.float32(0.37)
    acc = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reset_batched(acc, numel, so)
    oracle.accumulate_weighted_batched(g, acc, numel, so, fo, w)
    oracle.accumulate_weighted_batched(g, acc, numel, so, fo, 2.0)
    want = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    for t, n in enumerate(numel):
        gv = inputs.bf16_bits_to_f32(g[fo[t]:fo[t] + n]).astype(np.float64)
        first = (np.float64(w) * gv).astype(np.float32)      # exact product fits in float64, one rounding
        second = (2.0 * gv + first.astype(np.float64)).astype(np.float32)   # exact in float64: one rounding
        for r in range(R):
            lo, hi = r * S[t], min((r + 1) * S[t], n)
            if hi > lo:
                want[r][so[t]:so[t] + hi - lo] = second[lo:hi]
    for r in range(R):
        assert np.array_equal(bits32(acc[r]), bits32(want[r]))
    for dtype, cast in ((np.float32, lambda v: v), (np.uint16, inputs.f32_to_bf16_bits)):
        out = [np.full(arena, 7, dtype=dtype) for _ in range(R)]
        oracle.retrieve_batched(acc, out, numel, so, scale=0.25)
        for r in range(R):
            w_out = np.full(arena, 7, dtype=dtype)
            for t, n in enumerate(numel):
                valid = max(0, min(S[t], n - r * S[t]))
                w_out[so[t]:so[t] + valid] = cast(acc[r][so[t]:so[t] + valid] * np.float32(0.25))
            assert np.array_equal(out[r].view(np.uint32 if dtype == np.float32 else np.uint16),
                                  w_out.view(np.uint32 if dtype == np.float32 else np.uint16))
