"""Checks of the seeded input generators (no method arithmetic lives there)."""
import numpy as np
import pytest

from paper_2601_19362_amd import inputs


def test_bf16_rounding_matches_torch_and_hand_cases():
    import torch

    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(100_000).astype(np.float32) * 1e-3,
                        rng.uniform(-1, 1, 100_000).astype(np.float32),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, 1e-40],
                                 dtype=np.float32)])
    mine = inputs.f32_to_bf16_bits(x)
    theirs = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(mine, theirs)
    # ties: 1 + 2^-8 is halfway between bf16 neighbours 1.0 (even) and 1 + 2^-7 -> 1.0;
    # 1 + 3*2^-8 is halfway between 1 + 2^-7 (odd) and 1 + 2^-6 (even) -> 1 + 2^-6
    assert inputs.f32_to_bf16_bits(np.array([1.00390625], np.float32))[0] == 0x3F80
    assert inputs.f32_to_bf16_bits(np.array([1.01171875], np.float32))[0] == 0x3F82
    back = inputs.bf16_bits_to_f32(mine)
    assert np.array_equal(back.view(np.uint32), mine.astype(np.uint32) << 16)


def test_generators_are_seeded_and_shaped():
    a = inputs.uniform_bf16(10_000, -0.05, 0.05, seed=(1, 2))
    b = inputs.uniform_bf16(10_000, -0.05, 0.05, seed=(1, 2))
    c = inputs.uniform_bf16(10_000, -0.05, 0.05, seed=(1, 3))
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    v = inputs.bf16_bits_to_f32(a)
    assert v.min() >= -0.0501 and v.max() <= 0.0501 and abs(v.mean()) < 2e-3
    g = inputs.bf16_bits_to_f32(inputs.normal_bf16(200_000, 1e-3, seed=4))
    assert abs(g.std() - 1e-3) < 2e-5 and abs(g.mean()) < 2e-5


def test_workload_shapes():
    assert inputs.workload("tiny").numel == (1_048_589,)
    assert inputs.workload("1.5b").numel == (46_795_776,) and inputs.workload("1.5b").R == 8
    assert inputs.workload("7b").numel == (233_053_184,) and inputs.workload("7b").R == 16
    w32 = inputs.workload("32b")
    assert w32.numel == (487_598_080,) and w32.R == 32 and w32.layers == 64
    assert w32.resident_layers == 4
    s = inputs.workload("stress")
    assert s.T == 10_000 and s.R == 64
    n = np.array(s.numel)
    assert n.min() >= 1 and n.max() <= 65536
    # log-uniform: about as many sizes below 256 as above
    assert 0.4 < (n < 256).mean() < 0.6
    assert s.numel == inputs.workload("stress").numel
    with pytest.raises(ValueError):
        inputs.workload("nope")


def test_microbatch_counts():
    assert inputs.microbatch_counts(inputs.workload("tiny")) == [2, 2, 2, 2]
    m = inputs.microbatch_counts(inputs.workload("1.5b"))
    assert len(m) == 8 and all(1 <= v <= 8 for v in m) and len(set(m)) > 1
    m = inputs.microbatch_counts(inputs.workload("32b"))
    assert len(m) == 32 and all(1 <= v <= 16 for v in m)
    m = inputs.microbatch_counts(inputs.workload("stress"))
    assert len(m) == 64 and all(1 <= v <= 4 for v in m)
    m7 = inputs.microbatch_counts(inputs.workload("7b"))
    assert len(m7) == 16 and all(v >= 1 for v in m7) and len(set(m7)) > 1   # imbalanced
    assert m7 == inputs.microbatch_counts(inputs.workload("7b"))


def test_split_layer_workload_matches_the_flat_one():
    flat, split = inputs.workload("7b"), inputs.workload("7b-split")
    assert sum(split.numel) == flat.numel[0] and len(split.numel) == 9
    assert split.numel == inputs.decoder_layer_tensors(3584, 18944, 28, 4)
    assert (split.R, split.layers) == (flat.R, flat.layers)
    assert inputs.microbatch_counts(split) == inputs.microbatch_counts(flat)
