"""Seeded synthetic inputs for the ODC gather / scatter-accumulate path.

This module serves both the HIP path and the CPU oracle and therefore holds none of
the method's arithmetic: no partition rule, no copy, no accumulation.  It only draws
random bf16 bit patterns, per-rank microbatch counts and tensor sizes with the shapes
and distributions of the five workloads, which stand in for the paper's models
(DeepSeek-R1-Distill-Qwen 1.5B to 32B, Section 5.1) and for its long-tailed
sequence-length histograms (the sequence-length distribution figure of Section 5.1).

bf16 values travel as raw 16-bit patterns: numpy uint16 on the host, torch.bfloat16 on
the device (bit-identical after a view).  float32 -> bf16 uses round-to-nearest-even
and is input preparation, outside the path under test.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

HEAD_DIM = 128


# ----------------------------------------------------------------------------- bit helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed) -> np.random.Generator:
    # Philox is counter-based: a (seed, stream) pair names the sequence on any machine.
    if isinstance(seed, (tuple, list)):
        key = 0
        for s in seed:
            key = (key * 1_000_003 + int(s) + 1) % (1 << 64)
    else:
        key = int(seed)
    return np.random.Generator(np.random.Philox(key=key))


def uniform_bf16(n: int, lo: float, hi: float, seed) -> np.ndarray:
    """n bf16 bit patterns ~ Uniform[lo, hi) drawn in float32, then rounded."""
    r = _rng(seed)
    x = r.random(n, dtype=np.float32)
    x *= np.float32(hi - lo)
    x += np.float32(lo)
    return f32_to_bf16_bits(x)


def normal_bf16(n: int, sigma: float, seed) -> np.ndarray:
    """n bf16 bit patterns ~ Normal(0, sigma) (sigma = standard deviation)."""
    r = _rng(seed)
    x = r.standard_normal(n, dtype=np.float32)
    x *= np.float32(sigma)
    return f32_to_bf16_bits(x)


def device_uniform_bf16(n: int, lo: float, hi: float, seed: int, device):
    """Same distribution drawn on the device with torch's seeded generator (bf16 tensor).

    Used for the large resident buffers of the model-shaped workloads; a test that needs
    the oracle copies the tensor to the host, so both sides consume identical bits.
    """
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    out = torch.empty(n, dtype=torch.float32, device=device)
    out.uniform_(lo, hi, generator=g)
    return out.to(torch.bfloat16)


def device_normal_bf16(n: int, sigma: float, seed: int, device):
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    out = torch.empty(n, dtype=torch.float32, device=device)
    out.normal_(0.0, sigma, generator=g)
    return out.to(torch.bfloat16)


# ----------------------------------------------------------------------------- workloads
def decoder_layer_numel(hidden: int, ffn: int, q_heads: int, kv_heads: int) -> int:
    """Parameters of one decoder layer flattened into one flat param: q, k, v, o
    projections, gate/up/down MLP matrices and two RMSNorm vectors, no biases."""
    q = hidden * q_heads * HEAD_DIM
    kv = hidden * kv_heads * HEAD_DIM
    return 2 * q + 2 * kv + 3 * hidden * ffn + 2 * hidden


def decoder_layer_tensors(hidden: int, ffn: int, q_heads: int, kv_heads: int) -> Tuple[int, ...]:
    """The same layer kept as separate tensors (per-parameter sharding instead of one flat
    param): q, k, v, o, gate, up, down, two RMSNorm vectors."""
    q = hidden * q_heads * HEAD_DIM
    kv = hidden * kv_heads * HEAD_DIM
    return (q, kv, kv, q, hidden * ffn, hidden * ffn, hidden * ffn, hidden, hidden)


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration.  `numel` lists the flat params that one layout
    covers (one entry for a layer-shaped config, 10,000 for the stress test); `layers`
    is how many such parameter sets a minibatch touches; `resident_layers` how many
    of them are kept in HBM at once."""
    name: str
    R: int
    numel: Tuple[int, ...]
    layers: int
    resident_layers: int
    param_range: Tuple[float, float]
    grad_sigma: float
    seed: int
    microbatch_rule: str
    note: str = ""

    @property
    def T(self) -> int:
        return len(self.numel)

    @property
    def total_numel(self) -> int:
        return int(sum(self.numel))


def stress_tensor_sizes(T: int = 10_000, seed: int = 5) -> Tuple[int, ...]:
    """Sizes log-uniform in [1, 65536]: floor(exp(U * ln 65537)) clipped to the range."""
    u = _rng((seed, 101)).random(T)
    n = np.floor(np.exp(u * math.log(65537.0))).astype(np.int64)
    return tuple(int(v) for v in np.clip(n, 1, 65536))


def _long_tail_microbatches(R: int, seed: int, samples_per_rank: int = 16,
                            cap_tokens: int = 16384) -> List[int]:
    """Per-rank microbatch counts from a long-tailed length law.

    Lengths = clip(round(exp(7 + Z)), 128, 32768), Z ~ N(0, 1); every rank receives
    `samples_per_rank` samples at random (no balancing across ranks, which is what makes
    the counts differ) and packs them first-fit-decreasing into microbatches of at most
    `cap_tokens` tokens; a sample longer than the cap forms a microbatch alone.
    """
    r = _rng((seed, 303))
    counts = []
    for _ in range(R):
        z = r.standard_normal(samples_per_rank)
        lens = np.clip(np.rint(np.exp(7.0 + z)), 128, 32768).astype(np.int64)
        bins: List[int] = []
        for L in sorted((int(v) for v in lens), reverse=True):
            for k in range(len(bins)):
                if bins[k] + L <= cap_tokens:
                    bins[k] += L
                    break
            else:
                bins.append(L)
        counts.append(len(bins))
    return counts


def microbatch_counts(w: Workload) -> List[int]:
    """M_w for every logical rank (a property of the minibatch, equal for all layers)."""
    rule = w.microbatch_rule
    if rule.startswith("const:"):
        return [int(rule.split(":")[1])] * w.R
    if rule.startswith("uniform:"):
        lo, hi = (int(v) for v in rule.split(":")[1].split(","))
        r = _rng((w.seed, 202))
        return [int(v) for v in r.integers(lo, hi + 1, size=w.R)]
    if rule == "longtail":
        return _long_tail_microbatches(w.R, w.seed)
    raise ValueError(f"unknown microbatch rule {rule!r}")


def _cfg_tiny() -> Workload:
    return Workload("tiny", R=4, numel=(1_048_589,), layers=1, resident_layers=1,
                    param_range=(-0.05, 0.05), grad_sigma=1e-3, seed=0,
                    microbatch_rule="const:2",
                    note="R does not divide N: tail padding and 8-byte-misaligned shard boundaries")


def _cfg_1p5b() -> Workload:
    n = decoder_layer_numel(1536, 8960, 12, 2)
    return Workload("1.5b", R=8, numel=(n,), layers=28, resident_layers=28,
                    param_range=(-0.05, 0.05), grad_sigma=1e-3, seed=2,
                    microbatch_rule="uniform:1,8")


def _cfg_7b() -> Workload:
    n = decoder_layer_numel(3584, 18944, 28, 4)
    return Workload("7b", R=16, numel=(n,), layers=28, resident_layers=28,
                    param_range=(-0.05, 0.05), grad_sigma=1e-3, seed=3,
                    microbatch_rule="longtail")


def _cfg_7b_split() -> Workload:
    """The 7B-shaped workload with every layer kept as nine tensors in one multi-tensor layout
    (same elements, same ranks, same microbatch counts as "7b")."""
    return Workload("7b-split", R=16, numel=decoder_layer_tensors(3584, 18944, 28, 4), layers=28, resident_layers=28,
                    param_range=(-0.05, 0.05), grad_sigma=1e-3, seed=3, microbatch_rule="longtail",
                    note="per-parameter sharding: nine tensors per layer, batched kernels")


def _cfg_32b() -> Workload:
    n = decoder_layer_numel(5120, 27648, 40, 8)
    return Workload("32b", R=32, numel=(n,), layers=64, resident_layers=4,
                    param_range=(-0.05, 0.05), grad_sigma=1e-3, seed=4,
                    microbatch_rule="uniform:1,16",
                    note="rotating window of 4 resident layers")


def _cfg_stress() -> Workload:
    return Workload("stress", R=64, numel=stress_tensor_sizes(), layers=1, resident_layers=1,
                    param_range=(-1.0, 1.0), grad_sigma=1e-2, seed=5,
                    microbatch_rule="uniform:1,4",
                    note="10,000 small flat params, one batched launch per phase")


_BUILDERS = {"tiny": _cfg_tiny, "1.5b": _cfg_1p5b, "7b": _cfg_7b, "32b": _cfg_32b,
             "stress": _cfg_stress, "7b-split": _cfg_7b_split}
WORKLOAD_NAMES = tuple(_BUILDERS)


def workload(name: str) -> Workload:
    try:
        return _BUILDERS[name]()
    except KeyError:
        raise ValueError(f"unknown workload {name!r}; choose from {WORKLOAD_NAMES}") from None


def grad_seed(w: Workload, layer: int, worker: int, microbatch: int):
    """Seed tuple naming the gradient of contribution (layer, worker, microbatch)."""
    return (w.seed, 7, layer, worker, microbatch)


def param_seed(w: Workload, layer: int):
    return (w.seed, 11, layer)
