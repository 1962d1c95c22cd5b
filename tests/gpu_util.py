"""Helpers shared by the GPU parity tests: device buffers with sentinels around them and
comparisons against the CPU oracle.  bf16 data are numpy uint16 / torch int16 bit patterns."""
from __future__ import annotations

import numpy as np
import torch

from paper_2601_19362_amd import binding as odc

PAD16 = 0xDEAD
FULL16 = 0xBEEF
PAD32 = np.float32(-12345.678)
GUARD = 64  # guard elements placed before and after every device buffer


def to_dev_u16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def to_host_u16(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


class Guarded:
    """A device buffer of n elements inside a larger allocation whose GUARD-element margins
    hold a known pattern; `check()` asserts nothing wrote outside the buffer."""

    def __init__(self, n: int, dtype, fill):
        self.n = n
        self.whole = torch.empty(n + 2 * GUARD, dtype=dtype, device="cuda")
        self.fill = fill
        self.whole.fill_(fill)
        self.t = self.whole[GUARD:GUARD + n]
        assert self.t.data_ptr() % 16 == 0

    def check(self):
        lo = self.whole[:GUARD].cpu()
        hi = self.whole[GUARD + self.n:].cpu()
        assert bool((lo == self.fill).all()) and bool((hi == self.fill).all()), "wrote outside the buffer"


def i16(bits: int) -> int:
    return int(np.array([bits], dtype=np.uint16).view(np.int16)[0])


class DeviceCase:
    """Device-side state of one layout: R parameter arenas, R accumulator arenas, a full
    buffer and a gradient buffer, each guarded; plus host mirrors for the oracle."""

    def __init__(self, R: int, numel, with_params=True):
        self.R = R
        self.numel = [int(n) for n in numel]
        self.layout = odc.Layout(R, self.numel)
        L = self.layout
        self.T = L.num_tensors()
        self.arena = L.rank_arena_elems()
        self.full_n = L.full_elems()
        self.S = [L.shard_elems(t) for t in range(self.T)]
        self.shard_off = [L.shard_offset(t) for t in range(self.T)]
        self.full_off = [L.full_offset(t) for t in range(self.T)]
        self.params = [Guarded(self.arena, torch.int16, i16(PAD16)) for _ in range(R)] if with_params else None
        self.acc = [Guarded(self.arena, torch.float32, float(PAD32)) for _ in range(R)]
        self.full = Guarded(self.full_n, torch.int16, i16(FULL16))
        self.grad = Guarded(self.full_n, torch.int16, 0)
        self.acc_ptrs = odc.PtrArray([a.t for a in self.acc])
        self.param_ptrs = odc.PtrArray([p.t for p in self.params]) if with_params else None

    def load_params(self, arenas_host):
        for p, a in zip(self.params, arenas_host):
            p.t.copy_(to_dev_u16(a))

    def check_guards(self):
        for g in (self.params or []) + self.acc + [self.full, self.grad]:
            g.check()

    def acc_host(self):
        return [a.t.cpu().numpy() for a in self.acc]

    def close(self):
        self.layout.close()


def host_arenas_from_flats(oracle, flats, R, S, shard_off, arena):
    arenas = [np.full(arena, PAD16, dtype=np.uint16) for _ in range(R)]
    for t, flat in enumerate(flats):
        for r, sh in enumerate(oracle.make_shards(flat, R, pad_bits=PAD16)):
            arenas[r][shard_off[t]:shard_off[t] + S[t]] = sh
    return arenas


def assert_bits_equal(got: np.ndarray, want: np.ndarray, what: str):
    g = got.view(np.uint32) if got.dtype == np.float32 else got
    w = want.view(np.uint32) if want.dtype == np.float32 else want
    if not np.array_equal(g, w):
        bad = np.flatnonzero(g != w)
        raise AssertionError(f"{what}: {bad.size} of {g.size} elements differ, first at {bad[0]}: "
                             f"got {g[bad[0]]:#x} want {w[bad[0]]:#x}")
