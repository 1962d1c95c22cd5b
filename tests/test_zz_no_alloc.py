"""odc_stage_drain_noalloc (the drain whose snapshot list lives in a fixed device array inside
the library) against odc_stage_drain with a caller-provided workspace: same pushes, same
drains, accumulators and flags compared bit for bit -- on two calls in a row, the second with
a smaller layout, so that whatever the first call left in the shared array must not matter."""
import numpy as np
import pytest
import torch

from paper_2601_19362_amd import binding as odc
from paper_2601_19362_amd import inputs

from gpu_util import PAD32, DeviceCase, assert_bits_equal, to_dev_u16

pytestmark = pytest.mark.gpu


class Staged:
    def __init__(self, case):
        L = case.layout
        self.slot = L.stage_slot_elems()
        self.bufs = [torch.full((case.R * self.slot,), -3.0, dtype=torch.bfloat16, device="cuda") for _ in range(case.R)]
        self.flags = torch.full((L.stage_flag_count(),), 77, dtype=torch.int32, device="cuda")
        self.snap = torch.zeros(L.stage_snapshot_count(), dtype=torch.int32, device="cuda")
        L.stage_init(self.flags)


def run_both(numel, R, steps, seed):
    """The same push/drain sequence through both entry points; returns nothing, asserts equality."""
    print(f"no-alloc drain case R={R} T={len(numel)} total={sum(numel)} steps={steps}", flush=True)
    ref, new = DeviceCase(R, numel, with_params=False), DeviceCase(R, numel, with_params=False)
    st_ref, st_new = Staged(ref), Staged(new)
    for c in (ref, new):
        c.layout.reset_accum(c.acc_ptrs)
    for k, (kind, w) in enumerate(steps):
        if kind == "p":
            g = to_dev_u16(inputs.normal_bf16(ref.full_n, 1e-2, seed=(seed, k)))
            ref.layout.stage_push(g, st_ref.bufs, st_ref.flags, w)
            new.layout.stage_push(g, st_new.bufs, st_new.flags, w)
        else:
            ref.layout.stage_drain(st_ref.bufs, st_ref.flags, st_ref.snap, ref.acc_ptrs)
            new.layout.stage_drain_noalloc(st_new.bufs, st_new.flags, new.acc_ptrs)
    torch.cuda.synchronize()
    touched = False
    for r, (a, b) in enumerate(zip(new.acc_host(), ref.acc_host())):
        assert_bits_equal(a, b, f"accumulator of owner {r}")
        touched |= bool(((b != PAD32) & (b != 0)).any())
    assert touched, "the sequence accumulated nothing"
    assert np.array_equal(st_new.flags.cpu().numpy(), st_ref.flags.cpu().numpy())
    for c in (ref, new):
        c.check_guards()
        c.close()


def test_noalloc_drain_equals_workspace_drain_twice_in_a_row():
    hi = 69
    run_both([5] * 70 + [100_000], 70,
             [("p", hi), ("p", 0), ("p", 33), ("d", None), ("p", 0), ("p", 0), ("p", 1), ("d", None), ("d", None), ("p", hi)],
             seed=21)
    # second call: fewer owners and a smaller tensor; the array still holds the first call's lists
    run_both([1_048_589], 4, [("p", 3), ("p", 0), ("d", None), ("p", 3), ("p", 1), ("p", 3), ("d", None)], seed=22)


def test_noalloc_drain_refuses_layouts_beyond_its_scratch():
    R = odc.ODC_NOALLOC_MAX_RANKS + 1
    L = odc.Layout(R, [R * 8])
    arena = L.rank_arena_elems()
    slot = L.stage_slot_elems()
    bufs = [torch.zeros(R * slot, dtype=torch.bfloat16, device="cuda")] * R     # never touched: the call is refused
    acc = [torch.zeros(arena, dtype=torch.float32, device="cuda")] * R
    flags = torch.zeros(L.stage_flag_count(), dtype=torch.int32, device="cuda")
    assert odc.stage_drain_noalloc_rc(L, bufs, flags, acc) == odc.ODC_ERR_TOO_LARGE
    assert "scratch" in odc.strerror(odc.ODC_ERR_TOO_LARGE)
    assert odc.stage_drain_noalloc_rc(L, bufs, None, acc) == odc.ODC_ERR_INVALID_ARG
    L.close()
