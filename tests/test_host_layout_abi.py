"""Host-side checks of the C-ABI library that need no GPU: the library loads and exports every
symbol the header declares, the layout arithmetic agrees with the closed forms and with the
oracle, and argument errors are reported before anything is launched."""
import os
import re

import numpy as np
import pytest

from paper_2601_19362_amd import binding as odc
from paper_2601_19362_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "odc.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(odc_[a-z_0-9]+)\s*\(", header))
    assert declared == set(odc.EXPORTS)
    lib = odc.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_error_strings_and_codes():
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        assert odc.strerror(code) and "unknown" not in odc.strerror(code)
    assert "unknown" in odc.strerror(-99)
    header = open(os.path.join(ROOT, "include", "odc.h")).read()
    for name in ("ODC_ERR_INVALID_ARG", "ODC_ERR_ALIGNMENT", "ODC_ERR_ORDER", "ODC_ERR_OVERFLOW",
                 "ODC_ERR_HIP", "ODC_ERR_NO_DEVICE", "ODC_ERR_NOMEM", "ODC_MAX_RANKS",
                 "ODC_LAYOUT_HOST_ONLY", "ODC_ORDERED", "ODC_UNORDERED", "ODC_OUT_F32", "ODC_OUT_BF16"):
        m = re.search(rf"#define {name} \(?(-?\d+)\)?", header)
        assert m and int(m.group(1)) == getattr(odc, name), name


@pytest.mark.parametrize("R", [1, 2, 3, 4, 8, 16, 33, 64, 100])
def test_single_tensor_layout_matches_closed_form_and_oracle(oracle, R):
    for N in [1, 2, 7, 63, 64, 65, 1000, 4099, 1_048_589, 46_795_776, 487_598_080]:
        L = odc.Layout(R, [N], host_only=True)
        S = -(-N // R)
        assert L.num_ranks() == R and L.num_tensors() == 1 and L.numel(0) == N
        assert L.shard_elems(0) == S == oracle.shard_elems(N, R)
        assert L.rank_arena_elems() == S and L.full_elems() == N
        assert L.shard_offset(0) == 0 and L.full_offset(0) == 0
        valid = [L.valid_elems(0, r) for r in range(R)]
        assert valid == [oracle.valid_elems(N, R, r) for r in range(R)]
        assert sum(valid) == N
        L.close()


def test_multi_tensor_placement():
    """Tensor starts are multiples of 8 elements, in order, without overlap; the last tensor
    is not padded."""
    w = inputs.workload("stress")
    L = odc.Layout(w.R, w.numel, host_only=True)
    so = np.array([L.shard_offset(t) for t in range(w.T)])
    fo = np.array([L.full_offset(t) for t in range(w.T)])
    n = np.array(w.numel)
    S = -(-n // w.R)
    assert (so % 8 == 0).all() and (fo % 8 == 0).all()
    assert so[0] == 0 and fo[0] == 0
    assert np.array_equal(so[1:], np.cumsum((S + 7) // 8 * 8)[:-1])
    assert np.array_equal(fo[1:], np.cumsum((n + 7) // 8 * 8)[:-1])
    assert L.rank_arena_elems() == so[-1] + S[-1]
    assert L.full_elems() == fo[-1] + n[-1]
    assert [L.shard_elems(t) for t in range(0, w.T, 997)] == S[::997].tolist()
    L.close()


def test_query_range_errors():
    L = odc.Layout(4, [10, 20], host_only=True)
    assert L.numel(2) == -1 and L.numel(-1) == -1 and L.shard_elems(5) == -1
    assert L.valid_elems(0, 4) == -1 and L.valid_elems(0, -1) == -1 and L.valid_elems(2, 0) == -1
    assert L.shard_offset(2) == -1 and L.full_offset(-1) == -1
    lib = odc.lib()
    assert lib.odc_num_ranks(None) == -1 and lib.odc_full_elems(None) == -1
    lib.odc_free_layout(None)  # ignored


def test_init_argument_errors():
    def code(R, numel, flags=odc.ODC_LAYOUT_HOST_ONLY, T=None):
        import ctypes
        arr = (ctypes.c_int64 * max(len(numel), 1))(*numel)
        h = ctypes.c_void_p()
        rc = odc.lib().odc_init_layout(R, len(numel) if T is None else T, arr, flags, ctypes.byref(h))
        if rc == 0:
            odc.lib().odc_free_layout(h)
        else:
            assert not h.value
        return rc

    assert code(4, [10]) == 0
    assert code(0, [10]) == odc.ODC_ERR_INVALID_ARG
    assert code(-3, [10]) == odc.ODC_ERR_INVALID_ARG
    assert code(odc.ODC_MAX_RANKS + 1, [10]) == odc.ODC_ERR_INVALID_ARG
    assert code(odc.ODC_MAX_RANKS, [10]) == 0
    assert code(4, [], T=0) == odc.ODC_ERR_INVALID_ARG
    assert code(4, [10, 0]) == odc.ODC_ERR_INVALID_ARG
    assert code(4, [-5]) == odc.ODC_ERR_INVALID_ARG
    assert code(4, [10], flags=2) == odc.ODC_ERR_INVALID_ARG
    assert code(4, [2 ** 62]) == odc.ODC_ERR_OVERFLOW
    assert code(4, [2 ** 58, 2 ** 58, 2 ** 58]) == odc.ODC_ERR_OVERFLOW
    import ctypes
    assert odc.lib().odc_init_layout(4, 1, None, 1, ctypes.byref(ctypes.c_void_p())) == odc.ODC_ERR_INVALID_ARG
    arr = (ctypes.c_int64 * 1)(5)
    assert odc.lib().odc_init_layout(4, 1, arr, 1, None) == odc.ODC_ERR_INVALID_ARG


def test_launch_argument_errors_are_found_before_any_launch():
    """With a host-only layout nothing can be launched, so every code below comes from the
    host-side validation (fake, never dereferenced addresses stand in for device pointers)."""
    L = odc.Layout(4, [1000], host_only=True)
    good = [0x1000, 0x2000, 0x3000, 0x4000]
    assert odc.gather_rc(L, good, 0x8000, 0) == odc.ODC_ERR_NO_DEVICE
    assert odc.gather_rc(L, good, None, 0) == odc.ODC_ERR_INVALID_ARG
    assert odc.gather_rc(L, None, 0x8000, 0) == odc.ODC_ERR_INVALID_ARG
    assert odc.gather_rc(L, [0x1000, None, 0x3000, 0x4000], 0x8000, 0) == odc.ODC_ERR_INVALID_ARG
    assert odc.gather_rc(L, [0x1000, 0x2008, 0x3000, 0x4000], 0x8000, 0) == odc.ODC_ERR_ALIGNMENT
    assert odc.gather_rc(L, good, 0x8002, 0) == odc.ODC_ERR_ALIGNMENT
    assert odc.lib().odc_gather(None, None, None, None) == odc.ODC_ERR_INVALID_ARG

    sa = odc.scatter_accumulate_rc
    assert sa(L, 0x8000, good, 0, 0, odc.ODC_ORDERED, 0) == odc.ODC_ERR_NO_DEVICE
    assert sa(L, 0x8000, good, 3, 7, odc.ODC_UNORDERED, 0) == odc.ODC_ERR_NO_DEVICE
    assert sa(L, None, good, 0, 0, odc.ODC_ORDERED, 0) == odc.ODC_ERR_INVALID_ARG
    assert sa(L, 0x8000, good, 4, 0, odc.ODC_ORDERED, 0) == odc.ODC_ERR_INVALID_ARG
    assert sa(L, 0x8000, good, -1, 0, odc.ODC_ORDERED, 0) == odc.ODC_ERR_INVALID_ARG
    assert sa(L, 0x8000, good, 0, -1, odc.ODC_ORDERED, 0) == odc.ODC_ERR_INVALID_ARG
    assert sa(L, 0x8000, good, 0, 0, 5, 0) == odc.ODC_ERR_INVALID_ARG
    assert sa(L, 0x8004, good, 0, 0, odc.ODC_ORDERED, 0) == odc.ODC_ERR_ALIGNMENT
    assert sa(L, 0x8000, [0x1000, 0x2000, 0x3004, 0x4000], 0, 0, odc.ODC_ORDERED, 0) == odc.ODC_ERR_ALIGNMENT

    lib = odc.lib()
    import ctypes
    arr = (ctypes.c_void_p * 4)(*good)
    assert lib.odc_scatter_accumulate_weighted(L.handle, 0x8000, arr, 0, 0, 0.5, odc.ODC_ORDERED, None) == odc.ODC_ERR_NO_DEVICE
    assert lib.odc_scatter_accumulate_weighted(L.handle, 0x8000, arr, 9, 0, 0.5, odc.ODC_ORDERED, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_scatter_accumulate_weighted(L.handle, 0x8002, arr, 0, 0, 0.5, odc.ODC_ORDERED, None) == odc.ODC_ERR_ALIGNMENT
    assert odc.retrieve_grads_rc(L, good, good, 1.0, odc.ODC_OUT_F32, 0) == odc.ODC_ERR_NO_DEVICE
    assert odc.retrieve_grads_rc(L, good, good, 1.0, 5, 0) == odc.ODC_ERR_INVALID_ARG
    assert odc.retrieve_grads_rc(L, good, None, 1.0, 0, 0) == odc.ODC_ERR_INVALID_ARG
    assert odc.retrieve_grads_rc(L, good, [0x1000, 0x2000, 0x3002, 0x4000], 1.0, 0, 0) == odc.ODC_ERR_ALIGNMENT

    assert odc.reset_accum_rc(L, good, 0) == odc.ODC_ERR_NO_DEVICE
    assert odc.reset_accum_rc(L, None, 0) == odc.ODC_ERR_INVALID_ARG
    assert odc.reset_accum_rc(L, [0x1000, 0x2000, 0x3000, 0x4001], 0) == odc.ODC_ERR_ALIGNMENT
    L.close()


def test_hybrid_wide_and_staging_argument_errors_are_found_on_the_host():
    """The later entry points validate before they launch too (host-only layout, fake addresses)."""
    import ctypes
    L = odc.Layout(4, [1000], host_only=True)
    lib = odc.lib()
    good = [0x1000, 0x2000, 0x3000, 0x4000]
    two = good + [0x5000, 0x6000, 0x7000, 0x9000]                      # two groups of four owners
    out = [0xA000, 0xB000, 0xC000, 0xD000]
    assert odc.reduce_groups_rc(L, 2, two, out, stream=0) == odc.ODC_ERR_NO_DEVICE
    assert odc.reduce_groups_rc(L, 2, two, good, stream=0) == odc.ODC_ERR_NO_DEVICE          # into group 0: allowed
    assert odc.reduce_groups_rc(L, 2, two, [0xA000, 0x7000, 0xC000, 0xD000], stream=0) == odc.ODC_ERR_INVALID_ARG  # a later group's shard
    assert odc.reduce_groups_rc(L, 2, two, two[4:], stream=0) == odc.ODC_ERR_INVALID_ARG
    assert odc.reduce_groups_rc(L, 0, [], out, stream=0) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_reduce_groups(L.handle, odc.ODC_MAX_GROUPS + 1, (ctypes.c_void_p * 8)(*two), (ctypes.c_void_p * 4)(*out), None) == odc.ODC_ERR_INVALID_ARG
    assert odc.reduce_groups_rc(L, 2, two[:5] + [0x6004] + two[6:], out, stream=0) == odc.ODC_ERR_ALIGNMENT
    assert odc.reduce_groups_rc(L, 2, two, None, stream=0) == odc.ODC_ERR_INVALID_ARG
    assert L.hybrid_group_of(2, 0) == 0 and L.hybrid_group_of(2, 7) == 1 and L.hybrid_group_of(2, 8) == -1
    assert L.hybrid_group_of(2, -1) == -1 and L.hybrid_group_of(0, 0) == -1
    sah = odc.scatter_accumulate_hybrid_rc
    assert sah(L, 2, 0x8000, two, 5, 0, stream=0) == odc.ODC_ERR_NO_DEVICE
    assert sah(L, 2, 0x8000, two, 8, 0, stream=0) == odc.ODC_ERR_INVALID_ARG
    assert sah(L, 2, 0x8002, two, 5, 0, stream=0) == odc.ODC_ERR_ALIGNMENT
    arr, full = (ctypes.c_void_p * 8)(*two), ctypes.c_void_p(0x8000)
    assert lib.odc_gather_hybrid(L.handle, 2, arr, 7, full, None) == odc.ODC_ERR_NO_DEVICE
    assert lib.odc_gather_hybrid(L.handle, 2, arr, 8, full, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_gather_hybrid(L.handle, 2, None, 0, full, None) == odc.ODC_ERR_INVALID_ARG

    a4 = (ctypes.c_void_p * 4)(*good)
    o4 = (ctypes.c_void_p * 4)(*out)
    bad4 = (ctypes.c_void_p * 4)(0x1000, 0x2008, 0x3000, 0x4000)
    assert lib.odc_reset_accum_wide(L.handle, a4, None) == odc.ODC_ERR_NO_DEVICE
    assert lib.odc_reset_accum_wide(L.handle, None, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_reset_accum_wide(L.handle, bad4, None) == odc.ODC_ERR_ALIGNMENT
    assert lib.odc_scatter_accumulate_wide(L.handle, 0x8000, a4, None) == odc.ODC_ERR_NO_DEVICE
    assert lib.odc_scatter_accumulate_wide(L.handle, None, a4, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_scatter_accumulate_wide(L.handle, 0x8008, a4, None) == odc.ODC_ERR_ALIGNMENT
    assert lib.odc_retrieve_grads_wide(L.handle, a4, o4, 1.0, odc.ODC_OUT_BF16, None) == odc.ODC_ERR_NO_DEVICE
    assert lib.odc_retrieve_grads_wide(L.handle, a4, o4, 1.0, 7, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_retrieve_grads_wide(L.handle, a4, None, 1.0, odc.ODC_OUT_F32, None) == odc.ODC_ERR_INVALID_ARG

    flags = 0xE000
    assert odc.stage_push_rc(L, 0x8000, good, flags, 0, stream=0) == odc.ODC_ERR_NO_DEVICE
    assert odc.stage_push_rc(L, 0x8000, good, flags, 4, stream=0) == odc.ODC_ERR_INVALID_ARG
    assert odc.stage_push_rc(L, 0x8000, good, 0xE004, 0, stream=0) == odc.ODC_ERR_ALIGNMENT
    assert odc.stage_drain_rc(L, good, flags, 0xF000, out, stream=0) == odc.ODC_ERR_NO_DEVICE
    assert odc.stage_drain_rc(L, good, flags, None, out, stream=0) == odc.ODC_ERR_INVALID_ARG
    assert odc.stage_drain_noalloc_rc(L, good, flags, out, stream=0) == odc.ODC_ERR_NO_DEVICE
    assert odc.stage_drain_noalloc_rc(L, good, None, out, stream=0) == odc.ODC_ERR_INVALID_ARG
    L.close()
    big = odc.Layout(odc.ODC_NOALLOC_MAX_RANKS + 1, [100_000], host_only=True)
    ptrs = [0x1000 + 0x100 * r for r in range(big.R)]
    assert odc.stage_drain_noalloc_rc(big, ptrs, flags, ptrs, stream=0) == odc.ODC_ERR_TOO_LARGE
    big.close()


def test_probe_and_tune_argument_errors():
    lib = odc.lib()
    assert lib.odc_probe_copy(None, 0x1000, 16, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_probe_copy(0x1000, 0x2000, 24, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_probe_copy(0x1000, 0x2000, -16, None) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_probe_copy(0x1004, 0x2000, 16, None) == odc.ODC_ERR_ALIGNMENT
    assert lib.odc_tune(b"gather_unroll", 3) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_tune(b"no_such_knob", 1) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_tune(None, 1) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_tune(b"gather_threads", 100) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_tune(b"nontemporal", 2) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_tune(b"max_grid_x", -1) == odc.ODC_ERR_INVALID_ARG
    assert lib.odc_tune(b"defaults", 1) == odc.ODC_ERR_INVALID_ARG
    for knob, value in [(b"gather_threads", 64), (b"accum_threads", 128), (b"reset_threads", 256),
                        (b"gather_unroll", 1), (b"accum_unroll", 2), (b"reset_unroll", 4),
                        (b"nontemporal", 0), (b"tile_remap", 1), (b"gather_store_sc1", 0), (b"max_grid_x", 512), (b"defaults", 0)]:
        assert lib.odc_tune(knob, value) == 0


def test_headers_compile_as_plain_c_and_cxx(tmp_path):
    """The boundary is a C ABI: both headers must be usable from a C99 translation unit (and
    from C++) with warnings as errors."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "hdr.c"
    src.write_text('#include "odc.h"\n#include "odc_packing.h"\n'
                   'int main(void) { return odc_strerror(ODC_OK) == 0 && ODC_MAX_FUSED > 0; }\n')
    inc = os.path.join(root, "include")
    if shutil.which("gcc"):
        subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc,
                        str(src)], check=True)
    if shutil.which("g++"):
        subprocess.run(["g++", "-std=c++11", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc,
                        "-x", "c++", str(src)], check=True)


def test_forget_accum_is_host_only_and_checks_its_arguments():
    L = odc.Layout(4, [1000], host_only=True)
    import ctypes
    fake = (ctypes.c_void_p * 4)(0x1000, 0x2000, 0x3000, 0x4000)      # never dereferenced
    assert odc.lib().odc_forget_accum(L.handle, fake) == odc.ODC_OK     # no history: still fine
    assert odc.lib().odc_forget_accum(L.handle, None) == odc.ODC_ERR_INVALID_ARG
    assert odc.lib().odc_forget_accum(None, fake) == odc.ODC_ERR_INVALID_ARG
    empty = (ctypes.c_void_p * 4)()
    assert odc.lib().odc_forget_accum(L.handle, empty) == odc.ODC_ERR_INVALID_ARG
    L.close()


def test_tune_from_several_threads_keeps_every_knob_valid():
    """odc_tune is a read-modify-write of the whole knob set under a lock: calls racing from
    several threads must all be applied or refused cleanly, never tear the set.  Afterwards each
    knob holds one of the values some thread wrote, and "defaults" restores the built-in set."""
    import threading

    knobs = {"gather_threads": (64, 128, 256), "accum_unroll": (1, 2, 4), "nontemporal": (0, 1),
             "gather_tile_xcd_block": (1, 8, 64), "batch_rank_group": (0, 2, 8), "max_grid_x": (0, 7)}
    errors = []

    def worker(seed):
        rng = np.random.default_rng(seed)
        names = list(knobs)
        for _ in range(3000):
            k = names[rng.integers(len(names))]
            v = knobs[k][rng.integers(len(knobs[k]))]
            if odc.lib().odc_tune(k.encode(), int(v)) != odc.ODC_OK:
                errors.append((k, v))
            if odc.lib().odc_tune(b"gather_threads", 100) != odc.ODC_ERR_INVALID_ARG:     # refused, changes nothing
                errors.append("bad value accepted")

    threads = [threading.Thread(target=worker, args=(s,)) for s in range(6)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors
    odc.reset_tuning()
    assert odc.lib().odc_tune(b"no_such_knob", 1) == odc.ODC_ERR_INVALID_ARG
