"""The library driven from a plain C99 program (tests/c_abi/c_abi_check.c: hipMalloc, its own
stream, the C ABI and nothing else -- no Python binding, no torch), checked against the CPU
oracle.  The program is compiled by build() in __graft_entry__.py."""
import os
import subprocess

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "c_abi", "_build", "c_abi_check")


def placement(numel, R):
    S = [-(-n // R) for n in numel]
    so, fo, a, f = [], [], 0, 0
    for n, s in zip(numel, S):
        so.append(a)
        fo.append(f)
        a += (s + 7) // 8 * 8
        f += (n + 7) // 8 * 8
    return S, so, fo, so[-1] + S[-1], fo[-1] + numel[-1]


@pytest.mark.parametrize("numel,R", [([1_048_589], 4), ([4099, 1, 70_001, 12_345, 8, 300_000], 8), ([350, 9000], 70)])
def test_c_program_through_the_c_abi(oracle, tmp_path, numel, R):
    if not os.path.exists(EXE):
        # build() makes it; a tree that lost it gets it rebuilt here (gcc, one second), and a
        # failure to do so fails the test: a missing program must not pass as a skip
        import sys

        sys.path.insert(0, ROOT)
        import __graft_entry__

        __graft_entry__.build_c_abi_check()
    assert os.path.exists(EXE), "tests/c_abi/_build/c_abi_check could not be built"
    print(f"c abi case R={R} numel={numel}", flush=True)
    p = subprocess.run([EXE, str(tmp_path), str(R)] + [str(n) for n in numel], capture_output=True, text=True,
                       timeout=100)
    assert p.returncode == 0, p.stdout + p.stderr
    S, so, fo, arena, full_n = placement(numel, R)
    arenas = np.fromfile(tmp_path / "arenas.u16", dtype=np.uint16).reshape(R, arena)
    want_full = np.full(full_n, 0xBEEF, dtype=np.uint16)
    oracle.gather_batched(list(arenas), numel, so, fo, want_full)
    assert np.array_equal(np.fromfile(tmp_path / "full.out", dtype=np.uint16), want_full)

    acc = [np.full(arena, -7.5, dtype=np.float32) for _ in range(R)]
    oracle.reset_batched(acc, numel, so)
    for k in range(3):
        g = np.fromfile(tmp_path / f"grad{k}.u16", dtype=np.uint16)
        oracle.accumulate_batched(g, acc, numel, so, fo)
    got = np.fromfile(tmp_path / "acc.out", dtype=np.float32).view(np.uint32)
    assert np.array_equal(got, np.concatenate(acc).view(np.uint32))

    out = [np.full(arena, -7.5, dtype=np.float32) for _ in range(R)]
    oracle.retrieve_batched(acc, out, numel, so, scale=0.25)
    got = np.fromfile(tmp_path / "retrieved.out", dtype=np.float32).view(np.uint32)
    assert np.array_equal(got, np.concatenate(out).view(np.uint32))
