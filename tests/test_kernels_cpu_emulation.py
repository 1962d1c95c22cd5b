"""The kernel source run on the CPU, one thread at a time, under AddressSanitizer and UBSan.

tests/cpu_emu/emu_main.cpp compiles paper_2601_19362_amd/csrc/odc_device.h (the real kernels,
one odc_dev_*.h header per family) against a small host shim.  Every rank buffer is an
exactly-sized heap block, so an index error in a kernel shows up here, on the CPU, as a
sanitizer report instead of a GPU fault.
The outputs are compared with the CPU oracle bit for bit.  This checks the kernels' indexing
and arithmetic logic, not the GPU build: parity of the HIP path proper is tests/test_gpu_*.py.
"""
import os
import subprocess

import numpy as np
import pytest

from paper_2601_19362_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/lib/llvm/bin/clang++"
PAD16 = 0xDEAD
PAD32 = np.float32(-12345.678)

pytestmark = pytest.mark.skipif(not os.path.exists(CLANG), reason="ROCm clang++ not present")


def start_build(exe, *defines):
    return subprocess.Popen([CLANG, "-std=c++17", "-O0", "-g", "-fsanitize=address,undefined",
                             "-fno-sanitize-recover=all", "-ffp-contract=off", "-pthread", *defines,
                             os.path.join(ROOT, "tests", "cpu_emu", "emu_main.cpp"),
                             os.path.join(ROOT, "paper_2601_19362_amd", "csrc", "odc_layout.cpp"),
                             "-o", exe])


@pytest.fixture(scope="module")
def emu_builds(tmp_path_factory):
    """Both emulation binaries, compiled side by side (each takes a minute or more).  The second
    has the size limit of the 32-bit gather records lowered from 2^30 to 2^9 elements, so that
    ordinary test tensors take the 64-bit path meant for huge ones; it holds the gather
    kernels only."""
    d = tmp_path_factory.mktemp("emu")
    exes = {"default": str(d / "emu"), "low_limit": str(d / "emu_low")}
    procs = [start_build(exes["default"]),
             start_build(exes["low_limit"], "-DODC_GATHER_SMALL_SHIFT=9", "-DEMU_GATHER_ONLY")]
    for p in procs:
        assert p.wait() == 0, "emulation build failed"
    return exes


@pytest.fixture(scope="module")
def emu(emu_builds):
    return emu_builds["default"]


@pytest.fixture(scope="module")
def emu_low_limit(emu_builds):
    return emu_builds["low_limit"]


def placement(numel, R):
    """Tensor starts at multiples of 8 elements (the library's documented placement rule)."""
    S = [-(-n // R) for n in numel]
    so, fo, a, f = [], [], 0, 0
    for n, s in zip(numel, S):
        so.append(a)
        fo.append(f)
        a += (s + 7) // 8 * 8
        f += (n + 7) // 8 * 8
    return S, so, fo, so[-1] + S[-1], fo[-1] + numel[-1]


def run(emu, d, op, R, **knobs):
    p = subprocess.run([emu, str(d), op, str(R)] + [f"{k}={v}" for k, v in knobs.items()],
                       capture_output=True, text=True,
                       env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0"})
    assert p.returncode == 0, p.stderr[-3000:]


def make_case(oracle, numel, R, seed):
    S, so, fo, arena, full_n = placement(numel, R)
    arenas = [np.full(arena, PAD16, dtype=np.uint16) for _ in range(R)]
    flats = []
    for t, n in enumerate(numel):
        flat = inputs.uniform_bf16(n, -1, 1, seed=(seed, t))
        flats.append(flat)
        for r, sh in enumerate(oracle.make_shards(flat, R, pad_bits=PAD16)):
            arenas[r][so[t]:so[t] + S[t]] = sh
    return S, so, fo, arena, full_n, arenas, flats


CASES = [
    ([1], 1), ([1], 64), ([7], 3), ([64], 64), ([65], 64), ([1000], 7), ([4099], 8),
    ([8 * 1024 * 3 + 5], 4),          # several full tiles + ragged tail, misaligned boundaries
    ([262_148 * 2 + 13], 2),
    ([8 * 4097 - 3], 8),              # S = 4097: owner r's source is shifted by 16 - 2r bytes, every shift once
    ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8),
    ([3, 1, 1, 2, 70, 5000, 2, 2, 129, 1], 64),
    ([30000, 17, 2048, 2049], 5),
    ([5] * 70, 70),                   # more than 64 ranks: two launch groups
    ([1] * 600 + [9000] + [3] * 50, 4),   # tiles packed with the maximum number of tensors
    ([2047, 2049, 1, 4096, 8, 16384 + 7, 5], 3),  # tensors ending at, before and after tile edges
    ([129] * 40 + [70000], 66),       # batched with more than 64 ranks
    ([1] * 1100 + [20000, 2], 2),     # a gather tile whose LDS index is filled to the brim
    ([1300, 2000, 1043, 520, 8 * 130], 130),  # S = 10, 16, 9, 4, 8 over three launch groups: items
                                              # that straddle two owners of different launches
    ([100_000, 9, 50_001, 3], 2),     # shard pieces of 50,000 and 25,001 elements: whole tiles inside
                                      # one owner's piece of one tensor (the lean uniform-tile paths)
]


@pytest.mark.parametrize("numel,R", CASES)
@pytest.mark.parametrize("threads,unroll,nt,remap,cap", [(256, 4, 1, 0, 0), (64, 1, 0, 0, 3), (128, 2, 1, 1, 0),
                                                         (64, 1, 1, 1, 0), (256, 2, 1, 0, 1)])
def test_emulated_gather(oracle, emu, tmp_path, numel, R, threads, unroll, nt, remap, cap):
    S, so, fo, arena, full_n, arenas, flats = make_case(oracle, numel, R, seed=1)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    np.concatenate(arenas).tofile(tmp_path / "arenas.u16")
    np.full(full_n, 0xBEEF, dtype=np.uint16).tofile(tmp_path / "full.u16")
    run(emu, tmp_path, "gather", R, threads=threads, unroll=unroll, nt=nt, remap=remap, cap=cap)
    got = np.fromfile(tmp_path / "full.out", dtype=np.uint16)
    want = np.full(full_n, 0xBEEF, dtype=np.uint16)
    oracle.gather_batched(arenas, numel, so, fo, want)
    assert np.array_equal(got, want)
    for t, n in enumerate(numel):
        assert np.array_equal(got[fo[t]:fo[t] + n], flats[t])


@pytest.mark.parametrize("numel,R", CASES)
@pytest.mark.parametrize("nt,cap,lds_max", [(1, 0, 0), (0, 2, 1)])
def test_emulated_gather_64bit_path_and_large_lds(oracle, emu_low_limit, tmp_path, numel, R, nt, cap, lds_max):
    """Tensors of 512 elements or more go through the 64-bit item path in this build; lds_max = 1
    also forces the kernel variant with the full-size LDS index."""
    S, so, fo, arena, full_n, arenas, flats = make_case(oracle, numel, R, seed=3)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    np.concatenate(arenas).tofile(tmp_path / "arenas.u16")
    np.full(full_n, 0xBEEF, dtype=np.uint16).tofile(tmp_path / "full.u16")
    run(emu_low_limit, tmp_path, "gather", R, nt=nt, cap=cap, lds_max=lds_max)
    got = np.fromfile(tmp_path / "full.out", dtype=np.uint16)
    want = np.full(full_n, 0xBEEF, dtype=np.uint16)
    oracle.gather_batched(arenas, numel, so, fo, want)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("numel,R", CASES)
@pytest.mark.parametrize("threads,unroll,nt,remap,atomic,cap,rg", [
    (256, 4, 1, 0, 0, 0, 1), (64, 1, 1, 0, 0, 0, 8), (128, 2, 0, 1, 0, 0, 4), (64, 4, 1, 0, 1, 2, 2),
    (64, 1, 1, 1, 0, 0, 8)])
def test_emulated_reset_and_accumulate(oracle, emu, tmp_path, numel, R, threads, unroll, nt, remap, atomic, cap, rg):
    S, so, fo, arena, full_n = placement(numel, R)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    acc = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    np.concatenate(acc).tofile(tmp_path / "acc.f32")
    run(emu, tmp_path, "reset", R, threads=threads, unroll=unroll, nt=nt, remap=remap, cap=cap, rg=rg)
    got = np.fromfile(tmp_path / "acc.out", dtype=np.float32)
    oracle.reset_batched(acc, numel, so)
    assert np.array_equal(got.view(np.uint32), np.concatenate(acc).view(np.uint32))
    for k in range(3):
        g = inputs.normal_bf16(full_n, 1e-2, seed=(2, k))
        g.tofile(tmp_path / "grad.u16")
        got.tofile(tmp_path / "acc.f32")
        run(emu, tmp_path, "accum", R, threads=threads, unroll=unroll, nt=nt, remap=remap, atomic=atomic, cap=cap,
            rg=rg)
        got = np.fromfile(tmp_path / "acc.out", dtype=np.float32)
        oracle.accumulate_batched(g, acc, numel, so, fo)
        assert np.array_equal(got.view(np.uint32), np.concatenate(acc).view(np.uint32))


@pytest.mark.parametrize("numel,R", CASES)
@pytest.mark.parametrize("threads,unroll,nt,atomic,rg,weight", [(64, 1, 1, 0, 4, 0.37), (256, 4, 0, 0, 1, -1.5),
                                                                (128, 2, 1, 1, 8, 0.5)])
def test_emulated_weighted_accumulate(oracle, emu, tmp_path, numel, R, threads, unroll, nt, atomic, rg, weight):
    S, so, fo, arena, full_n = placement(numel, R)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    acc = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reset_batched(acc, numel, so)
    got = np.concatenate(acc)
    for k in range(2):
        g = inputs.normal_bf16(full_n, 1e-2, seed=(3, k))
        g.tofile(tmp_path / "grad.u16")
        got.tofile(tmp_path / "acc.f32")
        run(emu, tmp_path, "accum", R, threads=threads, unroll=unroll, nt=nt, atomic=atomic, rg=rg, weighted=1,
            weight=repr(float(np.float32(weight))))
        got = np.fromfile(tmp_path / "acc.out", dtype=np.float32)
        if atomic:
            # the unordered form rounds the product first: power-of-two weight keeps it exact
            assert weight == 0.5
        oracle.accumulate_weighted_batched(g, acc, numel, so, fo, weight)
        assert np.array_equal(got.view(np.uint32), np.concatenate(acc).view(np.uint32))


@pytest.mark.parametrize("numel,R", CASES)
@pytest.mark.parametrize("threads,unroll,nt,rg,bf16,scale", [(256, 1, 1, 4, 0, 1.0), (64, 4, 0, 1, 1, 0.125),
                                                             (128, 2, 1, 8, 1, 1.0 / 3.0), (256, 4, 1, 2, 0, 1.0 / 7.0)])
def test_emulated_retrieve(oracle, emu, tmp_path, numel, R, threads, unroll, nt, rg, bf16, scale):
    S, so, fo, arena, full_n = placement(numel, R)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    rng = np.random.default_rng(5)
    acc = [(rng.standard_normal(arena) * 1e-2).astype(np.float32) for _ in range(R)]
    dtype = np.uint16 if bf16 else np.float32
    fill = 0xDEAD if bf16 else PAD32
    out = [np.full(arena, fill, dtype=dtype) for _ in range(R)]
    np.concatenate(acc).tofile(tmp_path / "acc.f32")
    np.concatenate(out).tofile(tmp_path / "out.bin")
    run(emu, tmp_path, "retrieve", R, threads=threads, unroll=unroll, nt=nt, rg=rg, bf16=bf16,
        scale=repr(float(np.float32(scale))))
    got = np.fromfile(tmp_path / "out.out", dtype=dtype)
    oracle.retrieve_batched(acc, out, numel, so, scale=scale)
    view = np.uint16 if bf16 else np.uint32
    assert np.array_equal(got.view(view), np.concatenate(out).view(view))
    assert np.array_equal(np.fromfile(tmp_path / "acc.out", dtype=np.float32).view(np.uint32),
                          np.concatenate(acc).view(np.uint32))          # accumulators untouched


@pytest.mark.parametrize("numel,R", CASES)
@pytest.mark.parametrize("count,cap", [(2, 0), (5, 3), (8, 0)])
def test_emulated_fused_accumulate(oracle, emu, tmp_path, numel, R, count, cap):
    """K contributions in one pass equal K single ordered contributions bit for bit."""
    S, so, fo, arena, full_n = placement(numel, R)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    acc = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reset_batched(acc, numel, so)
    oracle.accumulate_batched(inputs.normal_bf16(full_n, 1e-2, seed=70), acc, numel, so, fo)  # non-zero start
    np.concatenate(acc).tofile(tmp_path / "acc.f32")
    for k in range(count):
        g = inputs.normal_bf16(full_n, 1e-2, seed=(71, k))
        g.tofile(tmp_path / f"grad{k}.u16")
        oracle.accumulate_batched(g, acc, numel, so, fo)
    run(emu, tmp_path, "accum_multi", R, count=count, cap=cap)
    got = np.fromfile(tmp_path / "acc.out", dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), np.concatenate(acc).view(np.uint32))


@pytest.mark.parametrize("numel,R", [([8 * 1024 * 3 + 5], 4), ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8),
                                     ([5] * 66, 66)])
@pytest.mark.parametrize("count", [2, 3, 5, 7, 8])
def test_emulated_fused_unordered_sums_every_gradient_once(oracle, emu, tmp_path, numel, R, count):
    """The unordered fused form adds the K values of an element as a binary tree.  With
    integer-valued gradients every association gives the same exact sum, so the result must
    equal K single contributions bit for bit: a value dropped or counted twice by the tree
    would show."""
    S, so, fo, arena, full_n = placement(numel, R)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    acc = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reset_batched(acc, numel, so)
    np.concatenate(acc).tofile(tmp_path / "acc.f32")
    rng = np.random.default_rng(count)
    for k in range(count):
        g = inputs.f32_to_bf16_bits((rng.integers(-100, 101, size=full_n) * 3 ** k % 251).astype(np.float32))
        g.tofile(tmp_path / f"grad{k}.u16")
        oracle.accumulate_batched(g, acc, numel, so, fo)
    run(emu, tmp_path, "accum_multi", R, count=count, atomic=1)
    got = np.fromfile(tmp_path / "acc.out", dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), np.concatenate(acc).view(np.uint32))


@pytest.mark.parametrize("numel,R", [([7], 3), ([8 * 1024 * 3 + 5], 4), ([4099], 8), ([1], 64),
                                     ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8), ([30000, 17, 2048, 2049], 5),
                                     ([5] * 66, 66), ([40_000, 9, 20_001, 3], 2)])
@pytest.mark.parametrize("nt,cap,rg", [(1, 0, 1), (0, 2, 2)])
def test_emulated_staging(oracle, emu, tmp_path, numel, R, nt, cap, rg):
    """Pushes into per-client slots, drains in ascending client order, refusal of a push into
    a slot that is still full; compared with the oracle's bookkeeping model."""
    S, so, fo, arena, full_n = placement(numel, R)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    acc = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reset_batched(acc, numel, so)
    np.concatenate(acc).tofile(tmp_path / "acc.f32")
    w_hi = R - 1
    steps = [("p", w_hi), ("p", 0), ("d", None), ("p", 0), ("p", 0), ("p", min(1, w_hi)), ("d", None), ("d", None),
             ("p", w_hi)]
    model = oracle.Staging(numel, R, so, fo)
    k = 0
    for kind, w in steps:
        if kind == "p":
            g = inputs.normal_bf16(full_n, 1e-2, seed=(9, k))
            g.tofile(tmp_path / f"grad{k}.u16")
            k += 1
            model.push(g, w)
        else:
            model.drain(acc)
    script = ",".join(f"p{w}" if kind == "p" else "d" for kind, w in steps)
    run(emu, tmp_path, "stage", R, nt=nt, cap=cap, rg=rg, script=script)   # rg: owners per workgroup of the push
    got = np.fromfile(tmp_path / "acc.out", dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), np.concatenate(acc).view(np.uint32))
    flags = np.fromfile(tmp_path / "flags.out", dtype=np.int32)
    assert flags[:R * R].reshape(R, R).astype(bool).tolist() == model.full
    assert flags[R * R] == model.refused and model.refused >= R     # at least the second push of worker 0


@pytest.mark.parametrize("numel,R", [([7], 3), ([8 * 1024 * 3 + 5], 4), ([4099], 20), ([1], 64),
                                     ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8), ([30000, 17, 2048, 2049], 5),
                                     ([5] * 34, 34), ([40_000, 9, 20_001, 3], 2)])
@pytest.mark.parametrize("K,inplace", [(1, 0), (2, 1), (8, 0), (9, 1), (19, 0)])
def test_emulated_reduce_groups(oracle, emu, tmp_path, numel, R, K, inplace):
    """Hybrid sharding: the sum of K groups' accumulator shards (one, two and three passes of up
    to 8 sources; more than 16 owners = two launches), into a separate output or in place into
    group 0; everything compared with the oracle, sentinels in padding and gaps included."""
    S, so, fo, arena, full_n = placement(numel, R)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    rng = np.random.default_rng(K * 100 + R)
    groups = [[(rng.standard_normal(arena) * 1e-2).astype(np.float32) for _ in range(R)] for _ in range(K)]
    out = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    np.concatenate([a for grp in groups for a in grp]).tofile(tmp_path / "groups.f32")
    np.concatenate(out).tofile(tmp_path / "out.f32")
    run(emu, tmp_path, "reduce", R, count=K, lds_max=inplace)
    got = np.fromfile(tmp_path / "out.out", dtype=np.float32)
    want = [g.copy() for g in groups[0]] if inplace else out
    src = [want] + groups[1:] if inplace else groups
    oracle.reduce_groups_batched(src, want, numel, so)
    assert np.array_equal(got.view(np.uint32), np.concatenate(want).view(np.uint32))


@pytest.mark.parametrize("numel,R", [([7], 3), ([8 * 1024 * 3 + 5], 4), ([1], 64), ([5] * 66, 66),
                                     ([1, 5, 8, 9, 64, 100, 1, 777, 3, 4096, 63], 8), ([30000, 17, 2048, 2049], 5)])
@pytest.mark.parametrize("count,cap", [(1, 0), (3, 2)])
def test_emulated_wide_accumulators(oracle, emu, tmp_path, numel, R, count, cap):
    """Binary64 accumulators: reset, contributions, retrieval to binary32 and to bf16; accumulators
    and both outputs compared bit for bit with the oracle, sentinels in padding and gaps included."""
    S, so, fo, arena, full_n = placement(numel, R)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    acc = [np.full(arena, -9876.5, dtype=np.float64) for _ in range(R)]
    out32 = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    out16 = [np.full(arena, PAD16, dtype=np.uint16) for _ in range(R)]
    np.concatenate(acc).tofile(tmp_path / "acc.f64")
    np.concatenate(out32).tofile(tmp_path / "out32.f32")
    np.concatenate(out16).tofile(tmp_path / "out16.u16")
    gs = [inputs.normal_bf16(full_n, 1e-2, seed=(23, k)) for k in range(count)]
    for k, g in enumerate(gs):
        g.tofile(tmp_path / f"grad{k}.u16")
    scale = float(np.float32(1.0 / 3.0))
    run(emu, tmp_path, "wide", R, count=count, cap=cap, scale=repr(scale))
    for t, n in enumerate(numel):
        va = oracle.wide_views(acc, numel, so, t, R)
        oracle.reset_wide(va, n)
        for g in gs:
            oracle.accumulate_wide(np.ascontiguousarray(g[fo[t]:fo[t] + n]), va, n)
        oracle.retrieve_wide(va, oracle.wide_views(out32, numel, so, t, R), n, scale=scale)
        oracle.retrieve_wide(va, oracle.wide_views(out16, numel, so, t, R), n, scale=scale)
    assert np.array_equal(np.fromfile(tmp_path / "acc.out", dtype=np.float64).view(np.uint64), np.concatenate(acc).view(np.uint64))
    assert np.array_equal(np.fromfile(tmp_path / "out32.out", dtype=np.float32).view(np.uint32), np.concatenate(out32).view(np.uint32))
    assert np.array_equal(np.fromfile(tmp_path / "out16.out", dtype=np.uint16), np.concatenate(out16))


INTERLEAVINGS = [
    # a client pushes again while its slot is full; a drain on another stream empties the slot
    # after the claim / between the copy workgroups / before the raise
    "p0,c0,s,a,z,x0,r0,d",
    "p0,c0,x0:0:2,s,a,z,x0:1:2,r0,d",
    "p0,c0,x0,s,a,z,r0,d",
    "p0,s,c0,a,x0,z,r0,d",
    # a drain begins while a push is being written: left for the next drain, added once
    "c1,s,x1,a,z,r1,d",
    "c1,x1:1:3,s,a,x1:0:3,z,x1:2:3,r1,s,a,z",
    # another client's push lands inside a drain
    "p0,s,c1,x1,r1,a,z,d",
    "p0,p1,s,a,c0,x0,r0,z,c0,x0,r0,d",
]


@pytest.mark.parametrize("numel,R", [([8 * 1024 * 3 + 5], 4), ([30000, 17, 2048, 2049], 5), ([5] * 66, 66)])
@pytest.mark.parametrize("script", INTERLEAVINGS)
def test_emulated_staging_interleavings(oracle, emu, tmp_path, numel, R, script):
    """The kernels of a push and of a drain run in a scripted order, as two streams could run
    them (including a drain that empties a slot between the workgroups of a push's copy kernel).
    The phased bookkeeping model decides once per push and owner; the kernels must agree: every
    accepted contribution is added exactly once, a refused one never, and no slot is left full
    that the model has empty."""
    S, so, fo, arena, full_n = placement(numel, R)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    acc = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    oracle.reset_batched(acc, numel, so)
    np.concatenate(acc).tofile(tmp_path / "acc.f32")
    model = oracle.Staging(numel, R, so, fo)
    k = 0
    for step in script.split(","):
        kind, w = step[0], int(step[1:].split(":")[0]) if len(step) > 1 else 0
        if kind in "pc":
            g = inputs.normal_bf16(full_n, 1e-2, seed=(19, k))
            g.tofile(tmp_path / f"grad{k}.u16")
            k += 1
            model.begin_push(g, w)
            if kind == "p":
                model.end_push(w)
        elif kind == "r":
            model.end_push(w)
        elif kind in "ds":
            model.begin_drain()
            model.add_noted(acc)
            if kind == "d":
                model.end_drain()
        elif kind == "z":
            model.end_drain()
    run(emu, tmp_path, "stage", R, rg=1 + len(script) % 2, script=script)
    got = np.fromfile(tmp_path / "acc.out", dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), np.concatenate(acc).view(np.uint32))
    flags = np.fromfile(tmp_path / "flags.out", dtype=np.int32)
    assert flags[:R * R].reshape(R, R).tolist() == model.state
    assert flags[R * R] == model.refused


def random_layout(seed):
    """A seeded random multi-tensor layout: tensor sizes from a mixture of tiny, small, medium
    and large, a rank count from single-launch and multi-launch values; at most about 250,000
    elements in all so that a case runs in a second."""
    rng = np.random.default_rng(seed)
    R = int(rng.choice([1, 2, 3, 5, 8, 16, 33, 64, 65, 130]))
    T = int(rng.integers(2, 40))
    sizes = []
    for _ in range(T):
        kind = rng.choice(4, p=[0.35, 0.3, 0.25, 0.1])
        hi = [16, 600, 20_000, 70_000][kind]
        lo = [1, 17, 601, 20_001][kind]
        sizes.append(int(rng.integers(lo, hi + 1)))
    while sum(sizes) > 250_000:
        sizes.remove(max(sizes))
    if len(sizes) < 2:
        sizes.append(5)
    return sizes, R


@pytest.mark.parametrize("seed", range(int(os.environ.get("ODC_EMU_RANDOM_LAYOUTS", "20"))))   # more on request
def test_emulated_random_layouts(oracle, emu, emu_low_limit, tmp_path, seed):
    """Gather (both builds), reset, one ordered and one unordered contribution and a retrieval on
    a random layout; every buffer compared in full with the oracle."""
    numel, R = random_layout(1000 + seed)
    rg = [1, 2, 4, 8][seed % 4]
    S, so, fo, arena, full_n, arenas, flats = make_case(oracle, numel, R, seed=40 + seed)
    np.array(numel, dtype=np.int64).tofile(tmp_path / "numel.i64")
    np.concatenate(arenas).tofile(tmp_path / "arenas.u16")
    want = np.full(full_n, 0xBEEF, dtype=np.uint16)
    oracle.gather_batched(arenas, numel, so, fo, want)
    for exe in (emu, emu_low_limit):
        np.full(full_n, 0xBEEF, dtype=np.uint16).tofile(tmp_path / "full.u16")
        run(exe, tmp_path, "gather", R, nt=seed % 2, remap=seed % 5)   # tiles in XCD blocks of 1 .. 16
        assert np.array_equal(np.fromfile(tmp_path / "full.out", dtype=np.uint16), want), (numel, R)

    acc = [np.full(arena, PAD32, dtype=np.float32) for _ in range(R)]
    np.concatenate(acc).tofile(tmp_path / "acc.f32")
    run(emu, tmp_path, "reset", R, rg=rg)
    got = np.fromfile(tmp_path / "acc.out", dtype=np.float32)
    oracle.reset_batched(acc, numel, so)
    assert np.array_equal(got.view(np.uint32), np.concatenate(acc).view(np.uint32)), (numel, R)
    for atomic in (0, 1):   # a single contribution onto zeros or onto one value: exact either way
        g = inputs.normal_bf16(full_n, 1e-2, seed=(41, seed, atomic))
        g.tofile(tmp_path / "grad.u16")
        got.tofile(tmp_path / "acc.f32")
        run(emu, tmp_path, "accum", R, atomic=atomic, rg=rg)
        got = np.fromfile(tmp_path / "acc.out", dtype=np.float32)
        oracle.accumulate_batched(g, acc, numel, so, fo)
        assert np.array_equal(got.view(np.uint32), np.concatenate(acc).view(np.uint32)), (numel, R, atomic)

    bf16 = seed % 2
    dtype, fill = (np.uint16, 0xDEAD) if bf16 else (np.float32, PAD32)
    out = [np.full(arena, fill, dtype=dtype) for _ in range(R)]
    np.concatenate(out).tofile(tmp_path / "out.bin")
    got.tofile(tmp_path / "acc.f32")
    scale = float(np.float32(1.0 / 3.0))
    run(emu, tmp_path, "retrieve", R, rg=rg, bf16=bf16, scale=repr(scale))
    got_out = np.fromfile(tmp_path / "out.out", dtype=dtype)
    oracle.retrieve_batched(acc, out, numel, so, scale=scale)
    assert np.array_equal(got_out.view(np.uint16 if bf16 else np.uint32),
                          np.concatenate(out).view(np.uint16 if bf16 else np.uint32)), (numel, R)
