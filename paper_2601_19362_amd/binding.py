"""ctypes binding of libodc.so: same names as the C ABI in include/odc.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels; torch is used
by callers for device memory and streams.  There is no fallback: if the built library is
missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libodc.so")

ODC_OK = 0
ODC_ERR_INVALID_ARG = -1
ODC_ERR_ALIGNMENT = -2
ODC_ERR_ORDER = -3
ODC_ERR_OVERFLOW = -4
ODC_ERR_HIP = -5
ODC_ERR_NO_DEVICE = -6
ODC_ERR_NOMEM = -7
ODC_ERR_TOO_LARGE = -8
ODC_NOALLOC_MAX_RANKS = 256
ODC_MAX_GROUPS = 1024
ODC_MAX_RANKS = 4096
ODC_LAYOUT_HOST_ONLY = 1
ODC_ORDERED = 0
ODC_UNORDERED = 1
ODC_MAX_FUSED = 8
ODC_OUT_F32 = 0
ODC_OUT_BF16 = 1

EXPORTS = (
    "odc_init_layout", "odc_free_layout", "odc_num_ranks", "odc_num_tensors", "odc_numel",
    "odc_shard_elems", "odc_valid_elems", "odc_rank_arena_elems", "odc_full_elems",
    "odc_shard_offset", "odc_full_offset", "odc_gather", "odc_scatter_accumulate",
    "odc_reset_accum", "odc_forget_accum", "odc_scatter_accumulate_weighted", "odc_scatter_accumulate_multi", "odc_retrieve_grads",
    "odc_stage_slot_elems", "odc_stage_flag_count", "odc_stage_snapshot_count", "odc_stage_init",
    "odc_stage_push", "odc_stage_drain", "odc_stage_drain_noalloc", "odc_reset_accum_wide",
    "odc_scatter_accumulate_wide", "odc_retrieve_grads_wide", "odc_hybrid_group_of",
    "odc_gather_hybrid", "odc_scatter_accumulate_hybrid", "odc_reduce_groups", "odc_strerror", "odc_last_hip_error", "odc_probe_copy", "odc_tune",
)

_i64 = ctypes.c_int64
_int = ctypes.c_int
_vp = ctypes.c_void_p
_lib = None


class OdcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = strerror(code)
        if code == ODC_ERR_HIP:
            detail += f" [hipError {lib().odc_last_hip_error()}]"
        super().__init__(f"{where}: {detail} ({code})")


def lib():
    """Load the built library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it first (python -m paper_2601_19362_amd.build); "
                "there is no CPU fallback")
        # torch ships its own HIP runtime; import it first so that the dynamic loader binds
        # this library to that same runtime (one runtime per process: streams and device
        # pointers made by torch must be valid in the launches made here).
        import torch  # noqa: F401

        L = ctypes.CDLL(LIB_PATH)
        L.odc_init_layout.restype = _int
        L.odc_init_layout.argtypes = [_int, _int, ctypes.POINTER(_i64), _int, ctypes.POINTER(_vp)]
        L.odc_free_layout.restype = None
        L.odc_free_layout.argtypes = [_vp]
        for name in ("odc_num_ranks", "odc_num_tensors"):
            getattr(L, name).restype = _int
            getattr(L, name).argtypes = [_vp]
        for name in ("odc_numel", "odc_shard_elems", "odc_shard_offset", "odc_full_offset"):
            getattr(L, name).restype = _i64
            getattr(L, name).argtypes = [_vp, _int]
        L.odc_valid_elems.restype = _i64
        L.odc_valid_elems.argtypes = [_vp, _int, _int]
        for name in ("odc_rank_arena_elems", "odc_full_elems"):
            getattr(L, name).restype = _i64
            getattr(L, name).argtypes = [_vp]
        L.odc_gather.restype = _int
        L.odc_gather.argtypes = [_vp, ctypes.POINTER(_vp), _vp, _vp]
        L.odc_scatter_accumulate.restype = _int
        L.odc_scatter_accumulate.argtypes = [_vp, _vp, ctypes.POINTER(_vp), _int, _int, _int, _vp]
        L.odc_scatter_accumulate_weighted.restype = _int
        L.odc_scatter_accumulate_weighted.argtypes = [_vp, _vp, ctypes.POINTER(_vp), _int, _int, ctypes.c_float,
                                                      _int, _vp]
        L.odc_scatter_accumulate_multi.restype = _int
        L.odc_scatter_accumulate_multi.argtypes = [_vp, _int, ctypes.POINTER(_vp), ctypes.POINTER(_vp),
                                                   ctypes.POINTER(_int), ctypes.POINTER(_int), _int, _vp]
        for name in ("odc_stage_slot_elems", "odc_stage_flag_count", "odc_stage_snapshot_count"):
            getattr(L, name).restype = _i64
            getattr(L, name).argtypes = [_vp]
        L.odc_stage_init.restype = _int
        L.odc_stage_init.argtypes = [_vp, _vp, _vp]
        L.odc_stage_push.restype = _int
        L.odc_stage_push.argtypes = [_vp, _vp, ctypes.POINTER(_vp), _vp, _int, _vp]
        L.odc_stage_drain.restype = _int
        L.odc_stage_drain.argtypes = [_vp, ctypes.POINTER(_vp), _vp, _vp, ctypes.POINTER(_vp), _vp]
        L.odc_stage_drain_noalloc.restype = _int
        L.odc_stage_drain_noalloc.argtypes = [_vp, ctypes.POINTER(_vp), _vp, ctypes.POINTER(_vp), _vp]
        L.odc_reset_accum_wide.restype = _int
        L.odc_reset_accum_wide.argtypes = [_vp, ctypes.POINTER(_vp), _vp]
        L.odc_scatter_accumulate_wide.restype = _int
        L.odc_scatter_accumulate_wide.argtypes = [_vp, _vp, ctypes.POINTER(_vp), _vp]
        L.odc_retrieve_grads_wide.restype = _int
        L.odc_retrieve_grads_wide.argtypes = [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.c_float, _int, _vp]
        L.odc_hybrid_group_of.restype = _int
        L.odc_hybrid_group_of.argtypes = [_vp, _int, _int]
        L.odc_gather_hybrid.restype = _int
        L.odc_gather_hybrid.argtypes = [_vp, _int, ctypes.POINTER(_vp), _int, _vp, _vp]
        L.odc_scatter_accumulate_hybrid.restype = _int
        L.odc_scatter_accumulate_hybrid.argtypes = [_vp, _int, _vp, ctypes.POINTER(_vp), _int, _int, _int, _vp]
        L.odc_reduce_groups.restype = _int
        L.odc_reduce_groups.argtypes = [_vp, _int, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _vp]
        L.odc_retrieve_grads.restype = _int
        L.odc_retrieve_grads.argtypes = [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.c_float, _int, _vp]
        L.odc_reset_accum.restype = _int
        L.odc_reset_accum.argtypes = [_vp, ctypes.POINTER(_vp), _vp]
        L.odc_forget_accum.restype = _int
        L.odc_forget_accum.argtypes = [_vp, ctypes.POINTER(_vp)]
        L.odc_strerror.restype = ctypes.c_char_p
        L.odc_strerror.argtypes = [_int]
        L.odc_last_hip_error.restype = _int
        L.odc_last_hip_error.argtypes = []
        L.odc_probe_copy.restype = _int
        L.odc_probe_copy.argtypes = [_vp, _vp, _i64, _vp]
        L.odc_tune.restype = _int
        L.odc_tune.argtypes = [ctypes.c_char_p, _int]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().odc_strerror(int(code)).decode()


def _ptr(x) -> Optional[int]:
    """Device (or raw) address of a torch tensor, an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _stream(stream) -> Optional[int]:
    """hipStream_t of a torch stream object, a raw handle, or torch's current stream."""
    if stream is None:
        import torch

        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


class PtrArray:
    """A host array of R device pointers, built once and reused across calls."""

    def __init__(self, tensors: Sequence):
        self.n = len(tensors)
        self.array = (_vp * self.n)(*[_ptr(t) for t in tensors])
        self.keepalive = list(tensors)


def _ptr_array(x, R: int):
    if isinstance(x, PtrArray):
        if x.n != R:
            raise ValueError(f"expected {R} pointers, got {x.n}")
        return x.array
    if x is None:
        return None
    if len(x) != R:
        raise ValueError(f"expected {R} pointers, got {len(x)}")
    return (_vp * R)(*[_ptr(t) for t in x])


class Layout:
    """Owner of an odc_layout_t handle.  Methods mirror the C entry points one to one."""

    def __init__(self, R: int, numel: Sequence[int], host_only: bool = False):
        T = len(numel)
        arr = (_i64 * max(T, 1))(*[int(n) for n in numel])
        handle = _vp()
        flags = ODC_LAYOUT_HOST_ONLY if host_only else 0
        rc = lib().odc_init_layout(int(R), T, arr, flags, ctypes.byref(handle))
        if rc != ODC_OK:
            raise OdcError(rc, "odc_init_layout")
        self._h = handle
        self.R = int(R)
        self.T = T

    # -- lifetime
    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().odc_free_layout(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    # -- queries
    def num_ranks(self) -> int:
        return lib().odc_num_ranks(self._h)

    def num_tensors(self) -> int:
        return lib().odc_num_tensors(self._h)

    def numel(self, t: int = 0) -> int:
        return lib().odc_numel(self._h, t)

    def shard_elems(self, t: int = 0) -> int:
        return lib().odc_shard_elems(self._h, t)

    def valid_elems(self, t: int, r: int) -> int:
        return lib().odc_valid_elems(self._h, t, r)

    def rank_arena_elems(self) -> int:
        return lib().odc_rank_arena_elems(self._h)

    def full_elems(self) -> int:
        return lib().odc_full_elems(self._h)

    def shard_offset(self, t: int) -> int:
        return lib().odc_shard_offset(self._h, t)

    def full_offset(self, t: int) -> int:
        return lib().odc_full_offset(self._h, t)

    # -- launches (raise OdcError on a non-zero code)
    def gather(self, param_shards, full_out, stream=None) -> None:
        rc = gather_rc(self, param_shards, full_out, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_gather")

    def scatter_accumulate(self, grad_full, accum_shards, worker: int, microbatch: int,
                           flags: int = ODC_ORDERED, stream=None) -> None:
        rc = scatter_accumulate_rc(self, grad_full, accum_shards, worker, microbatch, flags, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_scatter_accumulate")

    def scatter_accumulate_weighted(self, grad_full, accum_shards, worker: int, microbatch: int, weight: float,
                                    flags: int = ODC_ORDERED, stream=None) -> None:
        rc = lib().odc_scatter_accumulate_weighted(self.handle, _ptr(grad_full), _ptr_array(accum_shards, self.R),
                                                   int(worker), int(microbatch), float(weight), int(flags),
                                                   _stream(stream))
        if rc != ODC_OK:
            raise OdcError(rc, "odc_scatter_accumulate_weighted")

    def scatter_accumulate_multi(self, grads, accum_shards, workers, microbatches, flags: int = ODC_ORDERED,
                                 stream=None) -> None:
        rc = scatter_accumulate_multi_rc(self, grads, accum_shards, workers, microbatches, flags, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_scatter_accumulate_multi")

    def stage_slot_elems(self) -> int:
        return lib().odc_stage_slot_elems(self._h)

    def stage_flag_count(self) -> int:
        return lib().odc_stage_flag_count(self._h)

    def stage_snapshot_count(self) -> int:
        return lib().odc_stage_snapshot_count(self._h)

    def stage_init(self, flags, stream=None) -> None:
        rc = lib().odc_stage_init(self._h, _ptr(flags), _stream(stream))
        if rc != ODC_OK:
            raise OdcError(rc, "odc_stage_init")

    def stage_push(self, grad_full, staging_shards, flags, worker: int, stream=None) -> None:
        rc = stage_push_rc(self, grad_full, staging_shards, flags, worker, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_stage_push")

    def stage_drain(self, staging_shards, flags, snapshot, accum_shards, stream=None) -> None:
        rc = stage_drain_rc(self, staging_shards, flags, snapshot, accum_shards, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_stage_drain")

    def stage_drain_noalloc(self, staging_shards, flags, accum_shards, stream=None) -> None:
        rc = stage_drain_noalloc_rc(self, staging_shards, flags, accum_shards, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_stage_drain_noalloc")

    # -- wide (binary64) accumulators of the unordered mode
    def reset_accum_wide(self, accum64_shards, stream=None) -> None:
        rc = lib().odc_reset_accum_wide(self._h, _ptr_array(accum64_shards, self.R), _stream(stream))
        if rc != ODC_OK:
            raise OdcError(rc, "odc_reset_accum_wide")

    def scatter_accumulate_wide(self, grad_full, accum64_shards, stream=None) -> None:
        rc = lib().odc_scatter_accumulate_wide(self._h, _ptr(grad_full), _ptr_array(accum64_shards, self.R),
                                               _stream(stream))
        if rc != ODC_OK:
            raise OdcError(rc, "odc_scatter_accumulate_wide")

    def retrieve_grads_wide(self, accum64_shards, out_shards, scale: float = 1.0, out_dtype: int = ODC_OUT_F32,
                            stream=None) -> None:
        rc = lib().odc_retrieve_grads_wide(self._h, _ptr_array(accum64_shards, self.R), _ptr_array(out_shards, self.R),
                                           float(scale), int(out_dtype), _stream(stream))
        if rc != ODC_OK:
            raise OdcError(rc, "odc_retrieve_grads_wide")

    # -- hybrid sharding: group-major lists of groups * R buffers
    def hybrid_group_of(self, groups: int, world_worker: int) -> int:
        return lib().odc_hybrid_group_of(self._h, int(groups), int(world_worker))

    def gather_hybrid(self, groups: int, group_param_shards, world_worker: int, full_out, stream=None) -> None:
        rc = lib().odc_gather_hybrid(self._h, int(groups), _ptr_array(group_param_shards, groups * self.R),
                                     int(world_worker), _ptr(full_out), _stream(stream))
        if rc != ODC_OK:
            raise OdcError(rc, "odc_gather_hybrid")

    def scatter_accumulate_hybrid(self, groups: int, grad_full, group_accum_shards, world_worker: int,
                                  microbatch: int, flags: int = ODC_ORDERED, stream=None) -> None:
        rc = scatter_accumulate_hybrid_rc(self, groups, grad_full, group_accum_shards, world_worker, microbatch,
                                          flags, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_scatter_accumulate_hybrid")

    def reduce_groups(self, groups: int, group_accum_shards, out_shards, stream=None) -> None:
        rc = reduce_groups_rc(self, groups, group_accum_shards, out_shards, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_reduce_groups")

    def retrieve_grads(self, accum_shards, out_shards, scale: float = 1.0, out_dtype: int = ODC_OUT_F32,
                       stream=None) -> None:
        rc = retrieve_grads_rc(self, accum_shards, out_shards, scale, out_dtype, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_retrieve_grads")

    def forget_accum(self, accum_shards) -> None:
        rc = lib().odc_forget_accum(self._h, _ptr_array(accum_shards, self.R))
        if rc != ODC_OK:
            raise OdcError(rc, "odc_forget_accum")

    def reset_accum(self, accum_shards, stream=None) -> None:
        rc = reset_accum_rc(self, accum_shards, stream)
        if rc != ODC_OK:
            raise OdcError(rc, "odc_reset_accum")


# Raw-code variants (used by tests of the error paths; a stream of 0 skips the torch lookup).
def gather_rc(layout: Layout, param_shards, full_out, stream=None) -> int:
    return lib().odc_gather(layout.handle, _ptr_array(param_shards, layout.R), _ptr(full_out),
                            _stream(stream))


def scatter_accumulate_rc(layout: Layout, grad_full, accum_shards, worker: int, microbatch: int,
                          flags: int = ODC_ORDERED, stream=None) -> int:
    return lib().odc_scatter_accumulate(layout.handle, _ptr(grad_full),
                                        _ptr_array(accum_shards, layout.R), int(worker),
                                        int(microbatch), int(flags), _stream(stream))


def scatter_accumulate_multi_rc(layout: Layout, grads, accum_shards, workers, microbatches,
                                flags: int = ODC_ORDERED, stream=None) -> int:
    k = len(grads)
    garr = (_vp * max(k, 1))(*[_ptr(g) for g in grads])
    warr = (_int * max(k, 1))(*[int(w) for w in workers])
    marr = (_int * max(k, 1))(*[int(m) for m in microbatches])
    return lib().odc_scatter_accumulate_multi(layout.handle, k, garr, _ptr_array(accum_shards, layout.R), warr,
                                              marr, int(flags), _stream(stream))


def stage_push_rc(layout: Layout, grad_full, staging_shards, flags, worker: int, stream=None) -> int:
    return lib().odc_stage_push(layout.handle, _ptr(grad_full), _ptr_array(staging_shards, layout.R), _ptr(flags),
                                int(worker), _stream(stream))


def stage_drain_rc(layout: Layout, staging_shards, flags, snapshot, accum_shards, stream=None) -> int:
    return lib().odc_stage_drain(layout.handle, _ptr_array(staging_shards, layout.R), _ptr(flags), _ptr(snapshot),
                                 _ptr_array(accum_shards, layout.R), _stream(stream))


def stage_drain_noalloc_rc(layout: Layout, staging_shards, flags, accum_shards, stream=None) -> int:
    return lib().odc_stage_drain_noalloc(layout.handle, _ptr_array(staging_shards, layout.R), _ptr(flags),
                                         _ptr_array(accum_shards, layout.R), _stream(stream))


def scatter_accumulate_hybrid_rc(layout: Layout, groups: int, grad_full, group_accum_shards, world_worker: int,
                                 microbatch: int, flags: int = ODC_ORDERED, stream=None) -> int:
    return lib().odc_scatter_accumulate_hybrid(layout.handle, int(groups), _ptr(grad_full),
                                               _ptr_array(group_accum_shards, max(groups, 0) * layout.R),
                                               int(world_worker), int(microbatch), int(flags), _stream(stream))


def reduce_groups_rc(layout: Layout, groups: int, group_accum_shards, out_shards, stream=None) -> int:
    return lib().odc_reduce_groups(layout.handle, int(groups),
                                   _ptr_array(group_accum_shards, max(groups, 0) * layout.R),
                                   _ptr_array(out_shards, layout.R), _stream(stream))


def retrieve_grads_rc(layout: Layout, accum_shards, out_shards, scale: float = 1.0,
                      out_dtype: int = ODC_OUT_F32, stream=None) -> int:
    return lib().odc_retrieve_grads(layout.handle, _ptr_array(accum_shards, layout.R),
                                    _ptr_array(out_shards, layout.R), float(scale), int(out_dtype),
                                    _stream(stream))


def reset_accum_rc(layout: Layout, accum_shards, stream=None) -> int:
    return lib().odc_reset_accum(layout.handle, _ptr_array(accum_shards, layout.R), _stream(stream))


def probe_copy(dst, src, nbytes: int, stream=None) -> None:
    rc = lib().odc_probe_copy(_ptr(dst), _ptr(src), int(nbytes), _stream(stream))
    if rc != ODC_OK:
        raise OdcError(rc, "odc_probe_copy")


def tune(knob: str, value: int) -> None:
    rc = lib().odc_tune(knob.encode(), int(value))
    if rc != ODC_OK:
        raise OdcError(rc, f"odc_tune({knob}={value})")


def reset_tuning() -> None:
    tune("defaults", 0)
