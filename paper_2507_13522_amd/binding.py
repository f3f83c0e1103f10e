"""ctypes binding of include/shadow.h and include/shadow_measure.h: argument marshalling only.

Function names follow the C ABI (``shadow_layout_create`` -> ``Layout``,
``shadow_init`` -> ``Shadow`` and its methods ``apply_bucket``, ``snapshot``,
``sync`` ...).  Pointers are plain integers (for torch tensors: ``data_ptr()``),
streams are ``hipStream_t`` handles as integers (``torch.cuda.Stream.cuda_stream``).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

from . import build as _build

GRAD_F32, GRAD_BF16 = 0, 1
REDUCE_MEAN, REDUCE_SUM = 0, 1
OPT_ADAMW, OPT_ADAM, OPT_SGD = 0, 1, 2
K_FOLD_ADAMW, K_FOLD_SUMSQ, K_NORM, K_ADAMW, K_SNAPSHOT = 0, 1, 2, 3, 4

OK, EINVAL, EBUCKET, EDUP, ESTEP, EBUSY, EHIP, ENOMEM, ETOOBIG = 0, -1, -2, -3, -4, -5, -6, -7, -8
STATIC_MAX_ARENA_NUMEL, STATIC_MAX_BUCKETS = 1 << 27, 4096


class TensorDesc(C.Structure):
    _fields_ = [("numel", C.c_uint64), ("weight_decay", C.c_uint32), ("reserved", C.c_uint32)]


class LaunchShape(C.Structure):
    """shadow_launch_shape: every field 0 = the library's default."""
    _fields_ = [("fold_block", C.c_uint32), ("fused_block", C.c_uint32), ("sweep_block", C.c_uint32),
                ("fold_waves_per_cu", C.c_uint32), ("fused_waves_per_cu", C.c_uint32), ("sweep_waves_per_cu", C.c_uint32),
                ("drain_blocks", C.c_uint32), ("reserved", C.c_uint32), ("max_launch_threads", C.c_uint64)]


class HParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("max_grad_norm", C.c_float), ("num_workers", C.c_uint32),
                ("grad_dtype", C.c_uint32), ("reduce_op", C.c_uint32), ("num_streams", C.c_uint32),
                ("optimizer", C.c_uint32), ("batch_bytes", C.c_uint64), ("launch", LaunchShape)]


class DevicePlan(C.Structure):
    _fields_ = [("block_bytes", C.c_uint64), ("param_offset", C.c_uint64), ("m_offset", C.c_uint64), ("v_offset", C.c_uint64),
                ("scratch_offset", C.c_uint64), ("staging_offset", C.c_uint64), ("snap_param_offset", C.c_uint64),
                ("snap_m_offset", C.c_uint64), ("snap_v_offset", C.c_uint64)]


class ShadowError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = shadow_strerror(status)
        if status == EHIP:
            msg += ": " + lib().shadow_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({status})")


_lib = None

_SIGS = {
    "shadow_layout_create": [C.POINTER(C.c_void_p), C.POINTER(TensorDesc), C.c_uint32, C.POINTER(C.c_uint32), C.c_uint32, C.c_uint64],
    "shadow_layout_destroy": [C.c_void_p],
    "shadow_layout_num_buckets": [C.c_void_p, C.POINTER(C.c_uint32)],
    "shadow_layout_num_params": [C.c_void_p, C.POINTER(C.c_uint64)],
    "shadow_layout_arena_numel": [C.c_void_p, C.POINTER(C.c_uint64)],
    "shadow_layout_bucket": [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)],
    "shadow_layout_tensor": [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint32), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)],
    "shadow_layout_device_plan": [C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.POINTER(DevicePlan)],
    "shadow_layout_arena_stride": [C.c_void_p, C.POINTER(C.c_uint64)],
    "shadow_layout_staging_bytes": [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint64)],
    "shadow_layout_staging_view": [C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.POINTER(C.c_uint64)],
    "shadow_init": [C.POINTER(C.c_void_p), C.c_void_p, C.POINTER(HParams), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p)],
    "shadow_num_buckets": [C.c_void_p, C.POINTER(C.c_uint32)],
    "shadow_bucket_info": [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)],
    "shadow_apply_bucket": [C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p), C.c_uint64, C.c_void_p],
    "shadow_record_consumed": [C.c_void_p, C.c_uint32, C.c_void_p],
    "shadow_ingest_attach": [C.c_void_p, C.c_void_p, C.c_uint64],
    "shadow_ingest_bucket": [C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p), C.c_uint64, C.c_void_p],
    "shadow_snapshot": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64), C.c_void_p],
    "shadow_snapshot_attach": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "shadow_snapshot_arm": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "shadow_snapshot_record": [C.c_void_p, C.c_void_p],
    "shadow_snapshot_wait": [C.c_void_p, C.POINTER(C.c_uint64)],
    "shadow_apply_iteration_static": [C.c_void_p, C.POINTER(HParams), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.POINTER(C.c_void_p), C.c_uint64, C.c_void_p],
    "shadow_sync": [C.c_void_p],
    "shadow_destroy": [C.c_void_p],
    "shadow_step": [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)],
    "shadow_bucket_stream": [C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p)],
    "shadow_clip_state": [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_double)],
    "shadow_set_lr": [C.c_void_p, C.c_float],
    "shadow_profile_enable": [C.c_void_p, C.c_int32],
    "shadow_profile_kinds": [C.c_void_p, C.c_uint32],
    "shadow_profile_read": [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint64), C.POINTER(C.c_double)],
    "shadow_copy_probe": [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64],
    "shadow_stream_probe": [C.POINTER(C.c_void_p), C.c_uint32, C.POINTER(C.c_void_p), C.c_uint32, C.c_void_p, C.c_uint64, C.c_void_p,
                            C.c_uint32, C.c_uint32],
}
EXPORTS = sorted(list(_SIGS) + ["shadow_strerror", "shadow_last_hip_error", "shadow_build_id"])


def lib() -> C.CDLL:
    """Load libshadow.so.  The library is built with hipcc first when none exists or when the one that exists
    was built from other sources than the ones beside it (it embeds a hash of them)."""
    global _lib
    if _lib is None:
        path = _build.LIB
        if _build.stale():
            print("paper_2507_13522_amd: libshadow.so is missing or older than its sources, building it", flush=True)
            _build.build_library()
        L = C.CDLL(path)
        for name, args in _SIGS.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = C.c_int32
        L.shadow_strerror.argtypes = [C.c_int32]
        L.shadow_strerror.restype = C.c_char_p
        L.shadow_last_hip_error.argtypes = []
        L.shadow_last_hip_error.restype = C.c_char_p
        L.shadow_build_id.argtypes = []
        L.shadow_build_id.restype = C.c_char_p
        if L.shadow_build_id().decode() != _build.ID_TAG + _build.source_id():
            raise RuntimeError(f"{path} was not built from the sources beside it")
        _lib = L
    return _lib


def shadow_strerror(status: int) -> str:
    return lib().shadow_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise ShadowError(status, where)


def shadow_copy_probe(dst: int, src: int, nbytes: int, stream: int = 0, max_launch_threads: int = 0) -> None:
    _check(lib().shadow_copy_probe(dst, src, nbytes, stream, max_launch_threads), "shadow_copy_probe")


def shadow_stream_probe(dst: Sequence[int], src: Sequence[int], nbytes: int, sink: Optional[int] = None, stream: int = 0, block: int = 0,
                        waves_per_cu: int = 0) -> int:
    """Status of shadow_stream_probe (OK, or EINVAL for a mix of streams the kernel is not built for)."""
    d = (C.c_void_p * max(len(dst), 1))(*dst)
    s = (C.c_void_p * max(len(src), 1))(*src)
    return int(lib().shadow_stream_probe(d, len(dst), s, len(src), sink, nbytes, stream, block, waves_per_cu))


class Layout:
    """shadow_layout_*: tensors = [(numel, weight_decay_flag)] in model order."""

    def __init__(self, tensors: Sequence[Tuple[int, bool]], grad_elem_bytes: int, bucket_cap_bytes: int = 0,
                 bucket_of_tensor: Optional[Sequence[int]] = None):
        n = len(tensors)
        arr = (TensorDesc * max(n, 1))()
        for i, (numel, wd) in enumerate(tensors):
            arr[i].numel, arr[i].weight_decay, arr[i].reserved = int(numel), int(bool(wd)), 0
        fixed = None
        if bucket_of_tensor is not None:
            if len(bucket_of_tensor) != n:
                raise ValueError("bucket_of_tensor length")
            fixed = (C.c_uint32 * max(n, 1))(*[int(b) for b in bucket_of_tensor])
        h = C.c_void_p()
        _check(lib().shadow_layout_create(C.byref(h), arr, n, fixed, grad_elem_bytes, bucket_cap_bytes), "shadow_layout_create")
        self._h = h
        self.num_tensors = n
        v32, v64 = C.c_uint32(), C.c_uint64()
        _check(lib().shadow_layout_num_buckets(h, C.byref(v32)), "shadow_layout_num_buckets")
        self.num_buckets = v32.value
        _check(lib().shadow_layout_num_params(h, C.byref(v64)), "shadow_layout_num_params")
        self.num_params = v64.value
        _check(lib().shadow_layout_arena_numel(h, C.byref(v64)), "shadow_layout_arena_numel")
        self.arena_numel = v64.value

    def bucket(self, b: int) -> Tuple[int, int, int]:
        """-> (arena offset, numel, number of tensors)"""
        off, n, nt = C.c_uint64(), C.c_uint64(), C.c_uint32()
        _check(lib().shadow_layout_bucket(self._h, b, C.byref(off), C.byref(n), C.byref(nt)), "shadow_layout_bucket")
        return off.value, n.value, nt.value

    def tensor(self, t: int) -> Tuple[int, int, int]:
        """-> (bucket, offset in bucket, arena offset)"""
        b, ob, oa = C.c_uint32(), C.c_uint64(), C.c_uint64()
        _check(lib().shadow_layout_tensor(self._h, t, C.byref(b), C.byref(ob), C.byref(oa)), "shadow_layout_tensor")
        return b.value, ob.value, oa.value

    def device_plan(self, with_scratch: bool, staging_bytes: int, with_snapshot_set: bool = False) -> Optional[DevicePlan]:
        """Offsets of the arenas, of a snapshot staging set and of a gradient buffer of staging_bytes (0: none) inside
        one 256 GiB allocation, or None when they do not fit."""
        plan = DevicePlan()
        rc = lib().shadow_layout_device_plan(self._h, int(with_scratch), int(with_snapshot_set), staging_bytes, C.byref(plan))
        if rc == ENOMEM:
            return None
        _check(rc, "shadow_layout_device_plan")
        return plan

    def arena_stride(self) -> int:
        """Recommended byte distance between the arenas inside one device allocation."""
        v = C.c_uint64()
        _check(lib().shadow_layout_arena_stride(self._h, C.byref(v)), "shadow_layout_arena_stride")
        return v.value

    def staging_bytes(self, num_workers: int) -> int:
        v = C.c_uint64()
        _check(lib().shadow_layout_staging_bytes(self._h, num_workers, C.byref(v)), "shadow_layout_staging_bytes")
        return v.value

    def staging_view(self, num_workers: int, bucket: int, worker: int) -> int:
        v = C.c_uint64()
        _check(lib().shadow_layout_staging_view(self._h, num_workers, bucket, worker, C.byref(v)), "shadow_layout_staging_view")
        return v.value

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().shadow_layout_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def shadow_apply_iteration_static(layout: "Layout", hp: HParams, d_param: int, d_m: int, d_v: Optional[int],
                                  d_reduced: Optional[int], views: Sequence[int], step: int, stream: int = 0) -> int:
    """One whole iteration without a context and without any allocation; views: num_buckets * W device addresses,
    bucket-major.  Returns the status (no exception), so that callers can test for ETOOBIG."""
    arr = views if isinstance(views, C.Array) else (C.c_void_p * len(views))(*[int(p) for p in views])
    return int(lib().shadow_apply_iteration_static(layout._h, C.byref(hp), d_param, d_m, d_v or None, d_reduced or None, arr,
                                                   step, stream or None))


class Shadow:
    """shadow_init .. shadow_destroy.  Arena arguments are device addresses (ints)."""

    def __init__(self, layout: Layout, hp: HParams, d_param: int, d_m: int, d_v: int, d_reduced: Optional[int] = None,
                 start_step: int = 0, streams: Optional[Sequence[int]] = None):
        self.layout = layout
        self.hp = hp
        sarr = None
        if streams is not None:
            if len(streams) != hp.num_streams:
                raise ValueError("need hp.num_streams stream handles")
            sarr = (C.c_void_p * len(streams))(*[int(s) for s in streams])
        h = C.c_void_p()
        _check(lib().shadow_init(C.byref(h), layout._h, C.byref(hp), d_param, d_m, d_v or None, d_reduced or None,
                                 start_step, sarr), "shadow_init")
        self._h = h
        self._views = {}

    def views_array(self, ptrs: Sequence[int]):
        """Marshal W device addresses once; the result can be passed to apply_bucket repeatedly."""
        return (C.c_void_p * len(ptrs))(*[int(p) for p in ptrs])

    def num_buckets(self) -> int:
        v = C.c_uint32()
        _check(lib().shadow_num_buckets(self._h, C.byref(v)), "shadow_num_buckets")
        return v.value

    def bucket_info(self, bucket_id: int) -> Tuple[int, int]:
        """-> (arena offset, numel)"""
        off, n = C.c_uint64(), C.c_uint64()
        _check(lib().shadow_bucket_info(self._h, bucket_id, C.byref(off), C.byref(n)), "shadow_bucket_info")
        return off.value, n.value

    def apply_bucket(self, bucket_id: int, views, step: int, ready_event: Optional[int] = None) -> None:
        """ready_event: hipEvent_t handle (int) recorded by the producer of the views, or None."""
        if not isinstance(views, C.Array):
            views = self.views_array(views)
        _check(lib().shadow_apply_bucket(self._h, bucket_id, views, step, ready_event or None), "shadow_apply_bucket")

    def try_apply_bucket(self, bucket_id: int, views, step: int, ready_event: Optional[int] = None) -> int:
        if not isinstance(views, C.Array):
            views = self.views_array(views)
        return int(lib().shadow_apply_bucket(self._h, bucket_id, views, step, ready_event or None))

    def record_consumed(self, bucket_id: int, event: int) -> None:
        _check(lib().shadow_record_consumed(self._h, bucket_id, event), "shadow_record_consumed")

    def ingest_attach(self, d_ring: int, ring_bytes: int) -> None:
        _check(lib().shadow_ingest_attach(self._h, d_ring, ring_bytes), "shadow_ingest_attach")

    def ingest_bucket(self, bucket_id: int, host_views, step: int, ready_event: Optional[int] = None) -> None:
        if not isinstance(host_views, C.Array):
            host_views = self.views_array(host_views)
        _check(lib().shadow_ingest_bucket(self._h, bucket_id, host_views, step, ready_event or None), "shadow_ingest_bucket")

    def snapshot(self, dst_param: Optional[int], dst_m: Optional[int], dst_v: Optional[int],
                 done_event: Optional[int] = None) -> int:
        st = C.c_uint64()
        _check(lib().shadow_snapshot(self._h, dst_param or None, dst_m or None, dst_v or None, C.byref(st), done_event or None),
               "shadow_snapshot")
        return st.value

    def snapshot_attach(self, d_stage_param: int, d_stage_m: int, d_stage_v: Optional[int]) -> None:
        _check(lib().shadow_snapshot_attach(self._h, d_stage_param, d_stage_m, d_stage_v or None), "shadow_snapshot_attach")

    def snapshot_arm(self, h_dst_param: Optional[int] = None, h_dst_m: Optional[int] = None, h_dst_v: Optional[int] = None) -> None:
        _check(lib().shadow_snapshot_arm(self._h, h_dst_param or None, h_dst_m or None, h_dst_v or None), "shadow_snapshot_arm")

    def try_snapshot_arm(self, h_dst_param: Optional[int] = None, h_dst_m: Optional[int] = None, h_dst_v: Optional[int] = None) -> int:
        return int(lib().shadow_snapshot_arm(self._h, h_dst_param or None, h_dst_m or None, h_dst_v or None))

    def snapshot_record(self, event: int) -> None:
        _check(lib().shadow_snapshot_record(self._h, event), "shadow_snapshot_record")

    def snapshot_wait(self) -> int:
        st = C.c_uint64()
        _check(lib().shadow_snapshot_wait(self._h, C.byref(st)), "shadow_snapshot_wait")
        return st.value

    def sync(self) -> None:
        _check(lib().shadow_sync(self._h), "shadow_sync")

    def step(self) -> Tuple[int, int]:
        s, pend = C.c_uint64(), C.c_uint32()
        _check(lib().shadow_step(self._h, C.byref(s), C.byref(pend)), "shadow_step")
        return s.value, pend.value

    def bucket_stream(self, bucket_id: int) -> int:
        s = C.c_void_p()
        _check(lib().shadow_bucket_stream(self._h, bucket_id, C.byref(s)), "shadow_bucket_stream")
        return s.value or 0

    def clip_state(self) -> Tuple[float, float]:
        c, s = C.c_float(), C.c_double()
        _check(lib().shadow_clip_state(self._h, C.byref(c), C.byref(s)), "shadow_clip_state")
        return c.value, s.value

    def set_lr(self, lr: float) -> None:
        _check(lib().shadow_set_lr(self._h, lr), "shadow_set_lr")

    def profile_enable(self, on: bool) -> None:
        _check(lib().shadow_profile_enable(self._h, int(on)), "shadow_profile_enable")

    def profile_kinds(self, kind_mask: int) -> None:
        _check(lib().shadow_profile_kinds(self._h, kind_mask), "shadow_profile_kinds")

    def profile_read(self, kind: int) -> Tuple[int, float]:
        n, ms = C.c_uint64(), C.c_double()
        _check(lib().shadow_profile_read(self._h, kind, C.byref(n), C.byref(ms)), "shadow_profile_read")
        return n.value, ms.value

    def destroy(self) -> None:
        if getattr(self, "_h", None):
            lib().shadow_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
