"""ctypes binding of libhp.so - argument marshalling only.

Function names mirror the C ABI in include/hp.h (hp_plan_create, hp_forward,
hp_backward, ...).  Every step of the transform runs in the library's HIP
kernels; there is no Python or CPU fallback: if the library has not been built
or cannot be loaded, every entry point raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

from .workloads import Grid, TokenMap

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libhp.so")

HP_OK = 0
HP_EINVAL, HP_ELAYOUT, HP_EMAP, HP_ENOMEM, HP_EHIP, HP_ESTATE, HP_EALIGN = -1, -2, -3, -4, -5, -6, -7


class HpError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        msg = _lib().hp_strerror(code).decode()
        if code == HP_EHIP:
            msg += f" (hipError {_lib().hp_last_hip_error()})"
        super().__init__(f"{what}: {msg} [{code}]")


class hp_layout_t(C.Structure):
    _fields_ = [("tp", C.c_int32), ("cp", C.c_int32), ("dp", C.c_int32), ("pp", C.c_int32),
                ("rank_offset", C.c_int32), ("tp_mode", C.c_int32), ("cp_split", C.c_int32),
                ("row_order", C.c_int32)]


class hp_token_map_t(C.Structure):
    _fields_ = [("batch", C.c_int32), ("seq", C.c_int32), ("hidden", C.c_int32),
                ("dtype", C.c_int32), ("n_images", C.c_int32),
                ("img_sample", C.POINTER(C.c_int32)), ("img_start", C.POINTER(C.c_int32)),
                ("img_len", C.POINTER(C.c_int32)), ("img_src_dp", C.POINTER(C.c_int32))]


class hp_plan_info_t(C.Structure):
    _fields_ = [("n_src_bufs", C.c_int32), ("n_dst_bufs", C.c_int32),
                ("src_copies", C.c_int32), ("dst_copies", C.c_int32),
                ("n_rows", C.c_int64), ("row_bytes", C.c_int64), ("dst_rows_per_buf", C.c_int64),
                ("boundary_bytes", C.c_int64), ("fwd_bytes", C.c_int64), ("bwd_bytes", C.c_int64),
                ("n_segments", C.c_int32), ("n_tiles", C.c_int32),
                ("on_device", C.c_int32), ("device", C.c_int32), ("n_maps", C.c_int32),
                ("elem_bytes", C.c_int32), ("bwd_accum_bytes", C.c_int64),
                ("n_edges", C.c_int32), ("reserved", C.c_int32)]


class hp_segment_t(C.Structure):
    _fields_ = [("src_buf", C.c_int32), ("dst_buf0", C.c_int32), ("src_row0", C.c_int64),
                ("dst_row0", C.c_int64), ("n_rows", C.c_int64), ("dst_row_stride", C.c_int64)]


class hp_launch_t(C.Structure):
    _fields_ = [("tile_bytes", C.c_int32), ("block_threads", C.c_int32),
                ("waves_per_cu", C.c_int32), ("nontemporal", C.c_int32)]


EXPORTS = ["hp_plan_create", "hp_plan_create_host", "hp_plan_create_batched", "hp_plan_create_joined",
           "hp_plan_destroy",
           "hp_release_cached_memory", "hp_forget_tuned_shapes",
           "hp_plan_query", "hp_plan_src_rows", "hp_plan_segments", "hp_plan_get_launch",
           "hp_plan_set_launch", "hp_plan_tune", "hp_plan_tune_accumulate", "hp_forward", "hp_backward", "hp_backward_accumulate", "hp_forward_static", "hp_zero_image_rows",
           "hp_set_option", "hp_get_option", "hp_probe_stream", "hp_probe_stream_ex", "hp_profile_enable", "hp_profile_read",
           "hp_strerror", "hp_last_hip_error", "hp_version"]

_handle = None


def _lib():
    """Loads libhp.so once.  Raises if it is missing: there is no fallback."""
    global _handle
    if _handle is not None:
        return _handle
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2605_27678_amd.build or "
            "__graft_entry__.build()); the transform has no CPU or PyTorch fallback")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    L.hp_plan_create.argtypes = [C.POINTER(hp_layout_t), C.POINTER(hp_layout_t),
                                 C.POINTER(hp_token_map_t), C.POINTER(vp)]
    L.hp_plan_create_host.argtypes = L.hp_plan_create.argtypes
    L.hp_plan_create_batched.argtypes = [C.POINTER(hp_layout_t), C.POINTER(hp_layout_t),
                                         C.POINTER(hp_token_map_t), i32, i32, C.POINTER(vp)]
    L.hp_plan_create_joined.argtypes = [C.POINTER(hp_layout_t), i32, C.POINTER(hp_layout_t),
                                        C.POINTER(hp_token_map_t), i32, i32, C.POINTER(vp)]
    L.hp_plan_create_joined.restype = C.c_int
    L.hp_plan_get_launch.argtypes = [vp, i32, C.POINTER(hp_launch_t)]
    L.hp_plan_set_launch.argtypes = [vp, i32, C.POINTER(hp_launch_t)]
    L.hp_plan_tune.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), vp]
    L.hp_plan_tune_accumulate.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp]
    L.hp_plan_tune_accumulate.restype = C.c_int
    L.hp_plan_destroy.argtypes = [vp]
    L.hp_plan_destroy.restype = None
    L.hp_release_cached_memory.restype = None
    L.hp_forget_tuned_shapes.restype = None
    L.hp_plan_query.argtypes = [vp, C.POINTER(hp_plan_info_t)]
    L.hp_plan_src_rows.argtypes = [vp, C.POINTER(i64), i32]
    L.hp_plan_segments.argtypes = [vp, C.POINTER(hp_segment_t), i32]
    L.hp_forward.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp]
    L.hp_backward.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp]
    L.hp_zero_image_rows.argtypes = [vp, C.POINTER(vp), vp]
    L.hp_zero_image_rows.restype = C.c_int
    L.hp_forward_static.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp]
    L.hp_forward_static.restype = C.c_int
    L.hp_backward_accumulate.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), vp]
    L.hp_backward_accumulate.restype = C.c_int
    L.hp_set_option.argtypes = [C.c_char_p, i64]
    L.hp_get_option.argtypes = [C.c_char_p]
    L.hp_get_option.restype = i64
    L.hp_probe_stream.argtypes = [i32, i32, i64, C.POINTER(hp_launch_t), C.POINTER(C.c_double),
                                  C.POINTER(hp_launch_t)]
    L.hp_probe_stream.restype = C.c_int
    L.hp_probe_stream_ex.argtypes = [i32, i32, i64, C.POINTER(hp_launch_t), i32, C.POINTER(C.c_double)]
    L.hp_probe_stream_ex.restype = C.c_int
    L.hp_profile_enable.argtypes = [i32]
    L.hp_profile_read.argtypes = [C.POINTER(C.c_float), C.POINTER(i32), i32]
    L.hp_strerror.argtypes = [C.c_int]
    L.hp_strerror.restype = C.c_char_p
    L.hp_version.restype = C.c_char_p
    for f in ("hp_plan_create", "hp_plan_create_host", "hp_plan_query", "hp_plan_src_rows",
              "hp_plan_segments", "hp_forward", "hp_backward", "hp_set_option", "hp_last_hip_error",
              "hp_profile_enable", "hp_profile_read", "hp_plan_create_batched", "hp_plan_get_launch",
              "hp_plan_set_launch", "hp_plan_tune"):
        getattr(L, f).restype = C.c_int
    _handle = L
    return L


def _check(rc: int, what: str) -> int:
    if rc < 0:
        raise HpError(rc, what)
    return rc


def _layout(g: Grid) -> hp_layout_t:
    return hp_layout_t(g.tp, g.cp, g.dp, g.pp, g.rank_offset, g.tp_mode, g.cp_split, g.row_order)


def _i32p(a: Optional[np.ndarray]):
    return C.POINTER(C.c_int32)() if a is None else a.ctypes.data_as(C.POINTER(C.c_int32))


def _token_map(m: TokenMap):
    keep = [np.ascontiguousarray(x, dtype=np.int32) for x in (m.img_sample, m.img_start, m.img_len)]
    dp = None if m.img_src_dp is None else np.ascontiguousarray(m.img_src_dp, dtype=np.int32)
    t = hp_token_map_t(m.batch, m.seq, m.hidden, int(getattr(m, "dtype", 0)), m.n_images,
                       _i32p(keep[0]), _i32p(keep[1]), _i32p(keep[2]), _i32p(dp))
    return t, (keep, dp)


def hp_set_option(key: str, value: int) -> None:
    _check(_lib().hp_set_option(key.encode(), int(value)), f"hp_set_option({key})")


def hp_get_option(key: str) -> int:
    return int(_lib().hp_get_option(key.encode()))


def hp_probe_stream(n_read: int, n_write: int, bytes_per_array: int, shape: Optional[dict] = None):
    """(GB/s, launch shape) of a plain n_read : n_write streaming kernel."""
    out = C.c_double(0.0)
    best = hp_launch_t()
    arg = C.byref(hp_launch_t(**shape)) if shape else None
    _check(_lib().hp_probe_stream(n_read, n_write, int(bytes_per_array), arg, C.byref(out), C.byref(best)),
           "hp_probe_stream")
    return out.value, {f[0]: getattr(best, f[0]) for f in best._fields_}


PROBE_SCHEDULES = {"oneshot": 0, "xcd_chunked": 1, "persistent": 2, "persistent_xcd": 3, "phased": 4}


def hp_probe_stream_ex(n_read: int, n_write: int, bytes_per_array: int, shape: dict, schedule) -> float:
    """GB/s of the streaming probe in the given launch shape with tiles handed
    to workgroups by `schedule` (a name in PROBE_SCHEDULES or its number)."""
    out = C.c_double(0.0)
    sched = PROBE_SCHEDULES[schedule] if isinstance(schedule, str) else int(schedule)
    _check(_lib().hp_probe_stream_ex(n_read, n_write, int(bytes_per_array), C.byref(hp_launch_t(**shape)), sched,
                                     C.byref(out)), "hp_probe_stream_ex")
    return out.value


def hp_profile_enable(max_launches: int) -> None:
    _check(_lib().hp_profile_enable(int(max_launches)), "hp_profile_enable")


def hp_profile_read(cap: int):
    """[(kind, milliseconds)] of the launches recorded since the last read;
    kind 0 = hp_forward, 1 = hp_backward."""
    ms = (C.c_float * max(cap, 1))()
    kinds = (C.c_int32 * max(cap, 1))()
    n = _check(_lib().hp_profile_read(ms, kinds, cap), "hp_profile_read")
    return [(int(kinds[i]), float(ms[i])) for i in range(min(n, cap))]


def hp_forget_tuned_shapes() -> None:
    _lib().hp_forget_tuned_shapes()


def hp_release_cached_memory() -> None:
    _lib().hp_release_cached_memory()


def hp_version() -> str:
    return _lib().hp_version().decode()


def _stream_handle(stream) -> C.c_void_p:
    if stream is None:
        return C.c_void_p(0)
    if hasattr(stream, "cuda_stream"):
        return C.c_void_p(int(stream.cuda_stream))
    return C.c_void_p(int(stream))


class Plan:
    """Owns one hp_plan_t.  `host_only=True` builds the tables without touching
    the GPU (for inspection on machines without one)."""

    def __init__(self, src, dst: Grid, tmap, host_only: bool = False):
        L = _lib()
        self._h = C.c_void_p(0)
        if not isinstance(src, Grid):           # several source grids: tmap[e][m] = edge e, microbatch m
            srcs = list(src)
            if len(tmap) != len(srcs) or any(len(row) != len(tmap[0]) for row in tmap) or not tmap[0]:
                raise ValueError("joined plan: need one list of microbatch token maps per source grid, equally long")
            pairs = [_token_map(m) for row in tmap for m in row]
            arr = (hp_token_map_t * len(pairs))(*[p[0] for p in pairs])
            keep = [p[1] for p in pairs]
            layouts = (hp_layout_t * len(srcs))(*[_layout(g) for g in srcs])
            _check(L.hp_plan_create_joined(layouts, len(srcs), C.byref(_layout(dst)), arr, len(tmap[0]),
                                           1 if host_only else 0, C.byref(self._h)),
                   "hp_plan_create_joined")
            self.hidden = tmap[0][0].hidden
        elif isinstance(tmap, TokenMap):
            tm, keep = _token_map(tmap)
            fn = L.hp_plan_create_host if host_only else L.hp_plan_create
            _check(fn(C.byref(_layout(src)), C.byref(_layout(dst)), C.byref(tm), C.byref(self._h)),
                   "hp_plan_create")
            self.hidden = tmap.hidden
        else:                                   # a sequence of microbatch token maps
            pairs = [_token_map(m) for m in tmap]
            arr = (hp_token_map_t * len(pairs))(*[p[0] for p in pairs])
            keep = [p[1] for p in pairs]
            _check(L.hp_plan_create_batched(C.byref(_layout(src)), C.byref(_layout(dst)), arr, len(pairs),
                                            1 if host_only else 0, C.byref(self._h)),
                   "hp_plan_create_batched")
            self.hidden = tmap[0].hidden
        del keep
        self.info = hp_plan_info_t()
        _check(L.hp_plan_query(self._h, C.byref(self.info)), "hp_plan_query")
        self.elem_bytes = self.info.elem_bytes

    def get_launch(self, direction: int) -> dict:
        out = hp_launch_t()
        _check(_lib().hp_plan_get_launch(self._h, direction, C.byref(out)), "hp_plan_get_launch")
        return {f[0]: getattr(out, f[0]) for f in out._fields_}

    def set_launch(self, direction: int, **kw) -> None:
        cur = self.get_launch(direction)
        cur.update(kw)
        arg = hp_launch_t(**cur)
        _check(_lib().hp_plan_set_launch(self._h, direction, C.byref(arg)), "hp_plan_set_launch")
        _check(_lib().hp_plan_query(self._h, C.byref(self.info)), "hp_plan_query")

    def tune(self, src_bufs=None, dst_bufs=None, dst_grad_bufs=None, src_grad_bufs=None, stream=None) -> None:
        """Measures launch shapes on these buffers and keeps the fastest per direction."""
        ps = pd = pgd = pgs = None
        if src_bufs is not None:
            ps, pd = self._src_dst(src_bufs, dst_bufs)
        if dst_grad_bufs is not None:
            pgs, pgd = self._src_dst(src_grad_bufs, dst_grad_bufs)
        _check(_lib().hp_plan_tune(self._h, ps, pd, pgd, pgs, _stream_handle(stream)), "hp_plan_tune")
        _check(_lib().hp_plan_query(self._h, C.byref(self.info)), "hp_plan_query")

    # -- introspection ------------------------------------------------------
    def src_rows(self) -> List[int]:
        n = self.info.n_src_bufs
        buf = (C.c_int64 * n)()
        _check(_lib().hp_plan_src_rows(self._h, buf, n), "hp_plan_src_rows")
        return list(buf)

    def segments(self) -> List[hp_segment_t]:
        n = self.info.n_segments
        arr = (hp_segment_t * max(n, 1))()
        _check(_lib().hp_plan_segments(self._h, arr, n), "hp_plan_segments")
        return [arr[i] for i in range(n)]

    # -- marshalling --------------------------------------------------------
    def _pointers(self, tensors: Sequence, rows: Sequence[int], what: str, esize: Optional[int] = None):
        esize = esize or self.elem_bytes
        P = (C.c_void_p * len(tensors))()
        for i, (t, r) in enumerate(zip(tensors, rows)):
            if t is None:
                P[i] = None
                continue
            if not t.is_cuda or not t.is_contiguous() or t.element_size() != esize:
                raise ValueError(f"{what}[{i}]: need a contiguous CUDA tensor of {esize}-byte elements")
            if t.numel() < r * self.hidden:
                raise ValueError(f"{what}[{i}]: {t.numel()} elements, plan needs {r * self.hidden}")
            P[i] = t.data_ptr() if t.numel() else None
        return P

    def _src_dst(self, src_bufs, dst_bufs, src_esize: Optional[int] = None):
        if len(src_bufs) != self.info.n_src_bufs or len(dst_bufs) != self.info.n_dst_bufs:
            raise ValueError("wrong number of buffers for this plan")
        ps = self._pointers(src_bufs, self.src_rows(), "src", src_esize)
        pd = self._pointers(dst_bufs, [self.info.dst_rows_per_buf] * len(dst_bufs), "dst")
        return ps, pd

    def tune_accumulate(self, dst_grad_bufs, src_accum_scratch, stream=None) -> None:
        """Launch-shape search for backward_accumulate; adds into src_accum_scratch many times."""
        ps, pd = self._src_dst(src_accum_scratch, dst_grad_bufs, src_esize=4)
        _check(_lib().hp_plan_tune_accumulate(self._h, pd, ps, _stream_handle(stream)), "hp_plan_tune_accumulate")

    def forward(self, src_bufs: Sequence, dst_bufs: Sequence, stream=None) -> None:
        ps, pd = self._src_dst(src_bufs, dst_bufs)
        _check(_lib().hp_forward(self._h, ps, pd, _stream_handle(stream)), "hp_forward")

    def forward_static(self, src_bufs: Sequence, dst_bufs: Sequence, stream=None) -> None:
        """hp_forward through the library's fixed table array: works on host-only
        plans and allocates nothing."""
        ps, pd = self._src_dst(src_bufs, dst_bufs)
        _check(_lib().hp_forward_static(self._h, ps, pd, _stream_handle(stream)), "hp_forward_static")

    def zero_image_rows(self, dst_bufs: Sequence, stream=None) -> None:
        """Zeroes the image-token rows of destination-shaped buffers in place."""
        if len(dst_bufs) != self.info.n_dst_bufs:
            raise ValueError("wrong number of buffers for this plan")
        pd = self._pointers(dst_bufs, [self.info.dst_rows_per_buf] * len(dst_bufs), "dst")
        _check(_lib().hp_zero_image_rows(self._h, pd, _stream_handle(stream)), "hp_zero_image_rows")

    def backward(self, dst_grad_bufs: Sequence, src_grad_bufs: Sequence, stream=None) -> None:
        ps, pd = self._src_dst(src_grad_bufs, dst_grad_bufs)
        _check(_lib().hp_backward(self._h, pd, ps, _stream_handle(stream)), "hp_backward")

    def backward_accumulate(self, dst_grad_bufs: Sequence, src_accum_bufs: Sequence, stream=None) -> None:
        """src_accum_bufs: float32 accumulators [rows_i, hidden], added to in place."""
        ps, pd = self._src_dst(src_accum_bufs, dst_grad_bufs, src_esize=4)
        _check(_lib().hp_backward_accumulate(self._h, pd, ps, _stream_handle(stream)),
               "hp_backward_accumulate")

    # raw-pointer variants for timing loops (pointer arrays prepared once)
    def pointer_arrays(self, src_bufs: Sequence, dst_bufs: Sequence):
        return self._src_dst(src_bufs, dst_bufs)

    def forward_raw(self, ps, pd, stream=None) -> None:
        _check(_lib().hp_forward(self._h, ps, pd, _stream_handle(stream)), "hp_forward")

    def backward_raw(self, pd, ps, stream=None) -> None:
        _check(_lib().hp_backward(self._h, pd, ps, _stream_handle(stream)), "hp_backward")

    def backward_accumulate_raw(self, pd, ps, stream=None) -> None:
        _check(_lib().hp_backward_accumulate(self._h, pd, ps, _stream_handle(stream)), "hp_backward_accumulate")

    def pointer_arrays_accum(self, src_accum_bufs: Sequence, dst_grad_bufs: Sequence):
        return self._src_dst(src_accum_bufs, dst_grad_bufs, src_esize=4)

    def close(self) -> None:
        if self._h:
            _lib().hp_plan_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def hp_plan_create(src: Grid, dst: Grid, tmap: TokenMap) -> Plan:
    return Plan(src, dst, tmap)


def hp_plan_create_host(src: Grid, dst: Grid, tmap: TokenMap) -> Plan:
    return Plan(src, dst, tmap, host_only=True)


def hp_plan_create_batched(src: Grid, dst: Grid, tmaps: Sequence[TokenMap], host_only: bool = False) -> Plan:
    return Plan(src, dst, list(tmaps), host_only=host_only)


def hp_plan_create_joined(srcs: Sequence[Grid], dst: Grid, tmaps: Sequence[Sequence[TokenMap]],
                          host_only: bool = False) -> Plan:
    """tmaps[e][m]: token map of edge e (source grid srcs[e]) for microbatch m."""
    return Plan(list(srcs), dst, [list(row) for row in tmaps], host_only=host_only)


def hp_plan_tune(plan: Plan, src_bufs=None, dst_bufs=None, dst_grad_bufs=None, src_grad_bufs=None,
                 stream=None) -> None:
    plan.tune(src_bufs, dst_bufs, dst_grad_bufs, src_grad_bufs, stream)


def hp_forward(plan: Plan, src_bufs, dst_bufs, stream=None) -> None:
    plan.forward(src_bufs, dst_bufs, stream)


def hp_forward_static(plan: Plan, src_bufs, dst_bufs, stream=None) -> None:
    plan.forward_static(src_bufs, dst_bufs, stream)


def hp_zero_image_rows(plan: Plan, dst_bufs, stream=None) -> None:
    plan.zero_image_rows(dst_bufs, stream)


def hp_backward(plan: Plan, dst_grad_bufs, src_grad_bufs, stream=None) -> None:
    plan.backward(dst_grad_bufs, src_grad_bufs, stream)


def hp_backward_accumulate(plan: Plan, dst_grad_bufs, src_accum_bufs, stream=None) -> None:
    plan.backward_accumulate(dst_grad_bufs, src_accum_bufs, stream)
