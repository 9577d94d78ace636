"""ctypes front end of the CPU oracle (oracle/hp_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg; the product package never imports it.  Buffers are
numpy arrays on the host (bf16 payloads travel as uint16 bit patterns).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hp_oracle.c")
_LIB = os.path.join(_HERE, "libhp_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE arithmetic: no fast-math, no
    contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class _Grid(C.Structure):
    _fields_ = [("tp", C.c_int32), ("cp", C.c_int32), ("dp", C.c_int32),
                ("tp_mode", C.c_int32), ("cp_split", C.c_int32), ("row_order", C.c_int32)]


class _Map(C.Structure):
    _fields_ = [("batch", C.c_int32), ("seq", C.c_int32), ("hidden", C.c_int32),
                ("n_images", C.c_int32),
                ("img_sample", C.POINTER(C.c_int32)), ("img_start", C.POINTER(C.c_int32)),
                ("img_len", C.POINTER(C.c_int32)), ("img_src_dp", C.POINTER(C.c_int32))]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_src_rows.restype = C.c_int64
        _lib.orc_dst_rows.restype = C.c_int64
        _lib.orc_f32_to_bf16.restype = C.c_uint16
        _lib.orc_f32_to_bf16.argtypes = [C.c_float]
        _lib.orc_f32_bits_to_bf16.restype = C.c_uint16
        _lib.orc_f32_bits_to_bf16.argtypes = [C.c_uint32]
        _lib.orc_bf16_to_f32.restype = C.c_float
        _lib.orc_bf16_to_f32.argtypes = [C.c_uint16]
    return _lib


def set_threads(n: int) -> None:
    """Number of OpenMP threads the oracle's row loops use."""
    omp = C.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(n))


def _i32p(a: Optional[np.ndarray]):
    if a is None:
        return C.POINTER(C.c_int32)()
    return a.ctypes.data_as(C.POINTER(C.c_int32))


class Problem:
    """Grids + token map in the oracle's own structs (keeps the numpy arrays
    alive while the C side reads them)."""

    def __init__(self, src, dst, tmap):
        self.src_grid, self.dst_grid, self.tmap = src, dst, tmap
        self.src = _Grid(src.tp, src.cp, src.dp, src.tp_mode, src.cp_split, src.row_order)
        self.dst = _Grid(dst.tp, dst.cp, dst.dp, dst.tp_mode, dst.cp_split, dst.row_order)
        self._keep = [np.ascontiguousarray(x, dtype=np.int32) for x in
                      (tmap.img_sample, tmap.img_start, tmap.img_len)]
        self._dp = None if tmap.img_src_dp is None else np.ascontiguousarray(tmap.img_src_dp, np.int32)
        self.map = _Map(tmap.batch, tmap.seq, tmap.hidden, tmap.n_images,
                        _i32p(self._keep[0]), _i32p(self._keep[1]), _i32p(self._keep[2]),
                        _i32p(self._dp))
        self.n_src = src.tp * src.dp
        self.n_dst = dst.tp * dst.cp * dst.dp
        self.hidden = tmap.hidden

    def src_rows(self) -> List[int]:
        """Rows of each source buffer, index tp + TP*dp."""
        L = lib()
        out = []
        for d in range(self.src_grid.dp):
            r = int(L.orc_src_rows(C.byref(self.src), C.byref(self.map), C.c_int32(d)))
            out += [r] * self.src_grid.tp
        return out

    def dst_rows(self) -> int:
        return int(lib().orc_dst_rows(C.byref(self.dst), C.byref(self.map)))

    def forward_map(self, buf: int):
        rows = self.dst_rows()
        sb = np.empty(rows, np.int32)
        sr = np.empty(rows, np.int64)
        rc = lib().orc_forward_map(C.byref(self.src), C.byref(self.dst), C.byref(self.map),
                                   C.c_int32(buf), _i32p(sb),
                                   sr.ctypes.data_as(C.POINTER(C.c_int64)))
        if rc:
            raise ValueError("oracle: layout does not divide the token map")
        return sb, sr

    @staticmethod
    def _ptrs(arrs: Sequence[np.ndarray]):
        P = (C.c_void_p * len(arrs))()
        for i, a in enumerate(arrs):
            assert a.flags["C_CONTIGUOUS"]
            P[i] = a.ctypes.data if a.size else None
        return P

    def forward(self, src_bufs: Sequence[np.ndarray], dst_bufs: Sequence[np.ndarray]) -> None:
        """In place on dst_bufs (which already hold the text rows)."""
        assert len(src_bufs) == self.n_src and len(dst_bufs) == self.n_dst
        es = dst_bufs[0].dtype.itemsize
        for a, r in zip(src_bufs, self.src_rows()):
            assert a.dtype.itemsize == es and a.size == r * self.hidden
        for a in dst_bufs:
            assert a.size == self.dst_rows() * self.hidden
        rc = lib().orc_forward(C.byref(self.src), C.byref(self.dst), C.byref(self.map),
                               C.c_int32(es), self._ptrs(src_bufs), self._ptrs(dst_bufs))
        if rc:
            raise ValueError("oracle: layout does not divide the token map")

    def zero_image_rows(self, dst_bufs: Sequence[np.ndarray]) -> None:
        """In place: the image-token rows of every destination buffer become zero."""
        assert len(dst_bufs) == self.n_dst
        es = dst_bufs[0].dtype.itemsize
        for a in dst_bufs:
            assert a.dtype.itemsize == es and a.size == self.dst_rows() * self.hidden
        rc = lib().orc_zero_image_rows(C.byref(self.src), C.byref(self.dst), C.byref(self.map),
                                       C.c_int32(es), self._ptrs(dst_bufs))
        if rc:
            raise ValueError("oracle: layout does not divide the token map")

    def backward_bf16(self, dst_grads: Sequence[np.ndarray], src_grads: Sequence[np.ndarray]) -> None:
        """uint16 bf16 bit patterns in, uint16 out (in place on src_grads)."""
        assert len(dst_grads) == self.n_dst and len(src_grads) == self.n_src
        for a in list(dst_grads) + list(src_grads):
            assert a.dtype == np.uint16
        for a, r in zip(src_grads, self.src_rows()):
            assert a.size == r * self.hidden
        for a in dst_grads:
            assert a.size == self.dst_rows() * self.hidden
        rc = lib().orc_backward_bf16(C.byref(self.src), C.byref(self.dst), C.byref(self.map),
                                     self._ptrs(dst_grads), self._ptrs(src_grads))
        if rc:
            raise ValueError("oracle: layout does not divide the token map")

    def _backward(self, dtype: int, accumulate: bool, dst_grads, src_out) -> None:
        assert len(dst_grads) == self.n_dst and len(src_out) == self.n_src
        in_dt = np.uint16 if dtype == 0 else np.float32
        out_dt = np.float32 if (accumulate or dtype == 1) else np.uint16
        for a in dst_grads:
            assert a.dtype == in_dt and a.size == self.dst_rows() * self.hidden
        for a, r in zip(src_out, self.src_rows()):
            assert a.dtype == out_dt and a.size == r * self.hidden
        rc = lib().orc_backward(C.byref(self.src), C.byref(self.dst), C.byref(self.map),
                                C.c_int32(dtype), C.c_int32(1 if accumulate else 0),
                                self._ptrs(dst_grads), self._ptrs(src_out))
        if rc:
            raise ValueError("oracle: layout does not divide the token map")

    def backward_f32(self, dst_grads, src_grads) -> None:
        """binary32 gradients in, binary32 out (in place on src_grads)."""
        self._backward(1, False, dst_grads, src_grads)

    def backward_accumulate(self, dst_grads, src_accum) -> None:
        """bf16 (uint16 bits) or binary32 gradients in; the float32 arrays in
        src_accum are added to in place."""
        self._backward(0 if dst_grads[0].dtype == np.uint16 else 1, True, dst_grads, src_accum)



def f32_to_bf16(x: float) -> int:
    return int(lib().orc_f32_to_bf16(C.c_float(x)))


def f32_bits_to_bf16(bits: int) -> int:
    """Rounds the binary32 value with this bit pattern (keeps signalling NaNs
    as they are on the way in)."""
    return int(lib().orc_f32_bits_to_bf16(C.c_uint32(bits)))


def bf16_to_f32(h: int) -> float:
    return float(lib().orc_bf16_to_f32(C.c_uint16(h)))
