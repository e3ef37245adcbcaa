"""ctypes front end of the CPU oracle (oracle/hxt_oracle.c).

TEST INFRASTRUCTURE ONLY.  May be imported by tests/, by the smoke check and by
the benchmark's CPU-baseline leg; never by the product package.  It marshals
NumPy arrays into the C routines and does no arithmetic of the method itself.

A message is a list of ``TensorSpec(shape, strides, esize)`` (strides in
elements, as PyTorch reports them) plus one NumPy uint8 array per tensor holding
that tensor's *storage* (the bytes its base pointer points at).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hxt_oracle.c")
_LIB = os.path.join(_HERE, "libhxt_oracle.so")
MAXDIM = 8


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (about a second)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"],
            check=True,
        )
    return _LIB


@dataclass(frozen=True)
class TensorSpec:
    shape: tuple
    strides: tuple  # elements
    esize: int

    @staticmethod
    def contiguous(shape: Sequence[int], esize: int) -> "TensorSpec":
        st, acc = [], 1
        for s in reversed(shape):
            st.append(acc)
            acc *= max(int(s), 1)
        return TensorSpec(tuple(int(s) for s in shape), tuple(reversed(st)), int(esize))

    def storage_bytes(self) -> int:
        """Bytes of storage the view can touch (0 for an empty tensor)."""
        if any(s == 0 for s in self.shape):
            return 0
        return (sum((s - 1) * st for s, st in zip(self.shape, self.strides)) + 1) * self.esize


class _Msg(C.Structure):
    _fields_ = [
        ("T", C.c_int),
        ("ndim", C.POINTER(C.c_int32)),
        ("shape", C.POINTER(C.c_int64)),
        ("stride", C.POINTER(C.c_int64)),
        ("esize", C.POINTER(C.c_int32)),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        i64, i32, p = C.c_int64, C.c_int, C.c_void_p
        M = C.POINTER(_Msg)
        sigs = {
            "hxo_tensor_elems": (i64, [M, i32]),
            "hxo_tensor_bytes": (i64, [M, i32]),
            "hxo_tensor_offset": (i64, [M, i32]),
            "hxo_message_bytes": (i64, [M]),
            "hxo_stream_bytes": (i64, [M]),
            "hxo_num_chunks": (i64, [i64, i64]),
            "hxo_chunk_lane": (i64, [i64, i32]),
            "hxo_chunk_slot": (i64, [i64, i32]),
            "hxo_lane_chunks": (i64, [i64, i64, i32, i32]),
            "hxo_lane_offset": (i64, [i64, i64, i32, i32]),
            "hxo_packed_bytes": (i64, [i64, i64, i32]),
            "hxo_chunk_padded": (i64, [i64, i64, i64]),
            "hxo_chunk_packed_offset": (i64, [i64, i64, i32, i64]),
            "hxo_lane_used": (i64, [i64, i64, i32, i32]),
            "hxo_stream_to_packed": (i64, [i64, i64, i32, i64]),
            "hxo_chunk_payload": (i64, [M, i64, i64]),
            "hxo_element_storage_offset": (i64, [M, i32, i64]),
            "hxo_pack": (i32, [M, p, i64, i32, p, i32]),
            "hxo_unpack": (i32, [M, p, i64, i32, p, i32]),
            "hxo_stage_lane": (i32, [i64, i64, i32, i32, p, p]),
            "hxo_stage_slots": (i32, [i64, i64, i32, i32, i64, i64, p, p]),
            "hxo_checksum": (i32, [i64, i64, i32, p, p, i32]),
            "hxo_checksum2": (i32, [i64, i64, i32, p, p, i32]),
            "hxo_seal": (i32, [i64, i64, i32, p, C.c_uint64, C.c_uint32, p]),
            "hxo_verify": (i32, [i64, i64, i32, p, p, C.c_uint64, C.c_uint32, p]),
            "hxo_packed_origin": (i32, [M, i64, i32, i64, C.POINTER(C.c_int32), C.POINTER(C.c_int64)]),
            "hxo_max_threads": (i32, []),
            "hxo_round_to_bf16": (C.c_uint16, [C.c_float]),
            "hxo_add_f32_bits": (C.c_uint32, [C.c_uint32, C.c_uint32]),
            "hxo_add_bf16_bits": (C.c_uint16, [C.c_uint16, C.c_uint16]),
            "hxo_unpack_accumulate": (i32, [M, C.POINTER(C.c_int32), p, i64, i32, p, i32]),
        }
        for name, (res, args) in sigs.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


class Message:
    """Marshalled description of T tensors, kept alive for the C calls."""

    def __init__(self, specs: Sequence[TensorSpec]):
        self.specs: List[TensorSpec] = list(specs)
        T = len(self.specs)
        self._ndim = (C.c_int32 * max(T, 1))()
        self._shape = (C.c_int64 * (max(T, 1) * MAXDIM))()
        self._stride = (C.c_int64 * (max(T, 1) * MAXDIM))()
        self._esize = (C.c_int32 * max(T, 1))()
        for t, s in enumerate(self.specs):
            if len(s.shape) > MAXDIM or len(s.shape) != len(s.strides):
                raise ValueError("bad tensor spec")
            self._ndim[t] = len(s.shape)
            self._esize[t] = s.esize
            for d, (a, b) in enumerate(zip(s.shape, s.strides)):
                if a < 0 or b < 0:
                    raise ValueError("negative shape or stride")
                self._shape[t * MAXDIM + d] = a
                self._stride[t * MAXDIM + d] = b
        self.c = _Msg(T, self._ndim, self._shape, self._stride, self._esize)
        self.ref = C.byref(self.c)

    # sizes
    @property
    def N(self) -> int:
        return lib().hxo_message_bytes(self.ref)

    @property
    def L(self) -> int:
        return lib().hxo_stream_bytes(self.ref)

    def tensor_offset(self, t: int) -> int:
        return lib().hxo_tensor_offset(self.ref, t)

    def tensor_bytes(self, t: int) -> int:
        return lib().hxo_tensor_bytes(self.ref, t)


def _ptr_array(arrs: Sequence[np.ndarray]):
    P = (C.c_void_p * max(len(arrs), 1))()
    for i, a in enumerate(arrs):
        assert a.dtype == np.uint8 and a.flags.c_contiguous
        P[i] = a.ctypes.data
    return P


def _check_storage(msg: Message, storages: Sequence[np.ndarray]):
    assert len(storages) == len(msg.specs)
    for s, a in zip(msg.specs, storages):
        assert a.dtype == np.uint8 and a.ndim == 1 and a.size >= s.storage_bytes(), "storage too small for view"


# ---- layout queries ---------------------------------------------------------

def num_chunks(msg: Message, B: int) -> int:
    return lib().hxo_num_chunks(msg.L, B)


def packed_bytes(msg: Message, B: int, k: int) -> int:
    return lib().hxo_packed_bytes(msg.L, B, k)


def chunk_info(msg: Message, B: int, k: int, c: int) -> dict:
    L_ = msg.L
    l = lib()
    return dict(
        lane=l.hxo_chunk_lane(c, k),
        slot=l.hxo_chunk_slot(c, k),
        stream_off=c * B,
        padded=l.hxo_chunk_padded(L_, B, c),
        payload=l.hxo_chunk_payload(msg.ref, B, c),
        packed_off=l.hxo_chunk_packed_offset(L_, B, k, c),
    )


def stream_to_packed(L_: int, B: int, k: int, s: int) -> int:
    """Packed position of stream byte s of a stream of L_ bytes."""
    return lib().hxo_stream_to_packed(L_, B, k, s)


def lane_info(msg: Message, B: int, k: int, lane: int) -> dict:
    L_ = msg.L
    l = lib()
    return dict(
        packed_off=l.hxo_lane_offset(L_, B, k, lane),
        n_chunks=l.hxo_lane_chunks(L_, B, k, lane),
        bytes=l.hxo_lane_used(L_, B, k, lane),
    )


# ---- the transfer -----------------------------------------------------------

def pack(msg: Message, storages: Sequence[np.ndarray], B: int, k: int, packed: np.ndarray | None = None,
         nthreads: int = 1, fill: int = 0xA5) -> np.ndarray:
    """Return the packed buffer (unspecified bytes keep ``fill``)."""
    _check_storage(msg, storages)
    nb = packed_bytes(msg, B, k)
    if packed is None:
        packed = np.full(nb, fill, dtype=np.uint8)
    assert packed.dtype == np.uint8 and packed.size >= nb
    rc = lib().hxo_pack(msg.ref, _ptr_array(storages), B, k, packed.ctypes.data, nthreads)
    if rc:
        raise ValueError("hxo_pack rejected the arguments")
    return packed


def unpack(msg: Message, packed: np.ndarray, B: int, k: int, storages: Sequence[np.ndarray], nthreads: int = 1) -> None:
    """Scatter into the given storages in place."""
    _check_storage(msg, storages)
    assert packed.dtype == np.uint8 and packed.size >= packed_bytes(msg, B, k)
    rc = lib().hxo_unpack(msg.ref, packed.ctypes.data, B, k, _ptr_array(storages), nthreads)
    if rc:
        raise ValueError("hxo_unpack rejected the arguments")


KIND_BF16, KIND_F32 = 1, 2


def unpack_accumulate(msg: Message, kinds: Sequence[int], packed: np.ndarray, B: int, k: int,
                      storages: Sequence[np.ndarray], nthreads: int = 1) -> None:
    """storages[t] += arriving tensor t, element-wise, in the arithmetic stated in hxt_oracle.c."""
    _check_storage(msg, storages)
    kk = (C.c_int32 * max(len(kinds), 1))(*kinds)
    rc = lib().hxo_unpack_accumulate(msg.ref, kk, packed.ctypes.data, B, k, _ptr_array(storages), nthreads)
    if rc:
        raise ValueError("hxo_unpack_accumulate rejected the arguments")


def stage_lane(msg: Message, B: int, k: int, lane: int, src: np.ndarray, dst: np.ndarray) -> None:
    rc = lib().hxo_stage_lane(msg.L, B, k, lane, src.ctypes.data, dst.ctypes.data)
    if rc:
        raise ValueError("bad lane")


def stage_slots(msg: Message, B: int, k: int, lane: int, first: int, count: int, src: np.ndarray, dst: np.ndarray) -> None:
    rc = lib().hxo_stage_slots(msg.L, B, k, lane, first, count, src.ctypes.data, dst.ctypes.data)
    if rc:
        raise ValueError("bad lane or slots")


def checksum(msg: Message, packed: np.ndarray, B: int, k: int, nthreads: int = 1) -> np.ndarray:
    sums = np.zeros(num_chunks(msg, B), dtype=np.uint64)
    rc = lib().hxo_checksum(msg.L, B, k, packed.ctypes.data, sums.ctypes.data, nthreads)
    if rc:
        raise ValueError("hxo_checksum rejected the arguments")
    return sums


def checksum2(msg: Message, packed: np.ndarray, B: int, k: int, nthreads: int = 1) -> np.ndarray:
    """[C, 2] array: plain sum and position-weighted sum of every chunk."""
    out = np.zeros((num_chunks(msg, B), 2), dtype=np.uint64)
    rc = lib().hxo_checksum2(msg.L, B, k, packed.ctypes.data, out.ctypes.data, nthreads)
    if rc:
        raise ValueError("hxo_checksum2 rejected the arguments")
    return out


TAG_BYTES = 64
TAG_BAD_MAGIC, TAG_BAD_PLACE, TAG_BAD_SEQ, TAG_BAD_MICRO_BATCH, TAG_BAD_SUM, TAG_BAD_WSUM, TAG_BAD_RESERVED = \
    1, 2, 4, 8, 16, 32, 64


def seal(msg: Message, packed: np.ndarray, B: int, k: int, seq: int, micro_batch: int) -> np.ndarray:
    """[C, 64] uint8: the chunk tags in packed-slot order."""
    tags = np.zeros((num_chunks(msg, B), TAG_BYTES), dtype=np.uint8)
    rc = lib().hxo_seal(msg.L, B, k, packed.ctypes.data, seq, micro_batch, tags.ctypes.data)
    if rc:
        raise ValueError("hxo_seal rejected the arguments")
    return tags


def verify(msg: Message, packed: np.ndarray, tags: np.ndarray, B: int, k: int, seq: int, micro_batch: int) -> np.ndarray:
    """uint32[C + 1]: per-chunk bit masks, then the number of rejected chunks."""
    assert tags.dtype == np.uint8 and tags.flags.c_contiguous and tags.size == num_chunks(msg, B) * TAG_BYTES
    status = np.zeros(num_chunks(msg, B) + 1, dtype=np.uint32)
    rc = lib().hxo_verify(msg.L, B, k, packed.ctypes.data, tags.ctypes.data, seq, micro_batch, status.ctypes.data)
    if rc:
        raise ValueError("hxo_verify rejected the arguments")
    return status


def packed_origin(msg: Message, B: int, k: int, p: int):
    """(kind, tensor, storage_byte): kind 1 = tensor byte, 0 = zero pad, -1 = unspecified."""
    t = C.c_int32(-1)
    off = C.c_int64(-1)
    kind = lib().hxo_packed_origin(msg.ref, B, k, p, C.byref(t), C.byref(off))
    return kind, t.value, off.value


def max_threads() -> int:
    return lib().hxo_max_threads()
