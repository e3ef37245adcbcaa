"""Thin ctypes binding over libhxt.so (the C ABI declared in include/hxt.h).

Same names as the C entry points; this layer only marshals arguments (tensor ->
device pointer, stream -> hipStream_t, status -> exception).  Every step of the
transfer runs in the library's HIP kernels; there is no Python or CPU fallback:
if the library is missing, loading raises.

PyTorch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch  # imported before the library so both share one HIP runtime

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libhxt.so")

HXT_OK, HXT_EINVAL, HXT_EALIGN, HXT_EUNSUPPORTED, HXT_EOVERLAP, HXT_EHIP, HXT_ENOMEM = 0, -1, -2, -3, -4, -5, -6
HXT_U8, HXT_F16, HXT_BF16, HXT_F32, HXT_F64 = 1, 2, 3, 4, 5
HXT_MAX_DIMS = 8
KIND_NAMES = {0: "none", 1: "contig", 2: "rows", 3: "transpose", 4: "generic", 6: "rows_split", 7: "transpose_span"}

# every symbol include/hxt.h declares
EXPORTS = (
    "hxt_plan", "hxt_plan_multi", "hxt_plan_destroy", "hxt_plan_message_bytes", "hxt_plan_stream_bytes",
    "hxt_plan_packed_bytes", "hxt_plan_chunk_bytes", "hxt_plan_num_chunks", "hxt_plan_num_lanes",
    "hxt_plan_num_tensors", "hxt_plan_chunk_info", "hxt_plan_lane_info", "hxt_plan_tensor_unpack_safe",
    "hxt_plan_tensor_kind", "hxt_pack", "hxt_stage_d2h", "hxt_stage_h2d", "hxt_unpack", "hxt_checksum",
    "hxt_pack_batch", "hxt_unpack_batch", "hxt_exchange_stream", "hxt_unpack_accumulate",
    "hxt_host_forward", "hxt_stage_hop", "hxt_checksum2", "hxt_seal", "hxt_verify", "hxt_pack_seal", "hxt_unpack_verify",
    "hxt_pack_noalloc", "hxt_plan_set_option", "hxt_pack_seal_batch", "hxt_unpack_verify_batch",
    "hxt_stage_d2h_slots", "hxt_stage_h2d_slots", "hxt_unpack_accumulate_batch",
    "hxt_strerror", "hxt_last_hip_error", "hxt_version",
)

_DTYPE_BY_TORCH = {
    torch.uint8: HXT_U8, torch.int8: HXT_U8, torch.bool: HXT_U8,
    torch.float16: HXT_F16, torch.int16: HXT_F16, torch.bfloat16: HXT_BF16,
    torch.float32: HXT_F32, torch.int32: HXT_F32, torch.float64: HXT_F64, torch.int64: HXT_F64,
}
_DTYPE_BY_SIZE = {1: HXT_U8, 2: HXT_BF16, 4: HXT_F32, 8: HXT_F64}


class HxtError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().hxt_strerror(status).decode()
        if status == HXT_EHIP:
            msg += " [hipError %d]" % lib().hxt_last_hip_error()
        super().__init__("%s: %s (%d)" % (where, msg, status))


class _TensorDesc(C.Structure):
    _fields_ = [("ndim", C.c_int), ("shape", C.POINTER(C.c_int64)), ("strides", C.POINTER(C.c_int64)),
                ("dtype", C.c_int)]


class ChunkInfo(C.Structure):
    _fields_ = [("lane", C.c_int32), ("slot", C.c_int32), ("stream_off", C.c_uint64), ("padded", C.c_uint64),
                ("payload", C.c_uint64), ("packed_off", C.c_uint64)]


class _Exchange(C.Structure):
    _fields_ = [("n_messages", C.c_int), ("n_buffers", C.c_int), ("path", C.c_int),
                ("src", C.POINTER(C.c_void_p)), ("dst", C.POINTER(C.c_void_p)),
                ("packed_send", C.POINTER(C.c_void_p)), ("packed_recv", C.POINTER(C.c_void_p)),
                ("host_pinned", C.POINTER(C.c_void_p)), ("send_sums", C.c_void_p), ("recv_sums", C.c_void_p),
                ("stream_pack", C.c_void_p), ("stream_stage", C.c_void_p), ("stream_unpack", C.c_void_p),
                ("tags_send", C.POINTER(C.c_void_p)), ("tags_recv", C.POINTER(C.c_void_p)),
                ("tags_pinned", C.POINTER(C.c_void_p)), ("status", C.c_void_p), ("seq_base", C.c_uint64),
                ("direct_mode", C.c_int), ("drain_every", C.c_int)]


HXT_DEVICE_DIRECT, HXT_CPU_FORWARD = 0, 1
HXT_DIRECT_AUTO, HXT_DIRECT_TWO_CHAINS, HXT_DIRECT_FUSED, HXT_DIRECT_EVENTS = 0, 1, 2, 3


class LaneInfo(C.Structure):
    _fields_ = [("packed_off", C.c_uint64), ("bytes", C.c_uint64), ("n_chunks", C.c_int32)]


_lib = None


def lib():
    """Load libhxt.so; raises if it has not been built (python -m paper_2602_18007_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libhxt.so is not built: run `python -m paper_2602_18007_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i, sz, u64p = C.c_void_p, C.c_int, C.c_size_t, C.c_void_p
        i64p = C.POINTER(C.c_int64)
        sig = {
            "hxt_plan": (i, [i64p, i64p, i, i, i, sz, C.POINTER(vp)]),
            "hxt_plan_multi": (i, [C.POINTER(_TensorDesc), i, i, sz, C.POINTER(vp)]),
            "hxt_plan_destroy": (i, [vp]),
            "hxt_plan_set_option": (i, [vp, i, i]),
            "hxt_plan_message_bytes": (sz, [vp]),
            "hxt_plan_stream_bytes": (sz, [vp]),
            "hxt_plan_packed_bytes": (sz, [vp]),
            "hxt_plan_chunk_bytes": (sz, [vp]),
            "hxt_plan_num_chunks": (i, [vp]),
            "hxt_plan_num_lanes": (i, [vp]),
            "hxt_plan_num_tensors": (i, [vp]),
            "hxt_plan_chunk_info": (i, [vp, i, C.POINTER(ChunkInfo)]),
            "hxt_plan_lane_info": (i, [vp, i, C.POINTER(LaneInfo)]),
            "hxt_plan_tensor_unpack_safe": (i, [vp, i]),
            "hxt_plan_tensor_kind": (i, [vp, i]),
            "hxt_pack": (i, [vp, C.POINTER(vp), vp, u64p, vp]),
            "hxt_stage_d2h": (i, [vp, i, vp, vp, vp]),
            "hxt_stage_h2d": (i, [vp, i, vp, vp, vp]),
            "hxt_stage_d2h_slots": (i, [vp, i, i, i, vp, vp, vp]),
            "hxt_stage_h2d_slots": (i, [vp, i, i, i, vp, vp, vp]),
            "hxt_unpack": (i, [vp, vp, C.POINTER(vp), u64p, vp]),
            "hxt_checksum": (i, [vp, vp, u64p, vp]),
            "hxt_checksum2": (i, [vp, vp, u64p, vp]),
            "hxt_seal": (i, [vp, vp, C.c_uint64, C.c_uint32, vp, vp]),
            "hxt_verify": (i, [vp, vp, vp, C.c_uint64, C.c_uint32, vp, vp]),
            "hxt_pack_seal": (i, [vp, C.POINTER(vp), vp, C.c_uint64, C.c_uint32, vp, vp]),
            "hxt_unpack_verify": (i, [vp, vp, vp, C.c_uint64, C.c_uint32, C.POINTER(vp), vp, vp]),
            "hxt_host_forward": (i, [vp, i, vp, vp, i]),
            "hxt_stage_hop": (i, [vp, i, vp, vp, i, vp]),
            "hxt_unpack_accumulate": (i, [vp, vp, C.POINTER(vp), u64p, vp]),
            "hxt_pack_batch": (i, [i, C.POINTER(vp), C.POINTER(C.POINTER(vp)), C.POINTER(vp), C.POINTER(vp), vp]),
            "hxt_unpack_batch": (i, [i, C.POINTER(vp), C.POINTER(vp), C.POINTER(C.POINTER(vp)), C.POINTER(vp), vp]),
            "hxt_unpack_accumulate_batch": (i, [i, C.POINTER(vp), C.POINTER(vp), C.POINTER(C.POINTER(vp)), C.POINTER(vp), vp]),
            "hxt_exchange_stream": (i, [vp, C.POINTER(_Exchange)]),
            "hxt_pack_seal_batch": (i, [i, C.POINTER(vp), C.POINTER(C.POINTER(vp)), C.POINTER(vp), C.POINTER(C.c_uint64),
                                        C.POINTER(C.c_uint32), C.POINTER(vp), vp]),
            "hxt_unpack_verify_batch": (i, [i, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(C.c_uint64),
                                            C.POINTER(C.c_uint32), C.POINTER(C.POINTER(vp)), C.POINTER(vp), vp]),
            "hxt_pack_noalloc": (i, [vp, sz, i, sz, vp, u64p, vp]),
            "hxt_strerror": (C.c_char_p, [i]),
            "hxt_last_hip_error": (i, []),
            "hxt_version": (C.c_char_p, []),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != HXT_OK:
        raise HxtError(status, where)


def _dtype_code(dt) -> int:
    if isinstance(dt, torch.dtype):
        return _DTYPE_BY_TORCH[dt]
    if isinstance(dt, int) and dt in _DTYPE_BY_SIZE:       # element size in bytes
        return _DTYPE_BY_SIZE[dt]
    raise ValueError("unsupported dtype %r" % (dt,))


def _names_arithmetic(dt) -> bool:
    """True if dt says what the bits mean as numbers (the library adds bf16 and f32 only).  An integer
    torch dtype or a bare element size describes raw bits: such data can be moved, not added."""
    return isinstance(dt, torch.dtype) and dt in (torch.bfloat16, torch.float32)


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, torch.Tensor):
        return x.data_ptr()
    return int(x)


def _stream(s) -> Optional[int]:
    if s is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(s, torch.cuda.Stream):
        return s.cuda_stream
    return int(s)


def _ptr_array(xs: Sequence):
    arr = (C.c_void_p * max(len(xs), 1))()
    for j, x in enumerate(xs):
        arr[j] = _ptr(x)
    return arr


class Plan:
    """Owner of one hxt_plan_t handle."""

    def __init__(self, handle: int, arithmetic: bool = False):
        self.handle = C.c_void_p(handle)
        self.arithmetic = arithmetic      # every tensor was described by torch.bfloat16 / torch.float32

    def destroy(self):
        if self.handle:
            lib().hxt_plan_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # queries, named after the C functions without the prefix
    message_bytes = property(lambda self: lib().hxt_plan_message_bytes(self.handle))
    stream_bytes = property(lambda self: lib().hxt_plan_stream_bytes(self.handle))
    packed_bytes = property(lambda self: lib().hxt_plan_packed_bytes(self.handle))
    chunk_bytes = property(lambda self: lib().hxt_plan_chunk_bytes(self.handle))
    num_chunks = property(lambda self: lib().hxt_plan_num_chunks(self.handle))
    num_lanes = property(lambda self: lib().hxt_plan_num_lanes(self.handle))
    num_tensors = property(lambda self: lib().hxt_plan_num_tensors(self.handle))

    def chunk_info(self, c: int) -> dict:
        out = ChunkInfo()
        _check(lib().hxt_plan_chunk_info(self.handle, c, C.byref(out)), "hxt_plan_chunk_info")
        return {k: getattr(out, k) for k, _ in ChunkInfo._fields_}

    def lane_info(self, lane: int) -> dict:
        out = LaneInfo()
        _check(lib().hxt_plan_lane_info(self.handle, lane, C.byref(out)), "hxt_plan_lane_info")
        return {k: getattr(out, k) for k, _ in LaneInfo._fields_}

    def tensor_unpack_safe(self, t: int) -> bool:
        r = lib().hxt_plan_tensor_unpack_safe(self.handle, t)
        if r < 0:
            raise HxtError(r, "hxt_plan_tensor_unpack_safe")
        return bool(r)

    def tensor_kind(self, t: int) -> str:
        r = lib().hxt_plan_tensor_kind(self.handle, t)
        if r < 0:
            raise HxtError(r, "hxt_plan_tensor_kind")
        return KIND_NAMES[r]


def hxt_plan(shape, strides, dtype, n_lanes: int, chunk_bytes: int) -> Plan:
    nd = len(shape)
    shp = (C.c_int64 * max(nd, 1))(*shape)
    st = (C.c_int64 * max(nd, 1))(*strides) if strides is not None else None
    out = C.c_void_p()
    _check(lib().hxt_plan(shp, st, nd, _dtype_code(dtype), n_lanes, chunk_bytes, C.byref(out)), "hxt_plan")
    return Plan(out.value, _names_arithmetic(dtype))


def hxt_plan_multi(tensors: Sequence, n_lanes: int, chunk_bytes: int) -> Plan:
    """tensors: sequence of (shape, strides_or_None, dtype) or torch tensors (their views are described)."""
    n = len(tensors)
    descs = (_TensorDesc * max(n, 1))()
    keep = []
    arithmetic = True
    for j, t in enumerate(tensors):
        if isinstance(t, torch.Tensor):
            shape, strides, dt = tuple(t.shape), tuple(t.stride()), t.dtype
        else:
            shape, strides, dt = t
        nd = len(shape)
        shp = (C.c_int64 * max(nd, 1))(*shape)
        st = (C.c_int64 * max(nd, 1))(*strides) if strides is not None else None
        keep += [shp, st]
        descs[j].ndim = nd
        descs[j].shape = shp
        descs[j].strides = st
        descs[j].dtype = _dtype_code(dt)
        arithmetic = arithmetic and (_names_arithmetic(dt) or 0 in shape)
    out = C.c_void_p()
    _check(lib().hxt_plan_multi(descs, n, n_lanes, chunk_bytes, C.byref(out)), "hxt_plan_multi")
    return Plan(out.value, arithmetic)


HXT_OPT_PACKED_HINT, HXT_OPT_STAGE_D2H = 1, 2


def hxt_plan_set_option(plan: Plan, option: int, value: int) -> None:
    _check(lib().hxt_plan_set_option(plan.handle, option, value), "hxt_plan_set_option")


def hxt_plan_destroy(plan: Plan) -> None:
    plan.destroy()


def hxt_pack(plan: Plan, src: Sequence, packed, sums=None, stream=None) -> None:
    _check(lib().hxt_pack(plan.handle, _ptr_array(src), _ptr(packed), _ptr(sums), _stream(stream)), "hxt_pack")


def hxt_unpack(plan: Plan, packed, dst: Sequence, sums=None, stream=None) -> None:
    _check(lib().hxt_unpack(plan.handle, _ptr(packed), _ptr_array(dst), _ptr(sums), _stream(stream)), "hxt_unpack")


def _host_ptr(x) -> Optional[int]:
    """Address of a host buffer: a CPU torch tensor, a NumPy array, or an integer."""
    if x is None or isinstance(x, (int, torch.Tensor)):
        return _ptr(x)
    return int(x.ctypes.data)


def hxt_host_forward(plan: Plan, lane: int, src, dst, n_threads: int = 0) -> None:
    _check(lib().hxt_host_forward(plan.handle, lane, _host_ptr(src), _host_ptr(dst), n_threads), "hxt_host_forward")


def hxt_stage_hop(plan: Plan, lane: int, from_pinned, to_pinned, n_threads: int = 0, stream=None) -> None:
    _check(lib().hxt_stage_hop(plan.handle, lane, _ptr(from_pinned), _ptr(to_pinned), n_threads, _stream(stream)),
           "hxt_stage_hop")


def hxt_unpack_accumulate(plan: Plan, packed, dst: Sequence, sums=None, stream=None) -> None:
    if not plan.arithmetic:
        raise ValueError("hxt_unpack_accumulate adds bf16 or f32 values: build the plan with torch.bfloat16 / "
                         "torch.float32, not with an integer dtype or a bare element size (those only name raw bits)")
    _check(lib().hxt_unpack_accumulate(plan.handle, _ptr(packed), _ptr_array(dst), _ptr(sums), _stream(stream)),
           "hxt_unpack_accumulate")


class Batch:
    """Pre-marshalled arguments of hxt_pack_batch / hxt_unpack_batch for a fixed set of messages."""

    def __init__(self, plans: Sequence[Plan], tensors: Sequence[Sequence], packed: Sequence, sums: Optional[Sequence]):
        n = len(plans)
        assert len(tensors) == n and len(packed) == n and (sums is None or len(sums) == n)
        self.n = n
        self.plans = (C.c_void_p * max(n, 1))(*[p.handle.value for p in plans])
        self._rows = [_ptr_array(t) for t in tensors]
        self.tensors = (C.POINTER(C.c_void_p) * max(n, 1))(*[C.cast(r, C.POINTER(C.c_void_p)) for r in self._rows])
        self.packed = _ptr_array(packed)
        self.sums = _ptr_array(sums) if sums is not None else None
        self._keep = (plans, tensors, packed, sums)


def hxt_pack_batch(batch: Batch, stream=None) -> None:
    _check(lib().hxt_pack_batch(batch.n, batch.plans, batch.tensors, batch.packed, batch.sums, _stream(stream)),
           "hxt_pack_batch")


def hxt_unpack_batch(batch: Batch, stream=None) -> None:
    _check(lib().hxt_unpack_batch(batch.n, batch.plans, batch.packed, batch.tensors, batch.sums, _stream(stream)),
           "hxt_unpack_batch")


def hxt_unpack_accumulate_batch(batch: Batch, stream=None) -> None:
    for p in batch._keep[0]:
        if not p.arithmetic:
            raise ValueError("hxt_unpack_accumulate_batch adds bf16 or f32 values: build every plan with "
                             "torch.bfloat16 / torch.float32")
    _check(lib().hxt_unpack_accumulate_batch(batch.n, batch.plans, batch.packed, batch.tensors, batch.sums,
                                             _stream(stream)), "hxt_unpack_accumulate_batch")


class Exchange:
    """Pre-marshalled hxt_exchange_t: src/dst are lists (one entry per message) of lists of tensors."""

    def __init__(self, src, dst, packed_send, path=HXT_DEVICE_DIRECT, packed_recv=None, host_pinned=None,
                 send_sums=None, recv_sums=None, stream_pack=None, stream_stage=None, stream_unpack=None,
                 tags_send=None, tags_recv=None, tags_pinned=None, status=None, seq_base=0,
                 direct_mode=HXT_DIRECT_AUTO, drain_every=0):
        flat = lambda rows: [t for row in rows for t in row]
        opt = lambda rows: _ptr_array(rows) if rows is not None else None
        self._keep = (src, dst, packed_send, packed_recv, host_pinned, send_sums, recv_sums, tags_send, tags_recv,
                      tags_pinned, status)
        self._arrays = [_ptr_array(flat(src)), _ptr_array(flat(dst)), _ptr_array(packed_send),
                        opt(packed_recv), opt(host_pinned)]
        self._tag_arrays = [opt(tags_send), opt(tags_recv), opt(tags_pinned)]
        self.c = _Exchange(len(src), len(packed_send), path, *self._arrays, _ptr(send_sums), _ptr(recv_sums),
                           _stream(stream_pack), _stream(stream_stage), _stream(stream_unpack),
                           *self._tag_arrays, _ptr(status), seq_base, direct_mode, drain_every)


def hxt_exchange_stream(plan: Plan, x: Exchange) -> None:
    _check(lib().hxt_exchange_stream(plan.handle, C.byref(x.c)), "hxt_exchange_stream")


def hxt_checksum(plan: Plan, packed, sums, stream=None) -> None:
    _check(lib().hxt_checksum(plan.handle, _ptr(packed), _ptr(sums), _stream(stream)), "hxt_checksum")


def hxt_checksum2(plan: Plan, packed, sums2, stream=None) -> None:
    _check(lib().hxt_checksum2(plan.handle, _ptr(packed), _ptr(sums2), _stream(stream)), "hxt_checksum2")


TAG_BYTES = 64
HXT_TAG_BAD_MAGIC, HXT_TAG_BAD_PLACE, HXT_TAG_BAD_SEQ, HXT_TAG_BAD_MICRO_BATCH = 1, 2, 4, 8
HXT_TAG_BAD_SUM, HXT_TAG_BAD_WSUM, HXT_TAG_BAD_RESERVED = 16, 32, 64


def hxt_seal(plan: Plan, packed, seq: int, micro_batch: int, tags, stream=None) -> None:
    _check(lib().hxt_seal(plan.handle, _ptr(packed), seq, micro_batch, _ptr(tags), _stream(stream)), "hxt_seal")


def hxt_verify(plan: Plan, packed, tags, seq: int, micro_batch: int, status, stream=None) -> None:
    _check(lib().hxt_verify(plan.handle, _ptr(packed), _ptr(tags), seq, micro_batch, _ptr(status), _stream(stream)),
           "hxt_verify")


def hxt_pack_seal(plan: Plan, src: Sequence, packed, seq: int, micro_batch: int, tags, stream=None) -> None:
    _check(lib().hxt_pack_seal(plan.handle, _ptr_array(src), _ptr(packed), seq, micro_batch, _ptr(tags),
                               _stream(stream)), "hxt_pack_seal")


def hxt_unpack_verify(plan: Plan, packed, tags, seq: int, micro_batch: int, dst: Sequence, status, stream=None) -> None:
    _check(lib().hxt_unpack_verify(plan.handle, _ptr(packed), _ptr(tags), seq, micro_batch, _ptr_array(dst),
                                   _ptr(status), _stream(stream)), "hxt_unpack_verify")


def hxt_pack_noalloc(src, message_bytes: int, n_lanes: int, chunk_bytes: int, packed, sums=None, stream=None) -> None:
    _check(lib().hxt_pack_noalloc(_ptr(src), message_bytes, n_lanes, chunk_bytes, _ptr(packed), _ptr(sums),
                                  _stream(stream)), "hxt_pack_noalloc")


class TagBatch:
    """Pre-marshalled arguments of hxt_pack_seal_batch / hxt_unpack_verify_batch for a fixed set of messages;
    sequence numbers and micro-batch ids are given per call."""

    def __init__(self, plans: Sequence[Plan], tensors: Sequence[Sequence], packed: Sequence, tags: Sequence,
                 status: Optional[Sequence] = None):
        n = len(plans)
        assert len(tensors) == n and len(packed) == n and len(tags) == n and (status is None or len(status) == n)
        self.n = n
        self.plans = (C.c_void_p * max(n, 1))(*[p.handle.value for p in plans])
        self._rows = [_ptr_array(t) for t in tensors]
        self.tensors = (C.POINTER(C.c_void_p) * max(n, 1))(*[C.cast(r, C.POINTER(C.c_void_p)) for r in self._rows])
        self.packed = _ptr_array(packed)
        self.tags = _ptr_array(tags)
        self.status = _ptr_array(status) if status is not None else None
        self._keep = (plans, tensors, packed, tags, status)

    def ids(self, seq: Sequence[int], micro_batch: Sequence[int]):
        return (C.c_uint64 * max(self.n, 1))(*seq), (C.c_uint32 * max(self.n, 1))(*micro_batch)


def hxt_pack_seal_batch(batch: TagBatch, seq: Sequence[int], micro_batch: Sequence[int], stream=None) -> None:
    s_, m_ = batch.ids(seq, micro_batch)
    _check(lib().hxt_pack_seal_batch(batch.n, batch.plans, batch.tensors, batch.packed, s_, m_, batch.tags,
                                     _stream(stream)), "hxt_pack_seal_batch")


def hxt_unpack_verify_batch(batch: TagBatch, seq: Sequence[int], micro_batch: Sequence[int], stream=None) -> None:
    s_, m_ = batch.ids(seq, micro_batch)
    _check(lib().hxt_unpack_verify_batch(batch.n, batch.plans, batch.packed, batch.tags, s_, m_, batch.tensors,
                                         batch.status, _stream(stream)), "hxt_unpack_verify_batch")


def hxt_stage_d2h(plan: Plan, lane: int, packed_dev, host_pinned, stream=None) -> None:
    _check(lib().hxt_stage_d2h(plan.handle, lane, _ptr(packed_dev), _ptr(host_pinned), _stream(stream)),
           "hxt_stage_d2h")


def hxt_stage_h2d(plan: Plan, lane: int, host_pinned, packed_dev, stream=None) -> None:
    _check(lib().hxt_stage_h2d(plan.handle, lane, _ptr(host_pinned), _ptr(packed_dev), _stream(stream)),
           "hxt_stage_h2d")


def hxt_stage_d2h_slots(plan: Plan, lane: int, first_slot: int, n_slots: int, packed_dev, host_pinned, stream=None) -> None:
    _check(lib().hxt_stage_d2h_slots(plan.handle, lane, first_slot, n_slots, _ptr(packed_dev), _ptr(host_pinned),
                                     _stream(stream)), "hxt_stage_d2h_slots")


def hxt_stage_h2d_slots(plan: Plan, lane: int, first_slot: int, n_slots: int, host_pinned, packed_dev, stream=None) -> None:
    _check(lib().hxt_stage_h2d_slots(plan.handle, lane, first_slot, n_slots, _ptr(host_pinned), _ptr(packed_dev),
                                     _stream(stream)), "hxt_stage_h2d_slots")


def hxt_version() -> str:
    return lib().hxt_version().decode()
