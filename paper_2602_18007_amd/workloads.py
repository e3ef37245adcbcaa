"""Seeded synthetic inputs shaped like the paper's pipeline-boundary messages.

This module only *describes* messages (shapes, strides, lanes, chunk size) and
draws their bytes; it contains none of the transfer's arithmetic and imports
neither the HIP binding nor the CPU oracle, so both can be fed from it.

The paper (Section 3.1) trains LLaMA-8B and Qwen2-7B with pipeline parallelism
2 and does not state precision, sequence length or micro-batch size; the shapes
below use the public hidden sizes of those models (4096 and 3584), bf16, and a
sequence length of 4096.  Values are drawn on the host once, so every consumer
sees the same bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

KiB = 1024
MiB = 1024 * 1024
BASE_SEED = 18007


@dataclass(frozen=True)
class TensorDesc:
    shape: Tuple[int, ...]
    strides: Tuple[int, ...]  # in elements
    esize: int = 2            # bf16
    name: str = ""

    @staticmethod
    def contiguous(shape, esize=2, name="") -> "TensorDesc":
        st, acc = [], 1
        for s in reversed(shape):
            st.append(acc)
            acc *= max(int(s), 1)
        return TensorDesc(tuple(int(s) for s in shape), tuple(reversed(st)), esize, name)

    @property
    def elems(self) -> int:
        n = 1
        for s in self.shape:
            n *= s
        return n

    @property
    def nbytes(self) -> int:
        return self.elems * self.esize

    @property
    def storage_elems(self) -> int:
        if self.elems == 0:
            return 0
        return sum((s - 1) * st for s, st in zip(self.shape, self.strides)) + 1


@dataclass(frozen=True)
class Workload:
    name: str
    tensors: Tuple[TensorDesc, ...]
    n_lanes: int
    chunk_bytes: int
    dist: str                  # "bits16" = uniform 16-bit patterns, "normal" = N(0, std) cast to bf16
    std: float = 1.0
    seed: int = BASE_SEED
    messages: int = 1          # independent messages of this geometry (micro-batches, fwd/bwd pair)
    seed_step: int = 0         # message i uses seed + i * seed_step
    paths: Tuple[str, ...] = ("device_direct",)
    note: str = ""

    @property
    def message_bytes(self) -> int:
        return sum(t.nbytes for t in self.tensors)


def _llama_layer_grads() -> List[TensorDesc]:
    c = TensorDesc.contiguous
    return [
        c((4096,), name="ln1"), c((4096, 4096), name="q"), c((1024, 4096), name="k"),
        c((1024, 4096), name="v"), c((4096, 4096), name="o"), c((4096,), name="ln2"),
        c((14336, 4096), name="gate"), c((14336, 4096), name="up"), c((4096, 14336), name="down"),
    ]


def tiny() -> Workload:
    return Workload("tiny", (TensorDesc.contiguous((1, 128, 512)),), 2, 16 * KiB, "bits16",
                    seed=BASE_SEED + 1, note="one contiguous bf16 tensor, 128 KiB")


def llama8b_boundary() -> Workload:
    # message 0 = forward activation, message 1 = backward activation gradient
    return Workload("llama8b_boundary", (TensorDesc.contiguous((4096, 1, 4096)),), 4, 1 * MiB, "normal", 1.0,
                    seed=BASE_SEED + 2, messages=2, seed_step=1,
                    note="bf16 [seq=4096, mb=1, hidden=4096], forward activation + backward gradient")


def qwen2_7b_boundary() -> Workload:
    return Workload("qwen2_7b_boundary", (TensorDesc.contiguous((4096, 2, 3584)),), 8, 4 * MiB, "normal", 1.0,
                    seed=BASE_SEED + 3, paths=("device_direct", "cpu_forward"),
                    note="bf16 [seq=4096, mb=2, hidden=3584]")


def stream_1f1b(micro_batches: int = 32) -> Workload:
    # [seq, mb, hidden] view of [mb, seq, hidden] storage
    t = TensorDesc((4096, 1, 4096), (4096, 4096 * 4096, 1))
    return Workload("stream_1f1b", (t,), 4, 2 * MiB, "normal", 1.0, seed=BASE_SEED + 4,
                    messages=micro_batches, seed_step=100, paths=("device_direct", "cpu_forward"),
                    note="32 micro-batches, transposed [seq,mb,hidden] view, ping-pong buffers, 3 streams")


def grad_buckets(layers: int = 4) -> Workload:
    ts: List[TensorDesc] = []
    for i in range(layers):
        ts += [TensorDesc(t.shape, t.strides, t.esize, f"layer{i}.{t.name}") for t in _llama_layer_grads()]
    return Workload("grad_buckets", tuple(ts), 8, 25 * MiB, "normal", 0.02, seed=BASE_SEED + 5,
                    paths=("device_direct", "cpu_forward"),
                    note="per-layer bf16 grads of 4 LLaMA-8B layers, 25 MiB buckets")


def qwen_rows_view() -> Workload:
    """Supplementary: the Qwen2-7B tensor as a real strided gather (7168-byte runs, two interleaved streams)."""
    t = TensorDesc((4096, 2, 3584), (3584, 4096 * 3584, 1))
    return Workload("qwen_rows_view", (t,), 8, 4 * MiB, "normal", 1.0, seed=BASE_SEED + 3,
                    note="[seq,mb,hidden] view of [mb,seq,hidden] storage, mb=2")


def transpose_view() -> Workload:
    """Supplementary: inner stride != 1, needs a real transpose."""
    t = TensorDesc((4096, 4096), (1, 4096))
    return Workload("transpose_view", (t,), 4, 1 * MiB, "normal", 1.0, seed=BASE_SEED + 6,
                    note="bf16 logical [4096,4096] with strides (1,4096)")


def rows_split_view() -> Workload:
    """Supplementary: rows whose length is not a multiple of 16 bytes (200-byte runs at a pitch of 256 bytes)."""
    t = TensorDesc((327680, 100), (128, 1))
    return Workload("rows_split_view", (t,), 4, 1 * MiB, "normal", 1.0, seed=BASE_SEED + 7,
                    note="bf16 [327680,100] view with a row pitch of 128 elements (62.5 MiB)")


def inner_stride_view() -> Workload:
    """Supplementary: innermost stride of two elements and no dimension with stride one (every other column of a
    [4096, 8192] matrix): neither a row gather nor a transpose, so the per-element kernel takes it."""
    t = TensorDesc((4096, 4096), (8192, 2))
    return Workload("inner_stride_view", (t,), 4, 1 * MiB, "normal", 1.0, seed=BASE_SEED + 8,
                    note="bf16 [4096,4096] view with strides (8192,2) (32 MiB out of 64 MiB of storage)")


def wide_transpose_view() -> Workload:
    """Supplementary: a transposed view whose packed rows are long against the chunk (128 KiB rows, 1 MiB chunks:
    8 rows per chunk), so that full transpose tiles span chunks."""
    t = TensorDesc((256, 65536), (1, 256))
    return Workload("wide_transpose_view", (t,), 4, 1 * MiB, "normal", 1.0, seed=BASE_SEED + 9,
                    note="bf16 logical [256,65536] with strides (1,256) (32 MiB)")


ALL = {
    "tiny": tiny, "llama8b_boundary": llama8b_boundary, "qwen2_7b_boundary": qwen2_7b_boundary,
    "stream_1f1b": stream_1f1b, "grad_buckets": grad_buckets,
    "qwen_rows_view": qwen_rows_view, "transpose_view": transpose_view, "rows_split_view": rows_split_view,
    "inner_stride_view": inner_stride_view, "wide_transpose_view": wide_transpose_view,
}


# ---- value generation -------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even cast of float32 to the 16-bit bf16 pattern (format conversion, input side only)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def draw_u16(n: int, dist: str, std: float, rng: np.random.Generator) -> np.ndarray:
    """n 16-bit values: raw uniform bit patterns, or N(0, std) rounded to bf16."""
    if dist == "bits16":
        return rng.integers(0, 1 << 16, size=n, dtype=np.uint16)
    if dist == "normal":
        out = np.empty(n, dtype=np.uint16)
        step = 1 << 24                               # bounded temporaries for the 800M-element case
        for a in range(0, n, step):
            b = min(n, a + step)
            out[a:b] = f32_to_bf16_bits(rng.standard_normal(b - a, dtype=np.float32) * np.float32(std))
        return out
    raise ValueError(dist)


def make_storages(w: Workload, message: int = 0) -> List[np.ndarray]:
    """One uint8 array per tensor holding that tensor's storage for message ``message``."""
    rng = np.random.default_rng(w.seed + message * w.seed_step)
    out = []
    for t in w.tensors:
        nbytes = t.storage_elems * t.esize
        assert nbytes % 2 == 0
        out.append(draw_u16(nbytes // 2, w.dist, w.std, rng).view(np.uint8))
    return out
