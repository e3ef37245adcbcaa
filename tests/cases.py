"""Small message shapes shared by the CPU pins and the GPU parity tests.

Pure descriptions (shape, element strides, element size) plus a seeded byte
source; no arithmetic of the transfer lives here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np


@dataclass(frozen=True)
class Case:
    name: str
    tensors: Tuple[Tuple[tuple, tuple, int], ...]   # (shape, strides in elements, esize)
    k: int
    B: int


def contig(shape, esize):
    st, acc = [], 1
    for s in reversed(shape):
        st.append(acc)
        acc *= max(int(s), 1)
    return (tuple(shape), tuple(reversed(st)), esize)


def storage_bytes(shape, strides, esize):
    if any(s == 0 for s in shape):
        return 0
    return (sum((s - 1) * st for s, st in zip(shape, strides)) + 1) * esize


def permuted(shape, order, esize, scale=2, pad=1):
    """A view whose dims lie in memory in the given order (order[0] varies fastest), the fastest with a stride of
    `scale` elements and `pad` unused elements after every dim, so that no two dims merge."""
    strides, run = [0] * len(shape), scale
    for d in order:
        strides[d] = run
        run *= shape[d] + pad
    return (tuple(shape), tuple(strides), esize)


SMALL_CASES: List[Case] = [
    Case("u8_1000_not_256_multiple", (contig((1000,), 1),), 2, 256),
    Case("ragged_last_chunk_2p5", (contig((1280,), 2),), 3, 1024),          # 2560 B = 2.5 chunks
    Case("fewer_chunks_than_lanes", (contig((300,), 4),), 8, 512),          # 1200 B -> 3 chunks, 8 lanes
    Case("single_lane", (contig((17, 33), 2),), 1, 256),
    Case("chunk_larger_than_message", (contig((100,), 2),), 4, 4096),
    Case("three_tensors_with_gaps", (contig((10,), 1), contig((300,), 1), contig((4096,), 1)), 2, 1024),
    Case("rows_not_16B_multiple", (((7, 100), (128, 1), 2),), 2, 512),       # 200-byte rows, padded pitch
    Case("rows_interleaved_3d", (((6, 2, 64), (64, 6 * 64, 1), 2),), 3, 256),   # [seq,mb,h] view of [mb,seq,h]
    Case("true_transpose_64x48", (((64, 48), (1, 64), 2),), 2, 512),
    Case("transpose_f32_odd", (((33, 17), (1, 40), 4),), 2, 256),
    Case("transpose_batched", (((3, 20, 24), (600, 1, 24), 2),), 2, 256),
    Case("broadcast_stride0", (((5, 64), (0, 1), 4),), 2, 256),
    Case("esize1_2d_strided", (((9, 31), (40, 1), 1),), 2, 256),
    Case("esize8_strided", (((12, 10), (16, 1), 8),), 3, 256),
    Case("esize8_transpose", (((10, 12), (1, 16), 8),), 2, 256),
    Case("four_d_mixed", (((3, 4, 5, 6), (200, 6, 40, 1), 2),), 2, 256),     # middle dims permuted
    Case("size_one_dims", (((1, 50, 1, 8), (7777, 8, 9999, 1), 2),), 2, 256),
    Case("scalar_0d", (((), (), 4),), 1, 256),
    Case("empty_tensor", (((0, 16), (16, 1), 2),), 2, 256),
    Case("empty_between", (contig((100,), 2), ((0,), (1,), 2), contig((77,), 4)), 2, 256),
    Case("inner_stride_2", (((40, 24), (48, 2), 2),), 2, 256),               # every other element
    Case("eight_dims_permuted", (((2, 3, 2, 2, 3, 2, 2, 4), (288, 48, 2, 576, 4, 1, 144, 12), 2),), 3, 256),
    Case("five_dims_no_unit_stride", (permuted((3, 2, 4, 2, 5), (2, 0, 4, 1, 3), 2),), 3, 256),
    Case("six_dims_no_unit_stride_u8", (permuted((2, 3, 2, 3, 2, 5), (5, 3, 1, 0, 2, 4), 1, scale=3),), 2, 512),
    Case("eight_dims_no_unit_stride_f32", (permuted((2, 2, 3, 2, 2, 3, 2, 2), (7, 0, 6, 1, 5, 2, 4, 3), 4, pad=0),), 2, 256),
    Case("six_dims_rows_32_byte_runs", (((2, 3, 2, 3, 2, 16), (384, 96, 1152, 24, 3456, 1), 2),), 2, 512),
    Case("six_dims_rows_20_byte_runs", (permuted((2, 3, 2, 3, 2, 10), (5, 1, 3, 0, 4, 2), 2, scale=1),), 3, 256),
    Case("seven_dims_f64_no_unit_stride", (permuted((2, 2, 2, 3, 2, 2, 3), (3, 6, 0, 5, 1, 4, 2), 8),), 2, 1024),
    Case("transpose_inner_stride_2", (((24, 40), (2, 48), 2),), 2, 16384),   # storage-fast dim strided by two elements
    Case("transpose_inner_stride_3_u8", (((5, 17, 33), (4000, 3, 60), 1),), 3, 8192),
    Case("transpose_inner_stride_2_f64", (((20, 12), (2, 48), 8),), 2, 8192),  # 16 bytes from element to element
    Case("inner_stride_3_f64_too_wide", (((20, 12), (3, 72), 8),), 2, 8192),   # 24 bytes: the per-element kernel
    Case("inner_stride_2_flat_chunks", (((24, 40), (2, 48), 2),), 2, 256),     # chunks below 1 KiB that hold 3 packed rows: per element
    Case("transpose_span_bf16", (((40, 300), (1, 40), 2),), 3, 1024),          # 600-byte packed rows: tiles span chunks
    Case("transpose_span_f32_batched", (((3, 70, 90), (70 * 100, 1, 70), 4),), 4, 1024),
    Case("transpose_span_u8_long_rows", (((5, 3000), (1, 8), 1),), 2, 1024),   # a packed row is longer than a chunk
    Case("transpose_span_strided_f64", (((20, 50), (2, 48), 8),), 2, 2048),
    Case("transpose_span_between_contig", (contig((100,), 1), ((64, 200), (1, 64), 2), contig((700,), 4)), 4, 1024),
    Case("sixty_four_lanes", (contig((40000,), 2),), 64, 512),                # 157 chunks, lanes hold 3 or 2
    Case("mixed_dtypes_multi", (contig((33,), 1), ((8, 24), (32, 1), 2), ((16, 8), (1, 16), 4), contig((5,), 8)), 4, 512),
]


def case_by_name(name: str) -> Case:
    for c in SMALL_CASES:
        if c.name == name:
            return c
    raise KeyError(name)


def make_storages(case: Case, seed: int) -> List[np.ndarray]:
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, size=storage_bytes(*t), dtype=np.uint8) for t in case.tensors]


def random_view(rng, max_dims=4):
    """(shape, strides, esize) of a random non-negative-stride view with a small storage footprint."""
    esize = int(rng.choice([1, 2, 4, 8]))
    nd = int(rng.integers(0, max_dims + 1))
    sizes = [1, 2, 3, 5, 8, 16, 17, 40, 64, 72, 130] if max_dims <= 4 else [1, 2, 2, 3, 3, 4, 5, 8, 16, 17]
    shape = [int(rng.choice(sizes)) for _ in range(nd)]
    if rng.random() < 0.08 and nd:
        shape[int(rng.integers(0, nd))] = 0
    order = list(rng.permutation(nd))                      # order[0] is the fastest-varying dim in memory
    strides, run = [0] * nd, 1
    for d in order:
        pad = int(rng.choice([0, 0, 0, 1, 3, 8]))
        strides[d] = run
        run *= max(shape[d], 1) + pad
        if run > 60000:                                    # keep storage small: flatten the rest with stride reuse
            run = 60000
    if rng.random() < 0.1 and nd:
        strides[int(rng.integers(0, nd))] = 0              # broadcast
    if rng.random() < 0.1 and nd:
        d = int(rng.integers(0, nd))
        strides[d] *= 2                                    # holes
    return tuple(shape), tuple(int(x) for x in strides), esize
