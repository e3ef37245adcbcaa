"""Host logic of the library, on the CPU: the C ABI loads and exports what the header
declares, plan queries agree with the oracle, argument errors come back as codes, and the
planner's work tables (executed byte by byte by a bounds-checking interpreter) reproduce
the oracle's packed buffer without touching a byte twice or out of range."""
import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import hxt_oracle as ho
from paper_2602_18007_amd import build as hxt_build
from paper_2602_18007_amd import hxt
from paper_2602_18007_amd import workloads as wl
from tests.cases import SMALL_CASES, Case, contig, make_storages, random_view, storage_bytes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="session", autouse=True)
def built_library():
    hxt_build.build(force=False)


def oracle_msg(case):
    return ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])


def plan_of(case):
    return hxt.hxt_plan_multi([(s, st, e) for (s, st, e) in case.tensors], case.k, case.B)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "hxt.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(hxt_[a-z0-9_]+)\s*\(", header))
    assert declared == set(hxt.EXPORTS)
    raw = C.CDLL(hxt.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(raw, name), name
    assert hxt.hxt_version().startswith("hxt")


def test_a_plain_c_program_can_use_the_library(tmp_path):
    """The boundary is a C ABI: a C11 client, compiled with gcc against include/hxt.h and linked with the
    shared library, creates a plan and reads its geometry (control plane only, no GPU needed)."""
    exe = tmp_path / "abi_client"
    pkg = os.path.join(ROOT, "paper_2602_18007_amd")
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "host", "abi_client.c"), "-o", str(exe),
                    "-L", pkg, "-lhxt", "-Wl,-rpath," + pkg, "-Wl,-rpath-link,/opt/rocm/lib"], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "abi_client: ok" in r.stdout


def test_header_is_plain_c_and_the_tag_record_has_the_documented_offsets(tmp_path):
    """include/hxt.h must compile as C; the 64-byte tag record's field offsets are the ones the oracle documents."""
    src = tmp_path / "abi.c"
    src.write_text("""
#include <stddef.h>
#include "hxt.h"
_Static_assert(sizeof(hxt_chunk_tag_t) == 64, "size");
_Static_assert(offsetof(hxt_chunk_tag_t, magic) == 0 && offsetof(hxt_chunk_tag_t, chunk) == 4, "a");
_Static_assert(offsetof(hxt_chunk_tag_t, lane) == 8 && offsetof(hxt_chunk_tag_t, slot) == 12, "b");
_Static_assert(offsetof(hxt_chunk_tag_t, seq) == 16 && offsetof(hxt_chunk_tag_t, micro_batch) == 24, "c");
_Static_assert(offsetof(hxt_chunk_tag_t, n_chunks) == 28 && offsetof(hxt_chunk_tag_t, padded) == 32, "d");
_Static_assert(offsetof(hxt_chunk_tag_t, sum) == 40 && offsetof(hxt_chunk_tag_t, wsum) == 48, "e");
_Static_assert(offsetof(hxt_chunk_tag_t, zero) == 56, "f");
_Static_assert(HXT_TAG_MAGIC == 0x31545848u, "magic");
_Static_assert(HXT_TAG_BAD_MAGIC == 1 && HXT_TAG_BAD_PLACE == 2 && HXT_TAG_BAD_SEQ == 4 && HXT_TAG_BAD_MICRO_BATCH == 8
               && HXT_TAG_BAD_SUM == 16 && HXT_TAG_BAD_WSUM == 32 && HXT_TAG_BAD_RESERVED == 64, "bits");
int main(void) { return 0; }
""")
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", os.path.join(ROOT, "include"),
                    str(src)], check=True)


@pytest.mark.parametrize("case", SMALL_CASES, ids=lambda c: c.name)
def test_plan_queries_match_oracle(case):
    m, p = oracle_msg(case), plan_of(case)
    assert (p.message_bytes, p.stream_bytes) == (m.N, m.L)
    assert p.num_chunks == ho.num_chunks(m, case.B)
    assert p.packed_bytes == ho.packed_bytes(m, case.B, case.k)
    assert (p.num_lanes, p.chunk_bytes, p.num_tensors) == (case.k, case.B, len(case.tensors))
    for c in range(p.num_chunks):
        assert p.chunk_info(c) == ho.chunk_info(m, case.B, case.k, c)
    for l in range(case.k):
        assert p.lane_info(l) == ho.lane_info(m, case.B, case.k, l)


@pytest.mark.parametrize("name", list(wl.ALL))
def test_plan_queries_match_oracle_on_benchmark_messages(name):
    w = wl.ALL[name]()
    case = Case(name, tuple((t.shape, t.strides, t.esize) for t in w.tensors), w.n_lanes, w.chunk_bytes)
    test_plan_queries_match_oracle(case)


def test_receive_side_plan_is_interchangeable():
    # same five arguments on both sides -> same table (the receive is symmetric, Section 2.2)
    case = SMALL_CASES[5]
    a, b = plan_of(case), plan_of(case)
    assert [a.chunk_info(c) for c in range(a.num_chunks)] == [b.chunk_info(c) for c in range(b.num_chunks)]


def test_transposed_view_with_unit_dim_is_planned_as_contiguous():
    w = wl.stream_1f1b()
    t = w.tensors[0]
    view = hxt.hxt_plan(t.shape, t.strides, 2, w.n_lanes, w.chunk_bytes)
    flat = hxt.hxt_plan((1, 4096, 4096), None, 2, w.n_lanes, w.chunk_bytes)
    assert view.tensor_kind(0) == flat.tensor_kind(0) == "contig"
    assert [view.chunk_info(c) for c in range(16)] == [flat.chunk_info(c) for c in range(16)]


def test_kernel_family_per_view():
    kinds = {c.name: [plan_of(c).tensor_kind(t) for t in range(len(c.tensors))] for c in SMALL_CASES}
    assert kinds["rows_interleaved_3d"] == ["rows"]
    assert kinds["true_transpose_64x48"] == ["transpose"]
    assert kinds["transpose_batched"] == ["transpose"]
    assert kinds["rows_not_16B_multiple"] == ["rows_split"]   # 200-byte runs: the row gather in narrower pieces
    assert kinds["esize1_2d_strided"] == ["rows_split"]       # 31-byte runs
    assert kinds["four_d_mixed"] == ["generic"]               # 12-byte runs are too short for it
    assert kinds["inner_stride_2"] == ["generic"]
    for name in ("five_dims_no_unit_stride", "six_dims_no_unit_stride_u8", "eight_dims_no_unit_stride_f32",
                 "seven_dims_f64_no_unit_stride", "eight_dims_permuted"):
        assert kinds[name] == ["generic"], name                # more than four dims that do not merge
    for name in ("transpose_inner_stride_2", "transpose_inner_stride_3_u8", "transpose_inner_stride_2_f64"):
        assert kinds[name] == ["transpose"], name              # the storage-fast dim strided by up to 16 bytes
    for name in ("transpose_span_bf16", "transpose_span_f32_batched", "transpose_span_u8_long_rows",
                 "transpose_span_strided_f64"):
        assert kinds[name] == ["transpose_span"], name         # a chunk holds fewer rows of the packed side than a tile is high
    assert kinds["transpose_span_between_contig"] == ["contig", "transpose_span", "contig"]
    assert kinds["true_transpose_64x48"] == ["transpose"]      # chunks below 1 KiB: tiles stay inside chunks
    assert kinds["inner_stride_3_f64_too_wide"] == ["generic"]
    assert kinds["inner_stride_2_flat_chunks"] == ["generic"]
    assert kinds["six_dims_rows_32_byte_runs"] == ["rows"]
    assert kinds["six_dims_rows_20_byte_runs"] == ["rows_split"]
    assert kinds["size_one_dims"] == ["contig"]
    assert kinds["scalar_0d"] == ["contig"]
    assert kinds["empty_tensor"] == ["none"]
    assert kinds["mixed_dtypes_multi"] == ["contig", "rows", "transpose", "contig"]
    assert plan_of(Case("q", (((4096, 2, 3584), (3584, 4096 * 3584, 1), 2),), 8, 4 << 20)).tensor_kind(0) == "rows"


def test_unpack_safety_flag():
    assert not plan_of(Case("b", (((5, 64), (0, 1), 4),), 2, 256)).tensor_unpack_safe(0)      # broadcast
    assert not plan_of(Case("o", (((4, 8), (4, 1), 2),), 2, 256)).tensor_unpack_safe(0)       # rows overlap
    assert plan_of(Case("t", (((64, 48), (1, 64), 2),), 2, 256)).tensor_unpack_safe(0)
    assert plan_of(Case("p", (((3, 4, 5, 6), (200, 6, 40, 1), 2),), 2, 256)).tensor_unpack_safe(0)
    assert plan_of(Case("e", (((0, 4), (0, 0), 2),), 2, 256)).tensor_unpack_safe(0)           # empty


def test_plan_accepts_a_far_reaching_view_below_the_limit():
    p = hxt.hxt_plan((2, 64), (1 << 59, 1), 2, 2, 256)                         # 2^60 bytes apart: still addressable
    assert p.message_bytes == 256 and p.tensor_unpack_safe(0)


@pytest.mark.parametrize("kwargs,status", [
    (dict(n_lanes=0), hxt.HXT_EINVAL), (dict(n_lanes=1025), hxt.HXT_EINVAL),
    (dict(chunk_bytes=0), hxt.HXT_EINVAL), (dict(chunk_bytes=1000), hxt.HXT_EINVAL),
    (dict(shape=(4, -1)), hxt.HXT_EINVAL), (dict(strides=(-2, 1)), hxt.HXT_EINVAL),
    (dict(shape=(1,) * 9, strides=(1,) * 9), hxt.HXT_EINVAL),
    (dict(shape=(1 << 30, 1 << 20), strides=None), hxt.HXT_EUNSUPPORTED),
    (dict(shape=(4, 4), strides=(1 << 61, 1)), hxt.HXT_EUNSUPPORTED),          # farthest element past 2^62 bytes
    (dict(shape=(3, 1 << 20), strides=((1 << 63) - 1, (1 << 43))), hxt.HXT_EUNSUPPORTED),   # products that overflow 64 bits
])
def test_plan_rejects_bad_arguments(kwargs, status):
    args = dict(shape=(4, 4), strides=(4, 1), dtype=2, n_lanes=2, chunk_bytes=256)
    args.update(kwargs)
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_plan(**args)
    assert e.value.status == status


def test_raw_abi_null_and_dtype_errors():
    L = hxt.lib()
    shp = (C.c_int64 * 2)(4, 4)
    out = C.c_void_p()
    assert L.hxt_plan(shp, None, 2, 3, 2, 256, None) == hxt.HXT_EINVAL              # out == NULL
    assert L.hxt_plan(None, None, 2, 3, 2, 256, C.byref(out)) == hxt.HXT_EINVAL     # shape == NULL
    assert L.hxt_plan(shp, None, 2, 99, 2, 256, C.byref(out)) == hxt.HXT_EINVAL     # dtype
    assert L.hxt_plan(shp, None, -1, 3, 2, 256, C.byref(out)) == hxt.HXT_EINVAL
    assert out.value is None
    assert L.hxt_plan_destroy(None) == hxt.HXT_OK
    assert L.hxt_pack(None, None, None, None, None) == hxt.HXT_EINVAL
    assert L.hxt_stage_d2h(None, 0, None, None, None) == hxt.HXT_EINVAL
    p = hxt.hxt_plan((4, 4), None, 2, 2, 256)
    info = hxt.ChunkInfo()
    assert L.hxt_plan_chunk_info(p.handle, 7, C.byref(info)) == hxt.HXT_EINVAL
    assert L.hxt_plan_lane_info(p.handle, 2, None) == hxt.HXT_EINVAL
    assert L.hxt_stage_d2h(p.handle, 5, 256, 256, None) == hxt.HXT_EINVAL           # bad lane
    assert L.hxt_stage_d2h(p.handle, 0, 256 + 8, 256, None) == hxt.HXT_EALIGN
    assert L.hxt_pack(p.handle, None, 256 + 16, None, None) == hxt.HXT_EALIGN       # packed misaligned
    assert L.hxt_checksum(p.handle, None, None, None) == hxt.HXT_EINVAL
    assert b"align" in L.hxt_strerror(hxt.HXT_EALIGN)


def test_argument_errors_of_the_newer_entry_points():
    """Options, staging in runs of slots, the batched tag calls, the stream's mode fields and the plan-free pack:
    everything that is refused before a GPU is touched."""
    L = hxt.lib()
    p = hxt.hxt_plan((2560,), None, 1, 2, 1024)                       # 3 chunks: lane 0 holds 2, lane 1 holds 1
    assert L.hxt_plan_set_option(None, hxt.HXT_OPT_PACKED_HINT, 1) == hxt.HXT_EINVAL
    assert L.hxt_plan_set_option(p.handle, 99, 1) == hxt.HXT_EINVAL
    assert L.hxt_plan_set_option(p.handle, hxt.HXT_OPT_PACKED_HINT, 2) == hxt.HXT_EINVAL
    assert L.hxt_plan_set_option(p.handle, hxt.HXT_OPT_STAGE_D2H, -1) == hxt.HXT_EINVAL
    for opt, vals in ((hxt.HXT_OPT_PACKED_HINT, (-1, 0, 1)), (hxt.HXT_OPT_STAGE_D2H, (0, 1, 0))):
        for v in vals:
            assert L.hxt_plan_set_option(p.handle, opt, v) == hxt.HXT_OK
    for f in (L.hxt_stage_d2h_slots, L.hxt_stage_h2d_slots):
        assert f(None, 0, 0, 1, 256, 256, None) == hxt.HXT_EINVAL
        assert f(p.handle, -1, 0, 1, 256, 256, None) == hxt.HXT_EINVAL          # a run of slots belongs to one lane
        assert f(p.handle, 2, 0, 1, 256, 256, None) == hxt.HXT_EINVAL
        assert f(p.handle, 0, 1, 2, 256, 256, None) == hxt.HXT_EINVAL           # lane 0 has slots 0 and 1 only
        assert f(p.handle, 1, 1, 1, 256, 256, None) == hxt.HXT_EINVAL
        assert f(p.handle, 0, 0, -1, 256, 256, None) == hxt.HXT_EINVAL
        assert f(p.handle, 0, -1, 1, 256, 256, None) == hxt.HXT_EINVAL
        assert f(p.handle, 0, 2, 0, None, None, None) == hxt.HXT_OK             # the empty run
        assert f(p.handle, 0, 0, 1, 256 + 8, 256, None) == hxt.HXT_EALIGN
        assert f(p.handle, 0, 0, 1, None, 256, None) == hxt.HXT_EINVAL
    assert L.hxt_pack_seal_batch(-1, None, None, None, None, None, None, None) == hxt.HXT_EINVAL
    assert L.hxt_pack_seal_batch(1, None, None, None, None, None, None, None) == hxt.HXT_EINVAL
    assert L.hxt_unpack_verify_batch(1, None, None, None, None, None, None, None, None) == hxt.HXT_EINVAL
    assert L.hxt_pack_seal_batch(0, None, None, None, None, None, None, None) == hxt.HXT_OK
    assert L.hxt_unpack_accumulate_batch(-1, None, None, None, None, None) == hxt.HXT_EINVAL
    assert L.hxt_unpack_accumulate_batch(2, None, None, None, None, None) == hxt.HXT_EINVAL
    assert L.hxt_unpack_accumulate_batch(0, None, None, None, None, None) == hxt.HXT_OK
    assert L.hxt_pack_noalloc(None, 100, 0, 256, None, None, None) == hxt.HXT_EINVAL
    assert L.hxt_pack_noalloc(None, 100, 2, 100, None, None, None) == hxt.HXT_EINVAL
    assert L.hxt_pack_noalloc(None, 100, 2, 256, None, None, None) == hxt.HXT_EINVAL      # NULL buffers
    assert L.hxt_pack_noalloc(256, 100, 2, 256, 256 + 16, None, None) == hxt.HXT_EALIGN
    assert L.hxt_pack_noalloc(None, 0, 2, 256, None, None, None) == hxt.HXT_OK            # empty message
    assert L.hxt_pack_noalloc(256, (1 << 40) + 1, 2, 256, 256, None, None) == hxt.HXT_EUNSUPPORTED
    x = hxt._Exchange()
    x.n_messages, x.n_buffers, x.drain_every = 1, 1, -1
    assert L.hxt_exchange_stream(p.handle, C.byref(x)) == hxt.HXT_EINVAL


def test_without_a_gpu_the_data_plane_reports_an_error_instead_of_falling_back():
    import torch
    if torch.cuda.is_available():
        pytest.skip("needs a machine without a GPU")
    p = hxt.hxt_plan((1000,), None, 1, 2, 256)
    L = hxt.lib()
    fake = 1 << 20                                            # never dereferenced: the call fails before any launch
    ptrs = (C.c_void_p * 1)(fake)
    assert p.num_chunks == 4                                  # queries still work
    assert L.hxt_pack(p.handle, ptrs, fake, None, None) == hxt.HXT_EHIP
    assert L.hxt_unpack(p.handle, fake, ptrs, None, None) == hxt.HXT_EHIP
    assert L.hxt_checksum(p.handle, fake, fake, None) == hxt.HXT_EHIP
    assert L.hxt_checksum2(p.handle, fake, fake, None) == hxt.HXT_EHIP
    assert L.hxt_seal(p.handle, fake, 1, 1, fake, None) == hxt.HXT_EHIP
    assert L.hxt_pack_seal(p.handle, ptrs, fake, 1, 1, fake, None) == hxt.HXT_EHIP
    assert L.hxt_pack_noalloc(fake, 1000, 2, 256, fake, fake, None) == hxt.HXT_EHIP
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_pack(p, [fake], fake, None)
    assert e.value.status == hxt.HXT_EHIP and "HIP" in str(e.value)


def test_binding_raises_when_the_library_is_not_built(monkeypatch, tmp_path):
    monkeypatch.setattr(hxt, "_lib", None)
    monkeypatch.setattr(hxt, "LIB_PATH", str(tmp_path / "libhxt.so"))
    with pytest.raises(RuntimeError, match="not built"):
        hxt.hxt_plan((16,), None, 1, 1, 256)


def test_empty_message_calls_are_no_ops():
    p = hxt.hxt_plan((0, 16), None, 2, 2, 256)
    assert (p.message_bytes, p.num_chunks, p.packed_bytes) == (0, 0, 0)
    L = hxt.lib()
    assert L.hxt_pack(p.handle, None, None, None, None) == hxt.HXT_OK
    assert L.hxt_unpack(p.handle, None, None, None, None) == hxt.HXT_OK
    assert L.hxt_checksum(p.handle, None, None, None) == hxt.HXT_OK
    assert L.hxt_stage_d2h(p.handle, -1, None, None, None) == hxt.HXT_OK


# ---- the planner's work tables, executed on the CPU --------------------------------

class _Desc(C.Structure):
    _fields_ = [("ndim", C.c_int), ("shape", C.POINTER(C.c_int64)), ("strides", C.POINTER(C.c_int64)),
                ("dtype", C.c_int)]


@pytest.fixture(scope="session")
def interp():
    src = os.path.join(ROOT, "tests", "host", "plan_interp.cpp")
    out = os.path.join(ROOT, "tests", "host", "libplan_interp.so")
    csrc = os.path.join(ROOT, "paper_2602_18007_amd", "csrc")
    deps = [src, os.path.join(csrc, "hxt_plan.cpp"), os.path.join(csrc, "hxt_internal.h")]
    if not os.path.exists(out) or any(os.path.getmtime(d) > os.path.getmtime(out) for d in deps):
        subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-shared", "-fPIC", "-Wall", "-Wextra",
                        "-fsanitize=undefined", "-fno-sanitize-recover=all",
                        "-I", os.path.join(ROOT, "include"), "-I", csrc, "-o", out, src,
                        os.path.join(csrc, "hxt_plan.cpp")], check=True)
    L = C.CDLL(out)
    L.plan_interp.restype = C.c_int
    L.fastdiv_check.restype = C.c_int
    return L


def run_interp(L, case, storages, packed, direction, tile_bytes):
    n = len(case.tensors)
    descs = (_Desc * max(n, 1))()
    keep = []
    size_code = {1: 1, 2: 3, 4: 4, 8: 5}
    for j, (shape, strides, e) in enumerate(case.tensors):
        shp = (C.c_int64 * max(len(shape), 1))(*shape)
        st = (C.c_int64 * max(len(shape), 1))(*strides)
        keep += [shp, st]
        descs[j].ndim, descs[j].shape, descs[j].strides, descs[j].dtype = len(shape), shp, st, size_code[e]
    bases = (C.c_void_p * max(n, 1))(*[s.ctypes.data for s in storages])
    sizes = (C.c_uint64 * max(n, 1))(*[s.size for s in storages])
    written = np.zeros(max(packed.size, 1), np.uint8)
    kinds = (C.c_int32 * max(n, 1))()
    uniform = C.c_int32(0)
    rc = L.plan_interp(descs, n, case.k, C.c_uint64(case.B), C.c_uint32(tile_bytes), bases, sizes,
                       C.c_void_p(packed.ctypes.data), C.c_uint64(packed.size), C.c_void_p(written.ctypes.data),
                       direction, kinds, C.byref(uniform))
    run_interp.last_uniform = bool(uniform.value)
    return rc, written[:packed.size], list(kinds)[:n]


@pytest.mark.parametrize("tile_bytes", [256, 1024, 16384])
@pytest.mark.parametrize("case", SMALL_CASES, ids=lambda c: c.name)
def test_work_tables_reproduce_oracle_pack_and_unpack(interp, case, tile_bytes):
    m = oracle_msg(case)
    raws = make_storages(case, 77)
    want = ho.pack(m, raws, case.B, case.k, fill=0x99)
    got = np.full(want.size, 0x99, np.uint8)
    rc, written, _ = run_interp(interp, case, raws, got, 0, tile_bytes)
    assert rc == 0
    assert np.array_equal(got, want)
    # every specified byte written exactly once, unspecified bytes never
    spec = np.zeros(want.size, bool)
    for c in range(ho.num_chunks(m, case.B)):
        info = ho.chunk_info(m, case.B, case.k, c)
        spec[info["packed_off"]:info["packed_off"] + info["padded"]] = True
    assert np.all(written[spec] == 1) and np.all(written[~spec] == 0)
    # closed-form path (messages made of one contiguous tensor)
    got2 = np.full(want.size, 0x99, np.uint8)
    rc, _, kinds = run_interp(interp, case, raws, got2, 2, tile_bytes)
    assert rc == 0 and np.array_equal(got2, want)
    live = [i for i, t in enumerate(case.tensors) if 0 not in t[0]]
    assert run_interp.last_uniform == (len(live) == 1 and kinds[live[0]] == 1)
    if case.name == "broadcast_stride0":
        return
    dst_o = [np.full(r.size, 0x42, np.uint8) for r in raws]
    dst_t = [np.full(r.size, 0x42, np.uint8) for r in raws]
    ho.unpack(m, want, case.B, case.k, dst_o)
    rc, _, _ = run_interp(interp, case, dst_t, want.copy(), 1, tile_bytes)
    assert rc == 0
    for a, b in zip(dst_o, dst_t):
        assert np.array_equal(a, b)


def test_work_tables_for_mid_size_strided_messages(interp):
    # chunk borders in the middle of rows, several transpose tiles per row, ragged edges
    cases = [
        Case("rows_mid", (((300, 2, 112), (112, 300 * 112, 1), 2),), 3, 4096),
        Case("transpose_mid", (((200, 150), (1, 200), 2),), 2, 4096),
        Case("transpose_batch_mid", (((3, 70, 90), (70 * 100, 1, 70), 4),), 4, 1024),
        Case("transpose_u8", (((130, 67), (1, 130), 1),), 2, 512),
    ]
    for case in cases:
        m = oracle_msg(case)
        raws = make_storages(case, 5)
        want = ho.pack(m, raws, case.B, case.k, fill=0x99)
        got = np.full(want.size, 0x99, np.uint8)
        rc, _, kinds = run_interp(interp, case, raws, got, 0, 2048)
        assert rc == 0 and np.array_equal(got, want), case.name
        # 150- and 90-element rows against 4 KiB and 1 KiB chunks: fewer packed rows per chunk than a tile is high, tiles span chunks
        assert kinds[0] == {"rows_mid": 2, "transpose_mid": 7, "transpose_batch_mid": 7, "transpose_u8": 3}[case.name]


def test_multiply_shift_division_is_exact(interp):
    rng = np.random.default_rng(3)
    edge = np.array([0, 1, 2, 3, (1 << 31) - 1, (1 << 31) - 2, 1 << 30, (1 << 30) - 1], np.uint32)
    for d in [1, 2, 3, 5, 7, 16, 100, 7168, 3584, 4096, 4097, 65535, 65536, 65537, (1 << 30) - 1, 1 << 30,
              (1 << 31) - 1] + [int(x) for x in rng.integers(1, 1 << 31, 40)]:
        mult = (np.arange(0, 2000, dtype=np.uint64) * d)
        near = np.concatenate([mult, mult + d - 1, mult + 1])
        near = near[near < (1 << 31)].astype(np.uint32)
        ns = np.ascontiguousarray(np.concatenate([edge, near, rng.integers(0, 1 << 31, 5000).astype(np.uint32)]))
        assert interp.fastdiv_check(C.c_uint32(d), C.c_void_p(ns.ctypes.data), C.c_int(ns.size)) == 0, d


# ---- randomised views: planner tables vs oracle ------------------------------------

@pytest.mark.parametrize("seed", list(range(12)) + [100, 101, 102, 103])
def test_random_views_tables_reproduce_oracle(interp, seed):
    rng = np.random.default_rng(1000 + seed)
    max_dims = 4 if seed < 100 else 8                   # the later seeds draw views of up to eight dims
    for _ in range(25):
        tensors = tuple(random_view(rng, max_dims) for _ in range(int(rng.integers(1, 5))))
        case = Case("rand", tensors, int(rng.integers(1, 6)), int(rng.choice([256, 512, 1024, 4096, 16384])))
        if sum(storage_bytes(*t) for t in tensors) > 4_000_000 or sum(int(np.prod(t[0])) * t[2] for t in tensors) > 8_000_000:
            continue
        m = oracle_msg(case)
        raws = make_storages(case, seed)
        want = ho.pack(m, raws, case.B, case.k, fill=0x99)
        tile = int(rng.choice([256, 1024, 16384]))
        got = np.full(want.size, 0x99, np.uint8)
        rc, written, _ = run_interp(interp, case, raws, got, 2, tile)
        assert rc == 0 and np.array_equal(got, want), (tensors, case.k, case.B, tile)
        p = plan_of(case)
        assert p.packed_bytes == want.size
        if all(p.tensor_unpack_safe(t) for t in range(len(tensors))):
            dst_o = [np.full(r.size, 0x42, np.uint8) for r in raws]
            dst_t = [np.full(r.size, 0x42, np.uint8) for r in raws]
            ho.unpack(m, want, case.B, case.k, dst_o)
            rc, _, _ = run_interp(interp, case, dst_t, want.copy(), 1, tile)
            assert rc == 0
            for a, b in zip(dst_o, dst_t):
                assert np.array_equal(a, b), (tensors, case.k, case.B, tile)


def test_unpack_safety_flag_never_accepts_an_aliasing_view():
    # brute force on small random views: whenever the planner calls a view safe, all its element
    # addresses are distinct (the converse need not hold: the test is only sufficient)
    rng = np.random.default_rng(5)
    accepted = 0
    for i in range(600):
        shape, strides, e = random_view(rng, 4 if i < 400 else 8)
        if 0 in shape or int(np.prod(shape)) > 20000:
            continue
        p = hxt.hxt_plan(shape, strides, e, 2, 256)
        if p.tensor_unpack_safe(0):
            accepted += 1
            idx = np.zeros((), np.int64)
            for s_, st in zip(shape, strides):
                idx = idx[..., None] + np.arange(s_, dtype=np.int64) * st
            assert np.unique(idx).size == idx.size, (shape, strides)
    assert accepted > 50


# ---- host-side hop of the CPU-forwarding path (pure host code) ------------------------

@pytest.mark.parametrize("name", ["ragged_last_chunk_2p5", "fewer_chunks_than_lanes", "three_tensors_with_gaps",
                                  "mixed_dtypes_multi", "empty_tensor"])
@pytest.mark.parametrize("threads", [0, 1, 3])
def test_host_forward_copies_the_used_bytes_of_the_lanes(name, threads):
    case = [c for c in SMALL_CASES if c.name == name][0]
    m, p = oracle_msg(case), plan_of(case)
    raws = make_storages(case, 91)
    packed = ho.pack(m, raws, case.B, case.k, fill=0xB7)
    n = max(packed.size, 1)
    for lanes in ([-1], list(range(case.k))):
        got = np.full(n, 0x11, np.uint8)
        want = np.full(n, 0x11, np.uint8)
        for l in lanes:
            hxt.hxt_host_forward(p, l, packed if packed.size else want, got, threads)
        for l in range(case.k):
            if packed.size:
                ho.stage_lane(m, case.B, case.k, l, packed, want)
        assert np.array_equal(got, want)          # used bytes moved, everything else (unspecified tail) untouched
    L = hxt.lib()
    assert L.hxt_host_forward(p.handle, case.k, 256, 256, 1) == hxt.HXT_EINVAL
    if packed.size:
        assert L.hxt_host_forward(p.handle, 0, None, 256, 1) == hxt.HXT_EINVAL
