"""GPU parity of hxt_unpack_accumulate against the oracle: bit-exact, including NaN, infinities,
subnormals and rounding ties (both sides add in binary32 and round bf16 results to nearest even)."""
import zlib

import numpy as np
import pytest
import torch

from oracle import hxt_oracle as ho
from paper_2602_18007_amd import hxt
from tests.cases import Case, contig

pytestmark = pytest.mark.gpu
FLOAT_OF = {2: torch.bfloat16, 4: torch.float32}
DEV = "cuda:0"


def draw(rng, nbytes, esize, mode):
    """Element bit patterns: 'bits' = anything (NaN, inf, subnormals included), 'near' = values of
    similar magnitude so that sums need rounding, 'grad' = N(0, 0.02)."""
    n = nbytes // esize
    if mode == "bits":
        return rng.integers(0, 256, nbytes, dtype=np.uint8)
    x = (rng.standard_normal(n) * (0.02 if mode == "grad" else 1.0)).astype(np.float32)
    if esize == 4:
        return x.view(np.uint8).copy()
    u = x.view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16).view(np.uint8).copy()


CASES = [
    Case("bf16_vector_ragged", (contig((70001,), 2),), 3, 8192),
    Case("f32_vector_ragged", (contig((33335,), 4),), 2, 4096),
    Case("bf16_matrix_one_chunk", (contig((37, 24), 2),), 4, 65536),
    Case("mixed_bucket", (contig((4096,), 2), contig((1000, 37), 2), contig((511,), 4), contig((0,), 2), contig((300, 300), 4),
                          contig((5,), 2)), 4, 16384),
]


@pytest.mark.parametrize("mode", ["bits", "near", "grad"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: c.name)
def test_accumulate_matches_oracle(case, mode):
    print("accumulate", case.name, mode, flush=True)
    rng = np.random.default_rng(zlib.crc32((case.name + mode).encode()))
    m = ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])
    kinds = [ho.KIND_BF16 if e == 2 else ho.KIND_F32 for (_, _, e) in case.tensors]
    sizes = [int(np.prod(s)) * e for (s, _, e) in case.tensors]
    incoming = [draw(rng, n, e, mode) for n, (_, _, e) in zip(sizes, case.tensors)]
    local = [draw(rng, n, e, mode) for n, (_, _, e) in zip(sizes, case.tensors)]
    if mode == "near" and sizes[0] >= 8:                  # plant exact ties: 1.0 + 2^-8 and 1.0078125 + 2^-8 in bf16
        if case.tensors[0][2] == 2:
            local[0][:4] = np.array([0x3F80, 0x3F81], np.uint16).view(np.uint8)
            incoming[0][:4] = np.array([0x3B80, 0x3B80], np.uint16).view(np.uint8)
    packed_o = ho.pack(m, incoming, case.B, case.k, fill=0x5A)
    want_sums = ho.checksum(m, packed_o, case.B, case.k)
    want = [x.copy() for x in local]
    ho.unpack_accumulate(m, kinds, packed_o, case.B, case.k, want)

    p = hxt.hxt_plan_multi([(s, st, FLOAT_OF[e]) for (s, st, e) in case.tensors], case.k, case.B)
    packed = torch.from_numpy(packed_o).to(DEV)
    dst = [torch.from_numpy(x.copy()).to(DEV) for x in local]
    sums = torch.full((p.num_chunks,), -1, dtype=torch.int64, device=DEV)
    hxt.hxt_unpack_accumulate(p, packed, dst, sums)
    torch.cuda.synchronize()
    for t, (a, b) in enumerate(zip(want, dst)):
        got = b.cpu().numpy()
        if not np.array_equal(got, a):
            bad = np.flatnonzero(got != a)[0] // case.tensors[t][2]
            raise AssertionError("tensor %d element %d differs" % (t, bad))
    assert np.array_equal(sums.cpu().numpy().view(np.uint64), want_sums)
    # twice in a row without checksums: accumulates again
    ho.unpack_accumulate(m, kinds, packed_o, case.B, case.k, want)
    hxt.hxt_unpack_accumulate(p, packed, dst, None)
    torch.cuda.synchronize()
    for a, b in zip(want, dst):
        assert np.array_equal(b.cpu().numpy(), a)


def test_accumulate_refuses_what_it_does_not_support():
    strided = hxt.hxt_plan((8, 64), (128, 1), torch.bfloat16, 2, 256)
    half = hxt.hxt_plan((64,), None, torch.float16, 2, 256)
    bytes_ = hxt.hxt_plan((64,), None, 1, 2, 256)
    buf = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_unpack_accumulate(strided, buf, [buf], None)
    assert e.value.status == hxt.HXT_EUNSUPPORTED
    # the library refuses element kinds it cannot add ...
    ptrs = (hxt.C.c_void_p * 1)(buf.data_ptr())
    for p in (half, bytes_):
        assert hxt.lib().hxt_unpack_accumulate(p.handle, buf.data_ptr(), ptrs, None, None) == hxt.HXT_EUNSUPPORTED
    # ... and the binding refuses plans whose dtype only names raw bits: an integer dtype or a bare element size
    # would otherwise be added as if it were bf16 / f32
    for dt in (2, 4, torch.int16, torch.int32, torch.float16):
        raw_bits = hxt.hxt_plan((64,), None, dt, 2, 256)
        with pytest.raises(ValueError):
            hxt.hxt_unpack_accumulate(raw_bits, buf, [buf], None)
    ok = hxt.hxt_plan((64,), None, torch.bfloat16, 2, 256)
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_unpack_accumulate(ok, buf, [buf[1:]], None)              # not even element aligned
    assert e.value.status == hxt.HXT_EALIGN
    torch.cuda.synchronize()


OFFSET_CASES = [(c, o) for c in CASES for o in (2, 4, 8, 12, 6) if o % max(e for (_, _, e) in c.tensors) == 0]


@pytest.mark.parametrize("case,offset", OFFSET_CASES, ids=lambda v: v.name if isinstance(v, Case) else str(v))
def test_accumulate_into_element_aligned_destinations(case, offset):
    """Destinations that start 2 to 12 bytes off a 16-byte boundary (slices of a larger gradient buffer): same
    arithmetic, narrower accesses on the destination side."""
    rng = np.random.default_rng(zlib.crc32((case.name + str(offset)).encode()))
    m = ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])
    kinds = [ho.KIND_BF16 if e == 2 else ho.KIND_F32 for (_, _, e) in case.tensors]
    sizes = [int(np.prod(s)) * e for (s, _, e) in case.tensors]
    incoming = [draw(rng, n, e, "near") for n, (_, _, e) in zip(sizes, case.tensors)]
    local = [draw(rng, n, e, "near") for n, (_, _, e) in zip(sizes, case.tensors)]
    packed_o = ho.pack(m, incoming, case.B, case.k, fill=0)
    want = [x.copy() for x in local]
    ho.unpack_accumulate(m, kinds, packed_o, case.B, case.k, want)
    p = hxt.hxt_plan_multi([(s, st, FLOAT_OF[e]) for (s, st, e) in case.tensors], case.k, case.B)
    dst = []
    for x in local:
        buf = torch.full((x.size + offset + 32,), 0x3C, dtype=torch.uint8, device=DEV)
        buf[offset:offset + x.size].copy_(torch.from_numpy(x))
        dst.append(buf)
    views = [b[offset:offset + x.size] for b, x in zip(dst, local)]
    sums = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    hxt.hxt_unpack_accumulate(p, torch.from_numpy(packed_o).to(DEV), views, sums)
    torch.cuda.synchronize()
    for a, b, x in zip(want, dst, local):
        got = b.cpu().numpy()
        assert np.array_equal(got[offset:offset + x.size], a)
        assert (got[:offset] == 0x3C).all() and (got[offset + x.size:] == 0x3C).all(), "bytes outside the tensor were touched"
    assert np.array_equal(sums.cpu().numpy().view(np.uint64), ho.checksum(m, packed_o, case.B, case.k))


@pytest.mark.parametrize("hint", [-1, 1], ids=["hint_by_size", "all_cold_non_temporal"])
def test_batched_accumulate_equals_the_oracle_message_by_message(hint):
    """hxt_unpack_accumulate_batch over a mixed set: single-tensor bf16 and f32 messages (these share launches),
    one of them without checksums (it cannot share a launch with its neighbours), a multi-tensor bucket, an empty
    message, a destination that is only element aligned, and the LLaMA-shaped pair of 32 MiB messages."""
    big = Case("llama_shaped", (contig((4096, 1, 4096), 2),), 4, 1 << 20)
    cases = [CASES[0], CASES[1], CASES[0], CASES[3], Case("empty", (contig((0,), 2),), 2, 256), CASES[2], CASES[1], big, big]
    want_sums = [True, True, False, True, True, True, True, True, True]
    offsets = [0, 0, 0, 0, 0, 0, 4, 0, 0]
    rng = np.random.default_rng(77)
    plans, packed, dst, views, sums, wants, wsums, locals_ = [], [], [], [], [], [], [], []
    for c, ws, off in zip(cases, want_sums, offsets):
        m = ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in c.tensors])
        kinds = [ho.KIND_BF16 if e == 2 else ho.KIND_F32 for (_, _, e) in c.tensors]
        sizes = [int(np.prod(s)) * e for (s, _, e) in c.tensors]
        mode = "grad" if c is big else "near"
        incoming = [draw(rng, n, e, mode) for n, (_, _, e) in zip(sizes, c.tensors)]
        local = [draw(rng, n, e, mode) for n, (_, _, e) in zip(sizes, c.tensors)]
        packed_o = ho.pack(m, incoming, c.B, c.k, fill=0x5A, nthreads=8)
        want = [x.copy() for x in local]
        ho.unpack_accumulate(m, kinds, packed_o, c.B, c.k, want, nthreads=8)
        p = hxt.hxt_plan_multi([(s, st, FLOAT_OF[e]) for (s, st, e) in c.tensors], c.k, c.B)
        hxt.hxt_plan_set_option(p, hxt.HXT_OPT_PACKED_HINT, hint)
        plans.append(p)
        packed.append(torch.from_numpy(packed_o).to(DEV) if packed_o.size else torch.zeros(256, dtype=torch.uint8, device=DEV))
        bufs = []
        for x in local:
            buf = torch.full((x.size + off + 32,), 0x3C, dtype=torch.uint8, device=DEV)
            buf[off:off + x.size].copy_(torch.from_numpy(x))
            bufs.append(buf)
        dst.append(bufs)
        views.append([b[off:off + x.size] for b, x in zip(bufs, local)])
        sums.append(torch.full((max(p.num_chunks, 1),), -1, dtype=torch.int64, device=DEV) if ws else None)
        wants.append(want)
        wsums.append(ho.checksum(m, packed_o, c.B, c.k))
        locals_.append(local)
    print("batched accumulate of", len(cases), flush=True)
    hxt.hxt_unpack_accumulate_batch(hxt.Batch(plans, views, packed, sums))
    torch.cuda.synchronize()
    for i, c in enumerate(cases):
        off = offsets[i]
        for a, b, x in zip(wants[i], dst[i], locals_[i]):
            got = b.cpu().numpy()
            assert np.array_equal(got[off:off + x.size], a), (i, c.name)
            assert (got[:off] == 0x3C).all() and (got[off + x.size:] == 0x3C).all(), (i, c.name)
        if sums[i] is not None:
            assert np.array_equal(sums[i].cpu().numpy().view(np.uint64)[:wsums[i].size], wsums[i]), (i, c.name)
    # the same plan twice with checksums is refused, and so is a plan that cannot accumulate; nothing is enqueued
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_unpack_accumulate_batch(hxt.Batch([plans[0], plans[0]], [views[0], views[0]], [packed[0], packed[0]],
                                                  [sums[0], sums[0]]))
    assert e.value.status == hxt.HXT_EINVAL
    strided = hxt.hxt_plan((8, 64), (128, 1), torch.bfloat16, 2, 256)
    buf = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    before = [b.clone() for b in dst[0]]
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_unpack_accumulate_batch(hxt.Batch([plans[0], strided], [views[0], [buf]], [packed[0], buf], None))
    assert e.value.status == hxt.HXT_EUNSUPPORTED
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(before, dst[0]))


def test_accumulate_gradient_bucket_shape():
    # one LLaMA-8B layer's worth of bf16 gradients (218 M elements) is too slow for the per-byte oracle
    # to add in a test; a 1/64 scale model of the nine tensors keeps the structure (two tiny norms,
    # tensors straddling 25 MiB/64 buckets, 8 lanes)
    shapes = [(64,), (512, 512), (128, 512), (128, 512), (512, 512), (64,), (1792, 512), (1792, 512), (512, 1792)]
    case = Case("bucket", tuple(contig(s, 2) for s in shapes), 8, 25 * 1024 * 1024 // 64)
    rng = np.random.default_rng(3)
    m = ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])
    sizes = [int(np.prod(s)) * 2 for s in shapes]
    incoming = [draw(rng, n, 2, "grad") for n in sizes]
    local = [draw(rng, n, 2, "grad") for n in sizes]
    packed_o = ho.pack(m, incoming, case.B, case.k, nthreads=8)
    want = [x.copy() for x in local]
    ho.unpack_accumulate(m, [ho.KIND_BF16] * 9, packed_o, case.B, case.k, want, nthreads=8)
    p = hxt.hxt_plan_multi([(s, st, FLOAT_OF[e]) for (s, st, e) in case.tensors], case.k, case.B)
    src = [torch.from_numpy(x).to(DEV) for x in incoming]
    packed = torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV)
    s1 = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    s2 = torch.zeros_like(s1)
    dst = [torch.from_numpy(x.copy()).to(DEV) for x in local]
    hxt.hxt_pack(p, src, packed, s1)
    hxt.hxt_unpack_accumulate(p, packed, dst, s2)
    torch.cuda.synchronize()
    assert torch.equal(s1, s2)
    for a, b in zip(want, dst):
        assert np.array_equal(b.cpu().numpy(), a)


def test_accumulate_full_size_gradient_buckets():
    """The real gradient message (36 tensors, 1.7 GB, 25 MiB chunks of 1600 tiles, 8 lanes): hxt_pack then
    hxt_unpack_accumulate, every element against the oracle.  At this size the packed side is accessed with
    non-temporal hints and every chunk's checksum commit fans out over 16 first-level slots."""
    from paper_2602_18007_amd import workloads as wl
    w = wl.grad_buckets()
    T = len(w.tensors)
    print("full-size accumulate: drawing 2 x", w.message_bytes, "bytes", flush=True)
    incoming = wl.make_storages(w)
    rng = np.random.default_rng(18007 + 77)
    local = [wl.draw_u16(t.nbytes // 2, "normal", 0.02, rng).view(np.uint8) for t in w.tensors]
    local[1][:4] = np.array([0x3F80, 0x3F81], np.uint16).view(np.uint8)      # two exact ties, as in the small cases
    incoming[1][:4] = np.array([0x3B80, 0x3B80], np.uint16).view(np.uint8)
    m = ho.Message([ho.TensorSpec(t.shape, t.strides, t.esize) for t in w.tensors])
    p = hxt.hxt_plan_multi([(t.shape, t.strides, torch.bfloat16) for t in w.tensors], w.n_lanes, w.chunk_bytes)
    src = [torch.from_numpy(x).to(DEV) for x in incoming]
    dst = [torch.from_numpy(x).to(DEV) for x in local]
    packed = torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV)
    s1 = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    s2 = torch.full_like(s1, -1)
    hxt.hxt_pack(p, src, packed, s1)
    hxt.hxt_unpack_accumulate(p, packed, dst, s2)
    torch.cuda.synchronize()
    print("full-size accumulate: oracle", flush=True)
    nt = ho.max_threads()
    packed_o = ho.pack(m, incoming, w.chunk_bytes, w.n_lanes, fill=0, nthreads=nt)
    want_sums = ho.checksum(m, packed_o, w.chunk_bytes, w.n_lanes, nthreads=nt)
    ho.unpack_accumulate(m, [ho.KIND_BF16] * T, packed_o, w.chunk_bytes, w.n_lanes, local, nthreads=nt)   # in place
    assert np.array_equal(s1.cpu().numpy().view(np.uint64), want_sums)
    assert np.array_equal(s2.cpu().numpy().view(np.uint64), want_sums)
    for t, (a, b) in enumerate(zip(local, dst)):
        assert np.array_equal(b.cpu().numpy(), a), "tensor %d differs" % t


def test_accumulate_can_be_captured_in_a_hip_graph_and_replayed():
    """pack + receive-and-accumulate recorded once and replayed: every replay adds the arriving gradients again,
    bit for bit as the oracle does when applied the same number of times."""
    case = CASES[3]                                              # the mixed bf16 / f32 bucket
    rng = np.random.default_rng(4242)
    m = ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])
    kinds = [ho.KIND_BF16 if e == 2 else ho.KIND_F32 for (_, _, e) in case.tensors]
    sizes = [int(np.prod(s)) * e for (s, _, e) in case.tensors]
    incoming = [draw(rng, n, e, "grad") for n, (_, _, e) in zip(sizes, case.tensors)]
    local = [draw(rng, n, e, "grad") for n, (_, _, e) in zip(sizes, case.tensors)]
    p = hxt.hxt_plan_multi([(s, st, FLOAT_OF[e]) for (s, st, e) in case.tensors], case.k, case.B)
    src = [torch.from_numpy(x.copy()).to(DEV) if x.size else torch.zeros(16, dtype=torch.uint8, device=DEV) for x in incoming]
    dst = [torch.from_numpy(x.copy()).to(DEV) if x.size else torch.zeros(16, dtype=torch.uint8, device=DEV) for x in local]
    packed = torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV)
    s_send = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    s_recv = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())

    def calls():
        hxt.hxt_pack(p, src, packed, s_send, side)
        hxt.hxt_unpack_accumulate(p, packed, dst, s_recv, side)

    with torch.cuda.stream(side):
        calls()                                                  # eager once: the accumulator sets now belong to this stream
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        calls()
    packed_o = ho.pack(m, incoming, case.B, case.k, fill=0)
    want = [x.copy() for x in local]
    ho.unpack_accumulate(m, kinds, packed_o, case.B, case.k, want)           # the eager call
    for rep in range(3):
        g.replay()
        torch.cuda.synchronize()
        ho.unpack_accumulate(m, kinds, packed_o, case.B, case.k, want)
        for a, b in zip(want, dst):
            assert np.array_equal(b.cpu().numpy()[:a.size], a), "replay %d" % rep
        assert torch.equal(s_send, s_recv)
        assert np.array_equal(s_recv.cpu().numpy().view(np.uint64), ho.checksum(m, packed_o, case.B, case.k))
