"""GPU parity of the chunk tags: hxt_seal / hxt_verify through the C ABI against the oracle's
seal / verify, byte for byte and mask for mask; every fault is planted on the host."""
import numpy as np
import pytest
import torch

from oracle import hxt_oracle as ho
from paper_2602_18007_amd import hxt
from paper_2602_18007_amd import workloads as wl
from tests.cases import SMALL_CASES, Case, contig, make_storages, random_view, storage_bytes

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = SMALL_CASES + [
    Case("contig_1MB_ragged", (contig((1_000_001,), 1),), 3, 65536),
    Case("chunks_of_256_tiles", (contig((9 * 1024 * 1024 // 2 + 40,), 2),), 2, 4 << 20),
    Case("multi_mid", (contig((70001,), 1), ((64, 2, 128), (128, 64 * 128, 1), 2), ((96, 80), (1, 96), 4),
                       contig((3, 1000), 8), ((33, 10), (20, 2), 2)), 4, 8192),
]


def setup(case, seed=3):
    m = ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])
    p = hxt.hxt_plan_multi([(s, st, e) for (s, st, e) in case.tensors], case.k, case.B)
    raws = make_storages(case, seed)
    packed = ho.pack(m, raws, case.B, case.k, fill=0x5C)
    return m, p, packed


def dev(a):
    t = torch.empty(max(a.size, 16), dtype=torch.uint8, device=DEV)
    t[:a.size].copy_(torch.from_numpy(a.reshape(-1)))
    return t


def gpu_verify(p, packed_np, tags_np, seq, mb):
    C = p.num_chunks
    status = torch.full((C + 1,), 0x7FFFFFFF, dtype=torch.int32, device=DEV)
    hxt.hxt_verify(p, dev(packed_np), dev(tags_np), seq, mb, status)
    return status.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("case", CASES, ids=lambda c: c.name)
def test_seal_and_verify_match_the_oracle(case):
    m, p, packed = setup(case)
    C = p.num_chunks
    seq, mb = 0xA1B2C3D4E5F60718, 0xCAFE0001
    want = ho.seal(m, packed, case.B, case.k, seq, mb)
    tags = torch.full((max(C, 1) * 64,), 0xEE, dtype=torch.uint8, device=DEV)
    d_packed = dev(packed)
    hxt.hxt_seal(p, d_packed, seq, mb, tags)
    got = tags.cpu().numpy()[:C * 64].reshape(C, 64)
    assert np.array_equal(got, want)
    for args in ((seq, mb), (seq + 1, mb), (seq, mb ^ 1)):
        assert np.array_equal(gpu_verify(p, packed, got, *args), ho.verify(m, packed, want, case.B, case.k, *args))
    assert not gpu_verify(p, packed, got, seq, mb).any()


def test_planted_faults_get_the_oracles_masks():
    case = next(c for c in CASES if c.name == "multi_mid")
    m, p, packed = setup(case, 8)
    C = p.num_chunks
    seq, mb = 77, 5
    tags = ho.seal(m, packed, case.B, case.k, seq, mb)
    faults = []
    bad = packed.copy()
    bad[p.chunk_info(3)["packed_off"] + 1001] ^= 0x04
    faults.append(("flipped bit", bad, tags))
    sw = packed.copy()
    w = sw[p.chunk_info(6)["packed_off"]:][:case.B].view("<u4")
    i, j = next((i, j) for i in range(40) for j in range(1500, 1540) if w[i] != w[j])
    w[i], w[j] = int(w[j]), int(w[i])
    faults.append(("swapped words", sw, tags))
    t = tags.copy()
    t[[2, 9]] = tags[[9, 2]]
    faults.append(("two tags exchanged", packed, t))
    t = tags.copy()
    t[4, 3] ^= 0x80
    t[5, 60] = 9
    t[7, 32:40] = 0
    faults.append(("magic, reserved and length fields", packed, t))
    lane = packed.copy()                                   # a whole lane region overwritten by another lane's bytes
    a, b = p.lane_info(0), p.lane_info(1)
    n = min(a["bytes"], b["bytes"])
    lane[a["packed_off"]:a["packed_off"] + n] = packed[b["packed_off"]:b["packed_off"] + n]
    faults.append(("lane 1's bytes in lane 0's region", lane, tags))
    for name, pk, tg in faults:
        want = ho.verify(m, pk, tg, case.B, case.k, seq, mb)
        assert want[C] > 0, name
        assert np.array_equal(gpu_verify(p, pk, tg, seq, mb), want), name
    for rep in range(2):                                   # the accumulators are clean again after rejected chunks
        assert not gpu_verify(p, packed, tags, seq, mb).any()


def test_every_field_of_the_tag_is_checked_on_the_device():
    """One field of one received tag changed by one (on the host): the device reports what the oracle reports,
    from the stand-alone pass and from the pass fused into unpack."""
    TAG = np.dtype([("magic", "<u4"), ("chunk", "<u4"), ("lane", "<u4"), ("slot", "<u4"), ("seq", "<u8"),
                    ("micro_batch", "<u4"), ("C", "<u4"), ("padded", "<u8"), ("sum", "<u8"), ("wsum", "<u8"), ("zero", "<u8")])
    case = next(c for c in CASES if c.name == "contig_1MB_ragged")
    m, p, packed = setup(case, 21)
    C = p.num_chunks
    tags = ho.seal(m, packed, case.B, case.k, 5, 6)
    raws_like = [np.zeros(t[0][0] * t[2] if len(t[0]) == 1 else 0, np.uint8) for t in case.tensors]
    for field in TAG.names:
        t = tags.copy()
        t.reshape(-1).view(TAG)[field][C - 1] += 1
        want = ho.verify(m, packed, t, case.B, case.k, 5, 6)
        assert want[C] == 1, field
        assert np.array_equal(gpu_verify(p, packed, t, 5, 6), want), field
        dst = [dev(r) for r in raws_like]
        status = torch.full((C + 1,), -1, dtype=torch.int32, device=DEV)
        hxt.hxt_unpack_verify(p, dev(packed), dev(t), 5, 6, dst, status)
        assert np.array_equal(status.cpu().numpy().view(np.uint32), want), field


def test_full_size_boundary_message_round_trip_with_tags():
    w = wl.llama8b_boundary()
    case = Case(w.name, tuple((t.shape, t.strides, t.esize) for t in w.tensors), w.n_lanes, w.chunk_bytes)
    m = ho.Message([ho.TensorSpec(t.shape, t.strides, t.esize) for t in w.tensors])
    p = hxt.hxt_plan_multi([(t.shape, t.strides, t.esize) for t in w.tensors], w.n_lanes, w.chunk_bytes)
    raws = wl.make_storages(w, 1)
    src = [torch.from_numpy(r).to(DEV) for r in raws]
    packed = torch.empty(p.packed_bytes, dtype=torch.uint8, device=DEV)
    hxt.hxt_pack(p, src, packed, None)
    tags = torch.zeros(p.num_chunks * 64, dtype=torch.uint8, device=DEV)
    hxt.hxt_seal(p, packed, 1234567890123, 31, tags)
    want_packed = ho.pack(m, raws, w.chunk_bytes, w.n_lanes, fill=0, nthreads=8)
    assert np.array_equal(tags.cpu().numpy().reshape(-1, 64), ho.seal(m, want_packed, w.chunk_bytes, w.n_lanes, 1234567890123, 31))
    # the tags travel lane by lane with the chunks (slot order = lane order)
    host = torch.zeros(p.packed_bytes, dtype=torch.uint8).pin_memory()
    recv = torch.zeros_like(packed)
    recv_tags = torch.zeros_like(tags)
    for l in range(w.n_lanes):
        hxt.hxt_stage_d2h(p, l, packed, host)
        hxt.hxt_stage_h2d(p, l, host, recv)
        li = p.lane_info(l)
        s0 = li["packed_off"] // w.chunk_bytes
        recv_tags[s0 * 64:(s0 + li["n_chunks"]) * 64].copy_(tags[s0 * 64:(s0 + li["n_chunks"]) * 64])
    status = torch.full((p.num_chunks + 1,), -1, dtype=torch.int32, device=DEV)
    hxt.hxt_verify(p, recv, recv_tags, 1234567890123, 31, status)
    assert not status.cpu().numpy().any()
    hxt.hxt_verify(p, recv, recv_tags, 1234567890122, 31, status)          # the previous message's number
    st = status.cpu().numpy()
    assert list(st[:-1]) == [hxt.HXT_TAG_BAD_SEQ] * p.num_chunks and st[-1] == p.num_chunks


@pytest.mark.parametrize("case", CASES, ids=lambda c: c.name)
def test_fused_pack_seal_and_unpack_verify_match_the_oracle(case):
    """hxt_pack_seal = pack + seal, hxt_unpack_verify = verify + unpack: same bytes, tags and masks as the oracle's
    composition, in one pass for single contiguous tensors and in two passes for everything else."""
    m = ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])
    p = hxt.hxt_plan_multi([(s, st, e) for (s, st, e) in case.tensors], case.k, case.B)
    raws = make_storages(case, 12)
    C = p.num_chunks
    seq, mb = 0x1122334455667788, 9
    want_packed = ho.pack(m, raws, case.B, case.k, fill=0xA5)
    want_tags = ho.seal(m, want_packed, case.B, case.k, seq, mb)
    src = [dev(r) for r in raws]
    packed = torch.full((max(want_packed.size, 16),), 0xA5, dtype=torch.uint8, device=DEV)
    tags = torch.full((max(C, 1) * 64,), 0xEE, dtype=torch.uint8, device=DEV)
    hxt.hxt_pack_seal(p, src, packed, seq, mb, tags)
    assert np.array_equal(packed.cpu().numpy()[:want_packed.size], want_packed)
    assert np.array_equal(tags.cpu().numpy()[:C * 64].reshape(C, 64), want_tags)
    if not all(p.tensor_unpack_safe(t) for t in range(len(case.tensors))):
        return
    # receive: intact, then with a stale sequence number, then with a damaged chunk (fault planted on the host)
    damaged = want_packed.copy()
    if C:
        damaged[p.chunk_info(C - 1)["packed_off"] + 5] ^= 0x40
    for pk, args in ((want_packed, (seq, mb)), (want_packed, (seq - 1, mb)), (damaged, (seq, mb))):
        dst_o = [np.full(r.size, 0x3C, np.uint8) for r in raws]
        ho.unpack(m, pk, case.B, case.k, dst_o)
        want_status = ho.verify(m, pk, want_tags, case.B, case.k, *args)
        dst = [dev(np.full(r.size, 0x3C, np.uint8)) for r in raws]
        status = torch.full((C + 1,), 0x7FFFFFFF, dtype=torch.int32, device=DEV)
        hxt.hxt_unpack_verify(p, dev(pk), dev(want_tags), *args, dst, status)
        assert np.array_equal(status.cpu().numpy().view(np.uint32), want_status)
        for a, b in zip(dst_o, dst):
            assert np.array_equal(b.cpu().numpy()[:a.size], a)
    if C:
        assert want_status[C] == 1 and want_status[C - 1] == ho.TAG_BAD_SUM | ho.TAG_BAD_WSUM


def test_fused_calls_on_the_full_size_boundary_message():
    w = wl.llama8b_boundary()
    m = ho.Message([ho.TensorSpec(t.shape, t.strides, t.esize) for t in w.tensors])
    p = hxt.hxt_plan_multi([(t.shape, t.strides, t.esize) for t in w.tensors], w.n_lanes, w.chunk_bytes)
    raws = wl.make_storages(w, 0)
    src = [torch.from_numpy(r).to(DEV) for r in raws]
    packed = torch.empty(p.packed_bytes, dtype=torch.uint8, device=DEV)
    tags = torch.zeros(p.num_chunks * 64, dtype=torch.uint8, device=DEV)
    dst = [torch.zeros_like(s_) for s_ in src]
    status = torch.full((p.num_chunks + 1,), -1, dtype=torch.int32, device=DEV)
    for rep in range(3):                                         # repeated calls leave the accumulators clean
        hxt.hxt_pack_seal(p, src, packed, 500 + rep, 3, tags)
        hxt.hxt_unpack_verify(p, packed, tags, 500 + rep, 3, dst, status)
        assert not status.cpu().numpy().any()
    want_packed = ho.pack(m, raws, w.chunk_bytes, w.n_lanes, fill=0, nthreads=8)
    assert np.array_equal(packed.cpu().numpy(), want_packed)
    assert np.array_equal(tags.cpu().numpy().reshape(-1, 64), ho.seal(m, want_packed, w.chunk_bytes, w.n_lanes, 502, 3))
    assert torch.equal(src[0], dst[0])


BATCH_MESSAGES = [
    Case("uniform_a", (contig((5 * 1024 * 1024 // 2 + 24,), 2),), 4, 1 << 20),
    Case("uniform_b_fanned_out", (contig((9 * 1024 * 1024 // 2 + 40,), 2),), 2, 4 << 20),
    Case("bucket_all_contig", (contig((4096,), 2), contig((1000, 37), 2), contig((511,), 4), contig((0,), 2),
                               contig((300, 300), 4), contig((5,), 1)), 4, 16384),
    Case("strided_two_pass", (((300, 2, 112), (112, 300 * 112, 1), 2),), 3, 4096),
    Case("empty", (contig((0,), 2),), 2, 256),
    Case("uniform_c_small", (contig((1000,), 1),), 8, 256),
]


@pytest.mark.parametrize("offset", [0, 4])
def test_batched_fused_tag_calls_match_the_oracle(offset):
    """hxt_pack_seal_batch / hxt_unpack_verify_batch over a mixed set of messages (single tensors that share
    launches, a bucket of contiguous tensors served by the table-driven fused kernel, a strided message that
    takes two passes, an empty one): tags, packed bytes, destinations and masks against the oracle, with one
    message's sequence number stale and one message damaged on the host.  offset 4: bases that are only
    element aligned (every message falls back to its own call)."""
    cases = BATCH_MESSAGES
    n = len(cases)
    ms = [ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in c.tensors]) for c in cases]
    plans = [hxt.hxt_plan_multi([(s, st, e) for (s, st, e) in c.tensors], c.k, c.B) for c in cases]
    raws = [make_storages(c, 40 + i) for i, c in enumerate(cases)]
    seqs = [(1 << 50) + 3 * i for i in range(n)]
    mbs = [100 + i for i in range(n)]
    want_packed = [ho.pack(m, r, c.B, c.k, fill=0xA5) for m, r, c in zip(ms, raws, cases)]
    want_tags = [ho.seal(m, pk, c.B, c.k, sq, mb) for m, pk, c, sq, mb in zip(ms, want_packed, cases, seqs, mbs)]

    def at(a):
        t = torch.empty(max(a.size, 1) + 64, dtype=torch.uint8, device=DEV)
        v = t[offset:offset + a.size] if a.size else t[:0]
        v.copy_(torch.from_numpy(a))
        return v

    src = [[at(r) for r in rs] for rs in raws]
    packed = [torch.full((max(pk.size, 16),), 0xA5, dtype=torch.uint8, device=DEV) for pk in want_packed]
    tags = [torch.full((max(p.num_chunks, 1) * 64,), 0xEE, dtype=torch.uint8, device=DEV) for p in plans]
    status = [torch.full((p.num_chunks + 1,), 0x7FFFFFFF, dtype=torch.int32, device=DEV) for p in plans]
    dst = [[at(np.full(r.size, 0x3C, np.uint8)) for r in rs] for rs in raws]
    hxt.hxt_pack_seal_batch(hxt.TagBatch(plans, src, packed, tags), seqs, mbs)
    for i, c in enumerate(cases):
        C = plans[i].num_chunks
        assert np.array_equal(packed[i].cpu().numpy()[:want_packed[i].size], want_packed[i]), c.name
        assert np.array_equal(tags[i].cpu().numpy()[:C * 64].reshape(C, 64), want_tags[i]), c.name
    # receive side: message 1 is expected under another sequence number, message 2 was damaged on the way
    seqs_r = list(seqs)
    seqs_r[1] += 1
    hit = plans[2].chunk_info(plans[2].num_chunks - 1)["packed_off"] + 9
    packed[2][hit] = int(want_packed[2][hit]) ^ 0x04
    want_packed[2][hit] ^= 0x04
    hxt.hxt_unpack_verify_batch(hxt.TagBatch(plans, dst, packed, tags, status), seqs_r, mbs)
    for i, c in enumerate(cases):
        want_status = ho.verify(ms[i], want_packed[i], want_tags[i], c.B, c.k, seqs_r[i], mbs[i])
        assert np.array_equal(status[i].cpu().numpy().view(np.uint32), want_status), c.name
        dst_o = [np.full(r.size, 0x3C, np.uint8) for r in raws[i]]
        ho.unpack(ms[i], want_packed[i], c.B, c.k, dst_o)
        for a, b in zip(dst_o, dst[i]):
            assert np.array_equal(b.cpu().numpy(), a), c.name
    assert int(status[1][-1]) == plans[1].num_chunks and int(status[2][-1]) == 1 and int(status[0][-1]) == 0
    # a plan may appear only once in a batch
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_pack_seal_batch(hxt.TagBatch([plans[0], plans[0]], [src[0], src[0]], [packed[0], packed[0]], [tags[0], tags[0]]),
                                [1, 2], [0, 0])
    assert e.value.status == hxt.HXT_EINVAL
    torch.cuda.synchronize()


@pytest.mark.parametrize("hint", [-1, 1], ids=["hint_by_size", "all_cold_non_temporal"])
def test_batched_fused_tag_calls_on_the_full_size_boundary_step(hint):
    """The benchmark's tagged step: both LLaMA-shaped messages sealed inside one batched pack launch and verified
    inside one batched unpack launch (hint 1: with the packed side non-temporal, its all-cold figure)."""
    w = wl.llama8b_boundary()
    m = ho.Message([ho.TensorSpec(t.shape, t.strides, t.esize) for t in w.tensors])
    plans = [hxt.hxt_plan_multi([(t.shape, t.strides, t.esize) for t in w.tensors], w.n_lanes, w.chunk_bytes) for _ in range(2)]
    for p in plans:
        hxt.hxt_plan_set_option(p, hxt.HXT_OPT_PACKED_HINT, hint)
    raws = [wl.make_storages(w, i) for i in range(2)]
    src = [[torch.from_numpy(r).to(DEV) for r in rs] for rs in raws]
    dst = [[torch.zeros_like(t) for t in ts] for ts in src]
    C = plans[0].num_chunks
    packed = [torch.empty(plans[0].packed_bytes, dtype=torch.uint8, device=DEV) for _ in range(2)]
    tags = [torch.zeros(C * 64, dtype=torch.uint8, device=DEV) for _ in range(2)]
    status = [torch.full((C + 1,), -1, dtype=torch.int32, device=DEV) for _ in range(2)]
    send = hxt.TagBatch(plans, src, packed, tags)
    recv = hxt.TagBatch(plans, dst, packed, tags, status)
    for rep in range(3):
        hxt.hxt_pack_seal_batch(send, [700 + rep, 800 + rep], [0, 1])
        hxt.hxt_unpack_verify_batch(recv, [700 + rep, 800 + rep], [0, 1])
        assert not status[0].cpu().numpy().any() and not status[1].cpu().numpy().any()
    for i in range(2):
        want_packed = ho.pack(m, raws[i], w.chunk_bytes, w.n_lanes, fill=0, nthreads=8)
        assert np.array_equal(packed[i].cpu().numpy(), want_packed)
        assert np.array_equal(tags[i].cpu().numpy().reshape(-1, 64),
                              ho.seal(m, want_packed, w.chunk_bytes, w.n_lanes, [702, 802][i], i))
        assert torch.equal(src[i][0], dst[i][0])


def full_size_tag_check(w, tensors, raws):
    """seal / verify and the fused calls at full size against the oracle: tags byte for byte, masks word for word,
    packed and destination bytes, and a bit flipped on the host that must be reported in exactly its chunk."""
    B, k = w.chunk_bytes, w.n_lanes
    m = ho.Message([ho.TensorSpec(t.shape, t.strides, t.esize) for t in tensors])
    p = hxt.hxt_plan_multi([(t.shape, t.strides, t.esize) for t in tensors], k, B)
    C = p.num_chunks
    seq, mb = 0x0102030405060708, 17
    print("full-size tags:", w.name, m.N, "bytes,", C, "chunks: oracle", flush=True)
    want_packed = ho.pack(m, raws, B, k, fill=0xA5, nthreads=ho.max_threads())
    want_tags = ho.seal(m, want_packed, B, k, seq, mb)
    src = [torch.from_numpy(r).to(DEV) for r in raws]
    packed = torch.full((p.packed_bytes,), 0xA5, dtype=torch.uint8, device=DEV)
    tags = torch.full((C * 64,), 0xEE, dtype=torch.uint8, device=DEV)
    hxt.hxt_pack_seal(p, src, packed, seq, mb, tags)
    assert np.array_equal(packed.cpu().numpy(), want_packed), "fused pack+seal: packed bytes"
    assert np.array_equal(tags.cpu().numpy().reshape(C, 64), want_tags), "fused pack+seal: tags"
    tags2 = torch.full_like(tags, 0x11)
    hxt.hxt_seal(p, packed, seq, mb, tags2)
    assert torch.equal(tags, tags2), "stand-alone seal"
    status = torch.full((C + 1,), 0x7FFFFFFF, dtype=torch.int32, device=DEV)
    hxt.hxt_verify(p, packed, tags, seq, mb, status)
    assert not status.cpu().numpy().any()
    dst = [torch.zeros_like(s_) for s_ in src]
    status.fill_(0x7FFFFFFF)
    hxt.hxt_unpack_verify(p, packed, tags, seq, mb, dst, status)
    assert not status.cpu().numpy().any()
    for t, (a, b) in enumerate(zip(src, dst)):
        assert torch.equal(a, b), "tensor %d after unpack+verify" % t
    # damage planted from the host: one bit of a chunk in the middle, one byte of the last chunk
    hit = sorted({C // 2, C - 1})
    for c in hit:
        off = p.chunk_info(c)["packed_off"] + 4 * 1000 + 2
        packed[off] = int(want_packed[off]) ^ 0x10
        want_packed[off] ^= 0x10
    want_status = ho.verify(m, want_packed, want_tags, B, k, seq, mb)
    assert int(want_status[C]) == len(hit)
    for fused in (False, True):
        status.fill_(0x7FFFFFFF)
        if fused:
            hxt.hxt_unpack_verify(p, packed, tags, seq, mb, dst, status)
        else:
            hxt.hxt_verify(p, packed, tags, seq, mb, status)
        assert np.array_equal(status.cpu().numpy().view(np.uint32), want_status), "masks, fused=%s" % fused
    torch.cuda.synchronize()


def test_tags_on_the_full_size_gradient_buckets():
    w = wl.grad_buckets()
    full_size_tag_check(w, w.tensors, wl.make_storages(w))


def test_tags_on_a_single_tensor_larger_than_the_cacheable_limit():
    # one contiguous bf16 tensor of 160 MiB + 4 KiB + 6 bytes (above 128 MiB the packed side is non-temporal),
    # 4 lanes, 4 MiB chunks of 256 tiles (fanned-out commits), ragged last chunk
    n = (160 << 20) + 4096 + 6
    t = wl.TensorDesc.contiguous((n // 2,))
    w = wl.Workload("single_160MiB", (t,), 4, 4 << 20, "bits16", seed=18007 + 91)
    full_size_tag_check(w, w.tensors, wl.make_storages(w))


def test_a_stale_ping_pong_buffer_is_caught_by_its_tags():
    """Six micro-batches through two buffer sets; the sender skips message 4 (a lost send), so the receiver finds
    message 2 still sitting in the buffer: every chunk is rejected for its sequence number and micro-batch id, the
    sums still agree (the bytes are intact, just the wrong message), and the other messages pass."""
    case = next(c for c in CASES if c.name == "contig_1MB_ragged")
    m = ho.Message([ho.TensorSpec(tuple(s_), tuple(st), e) for (s_, st, e) in case.tensors])
    p = hxt.hxt_plan_multi([(s_, st, e) for (s_, st, e) in case.tensors], case.k, case.B)
    C = p.num_chunks
    raws = [make_storages(case, 40 + i) for i in range(6)]
    src = [[dev(r) for r in rs] for rs in raws]
    dst = [[torch.zeros_like(t) for t in s_] for s_ in src]
    packed = [torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV) for _ in range(2)]
    tags = [torch.zeros(C * 64, dtype=torch.uint8, device=DEV) for _ in range(2)]
    status = torch.full((6, C + 1), -1, dtype=torch.int32, device=DEV)
    for i in range(6):
        b = i % 2
        if i != 4:
            hxt.hxt_pack_seal(p, src[i], packed[b], 100 + i, i, tags[b])
        hxt.hxt_unpack_verify(p, packed[b], tags[b], 100 + i, i, dst[i], status[i])
    st = status.cpu().numpy().view(np.uint32)
    for i in range(6):
        if i == 4:
            assert list(st[i, :C]) == [hxt.HXT_TAG_BAD_SEQ | hxt.HXT_TAG_BAD_MICRO_BATCH] * C and st[i, C] == C
            assert torch.equal(dst[4][0], src[2][0])                 # what was delivered is message 2 again
            want = ho.verify(m, ho.pack(m, raws[2], case.B, case.k), ho.seal(m, ho.pack(m, raws[2], case.B, case.k),
                                                                               case.B, case.k, 102, 2), case.B, case.k, 104, 4)
            assert np.array_equal(st[i], want)
        else:
            assert not st[i].any() and torch.equal(dst[i][0], src[i][0])


def test_tag_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """pack_seal, checksum2, verify and unpack_verify recorded once (after one eager call on the capture stream)
    and replayed on fresh inputs; every replay against the oracle, with eager work between the replays."""
    case = next(c for c in CASES if c.name == "chunks_of_256_tiles")
    m = ho.Message([ho.TensorSpec(tuple(s_), tuple(st), e) for (s_, st, e) in case.tensors])
    p = hxt.hxt_plan_multi([(s_, st, e) for (s_, st, e) in case.tensors], case.k, case.B)
    C = p.num_chunks
    nbytes = make_storages(case, 0)[0].size
    src = [torch.zeros(nbytes, dtype=torch.uint8, device=DEV)]
    dst = [torch.zeros(nbytes, dtype=torch.uint8, device=DEV)]
    packed = torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV)
    tags = torch.zeros(C * 64, dtype=torch.uint8, device=DEV)
    strong = torch.zeros(C, 2, dtype=torch.int64, device=DEV)
    st1 = torch.zeros(C + 1, dtype=torch.int32, device=DEV)
    st2 = torch.zeros(C + 1, dtype=torch.int32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())

    def calls():
        hxt.hxt_pack_seal(p, src, packed, 900, 4, tags, side)
        hxt.hxt_checksum2(p, packed, strong, side)
        hxt.hxt_verify(p, packed, tags, 900, 4, st1, side)
        hxt.hxt_unpack_verify(p, packed, tags, 901, 4, dst, st2, side)      # expects the next sequence number

    with torch.cuda.stream(side):
        calls()
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        calls()
    for rep in range(4):
        raw = make_storages(case, 600 + rep)[0]
        src[0].copy_(torch.from_numpy(raw))
        for t in (dst[0], packed, tags):
            t.zero_()
        st1.fill_(-1)
        st2.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want = ho.pack(m, [raw], case.B, case.k, fill=0)
        want_tags = ho.seal(m, want, case.B, case.k, 900, 4)
        assert np.array_equal(packed.cpu().numpy(), want), "replay %d" % rep
        assert np.array_equal(tags.cpu().numpy().reshape(C, 64), want_tags)
        assert np.array_equal(strong.cpu().numpy().view(np.uint64), ho.checksum2(m, want, case.B, case.k))
        assert not st1.cpu().numpy().any()
        assert np.array_equal(st2.cpu().numpy().view(np.uint32), ho.verify(m, want, want_tags, case.B, case.k, 901, 4))
        assert np.array_equal(dst[0].cpu().numpy(), raw)
        hxt.hxt_checksum2(p, packed, strong)                       # eager work of the same accumulator set in between
        torch.cuda.synchronize()


@pytest.mark.parametrize("block", range(3))
def test_fused_tag_calls_on_random_messages(block):
    """Random messages (single contiguous tensors of random length, and random strided views), random lanes and
    chunk sizes, element-aligned base offsets, and one planted fault per message (a flipped payload bit, a flipped
    tag bit or a stale sequence number): tags, masks and destinations against the oracle."""
    done = 0
    seed = 1000 * block
    while done < 40:
        seed += 1
        rng = np.random.default_rng(77000 + seed)
        if rng.random() < 0.5:
            tensors = (contig((int(rng.integers(1, 400000)),), int(rng.choice([1, 2, 4, 8]))),)
        else:
            tensors = tuple(random_view(rng) for _ in range(int(rng.integers(1, 4))))
        if not 0 < sum(storage_bytes(*t) for t in tensors) <= 4_000_000:
            continue
        case = Case("ft%d" % seed, tensors, int(rng.integers(1, 9)), int(rng.choice([256, 1024, 4096, 65536, 262144])))
        m = ho.Message([ho.TensorSpec(tuple(s_), tuple(st), e) for (s_, st, e) in case.tensors])
        p = hxt.hxt_plan_multi([(s_, st, e) for (s_, st, e) in case.tensors], case.k, case.B)
        C = p.num_chunks
        if C == 0 or not all(p.tensor_unpack_safe(t) for t in range(len(tensors))):
            continue
        raws = make_storages(case, seed)
        off = int(rng.choice([0, 0, 8, 16]))

        def shifted(a):
            t = torch.empty(max(a.size, 16) + off + 16, dtype=torch.uint8, device=DEV)
            v = t[off:off + a.size]
            v.copy_(torch.from_numpy(a.reshape(-1)))
            return v

        seq, mb = int(rng.integers(0, 2**62)), int(rng.integers(0, 2**31))
        want = ho.pack(m, raws, case.B, case.k, fill=0x77)
        want_tags = ho.seal(m, want, case.B, case.k, seq, mb)
        packed = torch.full((want.size,), 0x77, dtype=torch.uint8, device=DEV)
        tags = torch.zeros(C * 64, dtype=torch.uint8, device=DEV)
        hxt.hxt_pack_seal(p, [shifted(r) for r in raws], packed, seq, mb, tags)
        assert np.array_equal(packed.cpu().numpy(), want), case
        assert np.array_equal(tags.cpu().numpy().reshape(C, 64), want_tags), case
        pk, tg = want.copy(), want_tags.copy()
        kind = int(rng.integers(0, 4))
        info = p.chunk_info(int(rng.integers(0, C)))
        if kind == 1:
            pk[info["packed_off"] + int(rng.integers(0, info["padded"]))] ^= 1 << int(rng.integers(0, 8))
        if kind == 2:
            tg[int(rng.integers(0, C)), int(rng.integers(0, 64))] ^= 1 << int(rng.integers(0, 8))
        eseq = seq + (1 if kind == 3 else 0)
        want_status = ho.verify(m, pk, tg, case.B, case.k, eseq, mb)
        dst_o = [np.full(r.size, 0x3C, np.uint8) for r in raws]
        ho.unpack(m, pk, case.B, case.k, dst_o)
        dst = [shifted(np.full(r.size, 0x3C, np.uint8)) for r in raws]
        status = torch.full((C + 1,), -1, dtype=torch.int32, device=DEV)
        hxt.hxt_unpack_verify(p, dev(pk), dev(tg), eseq, mb, dst, status)
        assert np.array_equal(status.cpu().numpy().view(np.uint32), want_status), (case, kind)
        for a, b in zip(dst_o, dst):
            assert np.array_equal(b.cpu().numpy(), a), case
        assert np.array_equal(gpu_verify(p, pk, tg, eseq, mb), want_status), (case, kind)
        done += 1


def test_empty_message_and_argument_errors():
    p0 = hxt.hxt_plan((0, 16), None, 2, 2, 256)
    status = torch.full((4,), 5, dtype=torch.int32, device=DEV)
    buf = torch.zeros(1024, dtype=torch.uint8, device=DEV)
    hxt.hxt_seal(p0, buf, 1, 1, buf)
    hxt.hxt_verify(p0, buf, buf, 1, 1, status)
    assert status.cpu().tolist() == [0, 5, 5, 5]
    p = hxt.hxt_plan((1000,), None, 1, 2, 256)
    L = hxt.lib()
    packed = torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV)
    tags = torch.zeros(p.num_chunks * 64 + 64, dtype=torch.uint8, device=DEV)
    st = torch.zeros(p.num_chunks + 1, dtype=torch.int32, device=DEV)
    assert L.hxt_seal(p.handle, packed.data_ptr(), 1, 1, None, None) == hxt.HXT_EINVAL
    assert L.hxt_seal(p.handle, packed.data_ptr(), 1, 1, tags.data_ptr() + 8, None) == hxt.HXT_EALIGN
    assert L.hxt_verify(p.handle, packed.data_ptr(), None, 1, 1, st.data_ptr(), None) == hxt.HXT_EINVAL
    assert L.hxt_verify(p.handle, packed.data_ptr(), tags.data_ptr(), 1, 1, None, None) == hxt.HXT_EINVAL
    assert L.hxt_verify(p.handle, packed.data_ptr(), tags.data_ptr() + 4, 1, 1, st.data_ptr(), None) == hxt.HXT_EALIGN
    assert L.hxt_verify(p.handle, None, tags.data_ptr(), 1, 1, st.data_ptr(), None) == hxt.HXT_EINVAL
    ptrs = (hxt.C.c_void_p * 1)(packed.data_ptr())
    assert L.hxt_pack_seal(p.handle, ptrs, packed.data_ptr(), 1, 1, None, None) == hxt.HXT_EINVAL
    assert L.hxt_pack_seal(p.handle, None, packed.data_ptr(), 1, 1, tags.data_ptr(), None) == hxt.HXT_EINVAL
    assert L.hxt_pack_seal(p.handle, ptrs, packed.data_ptr(), 1, 1, tags.data_ptr() + 8, None) == hxt.HXT_EALIGN
    assert L.hxt_unpack_verify(p.handle, packed.data_ptr(), None, 1, 1, ptrs, st.data_ptr(), None) == hxt.HXT_EINVAL
    assert L.hxt_unpack_verify(p.handle, packed.data_ptr(), tags.data_ptr(), 1, 1, ptrs, None, None) == hxt.HXT_EINVAL
    hxt.hxt_pack_seal(p0, [buf], buf, 1, 1, buf)
    hxt.hxt_unpack_verify(p0, buf, buf, 1, 1, [buf], status)
    assert status.cpu().tolist()[0] == 0
    torch.cuda.synchronize()
