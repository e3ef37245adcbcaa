"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
byte for byte, on the same seeded inputs.  Integer/byte work: the bar is bit-exact."""
import os
import zlib

import numpy as np
import pytest
import torch

from oracle import hxt_oracle as ho
from paper_2602_18007_amd import hxt
from paper_2602_18007_amd import workloads as wl
from tests.cases import SMALL_CASES, Case, case_by_name, contig, make_storages, random_view, storage_bytes

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
NT = max(1, min(16, os.cpu_count() or 1))


def say(*a):
    print(*a, flush=True)


def oracle_msg(case):
    return ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])


def plan_of(case, tile_bytes=None, two_word=False):
    """Plan for a case; tile size and the checksum commit variant are read from the environment at creation."""
    env = {}
    if tile_bytes:
        env["HXT_TILE_BYTES"] = str(tile_bytes)
    if two_word:
        env["HXT_TWO_WORD_COMMIT"] = "1"
    old = {k: os.environ.get(k) for k in env}
    os.environ.update(env)
    try:
        return hxt.hxt_plan_multi([(s, st, e) for (s, st, e) in case.tensors], case.k, case.B)
    finally:
        for k, v in old.items():
            if v is None:
                del os.environ[k]
            else:
                os.environ[k] = v


def to_dev(a: np.ndarray, offset: int = 0) -> torch.Tensor:
    """Device copy of a byte array inside a 256-byte aligned allocation, shifted by ``offset`` bytes."""
    buf = torch.empty(a.size + offset + 16, dtype=torch.uint8, device=DEV)
    view = buf[offset:offset + a.size]
    view.copy_(torch.from_numpy(a))
    return view


def specified_mask(m, B, k, nbytes):
    spec = np.zeros(nbytes, bool)
    for c in range(ho.num_chunks(m, B)):
        i = ho.chunk_info(m, B, k, c)
        spec[i["packed_off"]:i["packed_off"] + i["padded"]] = True
    return spec


def round_trip_check(case, raws, tile_bytes=None, base_offset=0, nthreads=1, two_word=False, hint=None):
    """pack / checksum / unpack on the GPU vs the oracle; returns the device packed buffer."""
    m = oracle_msg(case)
    p = plan_of(case, tile_bytes, two_word)
    if hint is not None:
        hxt.hxt_plan_set_option(p, hxt.HXT_OPT_PACKED_HINT, hint)
    B, k = case.B, case.k
    want = ho.pack(m, raws, B, k, fill=0xA5, nthreads=nthreads)
    want_sums = ho.checksum(m, want, B, k, nthreads=nthreads)
    assert p.packed_bytes == want.size and p.num_chunks == want_sums.size

    src = [to_dev(r, base_offset) for r in raws]
    packed = torch.full((max(want.size, 1),), 0xA5, dtype=torch.uint8, device=DEV)
    sums = torch.full((max(want_sums.size, 1),), -1, dtype=torch.int64, device=DEV)   # garbage on purpose
    hxt.hxt_pack(p, src, packed, sums)
    got = packed.cpu().numpy()[:want.size]
    assert np.array_equal(got, want), "packed bytes differ (unspecified bytes must keep their old value)"
    got_sums = sums.cpu().numpy().view(np.uint64)[:want_sums.size]
    assert np.array_equal(got_sums, want_sums), "send-side checksums differ"

    # pack without checksums gives the same bytes; stand-alone checksum agrees with the fused one
    packed2 = torch.full_like(packed, 0xA5)
    hxt.hxt_pack(p, src, packed2, None)
    assert torch.equal(packed, packed2)
    sums2 = torch.full_like(sums, 7)
    hxt.hxt_checksum(p, packed, sums2)
    assert np.array_equal(sums2.cpu().numpy().view(np.uint64)[:want_sums.size], want_sums)
    # the position-weighted pair of sums
    strong = torch.full((max(want_sums.size, 1), 2), 9, dtype=torch.int64, device=DEV)
    hxt.hxt_checksum2(p, packed, strong)
    assert np.array_equal(strong.cpu().numpy().view(np.uint64)[:want_sums.size], ho.checksum2(m, want, B, k, nthreads=nthreads))

    if all(p.tensor_unpack_safe(t) for t in range(len(case.tensors))):
        dst_o = [np.full(r.size, 0x3C, np.uint8) for r in raws]
        ho.unpack(m, want, B, k, dst_o, nthreads=nthreads)
        dst = [to_dev(np.full(r.size, 0x3C, np.uint8), base_offset) for r in raws]
        rsums = torch.full_like(sums, 5)
        hxt.hxt_unpack(p, packed, dst, rsums)
        for t, (a, b) in enumerate(zip(dst_o, dst)):
            assert np.array_equal(b.cpu().numpy(), a), "tensor %d differs after unpack (or canary overwritten)" % t
        assert np.array_equal(rsums.cpu().numpy().view(np.uint64)[:want_sums.size], want_sums)
        dst2 = [to_dev(np.full(r.size, 0x3C, np.uint8), base_offset) for r in raws]
        hxt.hxt_unpack(p, packed, dst2, None)
        for a, b in zip(dst, dst2):
            assert torch.equal(a, b)
    else:
        with pytest.raises(hxt.HxtError) as e:
            hxt.hxt_unpack(p, packed, src, None)
        assert e.value.status == hxt.HXT_EOVERLAP
    torch.cuda.synchronize()
    return p, packed, want, want_sums


# ---------------------------------------------------------------------------
# small shapes: every kernel family, ragged tails, empty lanes, gaps
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("tile_bytes", [256, 16384])
@pytest.mark.parametrize("case", SMALL_CASES, ids=lambda c: c.name)
def test_small_cases(case, tile_bytes):
    say("case", case.name, "tile", tile_bytes)
    round_trip_check(case, make_storages(case, 1234), tile_bytes)


@pytest.mark.parametrize("name", ["u8_1000_not_256_multiple", "three_tensors_with_gaps", "rows_interleaved_3d",
                                  "true_transpose_64x48", "mixed_dtypes_multi", "esize8_strided"])
def test_base_pointers_that_are_only_element_aligned(name):
    case = case_by_name(name)
    off = max(e for (_, _, e) in case.tensors)            # element aligned, not 16-byte aligned
    say("case", name, "base offset", off)
    round_trip_check(case, make_storages(case, 99), None, base_offset=off)


MID_CASES = [
    Case("contig_1MB_ragged", (contig((1_000_001,), 1),), 3, 65536),
    Case("contig_bf16_5MiB_tail", (contig((5 * 1024 * 1024 // 2 + 24,), 2),), 4, 1 << 20),
    Case("contig_chunks_of_256_tiles", (contig((9 * 1024 * 1024 // 2 + 40,), 2),), 2, 4 << 20),   # fanned-out commit
    Case("rows_mid", (((300, 2, 112), (112, 300 * 112, 1), 2),), 3, 4096),
    Case("rows_200_byte_runs", (((4096, 100), (128, 1), 2),), 4, 65536),          # runs that are not 16-byte multiples
    Case("rows_31_byte_runs_3d", (((50, 3, 31), (100, 5000, 1), 1),), 2, 1024),
    Case("rows_f32_odd_pitch", (((700, 37), (41, 1), 4),), 3, 8192),
    Case("rows_big_rows", (((96, 2, 3584), (3584, 96 * 3584, 1), 2),), 8, 65536),
    Case("rows_padded_pitch", (((1000, 256), (320, 1), 4),), 5, 32768),
    Case("rows_4d", (((5, 7, 3, 64), (64, 5 * 3 * 64, 5 * 64, 1), 2),), 2, 2048),
    Case("transpose_mid", (((200, 150), (1, 200), 2),), 2, 4096),
    Case("transpose_512", (((512, 384), (1, 512), 2),), 4, 65536),
    Case("transpose_512_tall_chunks", (((512, 384), (1, 512), 2),), 4, 131072),   # tiles confined to chunks, vector path
    Case("transpose_u8_vec_tall_chunks", (((128, 96), (1, 128), 1),), 2, 16384),
    Case("transpose_mid_tall_chunks", (((200, 150), (1, 200), 2),), 2, 65536),
    Case("transpose_batch_f32", (((3, 70, 90), (70 * 100, 1, 70), 4),), 4, 1024),
    Case("transpose_u8", (((130, 67), (1, 130), 1),), 2, 512),
    Case("transpose_f64", (((100, 60), (1, 128), 8),), 3, 2048),
    Case("transpose_u8_vec", (((128, 96), (1, 128), 1),), 2, 4096),
    Case("transpose_bf16_vec_partial", (((72, 40), (1, 80), 2),), 2, 8192),
    Case("transpose_f32_vec_batched", (((5, 128, 68), (128, 1, 5 * 128), 4),), 4, 32768),
    Case("transpose_storage_stride_2", (((4096, 512), (2, 8192), 2),), 4, 262144),        # the storage-fast dim strided
    Case("transpose_storage_stride_4_u8_batched", (((3, 200, 130), (4 * 200 * 130, 4, 800), 1),), 2, 8192),
    Case("transpose_storage_stride_3_f32", (((129, 131), (3, 400), 4),), 3, 32768),
    Case("transpose_span_one_row_per_chunk", (((64, 32768), (1, 64), 2),), 4, 65536),     # tiles that span 64 chunks
    Case("transpose_span_rows_longer_than_chunks", (((40, 3, 9000), (1, 40 * 9000, 40), 4),), 3, 8192),
    Case("generic_mid", (((50, 30, 20), (20, 1000, 1), 2),), 3, 4096),
    Case("multi_mid", (contig((70001,), 1), ((64, 2, 128), (128, 64 * 128, 1), 2), ((96, 80), (1, 96), 4),
                       contig((3, 1000), 8), ((33, 10), (20, 2), 2)), 4, 8192),
]


@pytest.mark.parametrize("name,offset", [("contig_1MB_ragged", 1), ("contig_1MB_ragged", 7), ("contig_1MB_ragged", 4),
                                         ("contig_bf16_5MiB_tail", 2), ("contig_bf16_5MiB_tail", 6),
                                         ("contig_bf16_5MiB_tail", 8), ("contig_chunks_of_256_tiles", 12),
                                         ("multi_mid", 8), ("rows_mid", 2), ("rows_mid", 4), ("rows_big_rows", 6),
                                         ("rows_padded_pitch", 4), ("rows_4d", 2), ("transpose_mid", 2), ("transpose_512", 6),
                                         ("transpose_f32_vec_batched", 4), ("transpose_f64", 8), ("transpose_u8_vec", 1),
                                         ("transpose_u8_vec", 4), ("transpose_bf16_vec_partial", 2), ("generic_mid", 2),
                                         ("rows_200_byte_runs", 2), ("rows_200_byte_runs", 4), ("rows_200_byte_runs", 8),
                                         ("rows_31_byte_runs_3d", 1), ("rows_31_byte_runs_3d", 3), ("rows_f32_odd_pitch", 4)])
def test_mid_size_messages_with_element_aligned_bases(name, offset):
    """Contiguous tensors and row gathers whose base is 1, 2, 4, 8 or 12 bytes off a 16-byte boundary take their
    kernels, with narrower accesses on the tensor side, and so do transposes.  Same bytes and sums."""
    case = [c for c in MID_CASES if c.name == name][0]
    round_trip_check(case, make_storages(case, 321), None, base_offset=offset)


@pytest.mark.parametrize("case", MID_CASES, ids=lambda c: c.name)
def test_mid_size_cases_with_the_packed_side_non_temporal(case):
    round_trip_check(case, make_storages(case, 12), hint=1)


@pytest.mark.parametrize("case", MID_CASES, ids=lambda c: c.name)
def test_mid_size_cases(case):
    say("case", case.name)
    round_trip_check(case, make_storages(case, 4321))


@pytest.mark.parametrize("case", [c for c in MID_CASES if c.name in ("contig_1MB_ragged", "rows_mid", "transpose_512", "multi_mid")],
                         ids=lambda c: c.name)
def test_two_word_checksum_commit(case):
    # the commit variant used when a chunk's sum and its arrival count do not fit one 64-bit word
    say("two-word commit", case.name)
    round_trip_check(case, make_storages(case, 777), two_word=True)
    round_trip_check(case, make_storages(case, 778), tile_bytes=1024, two_word=True)


def test_repeated_calls_leave_accumulators_clean():
    case = [c for c in MID_CASES if c.name == "contig_bf16_5MiB_tail"][0]
    raws = make_storages(case, 31)
    m = oracle_msg(case)
    p = plan_of(case)
    want = ho.checksum(m, ho.pack(m, raws, case.B, case.k), case.B, case.k)
    src = [to_dev(r) for r in raws]
    packed = torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV)
    other = torch.cuda.Stream()
    for it in range(6):
        sums = torch.full((p.num_chunks,), it, dtype=torch.int64, device=DEV)
        st = other if it % 2 else torch.cuda.current_stream()       # alternate streams: calls are ordered by the library
        st.wait_stream(torch.cuda.current_stream())
        hxt.hxt_pack(p, src, packed, sums, st)
        st.synchronize()
        assert np.array_equal(sums.cpu().numpy().view(np.uint64), want), "call %d" % it


def test_one_plan_used_from_several_threads_and_streams():
    """Four host threads, a stream each, one shared plan, checksums on: the calls must queue behind each
    other on the plan's accumulators (the claim and the launch are one critical section)."""
    import threading
    case = Case("threads", (contig((5 * 1024 * 1024 // 2 + 24,), 2),), 4, 1 << 20)
    m = oracle_msg(case)
    p = plan_of(case)
    n_threads, iters = 4, 25
    raws = [make_storages(case, 200 + i) for i in range(n_threads)]
    want_sums = [ho.checksum(m, ho.pack(m, r, case.B, case.k, fill=0), case.B, case.k) for r in raws]
    src = [[to_dev(a) for a in r] for r in raws]
    dst = [[torch.zeros_like(a) for a in s_] for s_ in src]
    packed = [torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV) for _ in range(n_threads)]
    s_send = [torch.zeros(iters, p.num_chunks, dtype=torch.int64, device=DEV) for _ in range(n_threads)]
    s_recv = [torch.zeros(iters, p.num_chunks, dtype=torch.int64, device=DEV) for _ in range(n_threads)]
    streams = [torch.cuda.Stream() for _ in range(n_threads)]
    torch.cuda.synchronize()
    errors = []

    strong = [torch.zeros(iters, p.num_chunks, 2, dtype=torch.int64, device=DEV) for _ in range(n_threads)]
    plain = [torch.zeros(iters, p.num_chunks, dtype=torch.int64, device=DEV) for _ in range(n_threads)]
    tags = [torch.zeros(p.num_chunks * 64, dtype=torch.uint8, device=DEV) for _ in range(n_threads)]
    status = [torch.full((iters, p.num_chunks + 1), -1, dtype=torch.int32, device=DEV) for _ in range(n_threads)]

    def work(i):
        try:
            for it in range(iters):
                hxt.hxt_pack(p, src[i], packed[i], s_send[i][it], streams[i])
                hxt.hxt_checksum(p, packed[i], plain[i][it], streams[i])
                hxt.hxt_checksum2(p, packed[i], strong[i][it], streams[i])
                hxt.hxt_seal(p, packed[i], 1000 * i + it, i, tags[i], streams[i])
                hxt.hxt_verify(p, packed[i], tags[i], 1000 * i + it, i, status[i][it], streams[i])
                hxt.hxt_unpack(p, packed[i], dst[i], s_recv[i][it], streams[i])
        except Exception as e:                                   # noqa: BLE001 - reported below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i in range(n_threads):
        for arr in (s_send[i], s_recv[i]):
            got = arr.cpu().numpy().view(np.uint64)
            assert (got == want_sums[i][None, :]).all(), "thread %d" % i
        assert all(torch.equal(a, b) for a, b in zip(src[i], dst[i]))
        want2 = ho.checksum2(m, ho.pack(m, raws[i], case.B, case.k, fill=0), case.B, case.k)
        assert (plain[i].cpu().numpy().view(np.uint64) == want_sums[i][None, :]).all()
        assert (strong[i].cpu().numpy().view(np.uint64) == want2[None, :, :]).all()
        assert not status[i].cpu().numpy().any()


def test_batched_calls_that_share_plans_from_two_threads():
    """Two host threads, a stream each, issue batched calls over the same three plans in opposite orders, with
    checksums (each plan's accumulators are claimed under that plan's own lock; a batched call takes the locks of
    its plans in one fixed order, so the two threads can neither deadlock nor interleave on a plan)."""
    import threading
    names = ["contig_1MB_ragged", "rows_mid", "contig_bf16_5MiB_tail"]
    cases = [c for n in names for c in MID_CASES if c.name == n]
    plans = [plan_of(c) for c in cases]
    iters = 20
    raws = [[make_storages(c, 310 + 10 * t + i) for i, c in enumerate(cases)] for t in range(2)]
    want_packed = [[ho.pack(oracle_msg(c), raws[t][i], c.B, c.k, fill=0) for i, c in enumerate(cases)] for t in range(2)]
    want = [[ho.checksum(oracle_msg(c), want_packed[t][i], c.B, c.k) for i, c in enumerate(cases)] for t in range(2)]
    src = [[[to_dev(a) for a in rs] for rs in raws[t]] for t in range(2)]
    dst = [[[torch.zeros_like(a) for a in row] for row in src[t]] for t in range(2)]
    packed = [[torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV) for p in plans] for _ in range(2)]
    s_send = [[torch.zeros(iters, p.num_chunks, dtype=torch.int64, device=DEV) for p in plans] for _ in range(2)]
    s_recv = [[torch.zeros(iters, p.num_chunks, dtype=torch.int64, device=DEV) for p in plans] for _ in range(2)]
    streams = [torch.cuda.Stream() for _ in range(2)]
    torch.cuda.synchronize()
    errors = []

    def work(t):
        order = [0, 1, 2] if t == 0 else [2, 1, 0]
        pick = lambda rows: [rows[i] for i in order]
        try:
            for it in range(iters):
                say("thread", t, "batched call", it)
                hxt.hxt_pack_batch(hxt.Batch(pick(plans), pick(src[t]), pick(packed[t]),
                                             [s_send[t][i][it] for i in order]), streams[t])
                hxt.hxt_unpack_batch(hxt.Batch(pick(plans), pick(dst[t]), pick(packed[t]),
                                               [s_recv[t][i][it] for i in order]), streams[t])
        except Exception as e:                                   # noqa: BLE001 - reported below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(t,)) for t in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for t in range(2):
        for i, c in enumerate(cases):
            for arr in (s_send[t][i], s_recv[t][i]):
                assert (arr.cpu().numpy().view(np.uint64) == want[t][i][None, :]).all(), (t, c.name)
            dst_o = [np.zeros(r.size, np.uint8) for r in raws[t][i]]
            ho.unpack(oracle_msg(c), want_packed[t][i], c.B, c.k, dst_o)
            assert all(np.array_equal(b.cpu().numpy(), a) for a, b in zip(dst_o, dst[t][i])), (t, c.name)


def test_batch_calls_equal_single_calls():
    # mixed batch: three uniform messages (one without checksums, so it cannot share a launch with its
    # neighbours), a strided one, an empty one and a multi-tensor one
    names = ["contig_1MB_ragged", "contig_bf16_5MiB_tail", "rows_mid", "contig_1MB_ragged", "multi_mid"]
    cases = [c for n in names for c in MID_CASES if c.name == n] + [case_by_name("empty_tensor"), case_by_name("single_lane")]
    want_sums = [True, True, True, False, True, True, True]
    plans = [plan_of(c) for c in cases]
    raws = [make_storages(c, 900 + i) for i, c in enumerate(cases)]
    src = [[to_dev(r) for r in rs] for rs in raws]
    packed = [torch.full((max(p.packed_bytes, 1),), 0xA5, dtype=torch.uint8, device=DEV) for p in plans]
    sums = [torch.full((max(p.num_chunks, 1),), -3, dtype=torch.int64, device=DEV) if w else None
            for p, w in zip(plans, want_sums)]
    say("batch of", len(cases))
    hxt.hxt_pack_batch(hxt.Batch(plans, src, packed, sums))
    dst = [[to_dev(np.full(r.size, 0x3C, np.uint8)) for r in rs] for rs in raws]
    rsums = [torch.full_like(s_, 9) if s_ is not None else None for s_ in sums]
    hxt.hxt_unpack_batch(hxt.Batch(plans, dst, packed, rsums))
    torch.cuda.synchronize()
    for i, c in enumerate(cases):
        m = oracle_msg(c)
        want = ho.pack(m, raws[i], c.B, c.k, fill=0xA5)
        assert np.array_equal(packed[i].cpu().numpy()[:want.size], want), c.name
        if want_sums[i]:
            ws = ho.checksum(m, want, c.B, c.k)
            assert np.array_equal(sums[i].cpu().numpy().view(np.uint64)[:ws.size], ws), c.name
            assert np.array_equal(rsums[i].cpu().numpy().view(np.uint64)[:ws.size], ws), c.name
        dst_o = [np.full(r.size, 0x3C, np.uint8) for r in raws[i]]
        ho.unpack(m, want, c.B, c.k, dst_o)
        for a, b in zip(dst_o, dst[i]):
            assert np.array_equal(b.cpu().numpy(), a), c.name
    # the same plan twice with checksums is refused
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_pack_batch(hxt.Batch([plans[0], plans[0]], [src[0], src[0]], [packed[0], packed[0]], [sums[0], sums[0]]))
    assert e.value.status == hxt.HXT_EINVAL


@pytest.mark.parametrize("seed", range(6))
def test_random_views(seed):
    rng = np.random.default_rng(7000 + seed)
    done = 0
    while done < 10:
        tensors = tuple(random_view(rng) for _ in range(int(rng.integers(1, 5))))
        if sum(storage_bytes(*t) for t in tensors) > 4_000_000:
            continue
        case = Case("rand%d_%d" % (seed, done), tensors, int(rng.integers(1, 6)), int(rng.choice([256, 1024, 4096, 16384])))
        say("random case", case.tensors, case.k, case.B)
        round_trip_check(case, make_storages(case, seed), tile_bytes=int(rng.choice([256, 1024, 16384])))
        done += 1


@pytest.mark.parametrize("seed", range(4))
def test_random_views_of_up_to_eight_dims(seed):
    rng = np.random.default_rng(7100 + seed)
    done = 0
    while done < 12:
        tensors = tuple(random_view(rng, max_dims=8) for _ in range(int(rng.integers(1, 4))))
        if sum(storage_bytes(*t) for t in tensors) > 4_000_000 or sum(int(np.prod(t[0])) * t[2] for t in tensors) > 8_000_000:
            continue
        case = Case("rand8_%d_%d" % (seed, done), tensors, int(rng.integers(1, 6)), int(rng.choice([256, 1024, 4096, 16384])))
        hint = int(rng.choice([-1, 0, 1]))
        say("random case", case.tensors, case.k, case.B, "hint", hint)
        round_trip_check(case, make_storages(case, seed), tile_bytes=int(rng.choice([256, 1024, 16384])), hint=hint)
        done += 1


def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    # batched pack + unpack with checksums of two messages, captured once and replayed with fresh inputs;
    # every replay is compared with the eager result (no memset nodes: the library zero-fills nothing)
    case = [c for c in MID_CASES if c.name == "contig_bf16_5MiB_tail"][0]
    plans = [plan_of(case), plan_of(case)]
    nbytes = [int(np.prod(s)) * e for (s, _, e) in case.tensors][0]
    src = [[torch.zeros(nbytes, dtype=torch.uint8, device=DEV)] for _ in plans]
    dst = [[torch.zeros(nbytes, dtype=torch.uint8, device=DEV)] for _ in plans]
    packed = [torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV) for p in plans]
    ssum = [torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV) for p in plans]
    rsum = [torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV) for p in plans]
    pb = hxt.Batch(plans, src, packed, ssum)
    ub = hxt.Batch(plans, dst, packed, rsum)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up on the capture stream (accumulator ownership settles)
        hxt.hxt_pack_batch(pb, side)
        hxt.hxt_unpack_batch(ub, side)
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        hxt.hxt_pack_batch(pb, side)
        hxt.hxt_unpack_batch(ub, side)
    m = oracle_msg(case)
    for rep in range(4):
        raws = [make_storages(case, 500 + 10 * rep + i)[0] for i in range(2)]
        for i in range(2):
            src[i][0].copy_(torch.from_numpy(raws[i]))
            dst[i][0].zero_()
            rsum[i].fill_(-1)
        torch.cuda.synchronize()                        # the program's own eager work between replays
        g.replay()
        torch.cuda.synchronize()
        for i in range(2):
            want = ho.pack(m, [raws[i]], case.B, case.k, fill=0)        # unspecified slot bytes keep the buffer's zeros
            ws = ho.checksum(m, want, case.B, case.k)
            assert np.array_equal(packed[i].cpu().numpy(), want), "replay %d message %d" % (rep, i)
            assert np.array_equal(ssum[i].cpu().numpy().view(np.uint64), ws)
            assert np.array_equal(rsum[i].cpu().numpy().view(np.uint64), ws)
            assert np.array_equal(dst[i][0].cpu().numpy(), raws[i])


def test_many_tensors_need_several_launch_groups():
    rng = np.random.default_rng(8)
    tensors = tuple(contig((int(rng.integers(1, 3000)),), int(rng.choice([1, 2, 4]))) for _ in range(150))
    case = Case("many", tensors, 4, 4096)
    say("case many tensors", len(tensors))
    round_trip_check(case, make_storages(case, 55))


# ---------------------------------------------------------------------------
# staging (CPU-forwarding path) and fault detection
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["ragged_last_chunk_2p5", "fewer_chunks_than_lanes", "three_tensors_with_gaps"])
def test_staging_lane_by_lane_and_all_lanes(name):
    case = case_by_name(name)
    say("staging", name)
    raws = make_storages(case, 17)
    m = oracle_msg(case)
    p, packed, want, _ = round_trip_check(case, raws)
    n = want.size
    for lanes in ([-1], list(range(case.k))):
        host = torch.full((n,), 0x11, dtype=torch.uint8).pin_memory()
        expect_host = np.full(n, 0x11, np.uint8)
        for l in lanes:
            hxt.hxt_stage_d2h(p, l, packed, host)
        for l in (range(case.k) if lanes == [-1] else lanes):
            ho.stage_lane(m, case.B, case.k, l, want, expect_host)
        torch.cuda.synchronize()
        assert np.array_equal(host.numpy(), expect_host), "D2H must move the used bytes of the lane(s) and nothing else"
        recv = torch.full((n,), 0x22, dtype=torch.uint8, device=DEV)
        expect_recv = np.full(n, 0x22, np.uint8)
        for l in lanes:
            hxt.hxt_stage_h2d(p, l, host, recv)
        for l in (range(case.k) if lanes == [-1] else lanes):
            ho.stage_lane(m, case.B, case.k, l, expect_host, expect_recv)
        torch.cuda.synchronize()
        assert np.array_equal(recv.cpu().numpy(), expect_recv)
        # the receive side sees the same message
        dst = [torch.zeros(r.size, dtype=torch.uint8, device=DEV) for r in raws]
        rs = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
        hxt.hxt_unpack(p, recv, dst, rs)
        dst_o = [np.zeros(r.size, np.uint8) for r in raws]
        ho.unpack(m, want, case.B, case.k, dst_o)
        for a, b in zip(dst_o, dst):
            assert np.array_equal(b.cpu().numpy(), a)


@pytest.mark.parametrize("d2h", [0, 1], ids=["copy_command", "copy_kernel"])
@pytest.mark.parametrize("name", ["ragged_last_chunk_2p5", "fewer_chunks_than_lanes", "sixty_four_lanes", "contig_1MB_ragged",
                                  "multi_mid"])
def test_staging_in_runs_of_slots(name, d2h):
    """A lane staged in pieces (runs of slots), each piece down by the copy command or by the library's copy kernel
    and up by a copy command: exactly the oracle's bytes move, untouched bytes keep their canaries."""
    case = ([c for c in MID_CASES if c.name == name] or [None])[0] or case_by_name(name)
    say("slot staging", name, "d2h mode", d2h)
    raws = make_storages(case, 19)
    m = oracle_msg(case)
    p, packed, want, _ = round_trip_check(case, raws)
    hxt.hxt_plan_set_option(p, hxt.HXT_OPT_STAGE_D2H, d2h)
    n = want.size
    rng = np.random.default_rng(5)
    host = torch.full((n,), 0x11, dtype=torch.uint8).pin_memory()
    recv = torch.full((n,), 0x22, dtype=torch.uint8, device=DEV)
    expect_host, expect_recv = np.full(n, 0x11, np.uint8), np.full(n, 0x22, np.uint8)
    for lane in range(case.k):
        slots = p.lane_info(lane)["n_chunks"]
        s = 0
        while s < slots:                                   # random cuts, the empty run included
            cnt = int(rng.integers(0, slots - s + 1)) if rng.random() < 0.8 else 0
            hxt.hxt_stage_d2h_slots(p, lane, s, cnt, packed, host)
            hxt.hxt_stage_h2d_slots(p, lane, s, cnt, host, recv)
            ho.stage_slots(m, case.B, case.k, lane, s, cnt, want, expect_host)
            ho.stage_slots(m, case.B, case.k, lane, s, cnt, expect_host, expect_recv)
            s += cnt
        with pytest.raises(hxt.HxtError) as e:
            hxt.hxt_stage_d2h_slots(p, lane, slots, 1, packed, host)
        assert e.value.status == hxt.HXT_EINVAL
    torch.cuda.synchronize()
    assert np.array_equal(host.numpy(), expect_host)
    assert np.array_equal(recv.cpu().numpy(), expect_recv)
    # whole lanes and the whole buffer through the copy kernel too
    host2 = torch.full((n,), 0x11, dtype=torch.uint8).pin_memory()
    hxt.hxt_stage_d2h(p, -1, packed, host2)
    torch.cuda.synchronize()
    assert np.array_equal(host2.numpy(), expect_host)
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_stage_d2h_slots(p, -1, 0, 1, packed, host)
    assert e.value.status == hxt.HXT_EINVAL


@pytest.mark.parametrize("name", ["contig_1MB_ragged", "multi_mid"])
def test_cpu_forwarding_chain_with_host_hop(name):
    # D2H into the sender's pinned buffer, host-to-host hop (stream ordered), H2D from the receiver's pinned
    # buffer, unpack; once on one stream, once lane by lane over three streams chained with events
    case = [c for c in MID_CASES if c.name == name][0]
    say("host hop", name)
    raws = make_storages(case, 71)
    m = oracle_msg(case)
    p, packed, want, want_sums = round_trip_check(case, raws)
    n = want.size
    dst_o = [np.zeros(r.size, np.uint8) for r in raws]
    ho.unpack(m, want, case.B, case.k, dst_o)
    for pipelined in (False, True):
        h_send = torch.full((n,), 0x11, dtype=torch.uint8).pin_memory()
        h_recv = torch.full((n,), 0x22, dtype=torch.uint8).pin_memory()
        recv = torch.full((n,), 0x33, dtype=torch.uint8, device=DEV)
        if not pipelined:
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            hxt.hxt_stage_d2h(p, -1, packed, h_send, s)
            hxt.hxt_stage_hop(p, -1, h_send, h_recv, 0, s)
            hxt.hxt_stage_h2d(p, -1, h_recv, recv, s)
            last = s
        else:
            s1, s2, s3 = (torch.cuda.Stream() for _ in range(3))
            s1.wait_stream(torch.cuda.current_stream())
            for l in range(case.k):
                hxt.hxt_stage_d2h(p, l, packed, h_send, s1)
                e1 = torch.cuda.Event(); e1.record(s1); s2.wait_event(e1)
                hxt.hxt_stage_hop(p, l, h_send, h_recv, 1, s2)
                e2 = torch.cuda.Event(); e2.record(s2); s3.wait_event(e2)
                hxt.hxt_stage_h2d(p, l, h_recv, recv, s3)
            last = s3
        dst = [torch.zeros(r.size, dtype=torch.uint8, device=DEV) for r in raws]
        rs = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
        last.wait_stream(torch.cuda.current_stream())       # the zero fills above ran on the current stream
        hxt.hxt_unpack(p, recv, dst, rs, last)
        torch.cuda.synchronize()
        expect = np.full(n, 0x22, np.uint8)
        for l in range(case.k):
            ho.stage_lane(m, case.B, case.k, l, want, expect)
        assert np.array_equal(h_recv.numpy(), expect)
        assert np.array_equal(rs.cpu().numpy().view(np.uint64), want_sums)
        for a, b in zip(dst_o, dst):
            assert np.array_equal(b.cpu().numpy(), a)


def test_bit_flip_in_host_buffer_shows_in_exactly_one_checksum():
    case = Case("flip", (contig((40000,), 2),), 3, 8192)
    raws = make_storages(case, 23)
    p, packed, want, want_sums = round_trip_check(case, raws)
    host = torch.zeros(want.size, dtype=torch.uint8).pin_memory()
    hxt.hxt_stage_d2h(p, -1, packed, host)
    torch.cuda.synchronize()
    info = p.chunk_info(4)
    byte, bit = info["packed_off"] + 4 * 100 + 1, 3
    was_set = bool(int(host[byte]) >> bit & 1)
    host[byte] = int(host[byte]) ^ (1 << bit)                # the fault, planted on the host
    recv = torch.zeros(want.size, dtype=torch.uint8, device=DEV)
    hxt.hxt_stage_h2d(p, -1, host, recv)
    dst = [torch.zeros(r.size, dtype=torch.uint8, device=DEV) for r in raws]
    rs = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    hxt.hxt_unpack(p, recv, dst, rs)
    got = rs.cpu().numpy().view(np.uint64)
    delta = 1 << (8 + bit)
    diff = [int(a) - int(b) for a, b in zip(got, want_sums)]
    assert diff == [0, 0, 0, 0, (-delta if was_set else delta)] + [0] * (len(diff) - 5)


def test_words_that_change_places_show_only_in_the_weighted_sum():
    """Two unequal words of one chunk swapped on the host: the plain sum stays, the weighted sum moves by
    (j - i) * (w_i - w_j) in that chunk alone; repeated calls leave the accumulators clean."""
    case = Case("swap", (contig((600000,), 2),), 2, 262144)          # 16 tiles per full chunk, ragged last chunk
    raws = make_storages(case, 29)
    p, packed, want, want_sums = round_trip_check(case, raws)
    m = oracle_msg(case)
    host = packed.cpu().numpy().copy()
    c = 2
    base = p.chunk_info(c)["packed_off"]
    words = host[base:base + case.B].view("<u4")
    i, j = 5, 40001                                                  # different tiles of the chunk
    assert words[i] != words[j]
    wi, wj = int(words[i]), int(words[j])
    words[i], words[j] = wj, wi
    want2 = ho.checksum2(m, host, case.B, case.k)
    clean2 = ho.checksum2(m, want, case.B, case.k)
    assert np.array_equal(want2[:, 0], clean2[:, 0])
    assert (int(want2[c, 1]) - int(clean2[c, 1])) % 2**64 == ((j - i) * (wi - wj)) % 2**64
    dev = to_dev(host)
    for rep in range(3):
        got = torch.full((p.num_chunks, 2), rep, dtype=torch.int64, device=DEV)
        hxt.hxt_checksum2(p, dev, got)
        assert np.array_equal(got.cpu().numpy().view(np.uint64), want2)
    plain = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    hxt.hxt_checksum(p, dev, plain)
    assert np.array_equal(plain.cpu().numpy().view(np.uint64), want_sums)   # blind to the swap


@pytest.mark.parametrize("case", [
    Case("beyond_4GiB_one_tensor", (contig((2**32 + 3 * 2**20 + 24,), 1),), 3, 32 << 20),
    Case("dim_beyond_2_30_every_other_byte", (((2**30 + 5,), (2,), 1),), 2, 64 << 20),
    Case("beyond_4GiB_table", (contig((2**32 + 4096,), 1), ((1000, 256), (320, 1), 4), ((512, 384), (1, 512), 2),
                               contig((70001,), 1)), 4, 16 << 20),
], ids=lambda c: c.name)
def test_offsets_beyond_32_bits(case):
    """Stream, packed and storage offsets past 2^32: the closed-form kernel, and the table-driven kernels
    whose tiles start beyond 4 GiB; a dim of more than 2^30 elements in a view without a unit stride (the
    per-element kernel then divides every index out in 64 bits)."""
    rng = np.random.default_rng(zlib.crc32(case.name.encode()))
    raws = []
    for t in case.tensors:
        n = storage_bytes(*t)
        raws.append(rng.integers(0, 2**63, size=n // 8 + 1, dtype=np.int64).view(np.uint8)[:n].copy())
    say("drawn", [r.size for r in raws])
    round_trip_check(case, raws, nthreads=NT)


def test_plans_release_their_device_memory():
    case = [c for c in MID_CASES if c.name == "multi_mid"][0]
    raws = make_storages(case, 4)
    src = [to_dev(r) for r in raws]
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    side = torch.cuda.Stream()
    for i in range(200):
        p = plan_of(case)
        packed = torch.empty(p.packed_bytes, dtype=torch.uint8, device=DEV) if i == 0 else packed
        sums = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV) if i == 0 else sums
        if i == 0:
            free0 = torch.cuda.mem_get_info()[0]                 # after the buffers of the test itself exist
        hxt.hxt_pack(p, src, packed, sums)
        hxt.hxt_pack(p, src, packed, sums, side)                 # another stream: the plan creates its ordering event
        hxt.hxt_plan_destroy(p)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free0 - (8 << 20), "device memory of destroyed plans was not returned"


def test_data_plane_argument_errors():
    case = case_by_name("single_lane")
    p = plan_of(case)
    raws = make_storages(case, 1)
    src = [to_dev(r) for r in raws]
    packed = torch.zeros(p.packed_bytes + 256, dtype=torch.uint8, device=DEV)
    L = hxt.lib()
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_pack(p, src, packed[8:], None)
    assert e.value.status == hxt.HXT_EALIGN
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_pack(p, [src[0].data_ptr() + 1], packed, None)          # bf16 base on an odd byte
    assert e.value.status == hxt.HXT_EALIGN
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_pack(p, [None], packed, None)
    assert e.value.status == hxt.HXT_EINVAL
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_stage_d2h(p, 1, packed, packed)                          # lane out of range (k = 1)
    assert e.value.status == hxt.HXT_EINVAL
    assert L.hxt_checksum(p.handle, packed.data_ptr(), None, None) == hxt.HXT_EINVAL
    assert L.hxt_checksum2(p.handle, packed.data_ptr(), None, None) == hxt.HXT_EINVAL
    assert L.hxt_checksum2(p.handle, None, packed.data_ptr(), None) == hxt.HXT_EINVAL
    torch.cuda.synchronize()


# ---------------------------------------------------------------------------
# the five benchmark messages at full size
# ---------------------------------------------------------------------------

def case_of(w):
    return Case(w.name, tuple((t.shape, t.strides, t.esize) for t in w.tensors), w.n_lanes, w.chunk_bytes)


def test_config_tiny():
    w = wl.tiny()
    round_trip_check(case_of(w), wl.make_storages(w))


def test_config_llama8b_boundary_forward_and_backward():
    w = wl.llama8b_boundary()
    for msg in range(w.messages):                 # forward activation, backward gradient
        say("llama message", msg)
        round_trip_check(case_of(w), wl.make_storages(w, msg), nthreads=NT)


@pytest.mark.parametrize("hint", [-1, 1, 0], ids=["hint_by_size", "all_cold_non_temporal", "cacheable"])
def test_config_llama8b_boundary_in_the_benchmarks_launch_configuration(hint):
    """Both messages of the step in one batched pack call and one batched unpack call, a plan each, fused
    checksums, as the benchmark times them (hint 1 is its all-cold region: the packed side non-temporal too);
    every byte and every sum against the oracle."""
    w = wl.llama8b_boundary()
    case = case_of(w)
    m = oracle_msg(case)
    plans = [plan_of(case) for _ in range(w.messages)]
    for p in plans:
        hxt.hxt_plan_set_option(p, hxt.HXT_OPT_PACKED_HINT, hint)
    raws = [wl.make_storages(w, i) for i in range(w.messages)]
    src = [[to_dev(r) for r in rs] for rs in raws]
    packed = [torch.full((p.packed_bytes,), 0xA5, dtype=torch.uint8, device=DEV) for p in plans]
    sums = [torch.full((p.num_chunks,), -1, dtype=torch.int64, device=DEV) for p in plans]
    rsums = [torch.full((p.num_chunks,), -2, dtype=torch.int64, device=DEV) for p in plans]
    dst = [[torch.full_like(t, 0x3C) for t in s_] for s_ in src]
    hxt.hxt_pack_batch(hxt.Batch(plans, src, packed, sums))
    hxt.hxt_unpack_batch(hxt.Batch(plans, dst, packed, rsums))
    torch.cuda.synchronize()
    for i in range(w.messages):
        want = ho.pack(m, raws[i], w.chunk_bytes, w.n_lanes, fill=0xA5, nthreads=NT)
        ws = ho.checksum(m, want, w.chunk_bytes, w.n_lanes, nthreads=NT)
        assert np.array_equal(packed[i].cpu().numpy(), want), "message %d" % i
        assert np.array_equal(sums[i].cpu().numpy().view(np.uint64), ws)
        assert np.array_equal(rsums[i].cpu().numpy().view(np.uint64), ws)
        dst_o = [np.full(r.size, 0x3C, np.uint8) for r in raws[i]]
        ho.unpack(m, want, w.chunk_bytes, w.n_lanes, dst_o, nthreads=NT)
        for a, b in zip(dst_o, dst[i]):
            assert np.array_equal(b.cpu().numpy(), a)
    assert not np.array_equal(raws[0][0], raws[1][0])


def test_config_llama8b_boundary_steps_dealt_onto_two_streams():
    """The issue order behind the benchmark's headline figure: consecutive steps go alternately to two streams,
    each stream with a plan set of its own (two plans, packed side non-temporal), batched calls, fused checksums,
    nothing ordering the two streams against each other.  Six steps on fresh data each; every step's packed bytes,
    sums and destination against the oracle."""
    w = wl.llama8b_boundary()
    case = case_of(w)
    m = oracle_msg(case)
    n_steps = 6
    plan_sets = [[plan_of(case) for _ in range(w.messages)] for _ in range(2)]
    for ps in plan_sets:
        for p in ps:
            hxt.hxt_plan_set_option(p, hxt.HXT_OPT_PACKED_HINT, 1)
    streams = [torch.cuda.Stream() for _ in range(2)]
    raws = [[wl.make_storages(w, (3 * s_ + i) % 7 + i) for i in range(w.messages)] for s_ in range(n_steps)]
    src = [[[to_dev(r) for r in rs] for rs in step] for step in raws]
    dst = [[[torch.full_like(t, 0x3C) for t in row] for row in step] for step in src]
    C, nb = plan_sets[0][0].num_chunks, plan_sets[0][0].packed_bytes
    packed = [[torch.full((nb,), 0xA5, dtype=torch.uint8, device=DEV) for _ in range(w.messages)] for _ in range(n_steps)]
    sums = [[torch.full((C,), -1, dtype=torch.int64, device=DEV) for _ in range(w.messages)] for _ in range(n_steps)]
    rsums = [[torch.full((C,), -2, dtype=torch.int64, device=DEV) for _ in range(w.messages)] for _ in range(n_steps)]
    torch.cuda.synchronize()
    for s_ in range(n_steps):
        say("step", s_, "on stream", s_ % 2)
        ps, st = plan_sets[s_ % 2], streams[s_ % 2]
        hxt.hxt_pack_batch(hxt.Batch(ps, src[s_], packed[s_], sums[s_]), st)
        hxt.hxt_unpack_batch(hxt.Batch(ps, dst[s_], packed[s_], rsums[s_]), st)
    torch.cuda.synchronize()
    known = {}
    for s_ in range(n_steps):
        for i in range(w.messages):
            key = raws[s_][i][0].tobytes()[:64]
            if key not in known:
                want = ho.pack(m, raws[s_][i], w.chunk_bytes, w.n_lanes, fill=0xA5, nthreads=NT)
                known[key] = (want, ho.checksum(m, want, w.chunk_bytes, w.n_lanes, nthreads=NT))
            want, ws = known[key]
            assert np.array_equal(packed[s_][i].cpu().numpy(), want), (s_, i)
            assert np.array_equal(sums[s_][i].cpu().numpy().view(np.uint64), ws), (s_, i)
            assert np.array_equal(rsums[s_][i].cpu().numpy().view(np.uint64), ws), (s_, i)
            assert np.array_equal(dst[s_][i][0].cpu().numpy(), raws[s_][i][0]), (s_, i)


def test_config_qwen2_both_paths_same_bytes():
    w = wl.qwen2_7b_boundary()
    case = case_of(w)
    raws = wl.make_storages(w)
    p, packed, want, want_sums = round_trip_check(case, raws, nthreads=NT)
    # CPU-forwarding: D2H per lane on one stream, H2D per lane on another, chained by events
    host = torch.zeros(want.size, dtype=torch.uint8).pin_memory()
    recv = torch.zeros(want.size, dtype=torch.uint8, device=DEV)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    s1.wait_stream(torch.cuda.current_stream())
    for l in range(w.n_lanes):
        hxt.hxt_stage_d2h(p, l, packed, host, s1)
        ev = torch.cuda.Event()
        ev.record(s1)
        s2.wait_event(ev)
        hxt.hxt_stage_h2d(p, l, host, recv, s2)
    torch.cuda.current_stream().wait_stream(s2)
    dst = [torch.zeros(r.size, dtype=torch.uint8, device=DEV) for r in raws]
    rs = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    hxt.hxt_unpack(p, recv, dst, rs)
    torch.cuda.synchronize()
    assert np.array_equal(host.numpy(), want)                       # identical packed bytes on the host
    assert torch.equal(recv, packed[:want.size])                    # and on the receive side
    assert np.array_equal(rs.cpu().numpy().view(np.uint64), want_sums)
    assert np.array_equal(dst[0].cpu().numpy(), raws[0])


@pytest.mark.parametrize("path", ["device_direct", "cpu_forward"])
def test_config_stream_1f1b_three_streams_ping_pong(path):
    w = wl.stream_1f1b(32)                      # CPU forwarding drains its streams after messages 12 and 24
    case = case_of(w)
    m = oracle_msg(case)
    p = plan_of(case)
    assert p.tensor_kind(0) == "contig"
    nmsg, C, nb = w.messages, p.num_chunks, p.packed_bytes
    say("stream", path, "messages", nmsg)
    raws = [wl.make_storages(w, i)[0] for i in range(nmsg)]
    src = [to_dev(r) for r in raws]
    dst = [torch.zeros(r.size, dtype=torch.uint8, device=DEV) for r in raws]
    send_sums = torch.zeros((nmsg, C), dtype=torch.int64, device=DEV)
    recv_sums = torch.zeros((nmsg, C), dtype=torch.int64, device=DEV)
    # two buffer sets, poisoned so that a premature read would be seen
    send_buf = [torch.full((nb,), 0xEE, dtype=torch.uint8, device=DEV) for _ in range(2)]
    recv_buf = [torch.full((nb,), 0xDD, dtype=torch.uint8, device=DEV) for _ in range(2)] if path == "cpu_forward" else send_buf
    host_buf = [torch.zeros(nb, dtype=torch.uint8).pin_memory() for _ in range(2)]
    sp, ss, su = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    for s in (sp, ss, su):
        s.wait_stream(torch.cuda.current_stream())
    packed_ev = [None, None]      # buffer i%2 holds message i (pack done)
    staged_ev = [None, None]      # receive buffer i%2 holds message i (H2D done)
    freed_ev = [None, None]       # buffer i%2 may be overwritten (unpack of its previous message done)
    sent_ev = [None, None]        # send buffer drained to the host
    for i in range(nmsg):
        b = i % 2
        if freed_ev[b] is not None:
            sp.wait_event(freed_ev[b] if path == "device_direct" else sent_ev[b])
        hxt.hxt_pack(p, [src[i]], send_buf[b], send_sums[i], sp)
        packed_ev[b] = torch.cuda.Event(); packed_ev[b].record(sp)
        if path == "cpu_forward":
            ss.wait_event(packed_ev[b])
            if freed_ev[b] is not None:
                ss.wait_event(freed_ev[b])
            hxt.hxt_stage_d2h(p, -1, send_buf[b], host_buf[b], ss)
            sent_ev[b] = torch.cuda.Event(); sent_ev[b].record(ss)
            hxt.hxt_stage_h2d(p, -1, host_buf[b], recv_buf[b], ss)
            staged_ev[b] = torch.cuda.Event(); staged_ev[b].record(ss)
            su.wait_event(staged_ev[b])
        else:
            su.wait_event(packed_ev[b])
        hxt.hxt_unpack(p, recv_buf[b], [dst[i]], recv_sums[i], su)
        freed_ev[b] = torch.cuda.Event(); freed_ev[b].record(su)
    torch.cuda.synchronize()
    ss_h = send_sums.cpu().numpy().view(np.uint64)
    rs_h = recv_sums.cpu().numpy().view(np.uint64)
    assert np.array_equal(ss_h, rs_h)
    for i in range(nmsg):
        assert np.array_equal(dst[i].cpu().numpy(), raws[i]), "micro-batch %d" % i
        if i % 8 == 0:                     # oracle checksums on a sample of the micro-batches
            want = ho.pack(m, [raws[i]], w.chunk_bytes, w.n_lanes, nthreads=NT)
            assert np.array_equal(ss_h[i], ho.checksum(m, want, w.chunk_bytes, w.n_lanes, nthreads=NT))


def run_exchange_tagged(case, raws_per_msg, path, n_buffers, streams, seq_base=1 << 40):
    """hxt_exchange_stream with chunk tags: every destination, a clean verdict for every message, and the tags
    left in the buffers (those of the last n_buffers messages) against the oracle's."""
    m = oracle_msg(case)
    p = plan_of(case)
    nmsg, C, nb = len(raws_per_msg), p.num_chunks, max(p.packed_bytes, 256)
    fwd = path == "cpu_forward"
    src = [[to_dev(r) for r in raws] for raws in raws_per_msg]
    dst = [[to_dev(np.full(r.size, 0x3C, np.uint8)) for r in raws] for raws in raws_per_msg]
    dev_bufs = lambda n, fill: [torch.full((n,), fill, dtype=torch.uint8, device=DEV) for _ in range(n_buffers)]
    pinned = lambda n: [torch.zeros(n, dtype=torch.uint8).pin_memory() for _ in range(n_buffers)]
    send_buf, tags_send = dev_bufs(nb, 0xEE), dev_bufs(max(C, 1) * 64, 0x11)
    recv_buf, tags_recv = (dev_bufs(nb, 0xDD), dev_bufs(max(C, 1) * 64, 0x22)) if fwd else (None, None)
    host_buf, tags_pinned = (pinned(nb), pinned(max(C, 1) * 64)) if fwd else (None, None)
    status = torch.full((nmsg, C + 1), -1, dtype=torch.int32, device=DEV)
    for s_ in streams:
        s_.wait_stream(torch.cuda.current_stream())
    x = hxt.Exchange(src, dst, send_buf, hxt.HXT_CPU_FORWARD if fwd else hxt.HXT_DEVICE_DIRECT, recv_buf, host_buf,
                     None, None, *streams, tags_send=tags_send, tags_recv=tags_recv, tags_pinned=tags_pinned,
                     status=status, seq_base=seq_base)
    hxt.hxt_exchange_stream(p, x)
    torch.cuda.synchronize()
    assert not status.cpu().numpy().any(), "a chunk was rejected"
    for i, raws in enumerate(raws_per_msg):
        want = ho.pack(m, raws, case.B, case.k, nthreads=NT)
        dst_o = [np.full(r.size, 0x3C, np.uint8) for r in raws]
        ho.unpack(m, want, case.B, case.k, dst_o, nthreads=NT)
        for a, b in zip(dst_o, dst[i]):
            assert np.array_equal(b.cpu().numpy(), a), "message %d" % i
        if i >= nmsg - n_buffers:
            want_tags = ho.seal(m, want, case.B, case.k, seq_base + i, i)
            for buf in ([tags_send, tags_recv] if fwd else [tags_send]):
                assert np.array_equal(buf[i % n_buffers].cpu().numpy()[:C * 64].reshape(C, 64), want_tags), "message %d" % i


def run_exchange(case, raws_per_msg, path, n_buffers, streams, **how):
    """hxt_exchange_stream on a list of messages; checks every destination and every checksum."""
    m = oracle_msg(case)
    p = plan_of(case)
    nmsg, C, nb = len(raws_per_msg), p.num_chunks, max(p.packed_bytes, 256)
    src = [[to_dev(r) for r in raws] for raws in raws_per_msg]
    dst = [[to_dev(np.full(r.size, 0x3C, np.uint8)) for r in raws] for raws in raws_per_msg]
    send_sums = torch.full((nmsg, max(C, 1)), -1, dtype=torch.int64, device=DEV)
    recv_sums = torch.full((nmsg, max(C, 1)), -2, dtype=torch.int64, device=DEV)
    send_buf = [torch.full((nb,), 0xEE, dtype=torch.uint8, device=DEV) for _ in range(n_buffers)]      # poisoned
    fwd = path == "cpu_forward"
    recv_buf = [torch.full((nb,), 0xDD, dtype=torch.uint8, device=DEV) for _ in range(n_buffers)] if fwd else None
    host_buf = [torch.zeros(nb, dtype=torch.uint8).pin_memory() for _ in range(n_buffers)] if fwd else None
    for s_ in streams:
        s_.wait_stream(torch.cuda.current_stream())
    x = hxt.Exchange(src, dst, send_buf, hxt.HXT_CPU_FORWARD if fwd else hxt.HXT_DEVICE_DIRECT, recv_buf, host_buf,
                     send_sums, recv_sums, *streams, **how)
    hxt.hxt_exchange_stream(p, x)
    torch.cuda.synchronize()
    ss_h = send_sums.cpu().numpy().view(np.uint64)[:, :C]
    rs_h = recv_sums.cpu().numpy().view(np.uint64)[:, :C]
    assert np.array_equal(ss_h, rs_h)
    for i, raws in enumerate(raws_per_msg):
        want = ho.pack(m, raws, case.B, case.k, nthreads=NT)
        assert np.array_equal(ss_h[i], ho.checksum(m, want, case.B, case.k, nthreads=NT)), "message %d" % i
        dst_o = [np.full(r.size, 0x3C, np.uint8) for r in raws]
        ho.unpack(m, want, case.B, case.k, dst_o, nthreads=NT)
        for a, b in zip(dst_o, dst[i]):
            assert np.array_equal(b.cpu().numpy(), a), "message %d" % i


@pytest.mark.parametrize("path", ["device_direct", "cpu_forward"])
@pytest.mark.parametrize("n_buffers", [1, 2, 3])
def test_exchange_stream_small_messages(path, n_buffers):
    say("exchange", path, "buffers", n_buffers)
    streams = [torch.cuda.Stream() for _ in range(3)]
    for name, nmsg in (("contig_1MB_ragged", 7), ("multi_mid", 5), ("rows_mid", 4), ("transpose_span_one_row_per_chunk", 4),
                       ("transpose_storage_stride_2", 3)):
        case = [c for c in MID_CASES if c.name == name][0]
        run_exchange(case, [make_storages(case, 3000 + i) for i in range(nmsg)], path, n_buffers, streams)
    # all three roles on one stream: the steps simply serialise
    case = [c for c in MID_CASES if c.name == "contig_1MB_ragged"][0]
    one = torch.cuda.Stream()
    run_exchange(case, [make_storages(case, 3100 + i) for i in range(3)], path, n_buffers, [one, one, one])


@pytest.mark.parametrize("path", ["device_direct", "cpu_forward"])
@pytest.mark.parametrize("n_buffers", [1, 2, 3, 4])
def test_exchange_stream_with_chunk_tags(path, n_buffers):
    streams = [torch.cuda.Stream() for _ in range(3)]
    for name, nmsg in (("contig_bf16_5MiB_tail", 7), ("multi_mid", 5), ("rows_mid", 4)):
        case = [c for c in MID_CASES if c.name == name][0]
        run_exchange_tagged(case, [make_storages(case, 3300 + i) for i in range(nmsg)], path, n_buffers, streams)


def test_exchange_stream_with_chunk_tags_rejects_mixed_requests():
    case = [c for c in MID_CASES if c.name == "contig_1MB_ragged"][0]
    p = plan_of(case)
    raws = make_storages(case, 1)
    src, dst = [[to_dev(r) for r in raws]], [[to_dev(r) for r in raws]]
    buf = [torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV)]
    tags = [torch.zeros(p.num_chunks * 64, dtype=torch.uint8, device=DEV)]
    sums = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    status = torch.zeros(p.num_chunks + 1, dtype=torch.int32, device=DEV)
    for kwargs in (dict(tags_send=tags, status=None), dict(tags_send=tags, status=status, send=sums),
                   dict(tags_send=[None], status=status)):
        x = hxt.Exchange(src, dst, buf, hxt.HXT_DEVICE_DIRECT, None, None, kwargs.get("send"), None, None, None, None,
                         tags_send=kwargs["tags_send"], status=kwargs["status"])
        with pytest.raises(hxt.HxtError) as e:
            hxt.hxt_exchange_stream(p, x)
        assert e.value.status == hxt.HXT_EINVAL
    x = hxt.Exchange(src, dst, buf, hxt.HXT_CPU_FORWARD, buf, [torch.zeros(p.packed_bytes, dtype=torch.uint8).pin_memory()],
                     None, None, None, None, None, tags_send=tags, status=status)          # CPU forwarding needs the other tag buffers
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_exchange_stream(p, x)
    assert e.value.status == hxt.HXT_EINVAL
    torch.cuda.synchronize()


@pytest.mark.parametrize("path,how", [("device_direct", {}), ("cpu_forward", {}), ("cpu_forward", {"drain_every": 12})],
                         ids=["device_direct", "cpu_forward_enqueue_only", "cpu_forward_drained_every_12"])
def test_config_stream_1f1b_native_exchange(path, how):
    w = wl.stream_1f1b(32)                      # with drain_every = 12 the call waits after messages 12 and 24
    say("native stream", path, how, "messages", w.messages)
    run_exchange(case_of(w), [wl.make_storages(w, i) for i in range(w.messages)], path, 2,
                 [torch.cuda.Stream() for _ in range(3)], **how)


@pytest.mark.parametrize("mode", [hxt.HXT_DIRECT_AUTO, hxt.HXT_DIRECT_TWO_CHAINS, hxt.HXT_DIRECT_FUSED, hxt.HXT_DIRECT_EVENTS])
@pytest.mark.parametrize("n_buffers", [2, 4])
def test_exchange_stream_device_direct_modes_agree(mode, n_buffers):
    # device-direct streams: two message chains on two streams, fused launches on one stream (single-tensor
    # messages only) and event-chained calls on three streams must give the same result, for single-tensor
    # and for multi-tensor messages
    streams = [torch.cuda.Stream() for _ in range(3)]
    for name, nmsg in (("contig_bf16_5MiB_tail", 7), ("multi_mid", 6)):
        case = [c for c in MID_CASES if c.name == name][0]
        raws = [make_storages(case, 3200 + i) for i in range(nmsg)]
        if mode == hxt.HXT_DIRECT_FUSED and name == "multi_mid":          # not a single-tensor message: refused
            with pytest.raises(hxt.HxtError) as e:
                run_exchange(case, raws, "device_direct", n_buffers, streams, direct_mode=mode)
            assert e.value.status == hxt.HXT_EINVAL
            continue
        run_exchange(case, raws, "device_direct", n_buffers, streams, direct_mode=mode)


def test_exchange_stream_refuses_modes_the_arguments_do_not_allow():
    case = [c for c in MID_CASES if c.name == "contig_1MB_ragged"][0]
    raws = [make_storages(case, 1), make_storages(case, 2)]
    streams = [torch.cuda.Stream() for _ in range(3)]
    for n_buffers, how in ((3, dict(direct_mode=hxt.HXT_DIRECT_TWO_CHAINS)), (1, dict(direct_mode=hxt.HXT_DIRECT_FUSED)),
                           (2, dict(direct_mode=7)), (2, dict(drain_every=-1))):
        with pytest.raises(hxt.HxtError) as e:
            run_exchange(case, raws, "device_direct", n_buffers, streams, **how)
        assert e.value.status == hxt.HXT_EINVAL
    torch.cuda.synchronize()


@pytest.mark.parametrize("seed", range(3))
def test_exchange_stream_random_shapes_many_rounds(seed):
    """The paper's bring-up kept running into hangs (subsection "Engineering Challenges"): stress the ping-pong
    stream with random message shapes, both paths, 1 to 4 buffer sets, several calls in a row on the same
    streams and buffers; every call must finish and every byte and checksum must match the oracle."""
    rng = np.random.default_rng(9100 + seed)
    streams = [torch.cuda.Stream() for _ in range(3)]
    done = 0
    while done < 6:
        tensors = tuple(random_view(rng) for _ in range(int(rng.integers(1, 4))))
        if not 0 < sum(storage_bytes(*t) for t in tensors) <= 1_500_000:
            continue
        case = Case("xrand%d_%d" % (seed, done), tensors, int(rng.integers(1, 6)), int(rng.choice([256, 4096, 65536])))
        p = plan_of(case)
        if not all(p.tensor_unpack_safe(t) for t in range(len(tensors))):
            continue
        nmsg = int(rng.integers(2, 9))
        say("stream of", nmsg, "x", case.tensors, "lanes", case.k, "chunk", case.B)
        for rounds in range(2):
            for path in ("device_direct", "cpu_forward"):
                run_exchange(case, [make_storages(case, 77 * done + i + 1000 * rounds) for i in range(nmsg)], path,
                             int(rng.integers(1, 5)), streams)
        done += 1


def test_packed_buffer_in_pinned_host_memory():
    # the packed buffer may live in pinned host memory (the kernels then move the bytes over the
    # host link themselves, with no device-side staging buffer)
    case = [c for c in MID_CASES if c.name == "multi_mid"][0]
    m = oracle_msg(case)
    p = plan_of(case)
    raws = make_storages(case, 64)
    want = ho.pack(m, raws, case.B, case.k, fill=0x77)
    want_sums = ho.checksum(m, want, case.B, case.k)
    host = torch.full((p.packed_bytes,), 0x77, dtype=torch.uint8).pin_memory()
    src = [to_dev(r) for r in raws]
    ssum = torch.zeros(p.num_chunks, dtype=torch.int64, device=DEV)
    hxt.hxt_pack(p, src, host, ssum)
    torch.cuda.synchronize()
    assert np.array_equal(host.numpy(), want)
    dst = [to_dev(np.full(r.size, 0x3C, np.uint8)) for r in raws]
    rsum = torch.zeros_like(ssum)
    hxt.hxt_unpack(p, host, dst, rsum)
    torch.cuda.synchronize()
    dst_o = [np.full(r.size, 0x3C, np.uint8) for r in raws]
    ho.unpack(m, want, case.B, case.k, dst_o)
    for a, b in zip(dst_o, dst):
        assert np.array_equal(b.cpu().numpy(), a)
    assert np.array_equal(ssum.cpu().numpy().view(np.uint64), want_sums)
    assert np.array_equal(rsum.cpu().numpy().view(np.uint64), want_sums)


def test_exchange_stream_argument_errors():
    case = case_by_name("single_lane")
    p = plan_of(case)
    raws = make_storages(case, 1)
    src, dst = [[to_dev(r) for r in raws]], [[to_dev(r) for r in raws]]
    buf = [torch.zeros(p.packed_bytes, dtype=torch.uint8, device=DEV)]
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_exchange_stream(p, hxt.Exchange(src, dst, buf, hxt.HXT_CPU_FORWARD))       # no host buffers
    assert e.value.status == hxt.HXT_EINVAL
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_exchange_stream(p, hxt.Exchange(src, dst, [buf[0][8:]]))                   # misaligned packed
    assert e.value.status == hxt.HXT_EALIGN
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_exchange_stream(p, hxt.Exchange(src, dst, buf, 7))
    assert e.value.status == hxt.HXT_EINVAL
    torch.cuda.synchronize()


def test_config_grad_buckets_full_size_both_paths():
    w = wl.grad_buckets()
    case = case_of(w)
    m = oracle_msg(case)
    p = plan_of(case)
    say("grad buckets: drawing", w.message_bytes, "bytes")
    raws = wl.make_storages(w)
    src = [torch.from_numpy(r).to(DEV) for r in raws]
    nb, C = p.packed_bytes, p.num_chunks
    packed = torch.full((nb,), 0xA5, dtype=torch.uint8, device=DEV)
    sums = torch.zeros(C, dtype=torch.int64, device=DEV)
    hxt.hxt_pack(p, src, packed, sums)
    say("grad buckets: oracle pack")
    want = ho.pack(m, raws, w.chunk_bytes, w.n_lanes, fill=0xA5, nthreads=NT)
    want_sums = ho.checksum(m, want, w.chunk_bytes, w.n_lanes, nthreads=NT)
    got = packed.cpu().numpy()
    assert np.array_equal(got, want)
    assert np.array_equal(sums.cpu().numpy().view(np.uint64), want_sums)
    del got
    strong = torch.zeros(C, 2, dtype=torch.int64, device=DEV)
    hxt.hxt_checksum2(p, packed, strong)
    assert np.array_equal(strong.cpu().numpy().view(np.uint64), ho.checksum2(m, want, w.chunk_bytes, w.n_lanes, nthreads=NT))
    say("grad buckets: cpu-forward leg")
    host = torch.zeros(nb, dtype=torch.uint8).pin_memory()
    recv = torch.full((nb,), 0x5A, dtype=torch.uint8, device=DEV)
    for l in range(w.n_lanes):
        hxt.hxt_stage_d2h(p, l, packed, host)
        hxt.hxt_stage_h2d(p, l, host, recv)
    for path_buf in (packed, recv):
        dst = [torch.zeros_like(s) for s in src]
        rs = torch.zeros(C, dtype=torch.int64, device=DEV)
        hxt.hxt_unpack(p, path_buf, dst, rs)
        torch.cuda.synchronize()
        assert np.array_equal(rs.cpu().numpy().view(np.uint64), want_sums)
        for t, (a, b) in enumerate(zip(src, dst)):
            assert torch.equal(a, b), "tensor %d" % t
    # unspecified tail of the last slot: untouched by pack and by staging
    last = p.chunk_info(C - 1)
    tail0 = last["packed_off"] + last["padded"]
    tail1 = last["packed_off"] + w.chunk_bytes
    assert bool((packed[tail0:tail1] == 0xA5).all()) and bool((recv[tail0:tail1] == 0x5A).all())
    assert bool((host[tail0:tail1] == 0).all())


@pytest.mark.parametrize("hint", [None, 1], ids=["hint_by_size", "all_cold_non_temporal"])
@pytest.mark.parametrize("name", ["qwen_rows_view", "transpose_view", "rows_split_view", "inner_stride_view",
                                  "wide_transpose_view"])
def test_supplementary_strided_messages_full_size(name, hint):
    """hint 1: the packed side non-temporal as well, as in the benchmark's all-cold figures."""
    w = wl.ALL[name]()
    say("supplementary", name, hint)
    round_trip_check(case_of(w), wl.make_storages(w), nthreads=NT, hint=hint)
