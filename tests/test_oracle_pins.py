"""Pins the CPU oracle to things other than itself (CPU only).

The transfer is an exact rearrangement of bytes, so the pins are: hand-written
layouts (tests/golden/), NumPy's own flattening of a strided view as the
logical stream, memcpy for the degenerate case, closed-form and big-integer
checksums, the round-trip identity, and the inverse map against the forward one.
Each is chosen to fail for one family of plausible mistakes (wrong lane rule,
chunk-major instead of lane-major, first index fastest, a dropped pad, a
byte-swapped word, an off-by-one last chunk ...).
"""
import numpy as np
import pytest

from oracle import hxt_oracle as ho
from paper_2602_18007_amd import workloads as wl
from tests.cases import SMALL_CASES, Case, case_by_name, contig, make_storages
from tests.conftest import read_golden


def msg_of(case: Case) -> ho.Message:
    return ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])


def numpy_stream(case: Case, storages, offsets=None, L=None):
    """Logical stream built with NumPy's own view flattening; offsets/L may be given by hand."""
    parts = []
    pos = 0
    for i, ((shape, strides, esize), raw) in enumerate(zip(case.tensors, storages)):
        start = offsets[i] if offsets is not None else -(-pos // 256) * 256
        parts.append(np.zeros(start - pos, np.uint8))
        if 0 in shape:
            flat = np.zeros(0, np.uint8)
        else:
            dt = np.dtype("V%d" % esize)
            view = np.lib.stride_tricks.as_strided(raw.view(dt), shape=shape, strides=tuple(s * esize for s in strides))
            flat = np.frombuffer(view.tobytes(order="C"), dtype=np.uint8)   # last index fastest
        parts.append(flat)
        pos = start + flat.size
    end = L if L is not None else -(-pos // 256) * 256
    parts.append(np.zeros(end - pos, np.uint8))
    return np.concatenate(parts) if parts else np.zeros(0, np.uint8)


def deal_order(C, k):
    """Chunk numbers in packed order, by literally dealing them into k lists."""
    hands = [[] for _ in range(k)]
    for c in range(C):
        hands[c % k].append(c)
    return [c for h in hands for c in h]


# ---------------------------------------------------------------------------
# 1. hand-written chunk orders
# ---------------------------------------------------------------------------

def golden_orders():
    out = []
    for ln in read_golden("chunk_orders.txt"):
        left, right = ln.split(":")
        C, k = (int(x) for x in left.split())
        out.append((C, k, [int(x) for x in right.split()]))
    return out


@pytest.mark.parametrize("C,k,order", golden_orders())
def test_packed_chunk_order_matches_hand_written(C, k, order):
    B = 256
    case = Case("g", (contig((C * B,), 1),), k, B)
    (raw,) = make_storages(case, 1)
    packed = ho.pack(msg_of(case), [raw], B, k)
    expect = np.concatenate([raw[c * B:(c + 1) * B] for c in order])
    assert packed.size == C * B
    assert np.array_equal(packed, expect)
    assert deal_order(C, k) == order          # the helper used below agrees with the fixture


@pytest.mark.parametrize("C,k,order", golden_orders())
def test_stream_byte_to_packed_position_matches_hand_written_orders(C, k, order):
    # The hand-dealt order says in which slot of the packed buffer a chunk sits; a stream byte keeps its
    # position inside its chunk.  Also with a short last chunk (it still owns a whole slot).
    B = 512
    for L_ in (C * B, (C - 1) * B + 256):
        for c in range(C):
            last = min((c + 1) * B, L_) - 1
            for s in (c * B, c * B + 77, last):
                assert ho.stream_to_packed(L_, B, k, s) == order.index(c) * B + (s - c * B)


def test_stream_byte_to_packed_position_agrees_with_pack():
    # pack moves stream byte s of a one-tensor byte message to exactly that position
    case = Case("g", (contig((7 * 256 + 100,), 1),), 3, 512)
    m = msg_of(case)
    raw = np.arange(case.tensors[0][0][0], dtype=np.uint32).astype(np.uint8)
    packed = ho.pack(m, [raw], 512, 3, fill=0xEE)
    for s in range(raw.size):
        assert packed[ho.stream_to_packed(m.L, 512, 3, s)] == raw[s]


def test_short_last_chunk_keeps_its_full_slot():
    # 5 chunks over 2 lanes, last chunk 256 of 512 bytes: lane 0 holds chunks 0,2,4 and the
    # short chunk 4 still occupies a whole slot, so lane 1 starts at 3*512.
    B, k = 512, 2
    case = Case("g", (contig((4 * 512 + 256,), 1),), k, B)
    (raw,) = make_storages(case, 2)
    packed = ho.pack(msg_of(case), [raw], B, k, fill=0xEE)
    assert packed.size == 5 * 512
    assert np.array_equal(packed[0:512], raw[0:512])
    assert np.array_equal(packed[512:1024], raw[1024:1536])
    assert np.array_equal(packed[1024:1280], raw[2048:2304])
    assert np.all(packed[1280:1536] == 0xEE)                 # unspecified: untouched
    assert np.array_equal(packed[1536:2048], raw[512:1024])
    assert np.array_equal(packed[2048:2560], raw[1536:2048])


# ---------------------------------------------------------------------------
# 2. hand-computed geometry of the benchmark messages and of a worked example
# ---------------------------------------------------------------------------

def golden_geometry():
    rows = []
    for ln in read_golden("config_geometry.txt"):
        f = [x.strip() for x in ln.split("|")]
        rows.append((f[0], int(f[1]), int(f[2]), int(f[3]), int(f[4]), [int(x) for x in f[5].split(",")], int(f[6])))
    return rows


@pytest.mark.parametrize("name,N,B,k,C,per_lane,last", golden_geometry())
def test_benchmark_geometry(name, N, B, k, C, per_lane, last):
    w = wl.ALL[name]()
    assert (w.chunk_bytes, w.n_lanes) == (B, k)
    m = ho.Message([ho.TensorSpec(t.shape, t.strides, t.esize) for t in w.tensors])
    assert m.N == N == w.message_bytes
    assert ho.num_chunks(m, B) == C
    assert [ho.lane_info(m, B, k, l)["n_chunks"] for l in range(k)] == per_lane
    assert ho.chunk_info(m, B, k, C - 1)["padded"] == last
    assert ho.packed_bytes(m, B, k) == C * B
    assert sum(ho.chunk_info(m, B, k, c)["payload"] for c in range(C)) == N


def test_worked_multi_tensor_example():
    g = {ln.split()[0]: [int(x) for x in ln.split()[1:]] for ln in read_golden("multi_tensor_stream.txt")}
    sizes, B = g["sizes"], g["chunk_bytes"][0]
    case = Case("g", tuple(contig((n,), 1) for n in sizes), 2, B)
    m = msg_of(case)
    assert [m.tensor_offset(t) for t in range(3)] == g["offsets"]
    assert m.L == g["stream"][0]
    C = ho.num_chunks(m, B)
    assert [ho.chunk_info(m, B, 2, c)["padded"] for c in range(C)] == g["padded"]
    assert [ho.chunk_info(m, B, 2, c)["payload"] for c in range(C)] == g["payload"]
    # bytes: stream assembled from the hand-written offsets, chunks in dealt order
    raws = make_storages(case, 3)
    stream = numpy_stream(case, raws, offsets=g["offsets"], L=g["stream"][0])
    packed = ho.pack(m, raws, B, 2, fill=0x5A)
    pos = 0
    for c in deal_order(C, 2):
        n = g["padded"][c]
        assert np.array_equal(packed[pos:pos + n], stream[c * B:c * B + n]), c
        assert np.all(packed[pos + n:pos + B] == 0x5A)
        pos += B
    # the gaps really are zero in the packed buffer (chunk 0 is first in lane 0)
    assert np.all(packed[10:256] == 0) and np.all(packed[556:768] == 0)


# ---------------------------------------------------------------------------
# 3. logical order of strided views == NumPy's flattening
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("case", SMALL_CASES, ids=lambda c: c.name)
def test_pack_equals_numpy_flatten_then_deal(case):
    m = msg_of(case)
    raws = make_storages(case, 11)
    stream = numpy_stream(case, raws)
    assert stream.size == m.L
    C = -(-stream.size // case.B)
    packed = ho.pack(m, raws, case.B, case.k, fill=0xC3)
    assert packed.size == C * case.B
    pos = 0
    for c in deal_order(C, case.k):
        piece = stream[c * case.B:(c + 1) * case.B]
        assert np.array_equal(packed[pos:pos + piece.size], piece), (case.name, c)
        assert np.all(packed[pos + piece.size:pos + case.B] == 0xC3)
        pos += case.B


def test_single_lane_contiguous_is_memcpy_plus_zero_tail():
    case = case_by_name("u8_1000_not_256_multiple")
    (raw,) = make_storages(case, 5)
    packed = ho.pack(msg_of(case), [raw], 512, 1, fill=0x77)
    assert packed.size == 1024
    assert packed[:1000].tobytes() == raw.tobytes()
    assert np.all(packed[1000:1024] == 0)


def test_threads_do_not_change_the_result():
    case = case_by_name("mixed_dtypes_multi")
    raws = make_storages(case, 6)
    m = msg_of(case)
    a = ho.pack(m, raws, case.B, case.k, nthreads=1)
    b = ho.pack(m, raws, case.B, case.k, nthreads=4)
    assert np.array_equal(a, b)
    assert np.array_equal(ho.checksum(m, a, case.B, case.k, 1), ho.checksum(m, a, case.B, case.k, 4))


# ---------------------------------------------------------------------------
# 4. round trip, untouched memory, symmetric receive
# ---------------------------------------------------------------------------

def touched_mask(shape, strides, esize, nbytes):
    mask = np.zeros(nbytes, bool)
    if 0 in shape:
        return mask
    idx = np.zeros((), np.int64)
    for s, st in zip(shape, strides):
        idx = idx[..., None] + np.arange(s, dtype=np.int64) * st
    for b in range(esize):
        mask[(idx.ravel() * esize + b)] = True
    return mask


@pytest.mark.parametrize("case", [c for c in SMALL_CASES if c.name != "broadcast_stride0"], ids=lambda c: c.name)
def test_round_trip_identity_and_canary(case):
    m = msg_of(case)
    raws = make_storages(case, 21)
    packed = ho.pack(m, raws, case.B, case.k)
    dst = [np.full(r.size, 0xA7, np.uint8) for r in raws]
    ho.unpack(m, packed, case.B, case.k, dst)
    for (shape, strides, esize), r, d in zip(case.tensors, raws, dst):
        mask = touched_mask(shape, strides, esize, r.size)
        assert np.array_equal(d[mask], r[mask])
        assert np.all(d[~mask] == 0xA7)            # bytes outside the view are not written


def test_unpack_into_other_layout_gives_same_logical_tensor():
    # Send a transposed view, receive into a contiguous tensor of the same shape.
    shape, e = (64, 48), 2
    src = Case("s", ((shape, (1, 64), e),), 2, 512)
    dstc = Case("d", (contig(shape, e),), 2, 512)
    (raw,) = make_storages(src, 8)
    packed = ho.pack(msg_of(src), [raw], 512, 2)
    out = np.zeros(64 * 48 * 2, np.uint8)
    ho.unpack(msg_of(dstc), packed, 512, 2, [out])
    want = raw.view(np.uint16).reshape(48, 64).T
    assert np.array_equal(out.view(np.uint16).reshape(64, 48), want)


# ---------------------------------------------------------------------------
# 5. checksums
# ---------------------------------------------------------------------------

def test_checksum_big_integer_brute_force():
    case = case_by_name("three_tensors_with_gaps")
    m = msg_of(case)
    packed = ho.pack(m, make_storages(case, 31), case.B, case.k)
    sums = ho.checksum(m, packed, case.B, case.k)
    for c in range(ho.num_chunks(m, case.B)):
        info = ho.chunk_info(m, case.B, case.k, c)
        raw = packed[info["packed_off"]:info["packed_off"] + info["padded"]].tobytes()
        big = sum(int.from_bytes(raw[i:i + 4], "little") for i in range(0, len(raw), 4))
        assert int(sums[c]) == big % (1 << 64)


def test_checksum_closed_forms():
    B, k = 1024, 3
    case = Case("z", (contig((5 * B,), 1),), k, B)
    m = msg_of(case)
    zeros = ho.pack(m, [np.zeros(5 * B, np.uint8)], B, k)
    assert np.all(ho.checksum(m, zeros, B, k) == 0)
    ones = ho.pack(m, [np.full(5 * B, 0xFF, np.uint8)], B, k)
    assert [int(x) for x in ho.checksum(m, ones, B, k)] == [(B // 4) * (2**32 - 1)] * 5
    # one byte set: its weight is 256**(position within the word)
    for pos, weight in ((0, 1), (1, 256), (2, 65536), (3, 1 << 24), (4, 1)):
        raw = np.zeros(5 * B, np.uint8)
        raw[2 * B + pos] = 1                       # inside chunk 2
        s = ho.checksum(m, ho.pack(m, [raw], B, k), B, k)
        assert [int(x) for x in s] == [0, 0, weight, 0, 0]


def test_checksum_sum_over_chunks_is_stream_sum_and_wraps_mod_2_64():
    case = case_by_name("ragged_last_chunk_2p5")
    m = msg_of(case)
    raws = make_storages(case, 33)
    packed = ho.pack(m, raws, case.B, case.k)
    stream = numpy_stream(case, raws)
    whole = int(stream.view("<u4").astype(object).sum())
    assert sum(int(x) for x in ho.checksum(m, packed, case.B, case.k)) == whole
    # pad bytes are zero, so the stream sum is also the sum of the tensor's own words
    assert whole == int(raws[0].view("<u4").astype(object).sum())


def test_bit_flip_in_flight_shows_in_exactly_one_chunk():
    case = case_by_name("ragged_last_chunk_2p5")
    m = msg_of(case)
    packed = ho.pack(m, make_storages(case, 34), case.B, case.k)
    before = ho.checksum(m, packed, case.B, case.k)
    info = ho.chunk_info(m, case.B, case.k, 1)
    byte, bit = info["packed_off"] + 4 * 10 + 2, 5          # byte 2 of word 10 of chunk 1
    was_set = bool(packed[byte] >> bit & 1)
    packed[byte] ^= 1 << bit
    after = ho.checksum(m, packed, case.B, case.k)
    diff = [int(a) - int(b) for a, b in zip(after, before)]
    delta = 1 << (16 + bit)
    assert diff == [0, -delta if was_set else delta, 0]


# ---------------------------------------------------------------------------
# 6. staging and the inverse map
# ---------------------------------------------------------------------------

def test_staging_copies_used_bytes_of_one_lane_only():
    case = case_by_name("ragged_last_chunk_2p5")      # lanes: chunk 0 | chunk 1 | chunk 2 (512 of 1024 bytes)
    m = msg_of(case)
    packed = ho.pack(m, make_storages(case, 41), case.B, case.k)
    for lane, (lo, hi) in enumerate([(0, 1024), (1024, 2048), (2048, 2560)]):
        host = np.full(packed.size, 0x11, np.uint8)
        ho.stage_lane(m, case.B, case.k, lane, packed, host)
        assert np.array_equal(host[lo:hi], packed[lo:hi])
        untouched = np.ones(packed.size, bool)
        untouched[lo:hi] = False
        assert np.all(host[untouched] == 0x11)
        info = ho.lane_info(m, case.B, case.k, lane)
        assert (info["packed_off"], info["bytes"]) == (lo, hi - lo)


def test_staging_a_run_of_slots_copies_exactly_those_chunks():
    # 7 chunks of 512 bytes over 2 lanes, last chunk 256 bytes: lane 0 holds chunks 0,2,4,6 at 0,512,1024,1536
    # (the last one short), lane 1 holds chunks 1,3,5 at 2048,2560,3072.  Ranges written out by hand.
    case = Case("g", (contig((6 * 512 + 256,), 1),), 2, 512)
    m = msg_of(case)
    packed = ho.pack(m, make_storages(case, 43), case.B, case.k, fill=0x77)
    hand = {(0, 0, 1): [(0, 512)], (0, 1, 2): [(512, 1536)], (0, 2, 2): [(1024, 1536 + 256)], (0, 3, 1): [(1536, 1536 + 256)],
            (1, 0, 3): [(2048, 3584)], (1, 2, 1): [(3072, 3584)], (0, 0, 0): [], (0, 0, 4): [(0, 1536 + 256)]}
    for (lane, first, count), ranges in hand.items():
        host = np.full(packed.size, 0x11, np.uint8)
        ho.stage_slots(m, case.B, case.k, lane, first, count, packed, host)
        touched = np.zeros(packed.size, bool)
        for lo, hi in ranges:
            touched[lo:hi] = True
        assert np.array_equal(host[touched], packed[touched]) and np.all(host[~touched] == 0x11), (lane, first, count)
    for bad in ((0, 3, 2), (1, 0, 4), (2, 0, 1), (0, -1, 1)):
        with pytest.raises(ValueError):
            ho.stage_slots(m, case.B, case.k, *bad, packed, np.zeros_like(packed))
    # all slots of a lane = the lane
    for lane, n in ((0, 4), (1, 3)):
        a, b = np.full(packed.size, 0x22, np.uint8), np.full(packed.size, 0x22, np.uint8)
        ho.stage_slots(m, case.B, case.k, lane, 0, n, packed, a)
        ho.stage_lane(m, case.B, case.k, lane, packed, b)
        assert np.array_equal(a, b)


@pytest.mark.parametrize("name", ["mixed_dtypes_multi", "four_d_mixed", "ragged_last_chunk_2p5", "fewer_chunks_than_lanes"])
def test_inverse_map_agrees_with_forward_pack(name):
    case = case_by_name(name)
    m = msg_of(case)
    raws = make_storages(case, 51)
    packed = ho.pack(m, raws, case.B, case.k, fill=0x3C)
    n_real = 0
    for p in range(packed.size):
        kind, t, off = ho.packed_origin(m, case.B, case.k, p)
        if kind == 1:
            assert packed[p] == raws[t][off]
            n_real += 1
        elif kind == 0:
            assert packed[p] == 0
        else:
            assert packed[p] == 0x3C
    assert n_real == m.N
    assert ho.packed_origin(m, case.B, case.k, packed.size)[0] == -1


def test_lane_balance_and_disjoint_slots():
    rng = np.random.default_rng(7)
    for _ in range(50):
        n = int(rng.integers(1, 40000))
        k = int(rng.integers(1, 12))
        B = 256 * int(rng.integers(1, 9))
        case = Case("r", (contig((n,), 1),), k, B)
        m = msg_of(case)
        C = ho.num_chunks(m, B)
        counts = [ho.lane_info(m, B, k, l)["n_chunks"] for l in range(k)]
        assert sum(counts) == C and max(counts) - min(counts) <= 1
        spans = sorted((ho.chunk_info(m, B, k, c)["packed_off"], ho.chunk_info(m, B, k, c)["padded"]) for c in range(C))
        for (a, la), (b, _) in zip(spans, spans[1:]):
            assert a + la <= b
        assert spans[-1][0] + spans[-1][1] <= ho.packed_bytes(m, B, k)
        assert all(p % 256 == 0 and q % 256 == 0 for p, q in spans)
        assert sum(ho.chunk_info(m, B, k, c)["payload"] for c in range(C)) == n


def test_empty_message():
    case = case_by_name("empty_tensor")
    m = msg_of(case)
    assert (m.N, m.L, ho.num_chunks(m, case.B), ho.packed_bytes(m, case.B, case.k)) == (0, 0, 0, 0)
    assert ho.checksum(m, np.zeros(0, np.uint8), case.B, case.k).size == 0


# ---------------------------------------------------------------------------
# 7. position-weighted second sum
# ---------------------------------------------------------------------------

def test_checksum2_big_integer_brute_force_and_closed_form():
    case = case_by_name("three_tensors_with_gaps")
    m = msg_of(case)
    packed = ho.pack(m, make_storages(case, 61), case.B, case.k)
    both = ho.checksum2(m, packed, case.B, case.k)
    assert np.array_equal(both[:, 0], ho.checksum(m, packed, case.B, case.k))
    for c in range(ho.num_chunks(m, case.B)):
        info = ho.chunk_info(m, case.B, case.k, c)
        raw = packed[info["packed_off"]:info["packed_off"] + info["padded"]].tobytes()
        big = sum((j + 1) * int.from_bytes(raw[4 * j:4 * j + 4], "little") for j in range(len(raw) // 4))
        assert int(both[c, 1]) == big % (1 << 64)
    # all-0xFF chunk of W words: (2^32 - 1) * W (W + 1) / 2
    B, k = 2048, 2
    z = Case("z", (contig((3 * B,), 1),), k, B)
    mz = msg_of(z)
    ones = ho.checksum2(mz, ho.pack(mz, [np.full(3 * B, 0xFF, np.uint8)], B, k), B, k)
    W = B // 4
    assert [int(x) for x in ones[:, 1]] == [((2**32 - 1) * W * (W + 1) // 2) % 2**64] * 3
    # one byte set in word j of chunk 1 (byte 1 of the word): weight (j + 1) * 256
    raw = np.zeros(3 * B, np.uint8)
    raw[B + 4 * 37 + 1] = 1
    one = ho.checksum2(mz, ho.pack(mz, [raw], B, k), B, k)
    assert [[int(a), int(b)] for a, b in one] == [[0, 0], [256, 38 * 256], [0, 0]]


def test_checksum2_sees_words_that_changed_places():
    case = case_by_name("ragged_last_chunk_2p5")
    m = msg_of(case)
    packed = ho.pack(m, make_storages(case, 62), case.B, case.k)
    before = ho.checksum2(m, packed, case.B, case.k)
    info = ho.chunk_info(m, case.B, case.k, 1)
    w = packed[info["packed_off"]:info["packed_off"] + info["padded"]].view("<u4")
    i, j = 5, 200
    wi, wj = int(w[i]), int(w[j])
    assert wi != wj
    w[i], w[j] = wj, wi
    after = ho.checksum2(m, packed, case.B, case.k)
    assert np.array_equal(after[:, 0], before[:, 0])                    # the plain sum is blind to it
    diff = (int(after[1, 1]) - int(before[1, 1])) % 2**64
    assert diff == ((j - i) * (wi - wj)) % 2**64 and diff != 0
    assert np.array_equal(after[[0, 2], 1], before[[0, 2], 1])
