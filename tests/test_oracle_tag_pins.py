"""Pins for the oracle's chunk tags (seal / verify): a worked example written out by hand
(tests/golden/chunk_tags.txt), an independent decoding of the records with a NumPy structured
dtype against values derived in the test with Python integers, and planted faults that must be
reported in exactly the chunk and the bit they belong to."""
import numpy as np
import pytest

from oracle import hxt_oracle as ho
from tests.cases import SMALL_CASES, make_storages
from tests.conftest import read_golden

TAG = np.dtype([("magic", "<u4"), ("chunk", "<u4"), ("lane", "<u4"), ("slot", "<u4"), ("seq", "<u8"),
                ("micro_batch", "<u4"), ("C", "<u4"), ("padded", "<u8"), ("sum", "<u8"), ("wsum", "<u8"),
                ("zero", "<u8")])
M64 = (1 << 64) - 1


def msg_of(case):
    return ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])


def worked_example():
    m = ho.Message([ho.TensorSpec.contiguous((700,), 1)])
    raw = np.zeros(700, np.uint8)
    raw[0:512:4] = 1
    raw[512:700:4] = 2
    return m, ho.pack(m, [raw], 512, 2, fill=0)


def test_record_is_64_bytes():
    assert TAG.itemsize == 64 == ho.TAG_BYTES


def test_worked_example_matches_the_hand_written_bytes():
    m, packed = worked_example()
    tags = ho.seal(m, packed, 512, 2, 0x0102030405060708, 7)
    want = {}
    for ln in read_golden("chunk_tags.txt"):
        head, body = ln.split(":")
        want[int(head.split()[1])] = bytes(int(x, 16) for x in body.split())
    assert len(want) == 2 and all(len(v) == 64 for v in want.values())
    for s in (0, 1):
        assert tags[s].tobytes() == want[s], "tag in slot %d" % s
    assert not ho.verify(m, packed, tags, 512, 2, 0x0102030405060708, 7).any()


@pytest.mark.parametrize("C,k,order", [(3, 2, [0, 2, 1]), (5, 2, [0, 2, 4, 1, 3]), (7, 3, [0, 3, 6, 1, 4, 2, 5]),
                                       (3, 5, [0, 1, 2])])
def test_tags_sit_in_packed_slot_order(C, k, order):
    """Deal chunks round-robin to k lanes, lay the lanes one after another: that is the order of the tags."""
    B = 256
    m = ho.Message([ho.TensorSpec.contiguous((C * B,), 1)])
    raw = np.arange(C * B, dtype=np.uint32).astype(np.uint8)
    packed = ho.pack(m, [raw], B, k, fill=0)
    rec = ho.seal(m, packed, B, k, 1, 2).reshape(-1).view(TAG)
    assert list(rec["chunk"]) == order
    assert list(rec["lane"]) == [c % k for c in order] and list(rec["slot"]) == [c // k for c in order]


@pytest.mark.parametrize("case", SMALL_CASES, ids=lambda c: c.name)
def test_fields_against_python_integers(case):
    m = msg_of(case)
    raws = make_storages(case, 5)
    B, k = case.B, case.k
    packed = ho.pack(m, raws, B, k, fill=0x77)
    seq, mb = 0xFEDCBA9876543210, 0x89ABCDEF
    tags = ho.seal(m, packed, B, k, seq, mb)
    C = -(-m.L // B) if m.N else 0
    assert tags.shape == (C, 64)
    rec = tags.reshape(-1).view(TAG)
    # lane-major slot of chunk c: chunks of lower lanes first, then the chunk's slot in its lane
    per_lane = [len(range(l, C, k)) for l in range(k)]
    for c in range(C):
        lane, slot = c % k, c // k
        s = sum(per_lane[:lane]) + slot
        r = rec[s]
        padded = min(B, m.L - c * B)
        words = packed[s * B:s * B + padded].view("<u4")
        assert r["magic"] == int.from_bytes(b"HXT1", "little")
        assert (r["chunk"], r["lane"], r["slot"], r["C"], r["padded"]) == (c, lane, slot, C, padded)
        assert r["seq"] == seq and r["micro_batch"] == mb and r["zero"] == 0
        assert int(r["sum"]) == sum(int(w) for w in words) & M64
        assert int(r["wsum"]) == sum((j + 1) * int(w) for j, w in enumerate(words)) & M64
    st = ho.verify(m, packed, tags, B, k, seq, mb)
    assert st.size == C + 1 and not st.any()


def planted(case_name="three_tensors_with_gaps"):
    case = next(c for c in SMALL_CASES if c.name == case_name)
    m = msg_of(case)
    raws = make_storages(case, 6)
    packed = ho.pack(m, raws, case.B, case.k, fill=0)
    return case, m, packed, ho.seal(m, packed, case.B, case.k, 41, 3)


def test_wrong_message_is_rejected_in_every_chunk():
    case, m, packed, tags = planted()
    C = tags.shape[0]
    assert C >= 3
    st = ho.verify(m, packed, tags, case.B, case.k, 42, 3)            # stale buffer: previous sequence number
    assert list(st[:C]) == [ho.TAG_BAD_SEQ] * C and st[C] == C
    st = ho.verify(m, packed, tags, case.B, case.k, 41, 4)            # another micro-batch's buffer
    assert list(st[:C]) == [ho.TAG_BAD_MICRO_BATCH] * C and st[C] == C
    st = ho.verify(m, packed, tags, case.B, case.k, 40, 0)
    assert list(st[:C]) == [ho.TAG_BAD_SEQ | ho.TAG_BAD_MICRO_BATCH] * C


def test_damaged_payload_is_rejected_in_its_chunk_only():
    case, m, packed, tags = planted()
    C = tags.shape[0]
    c = 2
    off = ho.chunk_info(m, case.B, case.k, c)["packed_off"]
    bad = packed.copy()
    bad[off + 9] ^= 0x10                                               # one flipped bit
    st = ho.verify(m, bad, tags, case.B, case.k, 41, 3)
    want = [0] * C
    want[c] = ho.TAG_BAD_SUM | ho.TAG_BAD_WSUM
    assert list(st[:C]) == want and st[C] == 1
    w = packed.copy()
    words = w[off:off + 256].view("<u4")
    assert words[3] != words[17]
    words[3], words[17] = int(words[17]), int(words[3])                # two words change places
    st = ho.verify(m, w, tags, case.B, case.k, 41, 3)
    want[c] = ho.TAG_BAD_WSUM
    assert list(st[:C]) == want and st[C] == 1


def test_damaged_or_misplaced_tags_are_rejected():
    case, m, packed, tags = planted()
    C = tags.shape[0]
    t = tags.copy()
    t[1, 0] ^= 0xFF                                                    # magic
    t[0, 56] = 1                                                       # reserved field
    st = ho.verify(m, packed, t, case.B, case.k, 41, 3)
    slot_chunk = tags.reshape(-1).view(TAG)["chunk"]                   # which chunk each slot holds
    want = [0] * C
    want[int(slot_chunk[1])] = ho.TAG_BAD_MAGIC
    want[int(slot_chunk[0])] = ho.TAG_BAD_RESERVED
    assert list(st[:C]) == want and st[C] == 2
    # the tags of two full chunks exchanged: both carry the other's place and the other's sums
    full = [s for s in range(C) if tags.reshape(-1).view(TAG)["padded"][s] == case.B][:2]
    assert len(full) == 2
    t = tags.copy()
    t[full[0]], t[full[1]] = tags[full[1]], tags[full[0]]
    st = ho.verify(m, packed, t, case.B, case.k, 41, 3)
    for s in full:
        assert st[int(slot_chunk[s])] == ho.TAG_BAD_PLACE | ho.TAG_BAD_SUM | ho.TAG_BAD_WSUM
    assert st[C] == 2
    # a tag whose length field lies
    t = tags.copy()
    t.reshape(-1).view(TAG)["padded"][0] += 256
    st = ho.verify(m, packed, t, case.B, case.k, 41, 3)
    assert st[int(slot_chunk[0])] == ho.TAG_BAD_PLACE and st[C] == 1


@pytest.mark.parametrize("field,want_bit", [("chunk", "PLACE"), ("lane", "PLACE"), ("slot", "PLACE"), ("C", "PLACE"),
                                             ("padded", "PLACE"), ("magic", "MAGIC"), ("seq", "SEQ"),
                                             ("micro_batch", "MICRO_BATCH"), ("sum", "SUM"), ("wsum", "WSUM"),
                                             ("zero", "RESERVED")])
def test_every_field_of_the_tag_is_checked(field, want_bit):
    """One field of one tag changed by one: exactly that field's bit, in exactly that chunk."""
    case, m, packed, tags = planted()
    C = tags.shape[0]
    t = tags.copy()
    rec = t.reshape(-1).view(TAG)
    s = 1                                                              # the tag in packed slot 1
    rec[field][s] += 1
    st = ho.verify(m, packed, t, case.B, case.k, 41, 3)
    c = int(tags.reshape(-1).view(TAG)["chunk"][s])
    want = [0] * C
    want[c] = getattr(ho, "TAG_BAD_" + want_bit)
    assert list(st[:C]) == want and st[C] == 1


def test_empty_message_has_no_tags():
    m = ho.Message([ho.TensorSpec((0, 16), (16, 1), 2)])
    packed = np.zeros(0, np.uint8)
    tags = ho.seal(m, packed, 256, 2, 1, 1)
    assert tags.shape == (0, 64)
    assert list(ho.verify(m, packed, tags, 256, 2, 1, 1)) == [0]
