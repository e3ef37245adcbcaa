"""Pins for the oracle's accumulate arithmetic (CPU only): exact rational arithmetic with a
search over neighbouring bf16 values, hand-worked ties, special values, and NumPy's binary32 add."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import hxt_oracle as ho
from tests.cases import Case, contig, make_storages


def bf16_value(bits: int):
    """Exact value of a bf16 pattern as a Fraction, or 'nan' / '+inf' / '-inf'."""
    s, e, m = bits >> 15, (bits >> 7) & 0xFF, bits & 0x7F
    if e == 0xFF:
        return "nan" if m else ("-inf" if s else "+inf")
    v = Fraction(m, 128) * Fraction(2) ** -126 if e == 0 else (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)
    return -v if s else v


def f32_value(bits: int):
    s, e, m = bits >> 31, (bits >> 23) & 0xFF, bits & 0x7FFFFF
    if e == 0xFF:
        return "nan" if m else ("-inf" if s else "+inf")
    v = Fraction(m, 1 << 23) * Fraction(2) ** -126 if e == 0 else (1 + Fraction(m, 1 << 23)) * Fraction(2) ** (e - 127)
    return -v if s else v


def nearest_bf16_by_search(x: Fraction, negative_zero: bool) -> int:
    """Nearest bf16 to the exact value x, ties to even mantissa, by scanning candidate patterns."""
    if x == 0:
        return 0x8000 if negative_zero else 0
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    lo, hi = 0, 0x7F80                        # magnitudes are ordered like their bit patterns; 0x7F80 stands for 2^128
    mag = lambda b: Fraction(2) ** 128 if b == 0x7F80 else bf16_value(b)
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if mag(mid) <= a:
            lo = mid
        else:
            hi = mid
    dl, dh = a - mag(lo), mag(hi) - a
    pick = lo if dl < dh else hi if dh < dl else (lo if lo % 2 == 0 else hi)
    return sign | pick


def oracle_bf16_add(a: int, b: int) -> int:
    return ho.lib().hxo_add_bf16_bits(a, b)


def test_bf16_rounding_hand_worked_ties():
    # 1.0 = 0x3F80, one bf16 ulp at 1.0 is 2^-7; 2^-8 = 0x3B80 is exactly half an ulp
    assert oracle_bf16_add(0x3F80, 0x3B80) == 0x3F80          # tie -> even mantissa (…0)
    assert oracle_bf16_add(0x3F81, 0x3B80) == 0x3F82          # tie -> even mantissa (…2)
    assert oracle_bf16_add(0x3F80, 0x3B81) == 0x3F81          # just above half -> up
    assert oracle_bf16_add(0x3F80, 0x3B7F) == 0x3F80          # just below half -> down
    assert oracle_bf16_add(0x3F80, 0xBF80) == 0x0000          # x + (-x) = +0
    assert oracle_bf16_add(0x8000, 0x8000) == 0x8000          # -0 + -0 = -0
    assert oracle_bf16_add(0x7F7F, 0x7F7F) == 0x7F80          # overflow -> +inf
    assert oracle_bf16_add(0x7F80, 0xFF80) == 0x7FC0          # inf - inf -> canonical NaN
    assert oracle_bf16_add(0x7FA3, 0x3F80) == 0x7FC0          # NaN in -> canonical NaN out
    assert oracle_bf16_add(0x0001, 0x0001) == 0x0002          # subnormals add exactly
    assert oracle_bf16_add(0x0001, 0x8001) == 0x0000


def test_bf16_add_against_exact_rational_arithmetic():
    rng = np.random.default_rng(11)
    pats = np.concatenate([
        rng.integers(0, 1 << 16, 3000, dtype=np.uint32),
        np.array([0, 0x8000, 1, 0x8001, 0x007F, 0x0080, 0x7F7F, 0xFF7F, 0x7F80, 0xFF80, 0x7FC0, 0x3F80, 0xBF80], np.uint32),
    ])
    a = rng.choice(pats, 6000)
    b = rng.choice(pats, 6000)
    # pairs of close exponents produce the interesting roundings: add some
    near = rng.integers(0x3E00, 0x4100, 3000, dtype=np.uint32)
    a = np.concatenate([a, near, near ^ 0x8000])
    b = np.concatenate([b, rng.integers(0x3A00, 0x4100, 3000, dtype=np.uint32), rng.integers(0x3E00, 0x4100, 3000, dtype=np.uint32)])
    for x, y in zip(a.tolist(), b.tolist()):
        vx, vy = bf16_value(x), bf16_value(y)
        got = oracle_bf16_add(x, y)
        if "nan" in (vx, vy) or {vx, vy} == {"+inf", "-inf"}:
            assert got == 0x7FC0, (hex(x), hex(y))
            continue
        if isinstance(vx, str) or isinstance(vy, str):
            assert got == (0x7F80 if "+inf" in (vx, vy) else 0xFF80)
            continue
        # step 1 of the contract: the exact sum rounded to binary32 (NumPy's float32 add is IEEE)
        s32 = np.array([x << 16], np.uint32).view(np.float32) + np.array([y << 16], np.uint32).view(np.float32)
        sbits = int(s32.view(np.uint32)[0])
        exact = vx + vy
        if (sbits & 0x7F800000) != 0x7F800000:
            # two bf16 values whose exponents differ by at most 16 add exactly in binary32
            if exact != 0 and abs(int(((x >> 7) & 0xFF) or 1) - int(((y >> 7) & 0xFF) or 1)) <= 16:
                assert f32_value(sbits) == exact
        v32 = f32_value(sbits)
        if isinstance(v32, str):
            want = 0x7F80 if v32 == "+inf" else 0xFF80
        else:
            want = nearest_bf16_by_search(v32, negative_zero=bool(sbits >> 31))
        assert got == want, (hex(x), hex(y), hex(got), hex(want))


def test_round_to_bf16_every_halfway_and_neighbour_in_a_binade():
    L = ho.lib()
    for hi in (0x3F80, 0x0000, 0x0080, 0x7F00):            # a normal binade, subnormals, smallest normals, largest binade
        for m in range(0, 128):
            base = (hi + m) << 16
            for low, want_delta in ((0x0000, 0), (0x7FFF, 0), (0x8000, m % 2), (0x8001, 1), (0xFFFF, 1)):
                f = np.array([base | low], np.uint32).view(np.float32)[0]
                want = hi + m + want_delta
                assert L.hxo_round_to_bf16(float(f)) == want, (hex(base | low),)


def test_f32_add_is_numpy_float32_add_with_canonical_nan():
    rng = np.random.default_rng(12)
    a = rng.integers(0, 1 << 32, 20000, dtype=np.uint64).astype(np.uint32)
    b = rng.integers(0, 1 << 32, 20000, dtype=np.uint64).astype(np.uint32)
    b[:5000] = a[:5000] ^ rng.integers(0, 1 << 12, 5000, dtype=np.uint64).astype(np.uint32)     # near cancellations
    with np.errstate(all="ignore"):
        s = (a.view(np.float32) + b.view(np.float32))
    want = np.where(np.isnan(s), np.uint32(0x7FC00000), s.view(np.uint32))
    got = np.array([ho.lib().hxo_add_f32_bits(int(x), int(y)) for x, y in zip(a, b)], np.uint32)
    assert np.array_equal(got, want)


def test_unpack_accumulate_is_elementwise_add_of_the_arriving_logical_tensor():
    # message: a bf16 matrix seen through a padded-pitch view plus an f32 vector; the arriving packed
    # buffer comes from ho.pack of another set of values
    case = Case("acc", (((9, 40), (48, 1), 2), contig((333,), 4)), 3, 512)
    m = ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])
    incoming = make_storages(case, 1)
    local = make_storages(case, 2)
    packed = ho.pack(m, incoming, case.B, case.k)
    before = [x.copy() for x in local]
    ho.unpack_accumulate(m, [ho.KIND_BF16, ho.KIND_F32], packed, case.B, case.k, local)
    # tensor 0: rows of 40 bf16 at pitch 48; bytes in the pitch gap are untouched
    for r in range(9):
        for c in range(48):
            i = (r * 48 + c)
            if i * 2 + 2 > before[0].size:
                break
            old = int(before[0][2 * i]) | int(before[0][2 * i + 1]) << 8
            new = int(local[0][2 * i]) | int(local[0][2 * i + 1]) << 8
            if c < 40:
                inc = int(incoming[0][2 * i]) | int(incoming[0][2 * i + 1]) << 8
                assert new == oracle_bf16_add(old, inc)
            else:
                assert new == old
    a = before[1].view("<u4"); b = incoming[1].view("<u4")
    want = np.array([ho.lib().hxo_add_f32_bits(int(x), int(y)) for x, y in zip(a, b)], np.uint32)
    assert np.array_equal(local[1].view("<u4"), want)
    with pytest.raises(ValueError):
        ho.unpack_accumulate(m, [ho.KIND_F32, ho.KIND_F32], packed, case.B, case.k, local)
