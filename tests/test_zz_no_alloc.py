"""The entry point for callers that cannot allocate (hxt_pack_noalloc), through the C ABI, against
hxt_pack on a plan of the same geometry and against the CPU oracle: bit-exact packed bytes (bytes the
layout leaves unspecified keep their old value) and checksums, on calls in a row that share the
library's fixed scratch array, the later ones smaller than the earlier ones."""
import numpy as np
import pytest
import torch

from oracle import hxt_oracle as ho
from paper_2602_18007_amd import hxt

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def both_ways(nbytes, k, B, seed, offset=0):
    """One message of nbytes random bytes: hxt_pack_noalloc vs hxt_pack vs the oracle."""
    say("no-alloc pack", nbytes, "bytes,", k, "lanes,", B, "byte chunks, base offset", offset)
    rng = np.random.default_rng(seed)
    raw = rng.integers(0, 256, size=nbytes, dtype=np.uint8)
    plan = hxt.hxt_plan((nbytes,), None, 1, k, B)
    C, nb = plan.num_chunks, plan.packed_bytes
    buf = torch.empty(nbytes + offset + 16, dtype=torch.uint8, device=DEV)
    src = buf[offset:offset + nbytes]
    src.copy_(torch.from_numpy(raw))

    packed_a = torch.full((nb,), 0xA5, dtype=torch.uint8, device=DEV)
    sums_a = torch.full((C,), -1, dtype=torch.int64, device=DEV)
    hxt.hxt_pack(plan, [src], packed_a, sums_a)

    packed_b = torch.full((nb,), 0xA5, dtype=torch.uint8, device=DEV)
    sums_b = torch.full((C,), -3, dtype=torch.int64, device=DEV)
    hxt.hxt_pack_noalloc(src, nbytes, k, B, packed_b, sums_b)
    packed_c = torch.full((nb,), 0xA5, dtype=torch.uint8, device=DEV)
    hxt.hxt_pack_noalloc(src, nbytes, k, B, packed_c, None)          # without checksums: same bytes
    torch.cuda.synchronize()

    assert torch.equal(packed_a, packed_b), "packed bytes differ from hxt_pack"
    assert torch.equal(sums_a, sums_b), "checksums differ from hxt_pack"
    assert torch.equal(packed_a, packed_c)
    m = ho.Message([ho.TensorSpec((nbytes,), (1,), 1)])
    want = ho.pack(m, [raw], B, k, fill=0xA5, nthreads=8)
    assert np.array_equal(packed_b.cpu().numpy(), want), "packed bytes differ from the oracle"
    assert np.array_equal(sums_b.cpu().numpy().view(np.uint64), ho.checksum(m, want, B, k, nthreads=8))


def test_no_alloc_pack_matches_pack_on_calls_in_a_row():
    # chunks of 256 tiles (accumulators fan out), ragged tail, not a multiple of 16 bytes
    both_ways(9 * 1024 * 1024 + 4 * 4096 + 81, 2, 4 << 20, 1)
    # smaller: the benchmark's 1 MiB chunks over 4 lanes, 5.x chunks
    both_ways(5 * 1024 * 1024 + 1000, 4, 1 << 20, 2)
    # smaller still: fewer chunks than lanes, then a tensor that is only byte aligned
    both_ways(1000, 8, 256, 3)
    both_ways(70001, 3, 4096, 4, offset=3)
    # and a large one again after the small ones (stale slots of earlier geometries must not matter)
    both_ways(32 << 20, 4, 1 << 20, 5)


def test_no_alloc_pack_rejects_what_the_scratch_cannot_serve():
    n = 5000 * 256                                           # 5000 chunks of 256 bytes need 10000 slots
    src = torch.zeros(n, dtype=torch.uint8, device=DEV)
    packed = torch.full((n,), 0x11, dtype=torch.uint8, device=DEV)
    sums = torch.full((5000,), 7, dtype=torch.int64, device=DEV)
    with pytest.raises(hxt.HxtError) as e:
        hxt.hxt_pack_noalloc(src, n, 2, 256, packed, sums)
    assert e.value.status == hxt.HXT_EUNSUPPORTED
    torch.cuda.synchronize()
    assert bool((packed == 0x11).all()) and bool((sums == 7).all()), "a rejected call wrote something"
    hxt.hxt_pack_noalloc(src, n, 2, 256, packed, None)       # without checksums no scratch is needed
    torch.cuda.synchronize()
    assert bool((packed == 0).all())
    for bad in (dict(n_lanes=0), dict(chunk_bytes=100), dict(chunk_bytes=0)):
        kw = dict(n_lanes=2, chunk_bytes=256)
        kw.update(bad)
        with pytest.raises(hxt.HxtError) as e:
            hxt.hxt_pack_noalloc(src, n, kw["n_lanes"], kw["chunk_bytes"], packed, None)
        assert e.value.status == hxt.HXT_EINVAL
    hxt.hxt_pack_noalloc(None, 0, 2, 256, None, None)        # empty message: no-op


def test_no_alloc_pack_can_be_captured_in_a_hip_graph_and_replayed():
    """What the entry point is for: a caller under stream capture.  The call records kernels only (its zero-fill
    is a kernel, not a memset node); every replay, with eager work and synchronisations between the replays, must
    give the eager result for the source's contents at that time."""
    n, k, B = 3 * 1024 * 1024 + 4096 + 32, 4, 1 << 20
    plan = hxt.hxt_plan((n,), None, 1, k, B)
    C = plan.num_chunks
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=DEV)
    packed = torch.full((plan.packed_bytes,), 0xA5, dtype=torch.uint8, device=DEV)
    sums = torch.full((C,), -1, dtype=torch.int64, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        hxt.hxt_pack_noalloc(src, n, k, B, packed, sums, side)      # first call on this device: before capture begins
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        hxt.hxt_pack_noalloc(src, n, k, B, packed, sums, side)
    for rep in range(3):
        src.copy_(torch.randint(0, 255, (n,), dtype=torch.uint8, device=DEV))       # eager work between the replays
        want_packed = torch.full_like(packed, 0xA5)
        want_sums = torch.full_like(sums, -2)
        hxt.hxt_pack(plan, [src], want_packed, want_sums)
        packed.fill_(0xA5)
        sums.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(packed, want_packed) and torch.equal(sums, want_sums), "replay %d" % rep
