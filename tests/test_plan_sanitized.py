"""The host planner under AddressSanitizer and UndefinedBehaviorSanitizer: a program of its own
(tests/host/plan_sanitized_main.cpp + the table interpreter + the planner source) runs the small cases, mid-size
strided messages and random views over heap buffers of exactly the size a plan may touch, and compares
with what the CPU oracle packed and unpacked."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import hxt_oracle as ho
from tests.cases import SMALL_CASES, Case, make_storages, random_view, storage_bytes

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SIZE_CODE = {1: 1, 2: 3, 4: 4, 8: 5}


def injective(shape, strides):
    """Brute force on small views: no two index tuples share an element offset."""
    if 0 in shape:
        return True
    offs = np.zeros(1, np.int64)
    for s, st in zip(shape, strides):
        offs = (offs[:, None] + np.arange(s, dtype=np.int64)[None, :] * st).reshape(-1)
    return np.unique(offs).size == offs.size


def encode(case, tile, seed):
    m = ho.Message([ho.TensorSpec(tuple(s), tuple(st), e) for (s, st, e) in case.tensors])
    raws = make_storages(case, seed)
    want = ho.pack(m, raws, case.B, case.k, fill=0x99)
    unpack_ok = all(injective(s, st) for (s, st, _) in case.tensors)
    out = [struct.pack("<IIQII", len(case.tensors), case.k, case.B, tile, int(unpack_ok))]
    for (shape, strides, e), raw in zip(case.tensors, raws):
        pad = [0] * (8 - len(shape))
        out.append(struct.pack("<II8q8qQ", len(shape), SIZE_CODE[e], *shape, *pad, *strides, *pad, raw.size))
        out.append(raw.tobytes())
    out.append(struct.pack("<Q", want.size))
    out.append(want.tobytes())
    if unpack_ok:
        dst = [np.full(r.size, 0x42, np.uint8) for r in raws]
        ho.unpack(m, want, case.B, case.k, dst)
        out += [d.tobytes() for d in dst]
    return b"".join(out)


def test_planner_and_its_tables_under_address_and_ub_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2602_18007_amd", "csrc")
    exe = tmp_path / "plan_sanitized"
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-static-libasan", "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"), "-I", csrc,
                    "-o", str(exe), os.path.join(ROOT, "tests", "host", "plan_sanitized_main.cpp"),
                    os.path.join(ROOT, "tests", "host", "plan_interp.cpp"), os.path.join(csrc, "hxt_plan.cpp")], check=True)
    blobs = []
    for case in SMALL_CASES:
        for tile in (256, 1024, 16384):
            blobs.append(encode(case, tile, 77))
    mid = [
        Case("rows_mid", (((300, 2, 112), (112, 300 * 112, 1), 2),), 3, 4096),
        Case("rows_odd_mid", (((257, 100), (128, 1), 2),), 2, 2048),
        Case("transpose_mid", (((200, 150), (1, 200), 2),), 2, 4096),
        Case("transpose_batch_mid", (((3, 70, 90), (70 * 100, 1, 70), 4),), 4, 1024),
        Case("transpose_u8", (((130, 67), (1, 130), 1),), 2, 512),
    ]
    blobs += [encode(c, 2048, 5) for c in mid]
    rng = np.random.default_rng(4711)
    for _ in range(150):
        tensors = tuple(random_view(rng) for _ in range(int(rng.integers(1, 5))))
        if sum(storage_bytes(*t) for t in tensors) > 1_000_000:
            continue
        case = Case("rand", tensors, int(rng.integers(1, 6)), int(rng.choice([256, 512, 1024, 4096, 16384])))
        blobs.append(encode(case, int(rng.choice([256, 1024, 16384])), 9))
    path = tmp_path / "cases.bin"
    path.write_bytes(struct.pack("<I", len(blobs)) + b"".join(blobs))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe), str(path)], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "plan_sanitized: ok, %d cases" % len(blobs) in r.stdout
