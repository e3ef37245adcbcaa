#!/usr/bin/env python3
"""Benchmark of the pipeline-boundary transfer hot path on one MI355X.

A step is one pass of the whole device-direct path over one batch of synthetic
input: the messages of the workload (default: the LLaMA-8B-shaped boundary, a
forward activation and a backward activation gradient, bf16 [4096,1,4096], one
plan each) are packed with send-side checksums by one batched call, then
unpacked with receive-side checksums by another.  Inputs are resident in HBM
before the timed region.  Buffer sets are rotated so that the working set is
several times the 256 MB last-level cache: the figures are cold.

Prints ONE JSON line.  `value` is the HBM traffic the pack and unpack kernels
must move (read N + write N each) divided by wall time over the timed steps.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X HBM3E vendor peak
METRIC = "pack+unpack GB/s (% HBM peak); staged round-trip GB/s (% host link)"
# The paper reports no bandwidth for this path, only relative end-to-end training throughput (Section 3.2,
# Performance); quoted as context with the hardware it names (Section 3.1), never as a target.
PAPER_CONTEXT = ("paper, Section 3.2: device-direct mixed training reaches 98.2 % (LLaMA-8B) and 94.4 % (Qwen2-7B) of "
                 "the NVIDIA-homogeneous throughput on 8 x H200 + 8 x MI325X with 8 BlueField-3 NICs per node; no "
                 "figure for pack/unpack or staging bandwidth is given, so vs_baseline is null")
# HBM-side bytes per k_uniform launch on the default workload from rocprofv3 counter passes
# (FETCH_SIZE, WRITE_SIZE, scaled by a plain copy of known size); None = not measured for the current kernel.
TRAFFIC_BYTES_PER_LAUNCH = 134501953


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="llama8b_boundary")
    ap.add_argument("--sets", type=int, default=8, help="rotating buffer sets (cold working set)")
    ap.add_argument("--two-streams", action="store_true",
                    help="issue the messages of a step one by one on separate streams instead of batched calls")
    ap.add_argument("--unbatched", action="store_true", help="one call per message on one stream")
    ap.add_argument("--path", default="device_direct", choices=["device_direct", "cpu_forward"],
                    help="for --workload stream_1f1b: how the packed buffer travels")
    ap.add_argument("--accumulate", action="store_true",
                    help="receive with hxt_unpack_accumulate (old + arriving) instead of hxt_unpack; one call per message")
    ap.add_argument("--tags", action="store_true",
                    help="hxt_pack_seal / hxt_unpack_verify (chunk tags written and checked inside the copies) "
                         "instead of the plain checksums; one call per message")
    ap.add_argument("--no-checksum", action="store_true", help="diagnostic only: copies without checksums")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-staged", action="store_true")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="also run this many plain device copies of one message (known size), so that hardware "
                         "counters collected over the run can be scaled against them")
    return ap.parse_args()


class MessageSet:
    """Device buffers of one message: source tensors, packed buffer, destination tensors, checksum arrays."""

    def __init__(self, torch, w, plan, seed):
        dev = "cuda:0"
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        self.src, self.dst = [], []
        for t in w.tensors:
            n = t.storage_elems
            if w.dist == "bits16":
                x = torch.randint(-32768, 32767, (n,), generator=g, device=dev, dtype=torch.int16).view(torch.bfloat16)
            else:
                x = (torch.randn(n, generator=g, device=dev, dtype=torch.float32) * w.std).to(torch.bfloat16)
            self.src.append(x)
            self.dst.append(torch.zeros_like(x))
        self.packed = torch.empty(max(plan.packed_bytes, 256), dtype=torch.uint8, device=dev)
        self.send_sums = torch.zeros(max(plan.num_chunks, 1), dtype=torch.int64, device=dev)
        self.recv_sums = torch.zeros_like(self.send_sums)
        self.tags = torch.zeros(max(plan.num_chunks, 1) * 64, dtype=torch.uint8, device=dev)
        self.status = torch.zeros(plan.num_chunks + 1, dtype=torch.int32, device=dev)


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this benchmark measures one GPU only (the transfer is per-GPU work with no collective); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2602_18007_amd import hxt
    from paper_2602_18007_amd import workloads as wl

    hxt.lib()                                   # fail loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    w = wl.ALL[a.workload]()
    if w.name == "stream_1f1b":
        print(json.dumps(stream_bench(torch, hxt, w, a)))
        return
    nmsg = w.messages
    plans = [hxt.hxt_plan_multi([(t.shape, t.strides, t.esize) for t in w.tensors], w.n_lanes, w.chunk_bytes)
             for _ in range(nmsg)]                  # independent messages: a plan each
    plan = plans[0]
    N = plan.message_bytes
    a.sets = max(1, min(a.sets, int(12e9 // (3 * N * nmsg))))      # keep the resident working set near 12 GB
    sets = [[MessageSet(torch, w, plan, w.seed + 1000 * s + m * w.seed_step) for m in range(nmsg)]
            for s in range(a.sets)]
    main_stream = torch.cuda.current_stream()
    streams = [torch.cuda.Stream() for _ in range(nmsg)] if a.two_streams else [main_stream] * nmsg
    use_sums = not a.no_checksum

    batched = not (a.two_streams or a.unbatched or a.accumulate or a.tags)
    pack_b = [hxt.Batch(plans, [ms.src for ms in S], [ms.packed for ms in S],
                        [ms.send_sums for ms in S] if use_sums else None) for S in sets]
    unpack_b = [hxt.Batch(plans, [ms.dst for ms in S], [ms.packed for ms in S],
                          [ms.recv_sums for ms in S] if use_sums else None) for S in sets]

    def step(i):
        if batched:
            hxt.hxt_pack_batch(pack_b[i % a.sets], main_stream)
            hxt.hxt_unpack_batch(unpack_b[i % a.sets], main_stream)
            return
        for m, ms in enumerate(sets[i % a.sets]):
            st = streams[m]
            if a.tags:                                   # sequence number = step, micro-batch id = message
                hxt.hxt_pack_seal(plans[m], ms.src, ms.packed, i, m, ms.tags, st)
                hxt.hxt_unpack_verify(plans[m], ms.packed, ms.tags, i, m, ms.dst, ms.status, st)
                continue
            hxt.hxt_pack(plans[m], ms.src, ms.packed, ms.send_sums if use_sums else None, st)
            recv = hxt.hxt_unpack_accumulate if a.accumulate else hxt.hxt_unpack
            recv(plans[m], ms.packed, ms.dst, ms.recv_sums if use_sums else None, st)

    def fence():
        if a.two_streams:
            for st in streams:
                main_stream.wait_stream(st)
        torch.cuda.synchronize()

    for i in range(a.calibration_copies):                 # plain copies: read N, write N each
        ms = sets[i % a.sets][0]
        ms.dst[0].copy_(ms.src[0])
    for i in range(a.warmup):
        step(i)
    fence()
    # HIP events on the launch streams bracket the timed region: their elapsed time is GPU time
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in set(streams)]
    t0 = time.perf_counter()
    for (e0, _), st in zip(ev, dict.fromkeys(streams)):
        e0.record(st)
    for i in range(a.steps):
        step(a.warmup + i)
    for (_, e1), st in zip(ev, dict.fromkeys(streams)):
        e1.record(st)
    fence()
    t1 = time.perf_counter()
    sec = t1 - t0
    gpu_ms = max(e0.elapsed_time(e1) for e0, e1 in ev)
    # pack: read N + write N; unpack: the same; accumulate: read N arriving + read N old + write N
    step_bytes = (5 if a.accumulate else 4) * N * nmsg
    gbps = step_bytes * a.steps / sec / 1e9

    # correctness of what was just timed: round trip identity and send == receive checksums
    for ms in sets[(a.warmup + a.steps - 1) % a.sets]:
        for s_, d_ in zip(ms.src, ms.dst):
            if not a.accumulate:
                assert torch.equal(s_.view(torch.int16), d_.view(torch.int16)), "round trip mismatch in the timed run"
        if a.tags:
            assert not bool(ms.status.any()), "a chunk was rejected in the timed run"
        elif use_sums:
            assert torch.equal(ms.send_sums, ms.recv_sums), "checksum mismatch in the timed run"

    # dominant kernel: hxt::k_uniform (pack and unpack instantiations); a launch moves 2N algorithmic bytes
    # (read N, write N) for every message it serves.  Average launch duration = GPU time of the timed
    # region (HIP events on the launch stream) / launches in it; the launches are back to back.
    uniform = plan.num_tensors == 1 and plan.tensor_kind(0) == "contig"
    per_launch = min(nmsg, 4) if batched and uniform else 1       # messages served by one launch
    kinds = sorted({plan.tensor_kind(t) for t in range(plan.num_tensors)} - {"none"})
    kernel = ("hxt::k_uniform_tag" if a.tags else "hxt::k_uniform") if uniform else " + ".join("hxt::k_" + k for k in kinds)
    default_run = w.name == "llama8b_boundary" and batched and use_sums
    launches = 2 * nmsg * a.steps // per_launch
    launch_ms = gpu_ms / (launches if not a.two_streams else launches / nmsg)
    launch_bytes = (2.5 if a.accumulate else 2) * N * per_launch      # accumulate: mean of a 2N pack and a 3N receive
    achieved = launch_bytes / (launch_ms * 1e-3) / 1e9
    out = {
        "metric": METRIC if not a.accumulate else "pack+accumulate GB/s",
        "value": round(gbps, 1),                       # the metric's first figure; its second is in "staged"
        "value_of": "pack+unpack GB/s" if not a.accumulate else "pack+accumulate GB/s",
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(sec / a.steps * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": w.name, "note": w.note, "message_bytes": N, "messages_per_step": nmsg,
                   "n_lanes": w.n_lanes, "chunk_bytes": w.chunk_bytes, "path": "device_direct",
                   "checksums": "chunk tags sealed and verified inside the copies" if a.tags else
                   ("fused send+receive" if use_sums else "off"),
                   "buffer_sets": a.sets, "cache_state": "cold (rotating sets)" if a.sets * 3 * N * nmsg > 1e9 else
                   "working set %d MiB" % (a.sets * 3 * N * nmsg >> 20),
                   "streams": nmsg if a.two_streams else 1,
                   "issue": "batched calls (one launch packs all messages of the step, one unpacks them)" if batched
                   else "one call per message"},
        "pct_hbm_peak": round(100 * gbps / HBM_PEAK_GBPS, 2),
        "roofline": {"bound": "hbm", "kernel": kernel + " (pack and unpack instantiations%s)" % (", fused checksum" if use_sums else ""),
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": TRAFFIC_BYTES_PER_LAUNCH if default_run else None,
                     "bytes_per_launch": launch_bytes, "avg_launch_ms": round(launch_ms, 6),
                     "launches": launches, "gpu_ms_timed_region": round(gpu_ms, 4)},
    }
    out["paper_context"] = PAPER_CONTEXT
    if not a.calibration_copies:        # a counter pass must see no other copy kernels than its calibration copies
        out["roofline"]["plain_copy"] = plain_copy_ceiling(torch, int(launch_bytes) // 2)
    if not a.no_staged:
        out["staged"] = staged_round_trip(torch, hxt, w, plans, sets[0])
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


def plain_copy_ceiling(torch, nbytes):
    """The runtime's own device-to-device copy of as many bytes as one launch of the dominant kernel reads
    (and writes), cold (rotating buffers), back to back on one stream: the machine's practical ceiling for a
    launch of that size, printed beside the kernel's figure."""
    dev = "cuda:0"
    nsets = max(2, min(8, int(3e9 // (2 * nbytes))))
    src = [torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(nsets)]
    dst = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(nsets)]
    iters = 64
    for i in range(8):
        dst[i % nsets].copy_(src[i % nsets])
    torch.cuda.synchronize()
    best = 1e9
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            dst[i % nsets].copy_(src[i % nsets])
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / iters)
    return {"what": "torch device-to-device copy, same bytes per launch, cold", "bytes_read_plus_written": 2 * nbytes,
            "avg_ms": round(best, 6), "gbps": round(2 * nbytes / (best * 1e-3) / 1e9, 1)}


def _wall(fn):
    t0 = time.perf_counter()
    fn()
    return time.perf_counter() - t0


def stream_bench(torch, hxt, w, a):
    """The micro-batch stream: one step = all micro-batches through hxt_exchange_stream (two buffer sets,
    three streams), so that pack of one micro-batch overlaps staging/unpack of the previous ones."""
    dev = "cuda:0"
    t = w.tensors[0]
    plan = hxt.hxt_plan(t.shape, t.strides, t.esize, w.n_lanes, w.chunk_bytes)
    N, C, nb, nmsg = plan.message_bytes, plan.num_chunks, plan.packed_bytes, w.messages
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed)
    src = [[(torch.randn(t.storage_elems, generator=g, device=dev) * w.std).to(torch.bfloat16)] for _ in range(nmsg)]
    dst = [[torch.zeros_like(s_[0])] for s_ in src]
    fwd = a.path == "cpu_forward"
    send = [torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(2)]
    recv = [torch.empty(nb, dtype=torch.uint8, device=dev) for _ in range(2)] if fwd else None
    host = [torch.empty(nb, dtype=torch.uint8).pin_memory() for _ in range(2)] if fwd else None
    s_send = torch.zeros((nmsg, C), dtype=torch.int64, device=dev)
    s_recv = torch.zeros_like(s_send)
    streams = [torch.cuda.Stream() for _ in range(3)]
    tag_kw = {}
    if a.tags:                                         # chunk tags instead of the plain checksums
        tag_dev = lambda: [torch.zeros(C * 64, dtype=torch.uint8, device=dev) for _ in range(2)]
        status = torch.zeros((nmsg, C + 1), dtype=torch.int32, device=dev)
        tag_kw = dict(tags_send=tag_dev(), tags_recv=tag_dev() if fwd else None,
                      tags_pinned=[torch.zeros(C * 64, dtype=torch.uint8).pin_memory() for _ in range(2)] if fwd else None,
                      status=status, seq_base=1)
    plain = not (a.no_checksum or a.tags)
    x = hxt.Exchange(src, dst, send, hxt.HXT_CPU_FORWARD if fwd else hxt.HXT_DEVICE_DIRECT, recv, host,
                     s_send if plain else None, s_recv if plain else None, *streams, **tag_kw)
    steps = a.steps if not fwd else max(1, min(a.steps, 20))
    warm = a.warmup if not fwd else max(1, min(a.warmup, 2))

    def one_pass():
        # One schedule's worth of micro-batches, then a host sync (as at the end of a training
        # iteration): the next pass reuses the buffer sets.
        hxt.hxt_exchange_stream(plan, x)
        torch.cuda.synchronize()

    torch.cuda.synchronize()                          # inputs were drawn on the default stream
    for _ in range(warm):
        one_pass()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_pass()
    sec = time.perf_counter() - t0
    for s_, d_ in zip(src, dst):
        assert torch.equal(s_[0].view(torch.int16), d_[0].view(torch.int16)), "round trip mismatch"
    if a.tags:
        assert not bool(status.any()), "a chunk was rejected in the timed run"
    elif not a.no_checksum:
        assert torch.equal(s_send, s_recv)
    gbps = 4 * N * nmsg * steps / sec / 1e9
    out = {"metric": METRIC, "value": round(gbps, 1), "value_of": "pack+unpack GB/s", "unit": "GB/s", "n_gpus": 1, "steps": steps,
           "warmup": warm, "ms_per_step": round(sec / steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "u32", "data": "synthetic",
           "config": {"workload": w.name, "note": w.note, "message_bytes": N, "messages_per_step": nmsg,
                      "n_lanes": w.n_lanes, "chunk_bytes": w.chunk_bytes, "path": a.path, "buffer_sets": 2,
                      "streams": 3, "checksums": "chunk tags sealed and verified inside the copies" if a.tags else
                      ("off" if a.no_checksum else "fused send+receive"),
                      "cache_state": "cold (%d MiB of sources per pass)" % (N * nmsg >> 20)},
           "pct_hbm_peak": round(100 * gbps / HBM_PEAK_GBPS, 2),
           "us_per_micro_batch": round(sec / steps / nmsg * 1e6, 2)}
    if fwd:
        out["staged_gbps_per_direction"] = round(N * nmsg * steps / sec / 1e9, 2)
    return out


def staged_round_trip(torch, hxt, w, plans, msgs):
    """CPU-forwarding leg: D2H lane by lane on one stream, H2D of each lane on another as soon as its D2H is
    done (events), through one pinned buffer per message; against a pinned hipMemcpy probe (256 MiB, each
    direction alone and both at once on separate buffers) taken in the same run."""
    dev = "cuda:0"
    k, N = w.n_lanes, plans[0].message_bytes
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()

    def best_of(fn, reps=10):
        fn()
        best = 1e9
        for _ in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            best = min(best, time.perf_counter() - t0)
        return best

    # link probe
    P = 256 << 20
    d_a, d_b = (torch.empty(P, dtype=torch.uint8, device=dev) for _ in range(2))
    h_a, h_b = (torch.empty(P, dtype=torch.uint8).pin_memory() for _ in range(2))

    def p_d2h():
        with torch.cuda.stream(s1):
            h_a.copy_(d_a, non_blocking=True)

    def p_h2d():
        with torch.cuda.stream(s2):
            d_b.copy_(h_b, non_blocking=True)

    def p_both():
        p_d2h()
        p_h2d()

    # Both directions together first: the HIP runtime in this process keeps using one DMA engine for
    # two streams whose first copies ran one after the other (57 GB/s for both directions instead of 97).
    t_both = best_of(p_both)

    host = [torch.empty(p.packed_bytes, dtype=torch.uint8).pin_memory() for p in plans]
    recv = [torch.empty(p.packed_bytes, dtype=torch.uint8, device=dev) for p in plans]

    def round_trip(which):
        for m in which:
            for l in range(k):
                hxt.hxt_stage_d2h(plans[m], l, msgs[m].packed, host[m], s1)
                ev = torch.cuda.Event()
                ev.record(s1)
                s2.wait_event(ev)
                hxt.hxt_stage_h2d(plans[m], l, host[m], recv[m], s2)

    t_one = best_of(lambda: round_trip([0]))
    t_all = best_of(lambda: round_trip(range(len(plans))))
    for m in range(len(plans)):
        assert torch.equal(recv[m], msgs[m].packed[:plans[m].packed_bytes]), "staged bytes differ"
    # the host-to-host hop of the chain (pinned to pinned), one thread per lane and one thread
    hop_dst = torch.empty(plans[0].packed_bytes, dtype=torch.uint8).pin_memory()
    t_hop = min(_wall(lambda: hxt.hxt_host_forward(plans[0], -1, host[0], hop_dst, 0)) for _ in range(5))
    t_hop1 = min(_wall(lambda: hxt.hxt_host_forward(plans[0], -1, host[0], hop_dst, 1)) for _ in range(5))
    assert torch.equal(hop_dst, host[0])
    t_d2h, t_h2d = best_of(p_d2h), best_of(p_h2d)
    link = min(P / t_d2h, P / t_h2d) / 1e9
    del d_a, d_b, h_a, h_b
    one, all_ = N / t_one / 1e9, N * len(plans) / t_all / 1e9
    return {"round_trip_gbps": round(one, 2), "pct_host_link": round(100 * one / link, 1),
            "step_round_trip_gbps": round(all_, 2), "step_pct_host_link": round(100 * all_ / link, 1),
            "messages_in_step": len(plans), "lanes": k, "message_bytes": N,
            "host_hop_gbps": round(N / t_hop / 1e9, 2), "host_hop_one_thread_gbps": round(N / t_hop1 / 1e9, 2),
            "probe_bytes": P, "probe_d2h_gbps": round(P / t_d2h / 1e9, 2), "probe_h2d_gbps": round(P / t_h2d / 1e9, 2),
            "probe_bidir_gbps": round(2 * P / t_both / 1e9, 2),
            "bidir_pct": round(100 * (2 * N * len(plans) / t_all / 1e9) / (2 * P / t_both / 1e9), 1),
            "note": "best of 10, wall clock around a synchronised region; round trip = first D2H start to last "
                    "H2D end of one message; step = all messages of the step pipelined lane by lane; "
                    "link = min one-direction probe; bidir_pct = 2 x step rate / both-directions probe"}


def cpu_baseline(w):
    """The CPU oracle, as it stands, on the same message geometry: one full step."""
    import numpy as np

    from oracle import hxt_oracle as ho
    from paper_2602_18007_amd import workloads as wl

    cores = ho.max_threads()
    m = ho.Message([ho.TensorSpec(t.shape, t.strides, t.esize) for t in w.tensors])
    raws = wl.make_storages(w, 0)
    B, k = w.chunk_bytes, w.n_lanes
    dst = [np.zeros_like(r) for r in raws]
    packed = np.zeros(ho.packed_bytes(m, B, k), np.uint8)
    t0 = time.perf_counter()
    reps = 0
    while True:
        ho.pack(m, raws, B, k, packed=packed, nthreads=cores)
        s_send = ho.checksum(m, packed, B, k, nthreads=cores)
        ho.unpack(m, packed, B, k, dst, nthreads=cores)
        s_recv = ho.checksum(m, packed, B, k, nthreads=cores)
        reps += 1
        if time.perf_counter() - t0 > 10.0:
            break
    sec = time.perf_counter() - t0
    assert np.array_equal(s_send, s_recv) and all(np.array_equal(a, b) for a, b in zip(raws, dst))
    t1 = time.perf_counter()                              # the same pass on one core
    ho.pack(m, raws, B, k, packed=packed, nthreads=1)
    ho.checksum(m, packed, B, k, nthreads=1)
    ho.unpack(m, packed, B, k, dst, nthreads=1)
    ho.checksum(m, packed, B, k, nthreads=1)
    sec1 = time.perf_counter() - t1
    return {"value": round(4 * m.N * reps / sec / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": "%d message(s) of %d bytes: pack + checksum + unpack + checksum, %.1f s" % (reps, m.N, sec),
            "one_core_value": round(4 * m.N / sec1 / 1e9, 3)}


if __name__ == "__main__":
    main()
