#!/usr/bin/env python3
"""Benchmark of the pipeline-boundary transfer hot path on one MI355X.

A step is one pass of the whole device-direct path over one batch of synthetic input: the messages
of the LLaMA-8B-shaped boundary (a forward activation and a backward activation gradient, bf16
[4096,1,4096], one plan each) are packed with send-side checksums by one batched call, then unpacked
with receive-side checksums by another.  Inputs are resident in HBM before the timed region.

The step is timed in several regions, each `repeats` blocks of `steps` steps back to back between
one pair of host synchronisations (HIP events between the blocks give every block's GPU time):
  cold          one stream, every access non-temporal: all 4N bytes per message come from and go
                to HBM, and a kernel has the machine to itself.  `roofline` is this region's.
  llc           one stream, packed buffer cacheable: unpack re-reads it from the 256 MB
                last-level cache ~25 us after pack wrote it (loopback only: at a real boundary the
                reader of a packed buffer is the NIC or the peer).  Reported, never the headline.
  chains_*      the same steps dealt alternately onto two streams with a plan set each, so that the
                kernels of consecutive steps overlap and fill each other's ramp-up and tail.  `value` and
                `ms_per_step` are chains_cold's: whole-job throughput, all-cold (kernel durations in these
                regions are not comparable with a roofline because the kernels share the machine).
Then every other benchmark message is timed once (`configs`), the CPU-forwarding path is timed
against a pinned-copy probe taken in the same run (`staged`), and the CPU oracle is timed on the
host cores (`cpu_baseline`).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
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
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "k_uniform_llama8b_boundary.md")
DEV = "cuda:0"
REGIONS = ("cold", "llc", "chains_cold", "chains_llc")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--repeats", type=int, default=0,
                    help="blocks of --steps steps per timed region (0: as many as make about 2000 steps, at least 5)")
    ap.add_argument("--workload", default="llama8b_boundary", help="the message the headline step is made of")
    ap.add_argument("--sets", type=int, default=8, help="rotating buffer sets (cold sources and destinations)")
    ap.add_argument("--regions", default=",".join(REGIONS),
                    help="which timed regions of the headline step to run (a profiler run names one)")
    ap.add_argument("--unbatched", action="store_true", help="one call per message instead of the batched calls")
    ap.add_argument("--tags", action="store_true",
                    help="chunk tags sealed and verified inside the copies instead of the plain checksums")
    ap.add_argument("--accumulate", action="store_true",
                    help="receive with hxt_unpack_accumulate_batch (old + arriving)")
    ap.add_argument("--no-checksum", action="store_true", help="diagnostic only: copies without checksums")
    ap.add_argument("--path", default="device_direct", choices=["device_direct", "cpu_forward"],
                    help="for --workload stream_1f1b")
    ap.add_argument("--window", type=int, default=-1,
                    help="for --workload stream_1f1b --path cpu_forward: micro-batches per hxt_exchange_stream call, the "
                         "streams being drained between calls (0: all at once; default 16)")
    ap.add_argument("--direct-mode", type=int, default=0, help="for --workload stream_1f1b: hxt_direct_mode_t (0 automatic)")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-message entries")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-staged", action="store_true")
    ap.add_argument("--calibration-copies", type=int, default=0,
                    help="also run this many plain device copies of one message (known size), so that hardware "
                         "counters collected over the run can be scaled against them")
    return ap.parse_args()


# ---------------------------------------------------------------------------------------------
# device-direct step of one workload
# ---------------------------------------------------------------------------------------------

class MessageSet:
    """Device buffers of one message: source tensors, packed buffer, destination tensors, checksum arrays."""

    def __init__(self, torch, w, plan, seed):
        g = torch.Generator(device=DEV)
        g.manual_seed(seed)
        self.src, self.dst = [], []
        for t in w.tensors:
            n = t.storage_elems
            if w.dist == "bits16":
                x = torch.randint(-32768, 32767, (n,), generator=g, device=DEV, dtype=torch.int16).view(torch.bfloat16)
            else:
                x = (torch.randn(n, generator=g, device=DEV, dtype=torch.float32) * w.std).to(torch.bfloat16)
            self.src.append(x)
            self.dst.append(torch.zeros_like(x))
        self.packed = torch.empty(max(plan.packed_bytes, 256), dtype=torch.uint8, device=DEV)
        self.send_sums = torch.zeros(max(plan.num_chunks, 1), dtype=torch.int64, device=DEV)
        self.recv_sums = torch.zeros_like(self.send_sums)
        self.tags = torch.zeros(max(plan.num_chunks, 1) * 64, dtype=torch.uint8, device=DEV)
        self.status = torch.zeros(plan.num_chunks + 1, dtype=torch.int32, device=DEV)


class DirectStep:
    """pack -> unpack of all messages of a workload's step, with rotating buffer sets."""

    def __init__(self, torch, hxt, w, sets, mode="sums", batched=True, budget=12e9):
        self.torch, self.hxt, self.w, self.mode, self.batched = torch, hxt, w, mode, batched
        self.nmsg = w.messages if w.name != "stream_1f1b" else 1
        dt = torch.bfloat16
        descr = [(t.shape, t.strides, dt) for t in w.tensors]
        # two plan sets: messages that overlap on two streams need their own checksum accumulators
        self.plans = [[hxt.hxt_plan_multi(descr, w.n_lanes, w.chunk_bytes) for _ in range(self.nmsg)] for _ in range(2)]
        p0 = self.plans[0][0]
        self.N, self.C = p0.message_bytes, p0.num_chunks
        store = sum(t.storage_elems * t.esize for t in w.tensors)
        self.sets = max(2, min(sets, int(budget // ((2 * store + p0.packed_bytes) * self.nmsg))))
        self.sets -= self.sets % 2                       # even: a set always belongs to the same chain
        self.S = [[MessageSet(torch, w, p0, w.seed + 1000 * s + m * max(w.seed_step, 1)) for m in range(self.nmsg)]
                  for s in range(self.sets)]
        use_sums = mode in ("sums", "accumulate")
        self.pack_b, self.unpack_b = [], []
        for s, S in enumerate(self.S):
            pl = self.plans[s % 2]
            if mode == "tags":
                self.pack_b.append(hxt.TagBatch(pl, [ms.src for ms in S], [ms.packed for ms in S], [ms.tags for ms in S]))
                self.unpack_b.append(hxt.TagBatch(pl, [ms.dst for ms in S], [ms.packed for ms in S], [ms.tags for ms in S],
                                                  [ms.status for ms in S]))
            else:
                self.pack_b.append(hxt.Batch(pl, [ms.src for ms in S], [ms.packed for ms in S],
                                             [ms.send_sums for ms in S] if use_sums else None))
                self.unpack_b.append(hxt.Batch(pl, [ms.dst for ms in S], [ms.packed for ms in S],
                                               [ms.recv_sums for ms in S] if use_sums else None))
        kinds = sorted({p0.tensor_kind(t) for t in range(p0.num_tensors)} - {"none"})
        self.uniform = p0.num_tensors == 1 and kinds == ["contig"]
        if self.uniform:
            self.kernel = "hxt::k_uniform_tag" if mode == "tags" else ("hxt::k_uniform_accumulate" if mode == "accumulate" else "hxt::k_uniform")
        elif kinds == ["contig"] and mode == "tags":
            self.kernel = "hxt::k_contig_tag"
        else:
            self.kernel = " + ".join("hxt::k_" + k for k in kinds)
        self.per_launch = min(self.nmsg, 4) if (batched and self.uniform) else 1
        self.launches_per_step = 2 * self.nmsg // self.per_launch if self.uniform or len(kinds) == 1 else None
        # pack: read N + write N; unpack: the same; accumulate: read N arriving + read N old + write N
        self.step_bytes = (5 if mode == "accumulate" else 4) * self.N * self.nmsg

    def hint(self, value):
        for ps in self.plans:
            for p in ps:
                self.hxt.hxt_plan_set_option(p, self.hxt.HXT_OPT_PACKED_HINT, value)

    def step(self, i, stream):
        hxt, s = self.hxt, i % self.sets
        if self.mode == "tags":
            seqs, mbs = [i] * self.nmsg, list(range(self.nmsg))
            if self.batched:
                hxt.hxt_pack_seal_batch(self.pack_b[s], seqs, mbs, stream)
                hxt.hxt_unpack_verify_batch(self.unpack_b[s], seqs, mbs, stream)
            else:
                for m, ms in enumerate(self.S[s]):
                    p = self.plans[s % 2][m]
                    hxt.hxt_pack_seal(p, ms.src, ms.packed, i, m, ms.tags, stream)
                    hxt.hxt_unpack_verify(p, ms.packed, ms.tags, i, m, ms.dst, ms.status, stream)
            return
        if self.batched:
            hxt.hxt_pack_batch(self.pack_b[s], stream)
            if self.mode == "accumulate":
                hxt.hxt_unpack_accumulate_batch(self.unpack_b[s], stream)
            else:
                hxt.hxt_unpack_batch(self.unpack_b[s], stream)
            return
        use = self.mode != "none"
        for m, ms in enumerate(self.S[s]):
            p = self.plans[s % 2][m]
            hxt.hxt_pack(p, ms.src, ms.packed, ms.send_sums if use else None, stream)
            recv = hxt.hxt_unpack_accumulate if self.mode == "accumulate" else hxt.hxt_unpack
            recv(p, ms.packed, ms.dst, ms.recv_sums if use else None, stream)

    def timed(self, steps, repeats, warmup, two_chains=False):
        """`repeats` blocks of `steps` steps between one pair of synchronisations.  Returns wall seconds for the
        whole region and, on one stream, every block's GPU time from HIP events recorded on the launch stream."""
        torch = self.torch
        main = torch.cuda.current_stream()
        if two_chains:
            if not hasattr(self, "side"):
                self.side = torch.cuda.Stream()
            streams = [main, self.side]
        else:
            streams = [main, main]
        for i in range(warmup):
            self.step(i, streams[i % 2])
        for st in set(streams):
            main.wait_stream(st)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(repeats + 1)]
        i = warmup + (warmup % 2)                        # keep the parity of step and buffer set aligned
        t0 = time.perf_counter()
        for r in range(repeats):
            if not two_chains:
                ev[r].record(main)
            for _ in range(steps):
                self.step(i, streams[i % 2])
                i += 1
        if not two_chains:
            ev[repeats].record(main)
        for st in set(streams):
            main.wait_stream(st)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        blocks = [ev[r].elapsed_time(ev[r + 1]) for r in range(repeats)] if not two_chains else []
        self.last_step = i - 1
        return wall, blocks

    def check(self):
        """Correctness of what was just timed, on the sets of the last two steps: round trip identity, equal send
        and receive checksums (or a clean verdict), and, when receiving with accumulate, the sums of the
        destination against a recomputation on the device (same binary32 additions, in torch)."""
        torch = self.torch
        for back in (0, 1):
            for ms in self.S[(self.last_step - back) % self.sets]:
                if self.mode != "accumulate":
                    for t, s_, d_ in zip(self.w.tensors, ms.src, ms.dst):       # the elements the view addresses
                        a = s_.view(torch.int16).as_strided(t.shape, t.strides)
                        b = d_.view(torch.int16).as_strided(t.shape, t.strides)
                        assert torch.equal(a, b), "round trip mismatch in the timed run"
                if self.mode == "tags":
                    assert not bool(ms.status.any()), "a chunk was rejected in the timed run"
                elif self.mode != "none":
                    assert torch.equal(ms.send_sums, ms.recv_sums), "checksum mismatch in the timed run"


def region_figures(d, wall, blocks, steps, repeats):
    total = steps * repeats
    out = {"gbps": round(d.step_bytes * total / wall / 1e9, 1), "ms_per_step": round(wall / total * 1e3, 5),
           "pct_hbm_peak": round(100 * d.step_bytes * total / wall / 1e9 / HBM_PEAK_GBPS, 2),
           "timed_steps": total, "wall_ms": round(wall * 1e3, 3)}
    if blocks:
        med = statistics.median(blocks)
        out["median_block_ms"] = round(med, 4)
        out["min_block_ms"], out["max_block_ms"] = round(min(blocks), 4), round(max(blocks), 4)
        if d.launches_per_step:
            launch_ms = med / (steps * d.launches_per_step)
            nbytes = d.step_bytes / d.launches_per_step
            out["avg_launch_ms"] = round(launch_ms, 6)
            out["bytes_per_launch"] = int(nbytes)
            out["launch_gbps"] = round(nbytes / (launch_ms * 1e-3) / 1e9, 1)
            out["frac"] = round(nbytes / (launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
    return out


def accumulate_check(torch, hxt, d):
    """One more pack + receive-and-accumulate on set 0 with known destinations, compared element by element with
    torch's own bf16 addition on the device (widen to binary32, add, round to nearest even: the same arithmetic)."""
    ms = d.S[0][0]
    p = d.plans[0][0]
    for t_ in ms.dst:
        t_.copy_(torch.randn(t_.numel(), device=DEV).to(torch.bfloat16) * d.w.std)
    want = [(a.float() + b.float()).to(torch.bfloat16) for a, b in zip(ms.dst, ms.src)]
    hxt.hxt_pack(p, ms.src, ms.packed, ms.send_sums)
    hxt.hxt_unpack_accumulate(p, ms.packed, ms.dst, ms.recv_sums)
    torch.cuda.synchronize()
    assert torch.equal(ms.send_sums, ms.recv_sums), "checksum mismatch"
    for a, b in zip(want, ms.dst):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "accumulated values differ from binary32 addition"


def traffic_from_profile(version):
    """HBM-side bytes per launch of the roofline's kernel from the tracked counter summary, or None when the summary
    was taken with another build of the library (its `library:` line must name this one)."""
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*(\d+)\s*\|\s*kernel:\s*(\S.*?)\s*\|\s*library:\s*(.+?)\s*$", text, re.M)
    if not m or m.group(3) != version:
        return None
    return int(m.group(1))


def plain_copy_ceiling(torch, nbytes):
    """The runtime's own device-to-device copy of as many bytes as one launch of the dominant kernel reads
    (and writes), cold (rotating buffers), back to back on one stream, printed beside the kernel's figure."""
    nsets = max(2, min(8, int(3e9 // (2 * nbytes))))
    src = [torch.empty(nbytes, dtype=torch.uint8, device=DEV).fill_(i + 1) for i in range(nsets)]
    dst = [torch.empty(nbytes, dtype=torch.uint8, device=DEV) for _ in range(nsets)]
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


# ---------------------------------------------------------------------------------------------
# CPU-forwarding path
# ---------------------------------------------------------------------------------------------

def _best_of(torch, fn, reps=10):
    fn()
    best = 1e9
    for _ in range(reps):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        best = min(best, time.perf_counter() - t0)
    return best


class Link:
    """Pinned-copy probe of the host link (256 MiB, each direction alone and both at once on separate buffers),
    taken once per run.  Both directions together first: the HIP runtime in this process keeps using one DMA
    engine for two streams whose first copies ran one after the other (57 GB/s for both directions instead of 97)."""

    def __init__(self, torch):
        self.s1, self.s2 = torch.cuda.Stream(), torch.cuda.Stream()
        P = self.P = 256 << 20
        d_a, d_b = (torch.empty(P, dtype=torch.uint8, device=DEV) for _ in range(2))
        h_a, h_b = (torch.empty(P, dtype=torch.uint8).pin_memory() for _ in range(2))

        def d2h():
            with torch.cuda.stream(self.s1):
                h_a.copy_(d_a, non_blocking=True)

        def h2d():
            with torch.cuda.stream(self.s2):
                d_b.copy_(h_b, non_blocking=True)

        def both():
            d2h()
            h2d()

        self.both = 2 * P / _best_of(torch, both) / 1e9
        self.d2h = P / _best_of(torch, d2h) / 1e9
        self.h2d = P / _best_of(torch, h2d) / 1e9
        self.one_way = min(self.d2h, self.h2d)
        # A round trip sends every byte up and down; with both directions busy each gets half of the
        # both-directions rate, so that is the most a pipelined round trip can show, as a share of one direction.
        self.bound_pct = 100 * (self.both / 2) / self.one_way

    def figures(self):
        return {"probe_bytes": self.P, "probe_d2h_gbps": round(self.d2h, 2), "probe_h2d_gbps": round(self.h2d, 2),
                "probe_bidir_gbps": round(self.both, 2), "bound_pct": round(self.bound_pct, 1)}


def staged_round_trip(torch, hxt, link, w, plans, packed, piece_bytes=8 << 20):
    """Every lane down and up in pieces (runs of slots of about piece_bytes): D2H of a piece on one stream, its H2D on
    another as soon as that D2H is done (an event), through one pinned buffer per message: first D2H start to last
    H2D end.  Pieces rather than whole lanes keep the part of the round trip in which only one direction is busy short."""
    k, N, B = w.n_lanes, plans[0].message_bytes, w.chunk_bytes
    s1, s2 = link.s1, link.s2
    host = [torch.empty(p.packed_bytes, dtype=torch.uint8).pin_memory() for p in plans]
    recv = [torch.empty(p.packed_bytes, dtype=torch.uint8, device=DEV) for p in plans]
    per = max(1, piece_bytes // B)
    pieces = [(l, s, min(per, plans[0].lane_info(l)["n_chunks"] - s)) for l in range(k)
              for s in range(0, plans[0].lane_info(l)["n_chunks"], per)]

    def round_trip(which):
        for m in which:
            for (l, s, n) in pieces:
                hxt.hxt_stage_d2h_slots(plans[m], l, s, n, packed[m], host[m], s1)
                ev = torch.cuda.Event()
                ev.record(s1)
                s2.wait_event(ev)
                hxt.hxt_stage_h2d_slots(plans[m], l, s, n, host[m], recv[m], s2)

    t_one = _best_of(torch, lambda: round_trip([0]))
    out = {"round_trip_gbps": round(N / t_one / 1e9, 2), "pct_host_link": round(100 * N / t_one / 1e9 / link.one_way, 1),
           "lanes": k, "pieces": len(pieces), "piece_bytes": per * B, "message_bytes": N}
    if len(plans) > 1:
        t_all = _best_of(torch, lambda: round_trip(range(len(plans))))
        all_ = N * len(plans) / t_all / 1e9
        out.update({"step_round_trip_gbps": round(all_, 2), "step_pct_host_link": round(100 * all_ / link.one_way, 1),
                    "messages_in_step": len(plans), "bidir_pct": round(100 * 2 * all_ / link.both, 1)})
    for m in range(len(plans)):
        used = plans[m].packed_bytes
        last = plans[m].chunk_info(plans[m].num_chunks - 1)
        if last["padded"] < B:                       # the unspecified tail of a short last chunk's slot is not transferred
            used = None
        if used:
            assert torch.equal(recv[m], packed[m][:used]), "staged bytes differ"
        else:
            a, b = last["packed_off"], last["packed_off"] + last["padded"]
            assert torch.equal(recv[m][:b], packed[m][:b]) and torch.equal(recv[m][a + B:], packed[m][a + B:plans[m].packed_bytes])
    out["host"], out["recv"] = host, recv
    return out


def _wall(fn):
    t0 = time.perf_counter()
    fn()
    return time.perf_counter() - t0


def stream_passes(torch, hxt, w, path, direct_mode=0, window=0, tags=False, checksums=True, passes=5, warm=1):
    """The micro-batch stream: one pass = all micro-batches through hxt_exchange_stream (two buffer sets, three
    streams) and a host synchronisation.  window > 0: the stream is issued in calls of that many messages with a
    wait for the three streams between them (the library itself only enqueues)."""
    t = w.tensors[0]
    plan = hxt.hxt_plan(t.shape, t.strides, torch.bfloat16, w.n_lanes, w.chunk_bytes)
    N, C, nb, nmsg = plan.message_bytes, plan.num_chunks, plan.packed_bytes, w.messages
    g = torch.Generator(device=DEV)
    g.manual_seed(w.seed)
    src = [[(torch.randn(t.storage_elems, generator=g, device=DEV) * w.std).to(torch.bfloat16)] for _ in range(nmsg)]
    dst = [[torch.zeros_like(s_[0])] for s_ in src]
    fwd = path == "cpu_forward"
    send = [torch.empty(nb, dtype=torch.uint8, device=DEV) for _ in range(2)]
    recv = [torch.empty(nb, dtype=torch.uint8, device=DEV) for _ in range(2)] if fwd else None
    host = [torch.empty(nb, dtype=torch.uint8).pin_memory() for _ in range(2)] if fwd else None
    s_send = torch.zeros((nmsg, C), dtype=torch.int64, device=DEV)
    s_recv = torch.zeros_like(s_send)
    streams = [torch.cuda.Stream() for _ in range(3)]
    status = torch.zeros((nmsg, C + 1), dtype=torch.int32, device=DEV)
    tag_dev = lambda: [torch.zeros(C * 64, dtype=torch.uint8, device=DEV) for _ in range(2)]
    tag_bufs = (tag_dev(), tag_dev() if fwd else None,
                [torch.zeros(C * 64, dtype=torch.uint8).pin_memory() for _ in range(2)] if fwd else None) if tags else None
    plain = checksums and not tags
    step = window if window > 0 else nmsg
    calls = []
    for a in range(0, nmsg, step):
        b = min(nmsg, a + step)
        kw = {}
        if tags:
            kw = dict(tags_send=tag_bufs[0], tags_recv=tag_bufs[1], tags_pinned=tag_bufs[2], status=status[a:b], seq_base=1 + a)
        calls.append(hxt.Exchange(src[a:b], dst[a:b], send, hxt.HXT_CPU_FORWARD if fwd else hxt.HXT_DEVICE_DIRECT, recv, host,
                                  s_send[a:b] if plain else None, s_recv[a:b] if plain else None, *streams,
                                  direct_mode=direct_mode, **kw))

    def one_pass():
        for x in calls:
            hxt.hxt_exchange_stream(plan, x)
            if window > 0:
                for st in streams:
                    st.synchronize()
        torch.cuda.synchronize()

    torch.cuda.synchronize()                          # inputs were drawn on the default stream
    for _ in range(warm):
        one_pass()
    times = [_wall(one_pass) for _ in range(passes)]
    for s_, d_ in zip(src, dst):
        assert torch.equal(s_[0].view(torch.int16), d_[0].view(torch.int16)), "round trip mismatch"
    if tags:
        assert not bool(status.any()), "a chunk was rejected in the timed run"
    elif checksums:
        assert torch.equal(s_send, s_recv)
    sec = statistics.median(times)
    return {"us_per_micro_batch": round(sec / nmsg * 1e6, 2), "ms_per_pass": round(sec * 1e3, 3), "passes": passes,
            "message_bytes": N, "messages": nmsg, "gbps_per_direction": round(N * nmsg / sec / 1e9, 2),
            "pack_unpack_gbps": round(4 * N * nmsg / sec / 1e9, 1)}


# ---------------------------------------------------------------------------------------------
# CPU oracle
# ---------------------------------------------------------------------------------------------

def cpu_baseline(w, budget_s=10.0, max_tensors=None, one_core=True):
    """The CPU oracle, as it stands, on the message geometry: pack + checksum + unpack + checksum on all host cores
    for about budget_s seconds (at least one pass).  Values are seeded random 16-bit patterns: the oracle's time does
    not depend on them.  max_tensors: take only the first so many tensors of the message (a bounded sample)."""
    import numpy as np

    from oracle import hxt_oracle as ho

    cores = ho.max_threads()
    tensors = list(w.tensors)[:max_tensors] if max_tensors else list(w.tensors)
    m = ho.Message([ho.TensorSpec(t.shape, t.strides, t.esize) for t in tensors])
    rng = np.random.default_rng(w.seed)
    raws = [rng.integers(0, 1 << 16, size=t.storage_elems * t.esize // 2, dtype=np.uint16).view(np.uint8) for t in tensors]
    B, k = w.chunk_bytes, w.n_lanes
    dst = [np.zeros_like(r) for r in raws]
    packed = np.zeros(ho.packed_bytes(m, B, k), np.uint8)

    def one(nt):
        ho.pack(m, raws, B, k, packed=packed, nthreads=nt)
        a = ho.checksum(m, packed, B, k, nthreads=nt)
        ho.unpack(m, packed, B, k, dst, nthreads=nt)
        return a, ho.checksum(m, packed, B, k, nthreads=nt)

    t0 = time.perf_counter()
    reps = 0
    while True:
        s_send, s_recv = one(cores)
        reps += 1
        if time.perf_counter() - t0 > budget_s:
            break
    sec = time.perf_counter() - t0
    assert np.array_equal(s_send, s_recv)
    for t, a_, b_ in zip(tensors, raws, dst):             # round trip: the elements the view addresses
        el = np.dtype("u%d" % t.esize)
        view = lambda x: np.lib.stride_tricks.as_strided(x.view(el), t.shape, [st * t.esize for st in t.strides])
        assert np.array_equal(view(a_), view(b_)), "oracle round trip"
    out = {"value": round(4 * m.N * reps / sec / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
           "sample": "%d pass(es) over %s (%d bytes): pack + checksum + unpack + checksum, %.1f s"
                     % (reps, "the whole message" if not max_tensors else "the first %d tensors of the message" % len(tensors),
                        m.N, sec)}
    if one_core:
        t1 = time.perf_counter()
        one(1)
        out["one_core_value"] = round(4 * m.N / (time.perf_counter() - t1) / 1e9, 3)
    return out


# ---------------------------------------------------------------------------------------------

def config_entries(torch, hxt, wl, a, link, headline_regions):
    """One entry per benchmark message and path (the headline message's entries come from its timed regions)."""
    out = []

    def direct(name, hints=("cold", "llc"), mode="sums", steps=None, note=None, w=None):
        w = w or wl.ALL[name]()
        d = DirectStep(torch, hxt, w, a.sets, mode=mode)
        big = d.plans[0][0].packed_bytes > (128 << 20)
        for h in hints:
            if h == "llc" and big:
                continue                                  # beyond the last-level cache nothing is re-read from it
            d.hint(1 if h == "cold" else 0)
            n = steps or max(4, min(200, int(40e-3 / (d.step_bytes / 5.5e12))))
            wall, blocks = d.timed(n, 3, max(2, n // 10))
            d.check()
            e = {"workload": w.name, "path": "device_direct", "issue": "batched calls, one stream" if d.batched else "one call per message",
                 "checks": {"sums": "fused send+receive checksums", "tags": "chunk tags sealed and verified inside the copies",
                            "accumulate": "receive-and-accumulate, fused checksums", "none": "off"}[mode],
                 "cache_state": "all-cold (non-temporal both sides, rotating sets)" if h == "cold" else
                                "packed buffer re-read from the last-level cache",
                 "message_bytes": d.N, "messages_per_step": d.nmsg, "kernel": d.kernel}
            e.update(region_figures(d, wall, blocks, n, 3))
            if note:
                e["note"] = note
            out.append(e)
        if mode == "accumulate":
            accumulate_check(torch, hxt, d)
        return d

    def forward(d, w):
        plans = d.plans[0]
        st = staged_round_trip(torch, hxt, link, w, plans, [ms.packed for ms in d.S[0]])
        st.pop("host"), st.pop("recv")
        e = {"workload": w.name, "path": "cpu_forward", "issue": "lanes in pieces of up to 8 MiB (at least a chunk), D2H and H2D on two streams"}
        e.update(st)
        e["bound_pct"] = round(link.bound_pct, 1)
        out.append(e)

    # 1 tiny
    d = direct("tiny", hints=("llc",), steps=200, note="128 KiB: launch-latency bound, cache resident whatever the hint")
    del d
    # 2 the headline message: its regions
    for name, r in headline_regions.items():
        e = {"workload": a.workload, "path": "device_direct", "region": name}
        e.update(r)
        out.append(e)
    # 3 Qwen2-7B boundary, both paths
    w = wl.qwen2_7b_boundary()
    d = direct("qwen2_7b_boundary")
    if not a.no_staged:
        forward(d, w)
    del d
    # 4 the micro-batch stream, both paths
    w = wl.stream_1f1b()
    for mode, label in ((hxt.HXT_DIRECT_EVENTS, "pack and unpack on two streams, unpack waits for an event (boundary-shaped)"),
                        (hxt.HXT_DIRECT_FUSED, "one launch unpacks micro-batch i-1 and packs micro-batch i"),
                        (hxt.HXT_DIRECT_TWO_CHAINS, "even and odd micro-batches as two chains on two streams (loopback-shaped: "
                                                    "a micro-batch is unpacked right behind its own pack)")):
        e = {"workload": w.name, "path": "device_direct", "issue": label,
             "cache_state": "sources and destinations cold (1 GiB per pass), packed buffers (2 x 32 MiB) cache resident"}
        e.update(stream_passes(torch, hxt, w, "device_direct", direct_mode=mode, passes=8))
        e["gbps"] = e.pop("pack_unpack_gbps")
        e["pct_hbm_peak"] = round(100 * e["gbps"] / HBM_PEAK_GBPS, 2)
        e.pop("gbps_per_direction")
        out.append(e)
    if not a.no_staged:
        for window, label in ((16, "issued in windows of 16 micro-batches, the three streams drained between windows"),
                              (0, "all 32 micro-batches enqueued at once")):
            e = {"workload": w.name, "path": "cpu_forward", "issue": label}
            e.update(stream_passes(torch, hxt, w, "cpu_forward", window=window, passes=3))
            e.pop("pack_unpack_gbps")
            e["pct_host_link"] = round(100 * e["gbps_per_direction"] / link.one_way, 1)
            e["bound_pct"] = round(link.bound_pct, 1)
            out.append(e)
    # 5 gradient buckets, both paths, and the two widenings that use them
    w = wl.grad_buckets()
    d = direct("grad_buckets", hints=("cold",), steps=12)
    if not a.no_staged:
        forward(d, w)
    del d
    torch.cuda.empty_cache()
    d = direct("grad_buckets", hints=("cold",), steps=12, mode="tags")
    del d
    torch.cuda.empty_cache()
    d = direct("grad_buckets", hints=("cold",), steps=12, mode="accumulate")
    del d
    torch.cuda.empty_cache()
    # supplementary strided views
    direct("qwen_rows_view")
    direct("transpose_view")
    direct("rows_split_view", note="bf16 [327680, 100]: runs of 200 bytes at a pitch of 256 bytes")
    direct("wide_transpose_view", hints=("cold",), note="bf16 [256, 65536] with strides (1, 256): 8 rows of the packed side per "
           "chunk, transpose tiles span chunks")
    direct("inner_stride_view", hints=("cold",), note="bf16 [4096, 4096] with strides (8192, 2): every second element, "
           "so the tensor side moves two bytes of memory bursts per byte of payload")
    return out


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
        window = (16 if a.path == "cpu_forward" else 0) if a.window < 0 else a.window
        r = stream_passes(torch, hxt, w, a.path, direct_mode=a.direct_mode, window=window, tags=a.tags,
                          checksums=not a.no_checksum, passes=max(1, min(a.steps, 20)), warm=max(1, min(a.warmup, 2)))
        out = {"metric": METRIC, "value": r["pack_unpack_gbps"], "value_of": "pack+unpack GB/s", "unit": "GB/s", "n_gpus": 1,
               "steps": r["passes"], "warmup": max(1, min(a.warmup, 2)), "ms_per_step": r["ms_per_pass"],
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
               "config": {"workload": w.name, "note": w.note, "path": a.path, "buffer_sets": 2, "streams": 3,
                          "window": window, "direct_mode": a.direct_mode}}
        out.update(r)
        print(json.dumps(out))
        return
    repeats = a.repeats if a.repeats > 0 else max(5, -(-2000 // max(a.steps, 1)))
    link = None if a.no_staged else Link(torch)        # before any other copy touches the DMA engines
    mode = "tags" if a.tags else ("accumulate" if a.accumulate else ("none" if a.no_checksum else "sums"))
    d = DirectStep(torch, hxt, w, a.sets, mode=mode, batched=not a.unbatched)
    for i in range(a.calibration_copies):                 # plain copies: read N, write N each
        ms = d.S[i % d.sets][0]
        ms.dst[0].copy_(ms.src[0])
    regions = {}
    for name in [r for r in a.regions.split(",") if r]:
        if name not in REGIONS:
            print("bench.py: unknown region %r" % name, file=sys.stderr)
            sys.exit(2)
        d.hint(1 if name.endswith("cold") else 0)
        wall, blocks = d.timed(a.steps, repeats, a.warmup, two_chains=name.startswith("chains"))
        d.check()
        regions[name] = region_figures(d, wall, blocks, a.steps, repeats)
        regions[name]["cache_state"] = ("all-cold: every access non-temporal, sources and destinations rotate over %d sets"
                                        % d.sets if name.endswith("cold") else
                                        "packed buffer re-read from the last-level cache (sources and destinations cold)")
        regions[name]["issue"] = ("steps dealt alternately onto two streams (a plan set each), kernels of consecutive steps overlap"
                                  if name.startswith("chains") else "one stream, launches back to back")
    if a.accumulate:
        accumulate_check(torch, hxt, d)
    # value: whole-job throughput of the all-cold step as the library is meant to be driven (independent steps on two
    # streams); roofline: the dominant kernel's launches alone on the machine, back to back on one stream, all-cold
    head_name = next(n for n in ("chains_cold", "cold", "chains_llc", "llc") if n in regions)
    roof_name = next((n for n in ("cold", "llc") if n in regions), None)
    head = regions[head_name]
    out = {
        "metric": METRIC if not a.accumulate else "pack+accumulate GB/s",
        "value": head["gbps"],                          # the metric's first figure; its second is in "staged"
        "value_of": "pack+unpack GB/s" if not a.accumulate else "pack+accumulate GB/s",
        "value_region": head_name,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "repeats": repeats,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": w.name, "note": w.note, "message_bytes": d.N, "messages_per_step": d.nmsg,
                   "n_lanes": w.n_lanes, "chunk_bytes": w.chunk_bytes, "path": "device_direct",
                   "checks": {"sums": "fused send+receive checksums", "tags": "chunk tags sealed and verified inside the copies",
                              "accumulate": "receive-and-accumulate, fused checksums", "none": "off"}[mode],
                   "buffer_sets": d.sets, "cache_state": head["cache_state"],
                   "streams": 2 if head_name.startswith("chains") else 1,
                   "issue": ("batched calls (one launch packs all messages of the step, one unpacks them)"
                             if d.batched and d.per_launch > 1 else "one call per message") + "; " + head["issue"],
                   "timing": "%d blocks of %d steps between one pair of host synchronisations; value = bytes / wall time of the "
                             "whole region" % (repeats, a.steps)},
        "pct_hbm_peak": head["pct_hbm_peak"],
        "regions": regions,
    }
    roof = regions.get(roof_name) if roof_name else None
    if roof and "avg_launch_ms" in roof:
        out["roofline"] = {"bound": "hbm", "kernel": d.kernel + " (pack and unpack instantiations%s)"
                           % ("" if mode == "none" else ", checks fused"), "region": roof_name,
                           "region_is": "one stream, launches back to back (a kernel has the machine to itself), " + roof["cache_state"],
                           "achieved": roof["launch_gbps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": roof["frac"],
                           "traffic": traffic_from_profile(hxt.hxt_version()) if (roof_name == "cold" and mode == "sums"
                                                                                  and w.name == "llama8b_boundary" and d.batched) else None,
                           "traffic_is": "L2<->fabric bytes per launch (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy of known "
                                         "size); last-level-cache hits are not separated from HBM accesses",
                           "bytes_per_launch": roof["bytes_per_launch"], "avg_launch_ms": roof["avg_launch_ms"],
                           "launches": a.steps * repeats * d.launches_per_step,
                           "gpu_ms_median_block": roof["median_block_ms"]}
        if not a.calibration_copies:        # a counter pass must see no other copy kernels than its calibration copies
            out["roofline"]["plain_copy"] = plain_copy_ceiling(torch, roof["bytes_per_launch"] // 2)
        if roof_name == "cold" and "llc" in regions and "frac" in regions["llc"]:
            out["roofline_llc_assisted"] = {k: regions["llc"][k] for k in ("launch_gbps", "frac", "avg_launch_ms", "cache_state")}
    out["paper_context"] = PAPER_CONTEXT
    if not a.no_staged:
        st = staged_round_trip(torch, hxt, link, w, d.plans[0], [ms.packed for ms in d.S[0]])
        host, recv = st.pop("host"), st.pop("recv")
        # the host-to-host hop of the chain (pinned to pinned), one thread per lane and one thread
        hop_dst = torch.empty(d.plans[0][0].packed_bytes, dtype=torch.uint8).pin_memory()
        t_hop = min(_wall(lambda: hxt.hxt_host_forward(d.plans[0][0], -1, host[0], hop_dst, 0)) for _ in range(5))
        t_hop1 = min(_wall(lambda: hxt.hxt_host_forward(d.plans[0][0], -1, host[0], hop_dst, 1)) for _ in range(5))
        assert torch.equal(hop_dst, host[0])
        st.update({"host_hop_gbps": round(d.N / t_hop / 1e9, 2), "host_hop_one_thread_gbps": round(d.N / t_hop1 / 1e9, 2)})
        st.update(link.figures())
        st["note"] = ("best of 10, wall clock around a synchronised region; round trip = first D2H start to last H2D end of one "
                      "message; step = all messages of the step pipelined lane by lane; link = min one-direction probe; "
                      "bound_pct = (both-directions probe / 2) / one-direction probe: the most a round trip that keeps both "
                      "directions busy can reach; bidir_pct = 2 x step rate / both-directions probe")
        out["staged"] = st
        del host, recv, hop_dst
    default_run = mode == "sums" and d.batched
    del d
    torch.cuda.empty_cache()
    if not a.no_configs and default_run and w.name == "llama8b_boundary":
        out["configs"] = config_entries(torch, hxt, wl, a, link, regions)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
        if "configs" in out:
            seen = {}
            for e in out["configs"]:
                name = e["workload"]
                if name == w.name:
                    e["cpu_oracle_gbps"] = out["cpu_baseline"]["value"]
                    continue
                if name not in seen:
                    wc = wl.ALL[name]()
                    big = wc.message_bytes > (1 << 30)
                    seen[name] = cpu_baseline(wc, budget_s=1.5, max_tensors=9 if big else None, one_core=False)
                e["cpu_oracle_gbps"] = seen[name]["value"]
                e["cpu_oracle_sample"] = seen[name]["sample"]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
