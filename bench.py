#!/usr/bin/env python3
"""Throughput of the AQ-SGD boundary codec on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

One *step* is one pass of the whole hot path over one micro-batch of the
GPT2-1.5B-shaped boundary (float16 [4, 1024, 1600], 8192-sample buffers):

    aqsgd_encode   (sender:   gather m rows, delta, per-row scale, 4-bit pack, update m)
    aqsgd_decode   (receiver: unpack, update its m, emit the activation)
    aqsgd_grad_quant / aqsgd_grad_dequant   (backward message, 8-bit, direct)

All inputs are resident in HBM before the clock starts.  Buffers rotate: sample ids
sweep a random permutation of the 8192 rows of the two 26.8 GB buffers and the
activation / codes / output tensors cycle through pools of > 1 GB each, far beyond
the 256 MB of last-level cache, so every call reads cold rows from HBM.  The
buffers are pre-seeded by one full pass and the activations then drift by
0.05 sigma, so the timed steps encode changes, as in steady-state fine-tuning.

The K timed steps are recorded into HIP graphs (256 steps each), replayed once
untimed (the first replay of a new graph uploads it), and then replayed back to back
between two HIP events on the launching stream, with device synchronisation on both
sides; event time / K is ms_per_step.  `value` is the metric's own quantity: the
activation bytes of a micro-batch over the time of its encode + decode, from a second
timed run of the same K micro-batches without the backward message.
How the messages are launched (--schedule):
  pipeline  (default) one aqsgd_run_jobs launch per time slot of the two stages, as when
            the sending and the receiving stage work on neighbouring micro-batches at the
            same time: encode of micro-batch k, decode and grad_quant of k-1, grad_dequant
            of k-2, all independent, 124.6 MB in one grid.  Every message of every timed
            micro-batch is launched exactly once (the first and last slots of a chain carry
            fewer jobs).
  stage     one launch per stage and micro-batch: the sending stage's encode(k) +
            grad_dequant(k-1), the receiving stage's decode(k) + grad_quant(k).
  calls     the four single-message calls.
Micro-batches touch disjoint samples and pool slots, so their chains are independent, as
they are in a pipeline that has several micro-batches in flight: they are dealt
round-robin over --streams streams (default 2; 4 for `calls`, half of them for the forward
and half for the backward messages), and one launch's fill and drain overlaps another's
streaming.  --streams 1 runs every launch strictly after the one before.

A further pass launches every kind of launch on its own, one after the other, through
the library's timed-launch hook, which stamps a HIP event pair with the kernel's own
begin and end on its stream: the four single-message calls and the schedule's fused
launch.  The longest launch of the schedule feeds the roofline figure (kernel quality),
independent of how launches are overlapped.

Secondary lines: --first-visit (Algorithm 1's uncompressed first visits against a same-run
copy), --ceilings (what launches of this size reach on this GPU), --config, --m-bits,
--bwd-keep.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from pathlib import Path

ROOT = Path(__file__).resolve().parent
for p in (ROOT, ROOT / "tests"):
    if str(p) not in sys.path:
        sys.path.insert(0, str(p))

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
GRAPH_STEPS = 256               # steps recorded per HIP graph


WORKLOAD_TEXT = {
    "gpt2_4bit": "GPT2-1.5B-shaped stage boundary: float16 activations [4,1024,1600], 8192-sample "
                 "float16 m_buf x2 (sender, receiver), forward 4-bit per-row delta codec, backward "
                 "8-bit direct",
    "gpt2_2bit_stochastic": "GPT2-1.5B-shaped stage boundary: float16 [4,1024,1600], 8192-sample m_buf "
                            "x2, forward 2-bit delta with Philox stochastic rounding in groups of 128, "
                            "backward 4-bit stochastic",
    "deberta_3bit": "DeBERTa-1.5B-shaped stage boundary: bfloat16 activations [32,256,1536], "
                    "100k-sample bfloat16 m_buf x2 (78.6 GB each), forward 3-bit delta in groups of 64, "
                    "backward 6-bit",
    "stress": "stress boundary: float32 activations [8,2048,4096] with outlier tokens, 256-sample "
              "float32 m_buf x2, forward 4-bit per-row delta, backward 8-bit",
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2048)
    ap.add_argument("--warmup", type=int, default=128)
    ap.add_argument("--launch", choices=["graph", "eager"], default="graph")
    ap.add_argument("--streams", type=int, choices=[0, 1, 2, 3, 4, 6, 8], default=0,
                    help="streams the micro-batches are dealt over (they touch disjoint samples and pool "
                         "slots, so their chains are independent); 0 = 2 for the fused schedules, 8 for "
                         "`calls` (short single-message launches one after the other need more chains in "
                         "flight to keep the memory system busy); "
                         "1: every launch strictly after the one before")
    ap.add_argument("--schedule", choices=["calls", "stage", "pipeline"], default="pipeline",
                    help="calls: four single-message calls per step; stage / pipeline: the same messages "
                         "through aqsgd_run_jobs, two launches (one per stage) or one launch (one time "
                         "slot of both stages) per micro-batch")
    ap.add_argument("--pool", type=int, default=0,
                    help="micro-batch slots per rotating pool (0 = enough for 1.25 GB per pool)")
    ap.add_argument("--config", default="gpt2_4bit",
                    choices=["gpt2_4bit", "gpt2_2bit_stochastic", "deberta_3bit", "stress"],
                    help="workload; the default is the one the headline metric is quoted on, the "
                         "others give secondary lines")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-legs", action="store_true")
    ap.add_argument("--cpu-calls", type=int, default=0, help="oracle sample size (0 = auto)")
    ap.add_argument("--m-bits", type=int, choices=[0, 2, 8], default=0,
                    help="keep the previous messages as z-bit levels (Appendix H.5) instead of the "
                         "activation dtype; 0 = full precision (the headline configuration)")
    ap.add_argument("--bwd-keep", type=float, default=0.0,
                    help="sparsify the backward message (Appendix H.6): fraction of each group's "
                         "entries that is sent, at 8 bits; 0 = dense (the headline configuration)")
    ap.add_argument("--first-visit", action="store_true",
                    help="secondary line: Algorithm 1's uncompressed first visits (aqsgd_seed, "
                         "aqsgd_encode_seen / aqsgd_decode_seen on new samples) against a same-run copy "
                         "of the same size, then the second visits through the same entry points")
    ap.add_argument("--ceilings", action="store_true",
                    help="secondary line: what this GPU does with launches of this size: a near-empty "
                         "launch, the library's plain row copy and its encode / decode at growing "
                         "micro-batch sizes, and large fill / copy kernels")
    ap.add_argument("--region-sweep", action="store_true",
                    help="secondary line: the timed region at 10, 20, 40, 80, 160 and 320 steps in one process "
                         "(whole step and forward messages alone), to show what the length of the region "
                         "does to the per-step figures")
    ap.add_argument("--boundaries", type=int, default=1,
                    help="secondary line, with --config stress: this many stage boundaries (2/4/8-bit "
                         "forward messages mixed) worked on at the same time, every launch carrying the "
                         "messages of all of them; each boundary has its own buffers (17 GB)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run three plain 1 GiB device-to-device tensor copies (known traffic: "
                         "1 GiB read, 1 GiB written) so hardware byte counters can be scaled")
    return ap.parse_args()


class Workload:
    """Device-resident state of the benchmarked boundary."""

    def __init__(self, cfg, pool: int, seed: int = 1234, m_bits: int = 0, bwd_keep: float = 0.0):
        import torch
        from paper_2206_01299_amd import binding as B
        self.torch, self.B, self.cfg = torch, B, cfg
        d = torch.device("cuda:0")
        self.dev = d
        td = B.DTYPE_NAME[cfg.dtype]
        g = torch.Generator(device=d)
        g.manual_seed(seed)
        self.gen = g
        self.pool = pool
        Bn, n_per = cfg.batch, cfg.n_per

        self.fdesc = B.make_desc(batch=Bn, n_per=n_per, n_samples=cfg.n_samples, bits=cfg.fwd_bits,
                                 group=cfg.fwd_group, dtype=cfg.dtype, rounding=cfg.fwd_rounding)
        self.bdesc = B.make_desc(batch=Bn, n_per=n_per, n_samples=cfg.n_samples, bits=cfg.bwd_bits,
                                 group=cfg.bwd_group, dtype=cfg.dtype, rounding=cfg.bwd_rounding)

        self.m_bits = m_bits
        if m_bits:      # previous messages as z-bit levels + one scale per group (Appendix H.5)
            row = B.lowbit_row_bytes(self.fdesc, m_bits)
            gps = n_per // cfg.fwd_group
            self.m_send = torch.zeros((cfg.n_samples, row), dtype=torch.uint8, device=d)
            self.m_recv = torch.zeros((cfg.n_samples, row), dtype=torch.uint8, device=d)
            self.ms_send = torch.zeros((cfg.n_samples, gps), dtype=torch.float32, device=d)
            self.ms_recv = torch.zeros((cfg.n_samples, gps), dtype=torch.float32, device=d)
            # the plain codec's buffers too: its launches are timed in the same process, next to
            # the variant's, so that the two can be compared (kernel_legs)
            self.m_plain_send = torch.zeros((cfg.n_samples, n_per), dtype=td, device=d)
            self.m_plain_recv = torch.zeros((cfg.n_samples, n_per), dtype=td, device=d)
        else:
            self.m_send = torch.zeros((cfg.n_samples, n_per), dtype=td, device=d)
            self.m_recv = torch.zeros((cfg.n_samples, n_per), dtype=td, device=d)

        # outliers: a fraction of the hidden channels, or of the token rows, carries a larger scale
        chan = torch.ones((1, cfg.hidden), device=d)
        k = int(round(cfg.outlier_channel_frac * cfg.hidden))
        if k:
            chan[0, torch.randperm(cfg.hidden, generator=g, device=d)[:k]] = cfg.outlier_scale
        k = int(round(cfg.outlier_token_frac * cfg.seq))
        if k:
            tok = torch.ones((cfg.seq, 1), device=d)
            tok[torch.randperm(cfg.seq, generator=g, device=d)[:k], 0] = cfg.outlier_scale
            chan = chan * tok
        self.chan = chan

        shape = (pool, Bn, cfg.seq, cfg.hidden)
        self.act = torch.empty(shape, dtype=td, device=d)
        self.grad = torch.empty(shape, dtype=td, device=d)
        for s in range(pool):
            self.act[s] = (self._draw((Bn, cfg.seq, cfg.hidden)) * chan).to(td)
            self.grad[s] = (self._draw((Bn, cfg.seq, cfg.hidden)) * (chan * cfg.grad_scale)).to(td)
        self.out = torch.empty(shape, dtype=td, device=d)
        self.gout = torch.empty(shape, dtype=td, device=d)
        self.codes = torch.empty((pool, B.codes_bytes(self.fdesc)), dtype=torch.uint8, device=d)
        self.scales = torch.empty((pool, B.scales_count(self.fdesc)), dtype=torch.float32, device=d)
        self.bcodes = torch.empty((pool, B.codes_bytes(self.bdesc)), dtype=torch.uint8, device=d)
        self.bscales = torch.empty((pool, B.scales_count(self.bdesc)), dtype=torch.float32, device=d)

        self.keep = int(round(bwd_keep * cfg.bwd_group)) if bwd_keep else 0
        if self.keep:   # only the largest entries of each group travel (Appendix H.6)
            self.bitmap = torch.empty((pool, B.topk_bitmap_bytes(self.bdesc)), dtype=torch.uint8, device=d)
            self.bcodes = torch.empty((pool, B.topk_codes_bytes(self.bdesc, self.keep)), dtype=torch.uint8,
                                      device=d)
            self.bcodes_dense = torch.empty((pool, B.codes_bytes(self.bdesc)), dtype=torch.uint8, device=d)

        perm = torch.randperm(cfg.n_samples, generator=g, device=d)
        self.ids = perm.view(-1, Bn).contiguous()              # [calls per epoch, B]
        self.calls = self.ids.shape[0]
        self.evict = torch.zeros(1 << 28, dtype=torch.int32, device=d)     # 1 GiB, see evict_caches()
        torch.cuda.synchronize()

    def _draw(self, shape):
        """fp32 draws of the configuration's law, on the device."""
        torch, c = self.torch, self.cfg
        z = torch.randn(shape, device=self.dev, generator=self.gen)
        if c.law == "normal":
            return z
        if c.law == "student_t3":                  # z / sqrt(chi2_3 / 3)
            chi = torch.zeros(shape, device=self.dev)
            for _ in range(3):
                chi += torch.randn(shape, device=self.dev, generator=self.gen) ** 2
            return z / torch.sqrt(chi / 3.0)
        if c.law == "laplace":                     # exponential magnitude, random sign
            mag = torch.empty(shape, device=self.dev).exponential_(1.0, generator=self.gen)
            return torch.where(z >= 0, mag, -mag)
        raise NotImplementedError(c.law)

    def preseed_and_drift(self):
        """One full pass (every sample visited once), then the activations drift."""
        torch, c = self.torch, self.cfg
        for k in range(self.calls):
            self.step(k, backward=False)
        torch.cuda.synchronize()
        td = self.act.dtype
        for s in range(self.pool):
            noise = self._draw(self.act[s].shape) * (self.chan * c.drift)
            self.act[s] = (self.act[s].float() + noise).to(td)
        torch.cuda.synchronize()

    # -- the four launches of one step -----------------------------------------
    def encode(self, k):
        s = k % self.pool
        self.fdesc.rng_seed = 0x5EED0000 + 2 * k           # a fresh key per message
        if self.m_bits:
            self.B.encode_lowbit(self.fdesc, self.m_bits, self.act[s], self.ids[k % self.calls],
                                 self.m_send, self.ms_send, self.codes[s], self.scales[s])
        else:
            self.B.encode(self.fdesc, self.act[s], self.ids[k % self.calls], self.m_send,
                          self.codes[s], self.scales[s])

    def decode(self, k):
        s = k % self.pool
        if self.m_bits:
            self.B.decode_lowbit(self.fdesc, self.m_bits, self.codes[s], self.scales[s],
                                 self.ids[k % self.calls], self.m_recv, self.ms_recv, self.out[s])
        else:
            self.B.decode(self.fdesc, self.codes[s], self.scales[s], self.ids[k % self.calls],
                          self.m_recv, self.out[s])

    def grad_quant(self, k):
        s = k % self.pool
        self.bdesc.rng_seed = 0x5EED0001 + 2 * k
        if self.keep:
            self.B.grad_topk_quant(self.bdesc, self.keep, self.grad[s], self.bitmap[s], self.bcodes[s],
                                   self.bscales[s])
        else:
            self.B.grad_quant(self.bdesc, self.grad[s], self.bcodes[s], self.bscales[s])

    def grad_dequant(self, k):
        s = k % self.pool
        if self.keep:
            self.B.grad_topk_dequant(self.bdesc, self.keep, self.bitmap[s], self.bcodes[s], self.bscales[s],
                                     self.gout[s])
        else:
            self.B.grad_dequant(self.bdesc, self.bcodes[s], self.bscales[s], self.gout[s])

    # -- the same four messages as jobs of one aqsgd_run_jobs call ------------------
    def job(self, leg, k):
        s, B = k % self.pool, self.B
        if leg == "encode":
            self.fdesc.rng_seed = 0x5EED0000 + 2 * k
            return B.encode_job(self.fdesc, self.act[s], self.ids[k % self.calls], self.m_send,
                                self.codes[s], self.scales[s])
        if leg == "decode":
            return B.decode_job(self.fdesc, self.codes[s], self.scales[s], self.ids[k % self.calls],
                                self.m_recv, self.out[s])
        if leg == "grad_quant":
            self.bdesc.rng_seed = 0x5EED0001 + 2 * k
            return B.grad_quant_job(self.bdesc, self.grad[s], self.bcodes[s], self.bscales[s])
        return B.grad_dequant_job(self.bdesc, self.bcodes[s], self.bscales[s], self.gout[s])

    def fused_chain(self, ks, schedule, backward=True):
        """The messages of micro-batches `ks` (in this order) on the current stream, in
        launches that carry several independent jobs.
        stage:    what each stage of the boundary launches: the sending stage encode(k) together
                  with grad_dequant of the micro-batch before, the receiving stage decode(k)
                  together with grad_quant(k); two launches per micro-batch.
        pipeline: both stages' work of one time slot in one launch, as when the two stages
                  work on neighbouring micro-batches at the same time: encode(k), decode and
                  grad_quant of the micro-batch before, grad_dequant of the one before that.
        Every message of every micro-batch in `ks` is launched exactly once."""
        B, n = self.B, len(ks)
        if schedule == "stage":
            for t in range(n):
                B.run_jobs([self.job("encode", ks[t])] +
                           ([self.job("grad_dequant", ks[t - 1])] if backward and t >= 1 else []))
                B.run_jobs([self.job("decode", ks[t])] + ([self.job("grad_quant", ks[t])] if backward else []))
            if backward and n:
                B.run_jobs([self.job("grad_dequant", ks[-1])])
            return
        assert schedule == "pipeline"
        for t in range(n + (2 if backward else 1)):
            jobs = []
            if t < n:
                jobs.append(self.job("encode", ks[t]))
            if 0 <= t - 1 < n:
                jobs.append(self.job("decode", ks[t - 1]))
                if backward:
                    jobs.append(self.job("grad_quant", ks[t - 1]))
            if backward and 0 <= t - 2 < n:
                jobs.append(self.job("grad_dequant", ks[t - 2]))
            if jobs:
                B.run_jobs(jobs)

    # -- the plain codec's launches on the same micro-batches, for the variants' reference legs
    def plain_encode(self, k):
        s = k % self.pool
        self.B.encode(self.fdesc, self.act[s], self.ids[k % self.calls], self.m_plain_send,
                      self.codes[s], self.scales[s])

    def plain_decode(self, k):
        s = k % self.pool
        self.B.decode(self.fdesc, self.codes[s], self.scales[s], self.ids[k % self.calls],
                      self.m_plain_recv, self.out[s])

    def dense_grad_quant(self, k):
        s = k % self.pool
        self.B.grad_quant(self.bdesc, self.grad[s], self.bcodes_dense[s], self.bscales[s])

    def dense_grad_dequant(self, k):
        s = k % self.pool
        self.B.grad_dequant(self.bdesc, self.bcodes_dense[s], self.bscales[s], self.gout[s])

    def reference_legs(self):
        """Launches of the plain codec that a variant run times beside its own."""
        return ((("plain_encode", "plain_decode") if self.m_bits else ())
                + (("dense_grad_quant", "dense_grad_dequant") if self.keep else ()))

    LEGS = ("encode", "decode", "grad_quant", "grad_dequant")

    def step(self, k, backward=True):
        self.encode(k)
        self.decode(k)
        if backward:
            self.grad_quant(k)
            self.grad_dequant(k)

    # -- algorithmic bytes per launch (what the method must move) ----------------
    def leg_bytes(self):
        c = self.cfg
        n, E = c.n, c.elem_bytes
        fb, bb = c.fwd_bits / 8.0, c.bwd_bits / 8.0
        fs, bs = 4.0 * n / c.fwd_group, 4.0 * n / c.bwd_group
        M = self.m_bits / 8.0 if self.m_bits else E   # bytes per element of the stored m
        ss = 2 * fs if self.m_bits else 0.0           # storage scales, read and written
        if self.keep:                                 # a bit per entry + a byte per kept entry
            bb = 1.0 / 8.0 + self.keep / c.bwd_group
        dense = c.bwd_bits / 8.0
        return {
            "encode": n * (E + M + M + fb) + fs + ss,     # act, m read, m write, codes + scales
            "decode": n * (fb + M + M + E) + fs + ss,     # codes, m read, m write, out + scales
            "grad_quant": n * (E + bb) + bs,
            "grad_dequant": n * (bb + E) + bs,
            # the plain codec's launches that variant runs time for reference
            "plain_encode": n * (E + E + E + fb) + fs,
            "plain_decode": n * (fb + E + E + E) + fs,
            "dense_grad_quant": n * (E + dense) + bs,
            "dense_grad_dequant": n * (dense + E) + bs,
        }


class DeviceClock:
    """Times work queued on one stream with a HIP event pair recorded on that stream.

    The host cannot enqueue as fast as the GPU drains a few hundred microseconds of
    kernels, so a bracket taken on an idle stream would also hold the host's launch
    latency.  Here a spin kernel is queued first; while it runs the host records the
    start event, enqueues all the work and records the stop event, so when the spin
    ends the stream goes through start, the work and stop back to back and the event
    pair holds device time only.  Every kernel of the timed region lies between the two
    events; a wall clock around the same region (synchronised on both sides) is reported
    next to it."""

    def __init__(self, torch, stream):
        self.torch, self.stream = torch, stream
        # how long one million spin cycles take on this device
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            torch.cuda._sleep(1_000_000)
            a.record(stream)
            torch.cuda._sleep(1_000_000)
            b.record(stream)
        torch.cuda.synchronize()
        self.cycles_per_ms = 1_000_000 / max(a.elapsed_time(b), 1e-3)

    def time(self, enqueue, hold_ms=2.0):
        """enqueue() queues the work on self.stream.  Returns (device seconds, wall seconds)."""
        torch = self.torch
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(self.stream):
            torch.cuda._sleep(int(hold_ms * self.cycles_per_ms))
            a.record(self.stream)
            enqueue()
            b.record(self.stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0 - hold_ms * 1e-3
        return a.elapsed_time(b) * 1e-3, wall

    def time_streams(self, streams, enqueue, hold_ms=2.0):
        """Independent work on several streams: enqueue(i) queues stream i's part on the
        current stream.  Every stream waits for the end of one spin kernel (on
        self.stream), stamps a start event, runs its part and stamps a stop event; the
        region runs from the earliest start to the latest stop, so every kernel of every
        stream lies inside it and no fork or join between streams does.  Returns (device
        seconds, wall seconds)."""
        torch = self.torch
        ev = lambda: torch.cuda.Event(enable_timing=True)
        starts, stops = [ev() for _ in streams], [ev() for _ in streams]
        opened = torch.cuda.Event()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(self.stream):
            torch.cuda._sleep(int(hold_ms * self.cycles_per_ms))
            opened.record(self.stream)
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                st.wait_event(opened)
                starts[i].record(st)
                enqueue(i)
                stops[i].record(st)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0 - hold_ms * 1e-3
        first = min(range(len(streams)), key=lambda i: starts[0].elapsed_time(starts[i]))
        return max(starts[first].elapsed_time(b) for b in stops) * 1e-3, wall


_SIDE_BY_SIDE = {}


def side_by_side_streams(torch, n):
    """n streams whose kernels really run next to each other, the same ones for every timed
    region of the process.  A process has a few hardware queues and the runtime spreads its
    streams over them; two streams that share a queue take turns, and which streams of
    torch's pool do so depends on how many were handed out before (regions timed later in
    a process were 14 % slower for that reason alone).  So candidates are tried in pairs
    with two spin kernels and a stream is taken only if it overlaps with those already
    taken.  More streams than hardware queues cannot all overlap: past four, streams are
    taken as they come."""
    have = _SIDE_BY_SIDE.setdefault("streams", [])
    if "cycles_per_ms" not in _SIDE_BY_SIDE:
        _SIDE_BY_SIDE["cycles_per_ms"] = DeviceClock(torch, torch.cuda.Stream()).cycles_per_ms
    spin = int(0.3 * _SIDE_BY_SIDE["cycles_per_ms"])

    def spin_ms(streams_):
        """Device time from a common start to the end of one spin kernel per stream."""
        s0 = torch.cuda.Event(enable_timing=True)
        ends = [torch.cuda.Event(enable_timing=True) for _ in streams_]
        torch.cuda.synchronize()
        s0.record(streams_[0])
        for st, e in zip(streams_, ends):
            st.wait_event(s0)
            with torch.cuda.stream(st):
                torch.cuda._sleep(spin)
                e.record(st)
        torch.cuda.synchronize()
        return max(s0.elapsed_time(e) for e in ends)

    def overlap(a, b):
        return spin_ms([a, b]) < 1.5 * spin_ms([a])

    tries = 0
    while len(have) < n:
        c = torch.cuda.Stream()
        tries += 1
        if len(have) >= 4 or tries > 64 or all(overlap(h, c) for h in have):
            have.append(c)
    return have[:n]


def evict_caches(torch, scratch, footprint_bytes):
    """Make sure the next kernels find none of their rows cached.  A region that itself
    touches more than 1 GiB of distinct rows (four times the last-level cache) has evicted
    its own first rows by the time its untimed replay ends; a smaller one is followed by a
    pass over 1 GiB of scratch.  (That pass leaves the cache full of modified lines, whose
    write-back would be charged to the timed kernels: it is not made where it is not needed.)"""
    if footprint_bytes < (1 << 30):
        scratch.add_(1)
    torch.cuda.synchronize()


def stream_part(wl, i, n_streams, k0, k1, schedule, backward=True):
    """Queues on the current stream what stream i of n_streams does of steps k0..k1-1.
    Micro-batches touch disjoint samples and buffers, so the streams' parts are
    independent of each other: stream i takes the micro-batches k0+i, k0+i+n, ... — as one
    chain of fused launches, or as their single calls one after the other."""
    ks = list(range(k0 + i, k1, n_streams))
    if schedule != "calls":
        wl.fused_chain(ks, schedule, backward)
        return
    for k in ks:
        wl.step(k, backward)


def timed_steps(wl, first, count, launch, n_streams, backward=True, schedule="calls"):
    """Run `count` steps starting at step index `first`; returns (device seconds, wall
    seconds) of the whole region.  Each stream's part is recorded into HIP graphs of its
    own (one stream per capture, nothing between streams inside a graph); the graphs are
    built, instantiated and replayed once before the clock starts (the first replay of a
    new graph uploads it); the caches are then evicted, so the timed replay reads cold rows
    again.  The clock is DeviceClock.time_streams."""
    torch = wl.torch
    streams = side_by_side_streams(torch, n_streams)
    clock = DeviceClock(torch, torch.cuda.Stream())

    if launch == "eager":
        # the spin must outlast the host's enqueueing of every launch (about 10 us each)
        return clock.time_streams(
            streams, lambda i: stream_part(wl, i, n_streams, first, first + count, schedule, backward),
            hold_ms=2.0 + 0.05 * count)
    graphs = [[] for _ in streams]
    k = first
    while k < first + count:
        m = min(GRAPH_STEPS, first + count - k)
        # a multiple of the stream count per graph keeps every stream's share of a graph the same
        for i, st in enumerate(streams):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=st):
                stream_part(wl, i, n_streams, k, k + m, schedule, backward)
            graphs[i].append(g)
        k += m

    def replay(i):
        for g in graphs[i]:
            g.replay()
    for i, st in enumerate(streams):                     # untimed: uploads the graphs
        with torch.cuda.stream(st):
            replay(i)
    lb = wl.leg_bytes()
    evict_caches(torch, wl.evict, count * sum(lb[l] for l in (wl.LEGS if backward else wl.LEGS[:2])))
    return clock.time_streams(streams, replay)


def hot_forward_pairs(wl, k, count):
    """Footnote figure: the same forward pair (same samples, same pool slot) over and
    over on one stream, so its rows stay in the last-level cache.  Seconds per pair."""
    torch = wl.torch
    main = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=main):
        for _ in range(count):
            wl.step(k, backward=False)
    with torch.cuda.stream(main):
        g.replay()
    dev, _ = DeviceClock(torch, main).time(g.replay)
    return dev / count


def one_stream_forward_pairs(wl, first, count=256, warm=20):
    """The forward message on ONE stream: `count` encode -> decode pairs of successive
    cold micro-batches, strictly one kernel after the other, after `warm` untimed pairs;
    HIP events around the pairs.  Seconds per pair."""
    torch = wl.torch
    main = torch.cuda.Stream()
    with torch.cuda.stream(main):
        for k in range(first, first + warm):
            wl.step(k, backward=False)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=main):
        for k in range(first + warm, first + warm + count):
            wl.step(k, backward=False)
    with torch.cuda.stream(main):
        g.replay()
    lb = wl.leg_bytes()
    evict_caches(torch, wl.evict, count * (lb["encode"] + lb["decode"]))
    dev, _ = DeviceClock(torch, main).time(g.replay)
    return dev / count


def stream_copy_ceiling(torch, nbytes=1 << 30, reps=5):
    """Same-run achievable ceiling: a plain device-to-device copy of `nbytes`
    (read + written bytes per second, GB/s)."""
    src = torch.empty(nbytes // 2, dtype=torch.float16, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    return 2.0 * nbytes * reps / (a.elapsed_time(b) * 1e-3) / 1e9


def kernel_legs(wl, first, count, schedule="calls"):
    """Per-launch device durations over `count` steps (HIP events stamped by the launch
    itself, on the stream the kernel runs on), every launch on its own, one after the
    other: the four single-message calls, and the launches of the fused schedule (a
    launch that carries several jobs is timed as the one kernel it is)."""
    torch, B = wl.torch, wl.B
    count = min(count, 1024)
    fused = {}
    one_launch = (wl.cfg.fwd_rounding == wl.cfg.bwd_rounding and wl.cfg.fwd_group == wl.cfg.bwd_group
                  and not wl.m_bits and not wl.keep)
    if schedule == "stage" and not wl.m_bits and not wl.keep:
        fused = {"sender_launch(encode+grad_dequant)": ("encode", "grad_dequant"),
                 "receiver_launch(decode+grad_quant)": ("decode", "grad_quant")}
    elif schedule == "pipeline" and one_launch:
        fused = {"slot_launch(encode+decode+grad_quant+grad_dequant)": wl.LEGS}
    singles = list(wl.LEGS) + list(wl.reference_legs())
    names = singles + list(fused)
    pairs = {leg: [] for leg in names}
    for leg in names:
        for _ in range(count):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); b.record()                       # creates the HIP events
            pairs[leg].append((a, b))
    torch.cuda.synchronize()
    for k in range(first + 2 * count, first + 2 * count + 24):      # untimed: clocks in their working state
        for leg in singles:
            getattr(wl, leg)(k)
    torch.cuda.synchronize()
    for i, k in enumerate(range(first, first + count)):
        for leg in singles:
            a, b = pairs[leg][i]
            B.profile_next_launch(a, b)
            getattr(wl, leg)(k)
    torch.cuda.synchronize()
    # fused launches: the jobs of one launch come from different micro-batches, as in the
    # schedule (encode k, decode / grad_quant k-1, grad_dequant k-2), so they are independent
    lag = {"encode": 0, "decode": 1, "grad_quant": 1, "grad_dequant": 2}
    for name, members in fused.items():
        for i, k in enumerate(range(first + count, first + 2 * count)):
            a, b = pairs[name][i]
            B.profile_next_launch(a, b)
            B.run_jobs([wl.job(m, k - lag[m]) for m in members])
    torch.cuda.synchronize()
    out = {}
    for leg in names:
        ms = [a.elapsed_time(b) for a, b in pairs[leg]]
        ms.sort()
        out[leg] = {"avg_us": 1e3 * sum(ms) / len(ms), "median_us": 1e3 * ms[len(ms) // 2],
                    "min_us": 1e3 * ms[0], "launches": len(ms), "members": fused.get(leg, (leg,))}
    return out


def cpu_baseline(cfg, calls):
    """The oracle, as it stands, on this machine's host cores: the forward message
    (encode + decode, the metric's quantity) and the whole step on full-shape
    micro-batches of the same workload, each micro-batch with its own samples.  The
    samples are seeded by one untimed visit first, so the timed calls encode changes.
    Median over the micro-batches."""
    import numpy as np
    import oracle
    from oracle.boundary import OracleBoundary
    from paper_2206_01299_amd import workloads as W
    oracle.build()
    threads = oracle.max_threads()
    n_mb = calls if calls > 0 else 8
    visited = W.parity_ids(cfg, n_mb)
    stream = W.ActivationStream(cfg, visited=visited)
    cpu = OracleBoundary(cfg, visited)
    batches = stream.epoch_ids(0)
    grads = [stream.gradients(ids, 0) for ids in batches]
    for k, ids in enumerate(batches):                              # seed m: later calls send changes
        cpu.forward(stream.activations(ids, 0), ids, k)
    acts = [stream.activations(ids, 1) for ids in batches]

    def run(first_seed):
        fwd, step = [], []
        for k, ids in enumerate(batches):
            t0 = time.perf_counter()
            cpu.forward(acts[k], ids, first_seed + k)
            t1 = time.perf_counter()
            cpu.backward(grads[k], first_seed + k)
            t2 = time.perf_counter()
            fwd.append(t1 - t0)
            step.append(t2 - t0)
        return float(np.median(fwd)), float(np.median(step))

    fwd, step = run(1000)
    oracle.set_threads(1)                                          # the same on one thread
    one = min(n_mb, max(2, int(6.0 / max(step * threads, 1e-3))))
    keep = batches
    batches = batches[:one]
    fwd1, step1 = run(2000)
    batches = keep
    oracle.set_threads(threads)
    act_bytes = cfg.n * cfg.elem_bytes
    return {"value": act_bytes / fwd / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "ms_per_fwd_pair": fwd * 1e3, "ms_per_step": step * 1e3,
            "step_act_GBps": round(act_bytes / step / 1e9, 4),
            "one_thread": {"value": round(act_bytes / fwd1 / 1e9, 4), "ms_per_fwd_pair": round(fwd1 * 1e3, 1),
                           "ms_per_step": round(step1 * 1e3, 1), "microbatches": one},
            "sample": f"{n_mb} distinct full-shape micro-batches of {cfg.name} ({cfg.batch} samples each), "
                      f"second visit of every sample; value = activation bytes / median time of "
                      f"encode + decode; OpenMP over groups"}


def read_traffic():
    """HBM bytes per launch from the committed rocprofv3 counter summary (a stored value,
    labelled as such in the line; None if it has not been collected)."""
    f = ROOT / "profiles" / "hbm_traffic_gpt2_fw4.txt"
    if not f.exists():
        return None
    vals = {}
    for line in f.read_text().splitlines():
        if ":" in line and not line.startswith("#"):
            k, v = line.split(":", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except (ValueError, IndexError):
                pass
    return vals or None


def read_slot_traffic(config):
    """The same for the slot launch of configurations 3, 4 and 5: read + written HBM bytes from
    the committed counter summary of that configuration (None if there is none)."""
    f = ROOT / "profiles" / "hbm_traffic_configs_3_4_5.md"
    if not f.exists():
        return None
    rows = f.read_text().splitlines()
    for i, line in enumerate(rows):
        if line.startswith(f"## {config} "):
            for data in rows[i + 1:i + 5]:
                cols = data.split()
                if len(cols) == 6:
                    try:
                        return (float(cols[0]) + float(cols[3])) * 1e6
                    except ValueError:
                        continue
    return None


def isolated_launches(torch, B, count, launch):
    """Average device duration (us) of `count` single launches made by launch(i), each
    stamped by the library's timed-launch hook on its own stream."""
    pairs = []
    for _ in range(count):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(); b.record()
        pairs.append((a, b))
    for i in range(count, count + 24):                   # untimed: clocks and caches in their working state
        launch(i)
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(pairs):
        B.profile_next_launch(a, b)
        launch(i)
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in pairs)
    return {"avg_us": round(1e3 * sum(ms) / len(ms), 3), "median_us": round(1e3 * ms[len(ms) // 2], 3),
            "min_us": round(1e3 * ms[0], 3), "launches": count}


def torch_copy_us(torch, src_pool, dst_pool, reps):
    """A plain device-to-device copy of one pool slot per launch, cold rotating slots (us)."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = src_pool.shape[0]
    for i in range(4):
        dst_pool[i % n].copy_(src_pool[i % n])
    torch.cuda.synchronize()
    a.record()
    for i in range(reps):
        dst_pool[i % n].copy_(src_pool[(i + n // 2) % n])
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / reps


class Boundaries:
    """Several stage boundaries handled at the same time (Appendix A.1's K machines are K-1
    independent instances of the two-machine scheme; a machine in the middle has two of
    them): the same schedules as Workload's, every launch carrying the messages of all the
    boundaries.  Has what timed_steps() uses of a Workload."""

    LEGS = Workload.LEGS

    def __init__(self, wls):
        self.wls = wls
        self.torch, self.B, self.evict = wls[0].torch, wls[0].B, wls[0].evict

    def step(self, k, backward=True):
        for w in self.wls:
            w.step(k, backward)

    def leg_bytes(self):
        out = {}
        for w in self.wls:
            for l, v in w.leg_bytes().items():
                out[l] = out.get(l, 0.0) + v
        return out

    def fused_chain(self, ks, schedule, backward=True):
        B, n = self.B, len(ks)
        assert schedule == "pipeline"
        for t in range(n + (2 if backward else 1)):
            jobs = []
            for w in self.wls:                           # the slot of Workload.fused_chain, per boundary
                if t < n:
                    jobs.append(w.job("encode", ks[t]))
                if 0 <= t - 1 < n:
                    jobs.append(w.job("decode", ks[t - 1]))
                    if backward:
                        jobs.append(w.job("grad_quant", ks[t - 1]))
                if backward and 0 <= t - 2 < n:
                    jobs.append(w.job("grad_dequant", ks[t - 2]))
            if jobs:
                B.run_jobs(jobs)


def boundaries_line(args):
    """The stress configuration as it is written: several boundaries with forward messages of
    2, 4 and 8 bits worked on concurrently.  One aqsgd_run_jobs call per time slot holds the
    slot's messages of every boundary (the library packs them into launches of up to 8 + 8
    jobs); micro-batches are dealt over two streams as in the default schedule."""
    import torch
    from paper_2206_01299_amd import workloads as W
    n_b = args.boundaries
    cfgs = [W.stress(W.STRESS_BITS[i % len(W.STRESS_BITS)], i) for i in range(n_b)]
    pool = max(4, -(-1_250_000_000 // (cfgs[0].n * cfgs[0].elem_bytes * n_b)))
    wls = []
    for i, c in enumerate(cfgs):
        w = Workload(c, pool, seed=1234 + i)
        w.preseed_and_drift()
        wls.append(w)
    both = Boundaries(wls)
    K, Wm = args.steps, args.warmup
    for k in range(Wm):
        both.step(k)
    torch.cuda.synchronize()
    n_streams = args.streams or 2
    step_dev, step_wall = timed_steps(both, Wm, K, args.launch, n_streams, schedule="pipeline")
    fwd_dev, fwd_wall = timed_steps(both, Wm, K, args.launch, n_streams, backward=False, schedule="pipeline")
    lb = both.leg_bytes()
    act_bytes = sum(c.n * c.elem_bytes for c in cfgs)
    fwd_bytes, step_bytes = lb["encode"] + lb["decode"], sum(lb[l] for l in Workload.LEGS)
    value = act_bytes / (fwd_dev / K) / 1e9
    line = {
        "metric": "encode+decode GB/s of activations, %d stress-shaped boundaries at the same time" % n_b,
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(step_dev / K * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%d stage boundaries, each float32 activations [8,2048,4096], 256-sample m_buf x2, "
                               "forward %s-bit per-row delta codec, backward 8-bit direct; a step is one "
                               "micro-batch of every boundary" % (n_b, "/".join(str(c.fwd_bits) for c in cfgs)),
                   "name": "stress_%d_boundaries" % n_b, "schedule": "pipeline", "streams": n_streams,
                   "value_is": "activation bytes of one micro-batch of every boundary / time of their encodes "
                               "and decodes (second timed run without the backward messages)"},
        "roofline": None, "cpu_baseline": None,
        "fwd_only": {"us_per_step": round(fwd_dev / K * 1e6, 2),
                     "hbm_GBps": round(fwd_bytes / (fwd_dev / K) / 1e9, 1),
                     "frac_of_hbm_peak": round(fwd_bytes / (fwd_dev / K) / 1e9 / HBM_PEAK_GBPS, 4)},
        "whole_step": {"us": round(step_dev / K * 1e6, 2),
                       "hbm_GBps": round(step_bytes / (step_dev / K) / 1e9, 1),
                       "frac_of_hbm_peak": round(step_bytes / (step_dev / K) / 1e9 / HBM_PEAK_GBPS, 4),
                       "algorithmic_bytes": step_bytes},
    }
    print(json.dumps(line))


def first_visit_line(args, cfg, wl):
    """Algorithm 1's first-visit branch: one epoch in which every sample is new (the message
    is the activation itself, both stages store it as m), then the same calls again (every
    sample seen: the ordinary codec path through the same entry points)."""
    torch, B = wl.torch, wl.B
    d = wl.dev
    # the untimed launches that precede every timed batch visit samples of their own
    n_calls = min(wl.calls - 32, max(64, args.steps))
    seen_s = torch.zeros(cfg.n_samples, dtype=torch.int32, device=d)
    seen_r = torch.zeros_like(seen_s)
    first = torch.zeros((wl.pool, cfg.batch), dtype=torch.int32, device=d)
    wl.m_send.zero_(); wl.m_recv.zero_()
    act_bytes = cfg.n * cfg.elem_bytes
    lb = wl.leg_bytes()

    def enc(k, stamp):
        s = k % wl.pool
        B.encode_seen(wl.fdesc, wl.act[s], wl.ids[k % wl.calls], wl.m_send, seen_s, stamp, first[s],
                      wl.codes[s], wl.scales[s])

    def dec(k, stamp):
        s = k % wl.pool            # on a first visit the uncompressed rows are the message
        B.decode_seen(wl.fdesc, wl.codes[s], wl.scales[s], wl.act[s], wl.ids[k % wl.calls], wl.m_recv, seen_r,
                      stamp, wl.out[s])

    res = {}
    res["encode_seen_first"] = isolated_launches(torch, B, n_calls, lambda i: enc(i, 1 + i))
    res["decode_seen_first"] = isolated_launches(torch, B, n_calls, lambda i: dec(i, 1 + i))
    assert int((seen_s != 0).sum()) >= n_calls * cfg.batch and bool((seen_s != 0).eq(seen_r != 0).all())
    assert bool(torch.equal(wl.m_send, wl.m_recv))
    res["encode_seen_second"] = isolated_launches(torch, B, n_calls, lambda i: enc(i, 100000 + i))
    res["decode_seen_second"] = isolated_launches(torch, B, n_calls, lambda i: dec(i, 100000 + i))
    assert bool(torch.equal(wl.m_send, wl.m_recv))
    res["seed"] = isolated_launches(
        torch, B, n_calls, lambda i: B.seed(wl.fdesc, wl.act[i % wl.pool], wl.ids[i % wl.calls], wl.m_send))
    # the same copies through the runtime's own copy kernel, same size, cold slots
    copy_us = torch_copy_us(torch, wl.act, wl.out, n_calls)
    bytes_of = {"encode_seen_first": 2 * act_bytes, "decode_seen_first": 3 * act_bytes, "seed": 2 * act_bytes,
                "encode_seen_second": lb["encode"], "decode_seen_second": lb["decode"]}
    for k, v in res.items():
        v["bytes"] = bytes_of[k]
        v["hbm_GBps"] = round(bytes_of[k] / v["avg_us"] / 1e3, 1)
        v["frac_of_hbm_peak"] = round(bytes_of[k] / v["avg_us"] / 1e3 / HBM_PEAK_GBPS, 4)

    # the whole first epoch as a pipeline would run it: sender and receiver alternate on one
    # stream; device time by events around a graph replay
    wl.m_send.zero_(); wl.m_recv.zero_(); seen_s.zero_(); seen_r.zero_()
    main = torch.cuda.Stream()
    clock = DeviceClock(torch, main)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=main):
        for k in range(n_calls):
            enc(k, 1 + k)
            dec(k, 1 + k)
    dev_first, _ = clock.time(g.replay)          # every sample new (the graph's first replay)
    dev_second, _ = clock.time(g.replay)         # same stamps again: the samples count as new once more
    pair_first = dev_second / n_calls
    copy_ceiling = 2 * act_bytes / (copy_us * 1e-6) / 1e9
    seed_gbps = res["seed"]["hbm_GBps"]
    line = {
        "metric": "first-visit path (uncompressed message, m <- a on both stages) GB/s against a same-run "
                  "copy of the same size",
        "value": round(seed_gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": n_calls, "warmup": 0,
        "ms_per_step": round(pair_first * 1e3, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.config] + "; first epoch: every sample new",
                   "value_is": "read + written bytes per second of aqsgd_seed (m_buf[ids] <- act), isolated "
                               "launches on cold rows",
                   "step": "aqsgd_encode_seen + aqsgd_decode_seen of one micro-batch of new samples "
                           "(ms_per_step: back to back on one stream, second replay of the graph)"},
        "seed_vs_copy": {"seed_GBps": seed_gbps, "copy_same_size_GBps": round(copy_ceiling, 1),
                         "ratio": round(seed_gbps / copy_ceiling, 3),
                         "copy_1GiB_GBps": round(stream_copy_ceiling(torch), 1)},
        "first_replay_us_per_pair": round(dev_first / n_calls * 1e6, 3),
        "launches": res, "roofline": {"bound": "hbm", "kernel": "seed", "achieved": seed_gbps,
                                      "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                      "frac": round(seed_gbps / HBM_PEAK_GBPS, 4), "traffic": None},
        "cpu_baseline": None,
    }
    print(json.dumps(line))


def ceilings_line(args, cfg, wl):
    """What launches of the codec's size can reach on this GPU, measured with the library's
    own kernels and the runtime's fill / copy: the fixed cost of a launch, and how the
    achieved bandwidth grows with the bytes per launch."""
    torch, B = wl.torch, wl.B
    d = wl.dev
    out = {}
    flag = torch.zeros(1, dtype=torch.int32, device=d)
    one_id = torch.zeros(1, dtype=torch.int64, device=d)
    out["near_empty_launch"] = isolated_launches(
        torch, B, 256, lambda i: B.check_ids(one_id, cfg.n_samples, flag))
    td = B.DTYPE_NAME[cfg.dtype]
    rows = 64                                    # a pool of 64-row micro-batches for the size sweep
    n_big = max(2, min(6, wl.pool * cfg.batch // rows))
    act = wl.act.view(-1, cfg.n_per)
    outp = wl.out.view(-1, cfg.n_per)
    perm = torch.randperm(cfg.n_samples, device=d)
    table = []
    for b in (1, 2, 4, 8, 16, 32, 64):
        if b * 8 > act.shape[0]:
            break
        desc = B.make_desc(batch=b, n_per=cfg.n_per, n_samples=cfg.n_samples, bits=cfg.fwd_bits,
                           group=cfg.fwd_group, dtype=cfg.dtype, rounding=cfg.fwd_rounding)
        codes = torch.empty((8, B.codes_bytes(desc)), dtype=torch.uint8, device=d)
        scales = torch.empty((8, B.scales_count(desc)), dtype=torch.float32, device=d)
        slots = act.shape[0] // b
        calls = cfg.n_samples // b
        reps = max(16, min(256, 4096 // b))

        def a_of(i): return act[(i % slots) * b:(i % slots + 1) * b]
        def o_of(i): return outp[(i % slots) * b:(i % slots + 1) * b]
        def ids_of(i): return perm[(i % calls) * b:(i % calls + 1) * b]
        row = {"batch": b, "bytes_encode": b * cfg.n_per * (3 * cfg.elem_bytes + cfg.fwd_bits / 8) +
                                           4.0 * b * cfg.n_per / cfg.fwd_group}
        row["seed_us"] = isolated_launches(torch, B, reps, lambda i: B.seed(desc, a_of(i), ids_of(i),
                                                                            wl.m_send))["avg_us"]
        row["encode_us"] = isolated_launches(torch, B, reps, lambda i: B.encode(
            desc, a_of(i), ids_of(i), wl.m_send, codes[i % 8], scales[i % 8]))["avg_us"]
        row["decode_us"] = isolated_launches(torch, B, reps, lambda i: B.decode(
            desc, codes[i % 8], scales[i % 8], ids_of(i), wl.m_recv, o_of(i)))["avg_us"]
        copy_bytes = 2.0 * b * cfg.n_per * cfg.elem_bytes
        row["seed_GBps"] = round(copy_bytes / row["seed_us"] / 1e3, 1)
        row["encode_GBps"] = round(row["bytes_encode"] / row["encode_us"] / 1e3, 1)
        row["decode_GBps"] = round(row["bytes_encode"] / row["decode_us"] / 1e3, 1)
        table.append(row)
    out["launch_size_sweep"] = table
    big = torch.empty(1 << 29, dtype=torch.float16, device=d)
    big2 = torch.empty_like(big)
    a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    big.fill_(1.0); big2.copy_(big); torch.cuda.synchronize()
    a.record()
    for _ in range(5):
        big.fill_(2.0)
    b_.record(); torch.cuda.synchronize()
    out["fill_1GiB_GBps"] = round((1 << 30) * 5 / (a.elapsed_time(b_) * 1e-3) / 1e9, 1)
    out["copy_1GiB_GBps"] = round(stream_copy_ceiling(torch), 1)
    seed64 = table[-1]
    line = {
        "metric": "ceilings of this GPU at the codec's launch sizes (GB/s of read + written bytes)",
        "value": seed64["seed_GBps"], "unit": "GB/s", "n_gpus": 1, "steps": 0, "warmup": 0,
        "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.config] + "; launch-size sweep",
                   "value_is": f"the library's row copy (aqsgd_seed) at {seed64['batch']} rows per launch",
                   "method": "every figure is the average device duration of isolated launches on cold rows, "
                             "stamped by HIP events on the launching stream"},
        "ceilings": out, "roofline": None, "cpu_baseline": None,
    }
    print(json.dumps(line))


def region_sweep_line(args, cfg, wl, sched, n_streams):
    """The timed region at growing step counts, same process, same schedule and streams."""
    for k in range(16):
        wl.step(k)
    wl.torch.cuda.synchronize()
    rows = []
    for K in (10, 20, 40, 80, 160, 320):
        step = [timed_steps(wl, 16, K, args.launch, n_streams, schedule=sched)[0] for _ in range(3)]
        fwd = [timed_steps(wl, 16, K, args.launch, n_streams, backward=False, schedule=sched)[0] for _ in range(3)]
        step.sort(); fwd.sort()
        rows.append({"steps": K, "step_region_us": round(step[1] * 1e6, 1), "us_per_step": round(step[1] / K * 1e6, 3),
                     "fwd_region_us": round(fwd[1] * 1e6, 1), "us_per_fwd_pair": round(fwd[1] / K * 1e6, 3)})
    act_bytes = cfg.n * cfg.elem_bytes
    line = {
        "metric": "timed region length sweep: device time of K steps and of their forward messages alone",
        "value": round(act_bytes / (rows[-1]["us_per_fwd_pair"] * 1e-6) / 1e9, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": rows[-1]["steps"], "warmup": 16, "ms_per_step": round(rows[-1]["us_per_step"] * 1e-3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.config] + "; region-length sweep", "schedule": sched,
                   "streams": n_streams, "launch": args.launch,
                   "value_is": "activation GB/s of encode + decode at the longest region",
                   "method": "median of three timed regions per length, the clock of the headline line"},
        "region_sweep": rows, "roofline": None, "cpu_baseline": None,
    }
    print(json.dumps(line))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the codec of one stage boundary; no collectives). "
              "Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the codec has no CPU path.", file=sys.stderr)
        sys.exit(3)
    from paper_2206_01299_amd import binding as B
    from paper_2206_01299_amd import build as _build
    from paper_2206_01299_amd import workloads as W
    if not _build.LIB.exists():          # load what is built; build only if nothing is
        _build.build(verbose=False)
    B.lib()

    cfg = {"gpt2_4bit": W.gpt2_4bit, "gpt2_2bit_stochastic": W.gpt2_2bit_stochastic,
           "deberta_3bit": W.deberta_3bit, "stress": W.stress}[args.config]()
    K, Wm = args.steps, args.warmup
    if args.boundaries > 1:
        if args.config != "stress" or args.boundaries > 8:
            print("bench.py: --boundaries (2..8) goes with --config stress.", file=sys.stderr)
            sys.exit(2)
        boundaries_line(args)
        return
    if args.pool <= 0:
        args.pool = max(4, -(-1_250_000_000 // (cfg.n * cfg.elem_bytes)))
    t_setup = time.perf_counter()
    wl = Workload(cfg, args.pool, m_bits=args.m_bits, bwd_keep=args.bwd_keep)
    wl.preseed_and_drift()
    t_setup = time.perf_counter() - t_setup

    if args.calibration_copy:
        src = torch.empty(1 << 29, dtype=torch.float16, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.first_visit:
        first_visit_line(args, cfg, wl)
        return
    if args.ceilings:
        ceilings_line(args, cfg, wl)
        return

    for k in range(Wm):                                  # untimed warm-up, eager
        wl.step(k)
    torch.cuda.synchronize()

    # K whole steps, then the forward messages of the same K micro-batches alone
    sched = args.schedule
    if args.m_bits or args.bwd_keep:
        sched = "calls"                                  # these variants have single-message calls only
    if args.streams == 0:
        args.streams = 8 if sched == "calls" else 2
    if args.region_sweep:
        region_sweep_line(args, cfg, wl, sched, args.streams)
        return
    step_dev, step_wall = timed_steps(wl, Wm, K, args.launch, args.streams, schedule=sched)
    fwd_dev, fwd_wall = timed_steps(wl, Wm, K, args.launch, args.streams, backward=False, schedule=sched)
    ms_per_step = step_dev / K * 1e3
    act_bytes = cfg.n * cfg.elem_bytes
    value = act_bytes / (fwd_dev / K) / 1e9              # the metric: encode + decode, activation bytes

    legs = None if args.no_kernel_legs else kernel_legs(wl, Wm, max(K, 512), sched)
    lb = wl.leg_bytes()
    roofline = None
    extra = {}
    if legs:
        for l in legs:                                   # a fused launch moves its members' bytes
            lb.setdefault(l, sum(lb[m] for m in legs[l]["members"]))
        # the dominant kernel: the longest launch among those the timed schedule makes
        ref = wl.reference_legs()
        in_schedule = [l for l in legs if l not in wl.LEGS and l not in ref] or list(wl.LEGS)
        dominant = max(in_schedule, key=lambda l: legs[l]["avg_us"])
        a_gbps = lb[dominant] / (legs[dominant]["avg_us"] * 1e-6) / 1e9
        traffic = (read_traffic() if args.config == "gpt2_4bit" and not args.m_bits and not args.bwd_keep
                   else None)
        roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(a_gbps, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(a_gbps / HBM_PEAK_GBPS, 4),
                    "algorithmic_bytes_per_launch": lb[dominant],
                    "avg_launch_us": round(legs[dominant]["avg_us"], 3),
                    "launches_timed": legs[dominant]["launches"],
                    "traffic": (traffic or {}).get(f"{dominant.split('(')[0]}_hbm_bytes_per_launch"),
                    "traffic_source": "stored rocprofv3 counter value (profiles/hbm_traffic_gpt2_fw4.txt), "
                                      "not measured in this run" if traffic else None}
        if (traffic is None and dominant.startswith("slot_launch") and not args.m_bits and not args.bwd_keep):
            slot = read_slot_traffic(args.config)        # configurations 3, 4, 5
            if slot:
                roofline["traffic"] = slot
                roofline["traffic_source"] = ("stored rocprofv3 counter value "
                                              "(profiles/hbm_traffic_configs_3_4_5.md), not measured in this run")
        pair_us = legs["encode"]["avg_us"] + legs["decode"]["avg_us"]
        pair_bytes = lb["encode"] + lb["decode"]
        extra["fwd_pair_isolated_launches"] = {"us": round(pair_us, 3),
                             "act_GBps": round(act_bytes / pair_us / 1e3, 1),
                             "hbm_GBps": round(pair_bytes / pair_us / 1e3, 1),
                             "frac_of_hbm_peak": round(pair_bytes / pair_us / 1e3 / HBM_PEAK_GBPS, 4)}
        extra["kernels"] = {l: {"avg_us": round(legs[l]["avg_us"], 3),
                                "median_us": round(legs[l]["median_us"], 3),
                                "hbm_GBps": round(lb[l] / legs[l]["avg_us"] / 1e3, 1)} for l in legs}
        if wl.reference_legs():
            extra["reference_legs"] = {
                "legs": list(wl.reference_legs()),
                "note": "the plain codec's launches on the same micro-batches, timed in this process in "
                        "turn with the variant's (same clocks, same box); not part of the timed steps"}
    fwd_bytes = lb["encode"] + lb["decode"]
    step_bytes = sum(lb[l] for l in wl.LEGS)
    extra["fwd_only"] = {"us_per_microbatch": round(fwd_dev / K * 1e6, 3),
                         "act_GBps": round(value, 1),
                         "hbm_GBps": round(fwd_bytes / (fwd_dev / K) / 1e9, 1),
                         "frac_of_hbm_peak": round(fwd_bytes / (fwd_dev / K) / 1e9 / HBM_PEAK_GBPS, 4),
                         "wall_us_per_microbatch": round(fwd_wall / K * 1e6, 3)}
    extra["whole_step"] = {"us": round(step_dev / K * 1e6, 3),
                           "act_GBps": round(act_bytes / (step_dev / K) / 1e9, 1),
                           "hbm_GBps": round(step_bytes / (step_dev / K) / 1e9, 1),
                           "frac_of_hbm_peak": round(step_bytes / (step_dev / K) / 1e9 / HBM_PEAK_GBPS, 4),
                           "wall_us": round(step_wall / K * 1e6, 3)}
    one = one_stream_forward_pairs(wl, Wm + K)
    extra["fwd_one_stream"] = {"us_per_microbatch": round(one * 1e6, 3),
                               "act_GBps": round(act_bytes / one / 1e9, 1),
                               "frac_of_hbm_peak": round(fwd_bytes / one / 1e9 / HBM_PEAK_GBPS, 4),
                               "note": "256 encode -> decode pairs of cold micro-batches on one stream after 20 "
                                       "untimed pairs, HIP events around them"}
    hot = hot_forward_pairs(wl, Wm, 256)
    extra["fwd_hot_buffers_footnote"] = {"us_per_microbatch": round(hot * 1e6, 3),
                                         "note": "one micro-batch repeated on one stream: rows stay in the "
                                                 "last-level cache; not the headline"}
    extra["stream_copy_ceiling_GBps"] = round(stream_copy_ceiling(torch), 1)

    base = None
    if not args.no_cpu_baseline:
        base = cpu_baseline(cfg, args.cpu_calls)
        base["value"] = round(base["value"], 4)
        base["ms_per_fwd_pair"] = round(base["ms_per_fwd_pair"], 2)
        base["ms_per_step"] = round(base["ms_per_step"], 2)

    line = {
        "metric": "encode+decode GB/s of activations (and % HBM peak), 4-bit GPT2-1.5B boundary",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.config],
                   "name": cfg.name,
                   "step": "encode + decode + grad_quant + grad_dequant of one micro-batch (ms_per_step)",
                   "value_is": "activation bytes of one micro-batch / time of its encode + decode "
                               "(the metric's quantity), from a second timed run of the same K "
                               "micro-batches without the backward message; the whole step is under "
                               "whole_step",
                   "timing": "each stream's chain of micro-batches is a sequence of HIP graphs of its own, "
                             "instantiated and replayed once beforehand; all streams wait for the end of one "
                             "spin kernel (host launch latency stays outside), each stamps a HIP event before "
                             "and after its replays, and the region runs from the earliest start stamp to the "
                             "latest stop stamp; caches evicted before the timed replay; every kernel of all "
                             "K steps is inside",
                   "storage_dtype": cfg.dtype, "batch": cfg.batch, "seq": cfg.seq, "hidden": cfg.hidden,
                   "n_samples": cfg.n_samples, "fwd_bits": cfg.fwd_bits, "bwd_bits": cfg.bwd_bits,
                   "group": cfg.fwd_group, "m_bits": args.m_bits or None, "bwd_keep": args.bwd_keep or None,
                   "pool_slots": args.pool, "launch": args.launch, "schedule": sched,
                   "streams": args.streams,
                   "streams_checked_to_overlap": args.streams in (2, 3, 4),
                   "cold_buffers": True, "device": torch.cuda.get_device_name(0),
                   "setup_s": round(t_setup, 1)},
        "roofline": roofline, "cpu_baseline": base,
    }
    line.update(extra)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
