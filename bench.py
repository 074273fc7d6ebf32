#!/usr/bin/env python3
"""Benchmark of the gradient path on one MI355X.

A step is one failure-free iteration of a workload through the C ABI: M x recover_accumulate,
recover_reduce, recover_adamw_step, recover_policy_adjust.  The headline workload (default) is the
largest single-GPU configuration, configs[4]: the Llama-70B-like 1/16 shard, 1,978,662,912 elements
in 259 tensors, bf16 gradients accumulated in fp32, R = 4 replicas, M = 16 microbatches per iteration.
Gradients are synthetic (seeded Philox streams), pre-generated into a pool of four HBM buffers before
the timed region: generating them stands in for the backward pass.

Prints ONE JSON line: effective HBM GB/s = algorithmic bytes per iteration / time, with
  roofline      the dominant kernel (the read-modify-write accumulate), timed with events on the launch
                stream inside the timed region
  cpu_baseline  the CPU oracle, as it stands, on a bounded slice of the same workload
  per_config    the other workloads (configs[1], [2], [3]), each timed the same way on a fresh context
                after the headline's buffers are freed, each with its own roofline block
and, timed separately after the headline region: every kernel's rate, snapshot and restore alone, the
one-pass variants, the non-blocking rewind, one whole failure iteration, and the read-only / copy
ceilings of this chip measured with the library's own kernels.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
POOL = 4
# Arithmetic type of the path: accumulators, contributor sum, the division and AdamW are all fp32 (bf16 is
# only the storage type of the incoming microbatch gradients of configs[2] and configs[4]).
ARITHMETIC = "f32"
SLAB = {"on": True, "pad": 4 << 20, "contiguous": True}          # buffer placement, see binding.alloc_slab

WORKLOAD_TEXT = {
    1: "configs[0] tiny: 1,048,576 fp32 elements, R=4, M=8 (cache- and launch-bound, not an HBM measurement)",
    2: "configs[1] GPT-2-small-sized shard: 123,589,632 fp32 elements in 148 tensors, R=8 replicas, "
       "M=32 microbatches/iteration, failure-free iteration",
    3: "configs[2] Llama-3-8B 1/8 HSDP shard: 1,003,749,376 elements in 30 tensors, bf16 gradients accumulated in "
       "fp32, R=8, M=64, failure-free iteration",
    4: "configs[3] heavy attrition shape: 100,663,296 fp32 elements in 12 tensors, R=64, M=128, failure-free iteration",
    5: "configs[4] Llama-70B-like 1/16 shard: 1,978,662,912 elements in 259 tensors, bf16 gradients accumulated in "
       "fp32, R=4 replicas, M=16 microbatches/iteration, failure-free iteration",
}
TRAFFIC_FILE = {5: "accumulate_bf16_llama70b_split16_shard_pmc.txt", 2: "accumulate_f32_gpt2_shard_pmc.txt"}


def bytes_per_elem(W, M, s_g, R_c):
    """Algorithmic bytes per element of one failure-free iteration: first microbatch of a
    replica writes acc and reads g; later ones also read acc; reduce reads R_c buffers and
    writes one; AdamW reads g,p,m,v and writes p,m,v."""
    acc = W * (s_g + 4) + (M - W) * (s_g + 8)
    return dict(accumulate=acc, reduce=4 * R_c + 4, adamw=28, total=acc + 4 * R_c + 4 + 28)


def read_traffic(workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary of this
    benchmark command (counters cannot be read from inside the run)."""
    name = TRAFFIC_FILE.get(workload)
    if not name:
        return None
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def quantiles(xs):
    xs = sorted(xs)
    pick = lambda q: xs[min(len(xs) - 1, int(round(q * (len(xs) - 1))))]
    return dict(mean=sum(xs) / len(xs), median=pick(0.5), p10=pick(0.1), p90=pick(0.9), n=len(xs))


def cpu_baseline(c, pool_slices, iters):
    """The oracle's fp32 protocol simulator on a contiguous slice: `iters` failure-free
    iterations (M accumulates, reduce, AdamW).  Only this leg touches oracle/."""
    import numpy as np
    from oracle.proto import Proto
    n = len(pool_slices[0])
    W, G = c["W"], c["G"]
    p = Proto(W, G, [0, n], dtype=np.float32)
    p.set_state(np.zeros(n, np.float32))
    t0 = time.perf_counter()
    for _ in range(iters):
        for k in range(G):
            for r in range(W):
                p.accumulate(r, r + W * k, pool_slices[(k * W + r) % POOL])
        p.reduce()
        p.adamw_step(**HP)
        p.advance()
    dt = time.perf_counter() - t0
    b = bytes_per_elem(W, W * G, 2 if c["bf16"] else 4, W)["total"]
    return dict(value=b * n * iters / dt / 1e9, unit="GB/s", cores=1, kind="oracle",
                sample="%d failure-free iterations of the same workload on a contiguous slice of %d elements "
                       "(oracle.proto.Proto, fp32, NumPy, one thread; %.1f s)" % (iters, n, dt),
                seconds=dt, host_cpus=os.cpu_count())


def pair_study(ballast_gib, NB=140):
    """Which pairs of buffers stream well together.  140 buffers of the configs[3] shard's size (100,663,296 fp32 elements,
    2 MiB-aligned, 4 MiB apart) in one physically contiguous slab; a one-replica context per accumulator buffer a, and
    recover_accumulate (read-modify-write: the second and later microbatches of an iteration) with buffer k as the gradient.
    Rows: a = 0, the middle, the last buffer; columns: k = 0, 4, 8, ...; and the diagonal (a, a + 4)."""
    import torch
    from paper_2605_11215_amd import binding as B
    from paper_2605_11215_amd.workloads import CONFIGS
    off = CONFIGS[4]["off"]
    N, T = off[-1], len(off) - 1
    ballast = torch.empty(ballast_gib << 30, dtype=torch.uint8, device="cuda:0") if ballast_gib else None
    if ballast is not None:
        ballast[:: 1 << 20].zero_()
    owner, bufs = B.alloc_slab([(torch.float32, N)] * NB, "cuda:0", SLAB["pad"], contiguous=True)
    stream = torch.cuda.current_stream().cuda_stream
    ctxs = {}

    def rate(a, k):
        if a not in ctxs:   # one replica, a quota that the study never reaches: every accumulate after the first is RMW
            code, ctx = B.recover_init(1, 1 << 20, off, [bufs[a].data_ptr()], None, bufs[a].data_ptr(), bufs[a].data_ptr(),
                                       bufs[a].data_ptr(), bufs[a].data_ptr(), 0, 0, 0)
            assert code == 0
            ctxs[a] = [ctx, 0]
        c = ctxs[a]
        g = bufs[k].data_ptr()
        for _ in range(2):
            assert B.recover_accumulate(c[0], 0, c[1], g, B.F32, 0, T, stream) == 0
            c[1] += 1
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(6):
            assert B.recover_accumulate(c[0], 0, c[1], g, B.F32, 0, T, stream) == 0
            c[1] += 1
        e1.record()
        torch.cuda.synchronize()
        return round(12 * N * 6 / e0.elapsed_time(e1) / 1e6)

    ks = list(range(0, NB, 4))
    # every second buffer against buffer 0: '.' = as fast as a neighbour (same zone), 'X' = 5 % or more below, '?' = between
    near = rate(0, 1)
    zone_map = "".join("." if r > 0.975 * near else ("X" if r < 0.95 * near else "?") for r in (rate(0, k) for k in range(1, NB, 2)))
    out = {"pair_study": "RMW accumulate GB/s, accumulator buffer a, gradient buffer k of %d buffers of %d fp32 elements in one slab" % (NB, N),
           "ballast_gib": ballast_gib, "contiguous": isinstance(owner, B.DeviceSlab), "slab_address": hex(owner.data_ptr()),
           "zone_map_vs_buffer_0": zone_map, "k": ks,
           "rows": {str(a): [rate(a, k) if k != a else None for k in ks] for a in (0, 68, NB - 1)},
           "diagonal_a_a_plus_4": [rate(a, a + 4) for a in range(0, NB - 4, 4)]}
    for c in ctxs.values():
        B.recover_destroy(c[0])
    return out


def one_pass_study(reps):
    """Where the one-pass reduce+AdamW kernel stops paying: for R contributors of the configs[3] shard (100,663,296 fp32
    elements, 12 tensors) the event-timed duration of recover_reduce_adamw_step forced to one kernel
    (RECOVER_TUNE_ONE_PASS_MAX = 64) and forced to k_reduce followed by k_adamw (= 0)."""
    import torch
    from paper_2605_11215_amd import binding as B
    from paper_2605_11215_amd import synth
    from paper_2605_11215_amd.synth import reference_np as S
    from paper_2605_11215_amd.workloads import CONFIGS
    c = CONFIGS[4]
    off, N, T = c["off"], c["off"][-1], len(c["off"]) - 1
    code, default = B.recover_get_tuning(B.TUNE_ONE_PASS_MAX)
    assert code == 0
    rows = []
    try:
        for R in (4, 8, 12, 16, 24, 32, 40, 48, 64):
            sh = B.Shard(R, 1, off, device="cuda:0", snapshots=False, slab=True, slab_pad=SLAB["pad"],
                         extra=[(torch.float32, N)] * 2, contiguous=SLAB["contiguous"])
            synth.fill_device(sh.param, 1, S.TAG_PARAM, 0, 0, 0.02, n=N)
            g = [synth.fill_device(x, 1, S.TAG_GRAD, j, 0, 1e-3) for j, x in enumerate(sh.extra)]
            stream = torch.cuda.current_stream().cuda_stream
            row = dict(contributors=R)
            for name, limit in (("one_kernel", 64), ("reduce_then_adamw", 0)):
                assert B.recover_set_tuning(B.TUNE_ONE_PASS_MAX, limit) == 0
                marks = []
                for it in range(reps + 2):
                    for r in range(R):
                        assert B.recover_accumulate(sh.ctx, r, r, g[r % 2].data_ptr(), B.F32, 0, T, stream) == 0
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    assert B.recover_reduce_adamw_step(sh.ctx, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"],
                                                       HP["weight_decay"], 0, stream) == 0
                    e1.record()
                    if it >= 2:
                        marks.append((e0, e1))
                torch.cuda.synchronize()
                ms = sorted(x.elapsed_time(y) for x, y in marks)[len(marks) // 2]
                bpe = 4 * R + (24 if limit else 32)
                row[name] = dict(ms=ms, bytes_per_elem=bpe, GBps=bpe * N / ms / 1e6)
            rows.append(row)
            sh.close()
            del sh, g
            torch.cuda.empty_cache()
    finally:
        assert B.recover_set_tuning(B.TUNE_ONE_PASS_MAX, default) == 0
    return {"one_pass_study": "configs[3] shard, 100,663,296 fp32 elements, median of %d calls" % reps,
            "library_limit": default, "rows": rows}


class Leg:
    """One workload resident in HBM: context, gradient pool, and the timed iteration."""

    def __init__(self, k):
        import torch
        from paper_2605_11215_amd import binding as B
        from paper_2605_11215_amd import synth
        from paper_2605_11215_amd.synth import reference_np as S
        from paper_2605_11215_amd.workloads import CONFIGS
        self.torch, self.B, self.synth, self.S = torch, B, synth, S
        self.k, self.c = k, CONFIGS[k]
        c = self.c
        self.s_g = 2 if c["bf16"] else 4
        self.W, self.G, self.off = c["W"], c["G"], c["off"]
        self.N, self.M, self.T = self.off[-1], c["W"] * c["G"], len(self.off) - 1
        gdt, self.gcode = (torch.bfloat16, B.BF16) if c["bf16"] else (torch.float32, B.F32)
        self.sh = B.Shard(self.W, self.G, self.off, device="cuda:0", snapshots=True, slab=SLAB["on"],
                          slab_pad=SLAB["pad"], extra=[(gdt, self.N)] * POOL, contiguous=SLAB["contiguous"])
        synth.fill_device(self.sh.param, c["seed"], S.TAG_PARAM, 0, 0, 0.02, n=self.N)
        self.pool = [synth.fill_device(g, c["seed"], S.TAG_GRAD, j, 0, c["scale"], c["kind"])
                     for j, g in enumerate(self.sh.extra)]
        self.gptr = [g.data_ptr() for g in self.pool]
        torch.cuda.synchronize()
        self.stream = torch.cuda.current_stream().cuda_stream
        self.ctx = self.sh.ctx
        self.bpe = bytes_per_elem(self.W, self.M, self.s_g, self.W)

    def close(self):
        self.sh.close()
        self.sh = self.pool = None
        self.torch.cuda.synchronize()
        self.torch.cuda.empty_cache()

    def ev(self):
        return self.torch.cuda.Event(enable_timing=True)

    def g_of(self, r, k):
        """The pool buffer that holds microbatch k of replica r: with the pool size dividing the replica count, buffer c
        serves replicas c W/POOL .. (c+1) W/POOL - 1 (Shard puts it next to their accumulators)."""
        if self.W % POOL == 0:
            return self.gptr[r // (self.W // POOL)]
        return self.gptr[(k * self.W + r) % POOL]

    def one_pass_tail_bytes(self):
        """Bytes per element of recover_reduce_adamw_step: one kernel (4 R_c + 24) up to the library's contributor limit,
        the reduction followed by the update (4 R_c + 32) beyond it."""
        code, limit = self.B.recover_get_tuning(self.B.TUNE_ONE_PASS_MAX)
        assert code == 0
        return 4 * self.W + (24 if self.W <= limit else 32)

    def iteration(self, marks=None, snapshot=False, fused=False, snapshot_every=False):
        """One failure-free iteration.  marks: list receiving the event list of the phases.  fused: the one-pass
        reduce+AdamW call; snapshot_every: the one-pass accumulate+snapshot call for every microbatch."""
        B, ctx, W, G, T, stream, gptr, gcode = self.B, self.ctx, self.W, self.G, self.T, self.stream, self.gptr, self.gcode
        acc_call = B.recover_accumulate_snapshot if snapshot_every else B.recover_accumulate
        e = [self.ev() for _ in range(5)] if marks is not None else None
        if e:
            e[0].record()
        for r in range(W):                                    # k = 0: overwrite variant
            rc = acc_call(ctx, r, r, self.g_of(r, 0), gcode, 0, T, stream)
            assert rc == 0, rc
        if e:
            e[1].record()
        for k in range(1, G):                                 # read-modify-write variant
            for r in range(W):
                rc = acc_call(ctx, r, r + W * k, self.g_of(r, k), gcode, 0, T, stream)
                assert rc == 0, rc
        if e:
            e[2].record()
        if snapshot:
            assert B.recover_snapshot(ctx, -1, 0, T, stream) == 0
        if fused:
            assert B.recover_reduce_adamw_step(ctx, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"],
                                               0, stream) == 0
        else:
            assert B.recover_reduce(ctx, 0, T, 0, stream) == 0
            if e:
                e[3].record()
            assert B.recover_adamw_step(ctx, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"],
                                        stream) == 0
        if e:
            e[4].record()
            marks.append(e)
        rc, _ = B.recover_policy_adjust(ctx, [], W)
        assert rc == 0

    def settle(self, limit_s):
        """Untimed: repeat iterations until three successive windows agree to 0.7 % (or the time limit).
        Memory that a previous process (or the previous leg) freed is wiped by the driver in the background
        and takes HBM bandwidth while it lasts, so a run started right after would otherwise time that."""
        torch = self.torch
        t_start, windows = time.perf_counter(), []
        n_win = max(2, int(0.2 / max(1e-4, self.bpe["total"] * self.N / 6e12)))         # about 0.2 s per window
        while time.perf_counter() - t_start < limit_s:
            torch.cuda.synchronize()
            t_w = time.perf_counter()
            for _ in range(n_win):
                self.iteration()
            torch.cuda.synchronize()
            windows.append((time.perf_counter() - t_w) / n_win)
            last = windows[-3:]
            if len(last) == 3 and max(last) <= 1.007 * min(last):
                break
        return time.perf_counter() - t_start, len(windows)

    def timed(self, n, **kw):
        torch = self.torch
        for _ in range(2):
            self.iteration(**kw)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            self.iteration(**kw)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / n

    def measure(self, steps, warmup, settle_seconds):
        """Settle, warm up, time exactly `steps` iterations bracketed by synchronisation; per-phase events inside
        the timed region give every kernel's rate and the per-iteration distribution."""
        torch = self.torch
        W, G, N, M, s_g, bpe = self.W, self.G, self.N, self.M, self.s_g, self.bpe
        settle_s, settle_windows = self.settle(settle_seconds) if settle_seconds > 0 else (0.0, 0)
        for _ in range(warmup):
            self.iteration()
        torch.cuda.synchronize()
        marks = []
        t0 = time.perf_counter()
        for _ in range(steps):
            self.iteration(marks)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        per_iter = [m[0].elapsed_time(m[4]) for m in marks]                                  # ms, events
        phase = [sum(m[i].elapsed_time(m[i + 1]) for m in marks) / len(marks) for i in range(4)]     # ms per iteration
        n_rmw = (G - 1) * W
        rmw_ms = phase[1] / n_rmw
        k_gbs = dict(accumulate_first=W * (s_g + 4) * N / phase[0] / 1e6, accumulate_rmw=(s_g + 8) * N / rmw_ms / 1e6,
                     reduce=bpe["reduce"] * N / phase[2] / 1e6, adamw=28 * N / phase[3] / 1e6)
        gbs = bpe["total"] * N / (dt / steps) / 1e9
        gname = "bf16" if self.c["bf16"] else "float"
        return dict(
            value=gbs, ms_per_step=dt * 1e3 / steps, steps=steps, warmup=warmup,
            pct_of_hbm_peak=100.0 * gbs / HBM_PEAK_GBS, microbatches_per_s=M / (dt / steps),
            iteration_ms_events=quantiles(per_iter),
            settle={"seconds": settle_s, "windows": settle_windows, "untimed": True},
            kernel_GBps=k_gbs,
            phase_ms=dict(accumulate_first=phase[0], accumulate_rmw=phase[1], reduce=phase[2], adamw=phase[3]),
            roofline={"bound": "hbm", "kernel": "k_accumulate<%s, RMW>" % gname, "achieved": k_gbs["accumulate_rmw"],
                      "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": k_gbs["accumulate_rmw"] / HBM_PEAK_GBS,
                      "traffic": read_traffic(self.k), "bytes_per_launch": (s_g + 8) * N, "avg_launch_ms": rmw_ms,
                      "launches_timed": n_rmw * len(marks)},
            config={"workload": WORKLOAD_TEXT[self.k], "grad_dtype": "bf16" if self.c["bf16"] else "f32",
                    "replicas": W, "microbatches": M, "n_elems": N, "n_tensors": self.T,
                    "bytes_per_elem": bpe["total"], "grad_pool_buffers": POOL})

    # ------------------------------------------------------------------------------------------ extras
    def extras(self, base_ms, steps):
        torch, B, ctx, W, G, T, N, M, s_g, bpe = self.torch, self.B, self.ctx, self.W, self.G, self.T, self.N, self.M, self.s_g, self.bpe
        stream, gptr, gcode, pool, c = self.stream, self.gptr, self.gcode, self.pool, self.c
        out = {}
        ns = max(3, steps // 5)
        # the same iteration with a snapshot of every replica before the reduction (Alg. 1, snapshot step)
        dts = self.timed(ns, snapshot=True)
        out["with_snapshot"] = dict(ms_per_step=dts * 1e3, bytes_per_elem=bpe["total"] + 8 * W,
                                    GBps=(bpe["total"] + 8 * W) * N / dts / 1e9)
        # one-pass variants: reduce+AdamW without writing the gradient (4 R_c + 24 B/element), and
        # accumulate+snapshot at every microbatch (s_g + 12 resp. s_g + 8 instead of s_g + 8 + 8 resp. s_g + 4 + 8)
        dtf = self.timed(ns, fused=True)
        b_fused = bpe["accumulate"] + self.one_pass_tail_bytes()
        out["fused_reduce_adamw"] = dict(ms_per_step=dtf * 1e3, bytes_per_elem=b_fused, GBps=b_fused * N / dtf / 1e9,
                                         microbatches_per_s=M / dtf, kernels=1 if self.one_pass_tail_bytes() == 4 * W + 24 else 2)
        marks = []
        for _ in range(ns):
            e0, e1 = self.ev(), self.ev()
            for r in range(W):
                for k in range(G):
                    assert B.recover_accumulate(ctx, r, r + W * k, self.g_of(r, k), gcode, 0, T, stream) == 0
            e0.record()
            assert B.recover_reduce_adamw_step(ctx, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"],
                                               0, stream) == 0
            e1.record()
            marks.append((e0, e1))
            assert B.recover_policy_adjust(ctx, [], W)[0] == 0
        torch.cuda.synchronize()
        fk = sorted(a.elapsed_time(b) for a, b in marks)[len(marks) // 2]
        out["fused_reduce_adamw"]["kernel_ms"] = fk
        out["fused_reduce_adamw"]["kernel_GBps"] = self.one_pass_tail_bytes() * N / fk / 1e6
        dte = self.timed(ns, fused=True, snapshot_every=True)
        b_every = W * (s_g + 8) + (M - W) * (s_g + 12) + self.one_pass_tail_bytes()
        out["fused_snapshot_every_microbatch"] = dict(ms_per_step=dte * 1e3, bytes_per_elem=b_every,
                                                      GBps=b_every * N / dte / 1e9, microbatches_per_s=M / dte)

        # snapshot and restore alone (one launch each for all replicas), and the chip's ceilings with the
        # library's own kernels on the same buffers: copy = the snapshot; read-only = recover_compare, which
        # streams two buffers and writes nothing.
        for k in range(G):
            for r in range(W):
                assert B.recover_accumulate(ctx, r, r + W * k, self.g_of(r, k), gcode, 0, T, stream) == 0
        snap_t, rest_t, cmp_t = [], [], []
        res = torch.empty(5, dtype=torch.int64, device="cuda:0")
        for i in range(6):
            e = [self.ev() for _ in range(4)]
            e[0].record()
            assert B.recover_snapshot(ctx, -1, 0, T, stream) == 0
            e[1].record()
            assert B.recover_restore(ctx, -1, 0, stream) == 0
            e[2].record()
            assert B.recover_compare(self.sh.acc[i % W].data_ptr(), self.sh.snap[(i + 1) % W].data_ptr(), N, res.data_ptr(),
                                     stream) == 0
            e[3].record()
            torch.cuda.synchronize()
            if i:
                snap_t.append(e[0].elapsed_time(e[1]))
                rest_t.append(e[1].elapsed_time(e[2]))
                cmp_t.append(e[2].elapsed_time(e[3]))
        med = lambda v: sorted(v)[len(v) // 2]
        out["snapshot_all_replicas"] = dict(ms=med(snap_t), GBps=8 * W * N / med(snap_t) / 1e6, launches=1)
        out["restore_all_replicas"] = dict(ms=med(rest_t), GBps=8 * W * N / med(rest_t) / 1e6, launches=1)
        out["ceilings"] = dict(copy_GBps=8 * W * N / min(snap_t) / 1e6, compare_two_reads_GBps=8 * N / min(cmp_t) / 1e6,
                               what="best of 5 with the library's own kernels on this workload's buffers: copy = "
                                    "recover_snapshot of all replicas (k_copy_many, 1 read : 1 write); compare = "
                                    "recover_compare over two buffers (k_compare: two reads, no write; a verification "
                                    "kernel with mismatch, NaN and checksum folds per element, two launches per call)")

        # Non-blocking restoration (Alg. 5): rewind every replica from its snapshot while the main stream
        # generates the next microbatch's gradient (the stand-in for the extended pass's forward/backward),
        # then re-reduce.  Serial = all on one stream; overlapped = the rewind on a side stream, ordered by
        # the context's events.
        S, synth = self.S, self.synth

        def restore_then_reduce(side):
            e0, e1 = self.ev(), self.ev()
            e0.record()
            assert B.recover_restore(ctx, -1, 0, stream if side is None else side.cuda_stream) == 0
            synth.fill_device(pool[0], c["seed"], S.TAG_GRAD, 99, 0, c["scale"], c["kind"])
            assert B.recover_reduce(ctx, 0, T, 0, stream) == 0
            e1.record()
            return e0, e1

        side = torch.cuda.Stream()
        pairs = {"serial": [], "overlapped": []}
        for i in range(8):
            for name, sd in (("serial", None), ("overlapped", side)):
                pairs[name].append(restore_then_reduce(sd))
        torch.cuda.synchronize()
        ro = {k: sum(a_.elapsed_time(b_) for a_, b_ in v[2:]) / len(v[2:]) for k, v in pairs.items()}
        out["nonblocking_restore"] = dict(serial_ms=ro["serial"], overlapped_ms=ro["overlapped"],
                                          what="restore of %d replicas + generation of one gradient + reduce" % W)
        assert B.recover_adamw_step(ctx, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], stream) == 0
        assert B.recover_policy_adjust(ctx, [], W)[0] == 0

        # One failure iteration of this workload, timed as a whole (Alg. 1 with Alg. 4-6): replicas crash
        # after two microbatches, half of the tensors are snapshotted and all-reduced in place before the
        # failure shows, then rewind, extended pass, snapshot, reduce, AdamW, advancement.
        if W >= 4 and G >= 2:
            from paper_2605_11215_amd.loop import run_iteration, view_shard
            lost = {W // 2 - 1: min(2, G), W - 2: min(2, G)} if W >= 8 else {W // 2 - 1: min(2, G)}
            torch.cuda.synchronize()
            t4 = time.perf_counter()
            res_ = run_iteration(self.sh, view_shard, 0, lambda t, mb: pool[(mb % W) * POOL // W if W % POOL == 0 else mb % POOL], W, dying=lost,
                                 fidelity_k=T // 2 or 1, hp=HP)
            torch.cuda.synchronize()
            dtf2 = time.perf_counter() - t4
            n_acc = sum(len(v) for v in res_["ids"].values()) + sum(lost.values())
            out["failure_iteration"] = dict(ms=dtf2 * 1e3, lost_replicas=sorted(lost), accumulates=n_acc,
                                            committed_microbatches=sum(len(v) for v in res_["ids"].values()),
                                            extra_slots=res_["decisions"][0]["G_ext"],
                                            vs_failure_free=dtf2 * 1e3 / base_ms)
        return out

    def batched(self, steps):
        """Launch-bound shards: one accumulate_many launch per microbatch slot + the fused step (G + 1 launches),
        and the same iteration captured once into a HIP graph (step count on the device) and replayed."""
        torch, B, W, G, N, M, gptr, gcode, stream, c = self.torch, self.B, self.W, self.G, self.N, self.M, self.gptr, self.gcode, self.stream, self.c
        b_fused = self.bpe["accumulate"] + 4 * W + 24
        hp = (HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"])

        def one(ctx, s):
            for k in range(G):
                rc, _ = B.recover_accumulate_many(ctx, list(range(W)), [r + W * k for r in range(W)],
                                                  [self.g_of(r, k) for r in range(W)], gcode, s)
                assert rc == 0, rc
            assert B.recover_reduce_adamw_step(ctx, *hp, 0, s) == 0
            assert B.recover_policy_adjust(ctx, [], W)[0] == 0

        for _ in range(3):
            one(self.ctx, stream)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(steps):
            one(self.ctx, stream)
        torch.cuda.synchronize()
        dtb = (time.perf_counter() - t2) / steps
        out = dict(ms_per_step=dtb * 1e3, launches=G + 1, bytes_per_elem=b_fused, GBps=b_fused * N / dtb / 1e9,
                   microbatches_per_s=M / dtb)
        sg = B.Shard(W, G, self.off, device="cuda:0", snapshots=False, device_step=True)
        self.synth.fill_device(sg.param, c["seed"], self.S.TAG_PARAM, 0, 0, 0.02, n=N)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one(sg.ctx, torch.cuda.current_stream().cuda_stream)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        dtg = (time.perf_counter() - t3) / steps
        out["graph_replay"] = dict(ms_per_step=dtg * 1e3, GBps=b_fused * N / dtg / 1e9, microbatches_per_s=M / dtg)
        sg.close()
        return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-slice", type=int, default=1 << 24)
    ap.add_argument("--cpu-iters", type=int, default=40)
    ap.add_argument("--settle-seconds", type=float, default=15.0,
                    help="upper bound of the untimed settling phase before the warmup (see Leg.settle)")
    ap.add_argument("--workload", type=int, default=5, choices=[1, 2, 3, 4, 5],
                    help="the headline workload (default 5 = configs[4], the largest single-GPU configuration)")
    ap.add_argument("--per-config", default="2,3,4",
                    help="comma list of further workloads timed after the headline ('' = none)")
    ap.add_argument("--no-extras", action="store_true", help="only the timed region (for profiling runs)")
    ap.add_argument("--fused-steps", type=int, default=0,
                    help="with --no-extras: also run this many iterations through the one-pass reduce+AdamW call "
                         "(so that a counter run sees that kernel)")
    ap.add_argument("--separate-allocations", action="store_true",
                    help="one device allocation per buffer instead of one slab per context (placement A/B)")
    ap.add_argument("--slab-pad-kib", type=int, default=4096, help="padding between the buffers of a slab")
    ap.add_argument("--no-contiguous", action="store_true",
                    help="ordinary allocation for the slab instead of asking for physically contiguous memory first")
    ap.add_argument("--realloc", type=int, default=0,
                    help="placement study instead of the benchmark: allocate, time and free the workload's buffers "
                         "this many times in ONE process and print every allocation's kernel rates")
    ap.add_argument("--one-pass-study", action="store_true",
                    help="instead of the benchmark: recover_reduce_adamw_step as one kernel against the reduction "
                         "followed by the update, over the number of contributors, on the 64-replica workload's shard")
    ap.add_argument("--pair-study", action="store_true",
                    help="instead of the benchmark: rate of the read-modify-write accumulate for pairs (accumulator, "
                         "gradient) of 403 MB buffers taken from different places of one 53 GB physically contiguous slab")
    ap.add_argument("--pair-buffers", type=int, default=140,
                    help="with --pair-study: number of 403 MB buffers in the slab (290 = the size of the headline slab)")
    ap.add_argument("--ballast-gib", type=int, default=0,
                    help="with --pair-study or --realloc: an ordinary allocation of this size is made first and held, "
                         "which moves the slab")
    ap.add_argument("--tuning", default="", help="launch-shape sweep: comma list of key=value for recover_set_tuning")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the R replicas are R buffers in one GPU's HBM); "
              "--gpus %d is not supported" % a.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_11215_amd import binding as B
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; this library has no CPU path", file=sys.stderr)
        sys.exit(3)
    B.lib()
    SLAB["on"], SLAB["pad"], SLAB["contiguous"] = not a.separate_allocations, a.slab_pad_kib << 10, not a.no_contiguous
    for kv in filter(None, a.tuning.split(",")):
        k, v = kv.split("=")
        assert B.recover_set_tuning(int(k), int(v)) == 0, kv
    torch.cuda.set_device(0)

    if a.pair_study:
        print(json.dumps(pair_study(a.ballast_gib, a.pair_buffers)))
        return
    if a.one_pass_study:
        print(json.dumps(one_pass_study(max(4, a.steps // 2))))
        return
    if a.realloc > 0:
        # Same process, same code, same virtual layout (the slab lands at the same address): what changes from one
        # allocation to the next is the physical memory behind it.  A 1 GiB allocation is kept after every second
        # round so that the driver cannot hand the same frames back.
        rows, keep = [], []
        if a.ballast_gib:
            keep.append(torch.empty(a.ballast_gib << 30, dtype=torch.uint8, device="cuda:0"))
            keep[-1][:: 1 << 20].zero_()
        for i in range(a.realloc):
            lk = Leg(a.workload)
            r = lk.measure(a.steps, a.warmup, min(a.settle_seconds, 3.0))
            dtf = lk.timed(max(2, a.steps // 4), fused=True)
            rows.append(dict(allocation=i, slab_address=hex(lk.sh._slab.data_ptr()) if SLAB["on"] else None,
                             contiguous=getattr(lk.sh, "contiguous", False),
                             GBps=r["value"], kernel_GBps=r["kernel_GBps"], fused_iteration_ms=dtf * 1e3))
            lk.close()
            if i % 2 == 0:
                keep.append(torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0"))
        print(json.dumps({"placement_study": WORKLOAD_TEXT[a.workload], "slab": SLAB["on"], "ballast_gib": a.ballast_gib,
                          "allocations": rows}))
        return
    leg = Leg(a.workload)
    head = leg.measure(a.steps, a.warmup, a.settle_seconds)
    out = {
        "metric": "effective HBM GB/s (and % of 8 TB/s) for accumulate+reduce+AdamW per iteration",
        "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ARITHMETIC, "data": "synthetic", "config": head["config"],
        "pct_of_hbm_peak": head["pct_of_hbm_peak"],
        "paper_context": "context only, other hardware: the paper reports 2.23x effective throughput over "
                         "checkpoint-restart after successive failures (128 x A100-40GB, 7B LLaMA-style model) and "
                         "evaluates up to 512 GPUs; it gives no bandwidth or per-kernel figure for this path",
    }
    for k in ("settle", "microbatches_per_s", "iteration_ms_events", "kernel_GBps", "phase_ms"):
        out[k] = head[k]
    if a.no_extras and a.fused_steps > 0:
        dtf = leg.timed(a.fused_steps, fused=True)
        out["fused_reduce_adamw"] = dict(ms_per_step=dtf * 1e3)
    if not a.no_extras:
        # before the extras: their failure leg leaves a replica dead
        out["batched_launches"] = leg.batched(a.steps) if a.workload == 1 else None
        out.update(leg.extras(head["ms_per_step"], a.steps))
    out["roofline"] = head["roofline"]
    cpu_slices = None
    if not a.no_cpu_baseline:
        n = min(a.cpu_slice, leg.N)
        cpu_slices = (leg.c, [g[:n].float().cpu().numpy() for g in leg.pool])
    leg.close()

    per = {}
    for k in [int(x) for x in a.per_config.split(",") if x]:
        if k == a.workload:
            continue
        lk = Leg(k)
        est_ms = lk.bpe["total"] * lk.N / 6.5e9
        r = lk.measure(max(5, min(40, int(1500.0 / est_ms))), 2, a.settle_seconds)
        if not a.no_extras:
            dtf = lk.timed(max(3, r["steps"] // 4), fused=True)
            b_fused = lk.bpe["accumulate"] + lk.one_pass_tail_bytes()
            r["fused_reduce_adamw"] = dict(ms_per_step=dtf * 1e3, bytes_per_elem=b_fused, GBps=b_fused * lk.N / dtf / 1e9)
        per["configs[%d]" % (k - 1)] = r
        lk.close()
    out["per_config"] = per
    if cpu_slices is not None:
        out["cpu_baseline"] = cpu_baseline(cpu_slices[0], cpu_slices[1], a.cpu_iters)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
