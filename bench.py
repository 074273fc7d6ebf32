#!/usr/bin/env python3
"""Benchmark of the gradient path on one MI355X.

A step is one failure-free iteration of the GPT-2-small-sized shard (8 replicas, 32
microbatches, fp32 gradients, 148 tensors, 123,589,632 elements) through the C ABI:
32 x recover_accumulate, recover_reduce, recover_adamw_step, recover_policy_adjust.
Gradients are synthetic (seeded Philox streams), pre-generated into a pool of four HBM
buffers before the timed region: generating them stands in for the backward pass.

Prints ONE JSON line: effective HBM GB/s = algorithmic bytes per iteration / time, with a
`roofline` object for the dominant kernel (the read-modify-write accumulate, timed with
events on the launch stream inside the timed region) and a `cpu_baseline` object (the CPU
oracle, as it stands, on a bounded slice of the same workload).  Extra keys, each timed
separately after the headline region: every kernel's rate, the iteration with a snapshot of every
replica, the one-pass variants, the non-blocking rewind, and one whole failure iteration.
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


WORKLOAD_TEXT = {
    1: "configs[0] tiny: 1,048,576 fp32 elements, R=4, M=8 (cache- and launch-bound, not an HBM measurement)",
    2: "configs[1] GPT-2-small-sized shard: 123,589,632 fp32 elements in 148 tensors, R=8 replicas, "
       "M=32 microbatches/iteration, failure-free iteration",
    3: "configs[2] Llama-3-8B 1/8 HSDP shard: 1,003,749,376 elements in 30 tensors, bf16 gradients, R=8, M=64",
    4: "configs[3] heavy attrition shape: 100,663,296 fp32 elements in 12 tensors, R=64, M=128",
    5: "configs[4] Llama-70B-like 1/16 shard: 1,978,662,912 elements in 259 tensors, bf16 gradients, R=4, M=16",
}


def workload(k=2):
    from paper_2605_11215_amd.workloads import CONFIGS
    return CONFIGS[k]


def bytes_per_elem(W, M, s_g, R_c):
    """Algorithmic bytes per element of one failure-free iteration: first microbatch of a
    replica writes acc and reads g; later ones also read acc; reduce reads R_c buffers and
    writes one; AdamW reads g,p,m,v and writes p,m,v."""
    acc = W * (s_g + 4) + (M - W) * (s_g + 8)
    return dict(accumulate=acc, reduce=4 * R_c + 4, adamw=28, total=acc + 4 * R_c + 4 + 28)


def read_traffic():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary."""
    path = os.path.join(ROOT, "profiles", "accumulate_f32_gpt2_shard_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("TRAFFIC_BYTES_PER_LAUNCH="):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def cpu_baseline(c, pool_slices, iters):
    """The oracle's fp32 protocol simulator on a contiguous slice: `iters` failure-free
    iterations (32 accumulates, reduce, AdamW).  Only this leg touches oracle/."""
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-slice", type=int, default=1 << 24)
    ap.add_argument("--cpu-iters", type=int, default=16)
    ap.add_argument("--settle-seconds", type=float, default=15.0,
                    help="upper bound of the untimed settling phase before the warmup (see settle())")
    ap.add_argument("--workload", type=int, default=2, choices=[1, 2, 3, 4, 5],
                    help="which of the five configs to time (default 2 = the headline workload, configs[1])")
    ap.add_argument("--tuning", default="", help="launch-shape sweep: comma list of key=value for recover_set_tuning")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the R replicas are R buffers in one GPU's HBM); "
              "--gpus %d is not supported" % a.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_11215_amd import binding as B
    from paper_2605_11215_amd import synth
    from paper_2605_11215_amd.synth import reference_np as S
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; this library has no CPU path", file=sys.stderr)
        sys.exit(3)
    B.lib()
    for kv in filter(None, a.tuning.split(",")):
        k, v = kv.split("=")
        assert B.recover_set_tuning(int(k), int(v)) == 0, kv

    c = workload(a.workload)
    s_g = 2 if c["bf16"] else 4
    W, G, off = c["W"], c["G"], c["off"]
    N, M = off[-1], c["W"] * c["G"]
    T = len(off) - 1
    torch.cuda.set_device(0)
    sh = B.Shard(W, G, off, device="cuda:0", snapshots=True)
    synth.fill_device(sh.param, c["seed"], S.TAG_PARAM, 0, 0, 0.02, n=N)
    gdt, gcode = (torch.bfloat16, B.BF16) if c["bf16"] else (torch.float32, B.F32)
    pool = [synth.fill_device(torch.empty(N, dtype=gdt, device="cuda:0"), c["seed"], S.TAG_GRAD, j, 0,
                              c["scale"], c["kind"]) for j in range(POOL)]
    gptr = [g.data_ptr() for g in pool]
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream().cuda_stream
    ctx = sh.ctx
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def iteration(marks=None, snapshot=False, fused=False, snapshot_every=False):
        """One failure-free iteration.  marks: list receiving event pairs per phase.  fused: the one-pass
        reduce+AdamW call; snapshot_every: the one-pass accumulate+snapshot call for every microbatch."""
        acc_call = B.recover_accumulate_snapshot if snapshot_every else B.recover_accumulate
        e = [ev() for _ in range(5)] if marks is not None else None
        if e:
            e[0].record()
        for r in range(W):                                    # k = 0: overwrite variant
            rc = acc_call(ctx, r, r, gptr[r % POOL], gcode, 0, T, stream)
            assert rc == 0, rc
        if e:
            e[1].record()
        for k in range(1, G):                                 # read-modify-write variant
            for r in range(W):
                rc = acc_call(ctx, r, r + W * k, gptr[(k * W + r) % POOL], gcode, 0, T, stream)
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

    def settle(limit_s):
        """Untimed: repeat iterations until three successive windows agree to 0.7 % (or the time limit).
        Memory that a previous process freed is wiped by the driver in the background and takes HBM
        bandwidth while it lasts (measured: 2 % for ~8 s after a process that held 200 GB), so a run
        started right after another GPU job would otherwise time that, not this path."""
        t_start, windows = time.perf_counter(), []
        n_win = max(5, int(0.2 / max(1e-4, 416 * N / 6e12)))         # about 0.2 s per window
        while time.perf_counter() - t_start < limit_s:
            torch.cuda.synchronize()
            t_w = time.perf_counter()
            for _ in range(n_win):
                iteration()
            torch.cuda.synchronize()
            windows.append((time.perf_counter() - t_w) / n_win)
            last = windows[-3:]
            if len(last) == 3 and max(last) <= 1.007 * min(last):
                break
        return time.perf_counter() - t_start, len(windows)

    settle_s, settle_windows = settle(a.settle_seconds) if a.settle_seconds > 0 else (0.0, 0)
    for _ in range(a.warmup):
        iteration()
    torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    for _ in range(a.steps):
        iteration(marks)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt * 1e3 / a.steps

    bpe = bytes_per_elem(W, M, s_g, W)
    gbs = bpe["total"] * N / (dt / a.steps) / 1e9
    phase = [sum(m[i].elapsed_time(m[i + 1]) for m in marks) / len(marks) for i in range(4)]     # ms per iteration
    n_rmw = (G - 1) * W
    rmw_ms = phase[1] / n_rmw
    k_gbs = dict(accumulate_first=W * (s_g + 4) * N / phase[0] / 1e6, accumulate_rmw=(s_g + 8) * N / rmw_ms / 1e6,
                 reduce=bpe["reduce"] * N / phase[2] / 1e6, adamw=28 * N / phase[3] / 1e6)

    # the same iteration with a snapshot of every replica before the reduction (Alg. 1, snapshot step)
    for _ in range(2):
        iteration(snapshot=True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ns = max(5, a.steps // 5)
    for _ in range(ns):
        iteration(snapshot=True)
    torch.cuda.synchronize()
    dts = (time.perf_counter() - t1) / ns
    with_snapshot = dict(ms_per_step=dts * 1e3, bytes_per_elem=bpe["total"] + 8 * W,
                         GBps=(bpe["total"] + 8 * W) * N / dts / 1e9)

    def timed(n, **kw):
        for _ in range(2):
            iteration(**kw)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            iteration(**kw)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / n

    # one-pass variants: reduce+AdamW without writing the gradient (4 R_c + 24 B/element), and
    # accumulate+snapshot at every microbatch (s_g + 12 resp. s_g + 8 instead of s_g + 8 + 8 resp. s_g + 4 + 8)
    dtf = timed(ns, fused=True)
    b_fused = bpe["accumulate"] + 4 * W + 24
    fused = dict(ms_per_step=dtf * 1e3, bytes_per_elem=b_fused, GBps=b_fused * N / dtf / 1e9,
                 microbatches_per_s=M / dtf)
    dte = timed(ns, fused=True, snapshot_every=True)
    b_every = W * (s_g + 8) + (M - W) * (s_g + 12) + 4 * W + 24
    every = dict(ms_per_step=dte * 1e3, bytes_per_elem=b_every, GBps=b_every * N / dte / 1e9,
                 microbatches_per_s=M / dte)

    # launch-bound shards: one accumulate_many launch per microbatch slot + the fused step (G + 1 launches)
    def iteration_batched():
        for k in range(G):
            rc, _ = B.recover_accumulate_many(ctx, list(range(W)), [r + W * k for r in range(W)],
                                              [gptr[(k * W + r) % POOL] for r in range(W)], gcode, stream)
            assert rc == 0, rc
        assert B.recover_reduce_adamw_step(ctx, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"],
                                           0, stream) == 0
        rc, _ = B.recover_policy_adjust(ctx, [], W)
        assert rc == 0

    batched = None
    if a.workload == 1:
        for _ in range(3):
            iteration_batched()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(a.steps):
            iteration_batched()
        torch.cuda.synchronize()
        dtb = (time.perf_counter() - t2) / a.steps
        batched = dict(ms_per_step=dtb * 1e3, launches=G + 1, bytes_per_elem=b_fused, GBps=b_fused * N / dtb / 1e9,
                       microbatches_per_s=M / dtb)
        # the same iteration captured once into a HIP graph (step count on the device) and replayed
        sg = B.Shard(W, G, off, device="cuda:0", snapshots=False, device_step=True)
        synth.fill_device(sg.param, c["seed"], S.TAG_PARAM, 0, 0, 0.02, n=N)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            cs = torch.cuda.current_stream().cuda_stream
            for k in range(G):
                rc, _ = B.recover_accumulate_many(sg.ctx, list(range(W)), [r + W * k for r in range(W)],
                                                  [gptr[(k * W + r) % POOL] for r in range(W)], gcode, cs)
                assert rc == 0, rc
            assert B.recover_reduce_adamw_step(sg.ctx, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"],
                                               HP["weight_decay"], 0, cs) == 0
            assert B.recover_policy_adjust(sg.ctx, [], W)[0] == 0
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t3 = time.perf_counter()
        for _ in range(a.steps):
            graph.replay()
        torch.cuda.synchronize()
        dtg = (time.perf_counter() - t3) / a.steps
        batched["graph_replay"] = dict(ms_per_step=dtg * 1e3, GBps=b_fused * N / dtg / 1e9, microbatches_per_s=M / dtg)

    # Non-blocking restoration (Alg. 5): rewind every replica from its snapshot while the main stream
    # generates the next microbatch's gradient (the stand-in for the extended pass's forward/backward),
    # then re-reduce.  Serial = all on one stream; overlapped = the rewind on a side stream, ordered by
    # the context's events.
    def restore_then_reduce(side):
        e0, e1 = ev(), ev()
        e0.record()
        if side is None:
            assert B.recover_restore(ctx, -1, 0, stream) == 0
        else:
            assert B.recover_restore(ctx, -1, 0, side.cuda_stream) == 0
        synth.fill_device(pool[0], c["seed"], S.TAG_GRAD, 99, 0, c["scale"], c["kind"])
        assert B.recover_reduce(ctx, 0, T, 0, stream) == 0
        e1.record()
        return e0, e1

    for k in range(G):
        for r in range(W):
            assert B.recover_accumulate(ctx, r, r + W * k, gptr[(k * W + r) % POOL], gcode, 0, T, stream) == 0
    assert B.recover_snapshot(ctx, -1, 0, T, stream) == 0
    side = torch.cuda.Stream()
    pairs = {"serial": [], "overlapped": []}
    for i in range(12):
        for name, sd in (("serial", None), ("overlapped", side)):
            pairs[name].append(restore_then_reduce(sd))
    torch.cuda.synchronize()
    restore_overlap = {k: sum(a_.elapsed_time(b_) for a_, b_ in v[2:]) / len(v[2:]) for k, v in pairs.items()}
    restore_overlap = dict(serial_ms=restore_overlap["serial"], overlapped_ms=restore_overlap["overlapped"],
                           what="restore of %d replicas + generation of one gradient + reduce" % W)
    assert B.recover_adamw_step(ctx, HP["lr"], HP["beta1"], HP["beta2"], HP["eps"], HP["weight_decay"], stream) == 0

    # One failure iteration of this workload's schedule, timed as a whole (Alg. 1 with Alg. 4-6): two
    # replicas crash after two microbatches, half of the tensors are snapshotted and all-reduced in
    # place before the failure shows, then rewind, extended pass, snapshot, reduce, AdamW, advancement.
    failure_iteration = None
    if W >= 4 and G >= 2:
        from paper_2605_11215_amd.loop import run_iteration, view_shard
        lost = {W // 2 - 1: min(2, G), W - 2: min(2, G)}
        torch.cuda.synchronize()
        t4 = time.perf_counter()
        res = run_iteration(sh, view_shard, 0, lambda t, mb: pool[mb % POOL], W, dying=lost, fidelity_k=T // 2 or 1,
                            hp=HP)
        torch.cuda.synchronize()
        dtf2 = time.perf_counter() - t4
        n_acc = sum(len(v) for v in res["ids"].values()) + sum(lost.values())
        failure_iteration = dict(ms=dtf2 * 1e3, lost_replicas=sorted(lost), accumulates=n_acc,
                                 committed_microbatches=sum(len(v) for v in res["ids"].values()),
                                 extra_slots=res["decisions"][0]["G_ext"], vs_failure_free=dtf2 / (dt / a.steps))

    out = {
        "metric": "effective HBM GB/s (and % of 8 TB/s) for accumulate+reduce+AdamW per iteration",
        "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[a.workload], "grad_dtype": "bf16" if c["bf16"] else "f32",
                   "replicas": W, "microbatches": M, "n_elems": N, "n_tensors": T,
                   "bytes_per_elem": bpe["total"], "grad_pool_buffers": POOL},
        "pct_of_hbm_peak": 100.0 * gbs / HBM_PEAK_GBS,
        "paper_context": "context only, other hardware: the paper reports 2.23x effective throughput over "
                         "checkpoint-restart after successive failures (128 x A100-40GB, 7B LLaMA-style model) and "
                         "evaluates up to 512 GPUs; it gives no bandwidth or per-kernel figure for this path",
        "settle": {"seconds": settle_s, "windows": settle_windows, "untimed": True},
        "microbatches_per_s": M / (dt / a.steps),
        "kernel_GBps": k_gbs,
        "phase_ms": dict(accumulate_first=phase[0], accumulate_rmw=phase[1], reduce=phase[2], adamw=phase[3]),
        "with_snapshot": with_snapshot,
        "fused_reduce_adamw": fused,
        "fused_snapshot_every_microbatch": every,
        "batched_launches": batched,
        "nonblocking_restore": restore_overlap,
        "failure_iteration": failure_iteration,
        "roofline": {"bound": "hbm", "kernel": "k_accumulate<%s, RMW>" % ("bf16" if c["bf16"] else "float"), "achieved": k_gbs["accumulate_rmw"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": k_gbs["accumulate_rmw"] / HBM_PEAK_GBS,
                     "traffic": read_traffic() if a.workload == 2 else None, "bytes_per_launch": (s_g + 8) * N, "avg_launch_ms": rmw_ms,
                     "launches_timed": n_rmw * len(marks)},
    }
    if not a.no_cpu_baseline:
        n = min(a.cpu_slice, N)
        slices = [g[:n].float().cpu().numpy() for g in pool]
        out["cpu_baseline"] = cpu_baseline(c, slices, a.cpu_iters)
    sh.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
