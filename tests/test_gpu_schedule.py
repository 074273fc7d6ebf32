"""Generated failure schedules through the HIP library (the stand-in for the paper's failure simulator,
implementation appendix, "Failure simulator"), side by side with the fp32 oracle; the attrition report
(effective throughput per alive replica, Sec. 5); and a context without snapshot buffers that gets past a
failure."""
import json

import numpy as np
import pytest

from oracle import adamw as oracle_adamw
from oracle.proto import Proto
from paper_2605_11215_amd import attrition, binding as B, schedule
from paper_2605_11215_amd.synth import reference_np as S
from tests.driver import run_iteration, view_oracle, HP
from tests.gpu_harness import HipEngine, view_hip, max_rel, bits_equal, assert_adamw_elementwise

pytestmark = pytest.mark.gpu


def hp32():
    return {k: float(np.float32(v)) for k, v in HP.items()}


def test_generated_schedule_through_the_library_matches_the_oracle():
    """12 replicas, 3 microbatches each, a ragged 6-tensor shard, 12 iterations.  The schedule has both kinds of
    location (crash at a microbatch boundary, crash during synchronisation after p % of the buckets were
    all-reduced), goes through YAML and back, and is consumed by `for_step` against each engine's own view of
    who is alive.  Per iteration: the injected failures, every decision field, the committed ids, Eq. 1, the
    gradient bit for bit, the AdamW state element by element; and the fields the attrition report prints."""
    import torch
    W, G = 12, 3
    off = [0, 5, 1029, 1030, 6000, 6003, 25000]
    N, T = off[-1], len(off) - 1
    entries = schedule.generate(W, 4, 11, 14, (0, 11), {"mb": 1, "sync": 1}, max_microbatch=G)
    entries = schedule.from_yaml(schedule.to_yaml(entries))
    kinds = {e["location"].split(":")[0] for e in entries}
    assert kinds == {"mb", "sync"}
    p0 = S.fill(N, 5, S.TAG_PARAM, 0, 0, 0.02)
    o = Proto(W, G, off, dtype=np.float32)
    o.set_state(p0)
    s = B.Shard(W, G, off, param_bf16=True)
    s.param[:N].copy_(torch.from_numpy(p0))
    eng = HipEngine(s)
    cache = {}

    def g(t, mb):
        if (t, mb) not in cache:
            cache[(t, mb)] = S.fill(N, 5, S.TAG_GRAD, mb, t, 1e-3)
        return cache[(t, mb)]

    lost, boundaries, in_sync = 0, 0, 0
    for t in range(12):
        va, vb = view_oracle(o), view_hip(s)
        assert va == vb
        da, fa = schedule.for_step(entries, t, va["alive"], va["target"], T)
        db, fb = schedule.for_step(entries, t, vb["alive"], vb["target"], T)
        assert (da, fa) == (db, fb)
        before = [x[:N].cpu().numpy().copy() for x in (s.param, s.exp_avg, s.exp_avg_sq)]
        a = run_iteration(o, view_oracle, t, g, W, dying=da, fidelity_k=fa, hp=hp32())
        b = run_iteration(eng, view_hip, t, g, W, dying=db, fidelity_k=fb, hp=hp32())
        assert a["ids"] == b["ids"]
        committed = sum(len(v) for v in b["ids"].values())
        assert committed == W * G                                             # Eq. 1
        assert len(a["decisions"]) == len(b["decisions"])
        for x, y in zip(a["decisions"], b["decisions"]):
            for k in x:
                assert x[k] == y[k], (t, k)
        g_gpu = s.grad_out[:N].cpu().numpy()
        assert bits_equal(g_gpu, o.grad_out), t
        ref = oracle_adamw.adamw_step(before[0], before[1], before[2], g_gpu, o.t, **hp32())
        got = [x[:N].cpu().numpy() for x in (s.param, s.exp_avg, s.exp_avg_sq)]
        assert_adamw_elementwise(before, g_gpu, o.t, hp32(), got, ref)
        for x, y in zip(got, (o.param, o.m, o.v)):
            assert max_rel(x, y) <= 1e-6
        # what the attrition report derives per iteration
        after = view_hip(s)
        assert len(after["alive"]) == len(vb["alive"]) - len(db)
        assert max(d["loop_bound"] for d in b["decisions"]) >= G
        lost += len(db)
        boundaries += int(any(d.get("at_boundary") for d in b["decisions"]))
        in_sync += int(fb > 0)
    assert lost >= 5 and boundaries >= 2 and in_sync >= 1, (lost, boundaries, in_sync)
    s.close()


def test_attrition_report_on_the_tiny_workload(capsys):
    """`python -m paper_2605_11215_amd.attrition` on configs[0]: every iteration commits exactly B microbatches
    and the report's fields are consistent with the schedule it prints."""
    assert attrition.main(["--workload", "1", "--iters", "6", "--failures", "3", "--seed", "7"]) == 0
    out = capsys.readouterr().out.strip().splitlines()
    doc = json.loads(out[-1])
    rows = doc["iterations"]
    assert len(rows) == 6 and all(r["committed"] == 8 for r in rows)
    assert all(r["alive_after"] == r["alive_before"] - len(r["failed"]) for r in rows)
    assert all(r["microbatches_per_s_per_alive_replica"] > 0 and r["ms"] > 0 for r in rows)
    assert rows[-1]["alive_after"] >= 1
    assert sum(len(r["failed"]) for r in rows) <= len(doc["schedule"])
    assert any(r["failed"] for r in rows)


def test_context_without_snapshot_buffers_gets_past_a_failure_on_the_gpu():
    """No snapshot buffers: a failure before the synchronisation leaves nothing to rewind (empty stale set), the
    rewind call lifts the quiesce, the extended pass, the reduction and the step match the oracle."""
    import torch
    off = [0, 3, 2051, 9000]
    N = off[-1]
    W, G = 4, 2
    p0 = S.fill(N, 9, S.TAG_PARAM, 0, 0, 0.02)
    o = Proto(W, G, off, dtype=np.float32)
    o.set_state(p0)
    s = B.Shard(W, G, off, snapshots=False)
    s.param[:N].copy_(torch.from_numpy(p0))
    eng = HipEngine(s)
    g = lambda mb: S.fill(N, 9, S.TAG_GRAD, mb, 0, 1e-3)
    for e in (o, eng):
        for r in range(W):
            assert e.accumulate(r, r, g(r))
        for r in (0, 1, 3):
            assert e.accumulate(r, r + W, g(r + W))
    assert B.recover_snapshot(s.ctx, -1, 0, 3) == B.ERR_NO_SNAPSHOT
    a, b = o.on_failure([2]), s.on_failure([2])
    assert a["at_boundary"] == b["at_boundary"] == 1 and a["target"] == b["target"]
    assert s.reduce() is False                                  # quiesced
    o.restore(None)
    s.restore(None)                                             # nothing to copy; lifts the quiesce
    before = [x[:N].cpu().numpy().copy() for x in (s.param, s.exp_avg, s.exp_avg_sq)]
    for e in (o, eng):
        for r in (0, 1):
            assert e.accumulate(r, r + 2 * W, g(r + 2 * W))
        e.reduce()
    g_gpu = s.grad_out[:N].cpu().numpy()
    assert bits_equal(g_gpu, o.grad_out)
    assert s.committed_ids_by_replica() == o.committed_ids_by_replica() == {0: [0, 4, 8], 1: [1, 5, 9], 3: [3, 7]}
    o.adamw_step(**hp32())
    s.adamw_step(**hp32())
    ref = oracle_adamw.adamw_step(before[0], before[1], before[2], g_gpu, 1, **hp32())
    assert_adamw_elementwise(before, g_gpu, 1, hp32(), [x[:N].cpu().numpy() for x in (s.param, s.exp_avg, s.exp_avg_sq)], ref)
    assert o.advance()["G_cur"] == s.advance()["G_cur"] == 3
    s.close()


def test_slab_placement_gives_the_same_bits_and_frees_its_memory():
    """All buffers of a context carved from one allocation (physically contiguous if the driver can give it, through
    recover_device_alloc): same results as separately allocated buffers, every buffer 2 MiB-aligned, and the memory
    is returned on close."""
    import torch
    off = [0, 7, 4099, 70000]
    N = off[-1]
    g = [torch.from_numpy(S.fill(N, 3, S.TAG_GRAD, j, 0, 1e-3)).cuda() for j in range(4)]
    p0 = torch.from_numpy(S.fill(N, 3, S.TAG_PARAM, 0, 0, 0.02)).cuda()
    free_before = torch.cuda.mem_get_info()[0]
    shards = [B.Shard(2, 2, off, param_bf16=True),
              B.Shard(2, 2, off, param_bf16=True, slab=True, extra=[(torch.float32, N)] * 2),
              B.Shard(2, 2, off, param_bf16=True, slab=True, contiguous=True, extra=[(torch.bfloat16, 5)])]
    assert shards[2].contiguous in (True, False)                    # the driver may refuse; then it is an ordinary slab
    for s in shards[1:]:
        bufs = s.acc + s.snap + [s.grad_out, s.param, s.exp_avg, s.exp_avg_sq, s.param_bf16] + s.extra
        assert all(b.data_ptr() % (2 << 20) == 0 for b in bufs)
        ends = sorted((b.data_ptr(), b.data_ptr() + b.numel() * b.element_size()) for b in bufs)
        assert all(a[1] + (4 << 20) <= b[0] for a, b in zip(ends, ends[1:]))            # padding between neighbours
        assert all(float(b.float().abs().max()) == 0 for b in bufs)                     # zero-filled
    for s in shards:
        s.param[:N].copy_(p0)
        for k in range(2):
            for r in range(2):
                assert s.accumulate(r, r + 2 * k, g[2 * k + r])
        s.snapshot()
        s.reduce()
        s.adamw_step(**hp32())
    ref = shards[0]
    for s in shards[1:]:
        for a, b in ((ref.grad_out, s.grad_out), (ref.param, s.param), (ref.exp_avg, s.exp_avg), (ref.exp_avg_sq, s.exp_avg_sq),
                     (ref.snap[1], s.snap[1])):
            assert torch.equal(a[:N].view(torch.int32), b[:N].view(torch.int32))
        assert torch.equal(ref.param_bf16[:N].view(torch.int16), s.param_bf16[:N].view(torch.int16))
    for s in shards:
        s.close()
    del shards, ref, s, bufs
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    assert torch.cuda.mem_get_info()[0] >= free_before - (64 << 20)
    assert B.lib().recover_device_free(None) == B.OK
