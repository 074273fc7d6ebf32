"""The C-ABI library without a GPU: it loads, exports what include/recover.h declares, and its
host logic (policy, bookkeeping, error returns) agrees with the oracle call by call on
host-only contexts (no kernel runs; nothing is computed).  CPU only."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

from oracle.proto import Proto, ProtocolError
from oracle import policy as OP
from paper_2605_11215_amd import binding as B
from tests.driver import run_iteration, view_oracle, HP

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "recover.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(recover_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    names = declared_functions()
    for must in ("recover_init", "recover_accumulate", "recover_snapshot", "recover_restore",
                 "recover_policy_adjust", "recover_reduce", "recover_adamw_step"):
        assert must in names
    L = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names


def test_synth_library_exports():
    from paper_2605_11215_amd import synth
    assert hasattr(ctypes.CDLL(synth.LIB_PATH), "synth_fill")


def test_device_calls_fail_loudly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    code, ctx = B.recover_init(2, 2, [0, 8], [16, 32], None, 16, 16, 16, 16)
    assert code == B.ERR_HIP and "no CPU path" in B.recover_last_error(None)


def test_argument_errors():
    assert B.recover_init(0, 2, [0, 8], None, None, 0, 0, 0, 0, flags=B.FLAG_HOST_ONLY)[0] == B.ERR_ARG
    assert B.recover_init(65, 2, [0, 8], None, None, 0, 0, 0, 0, flags=B.FLAG_HOST_ONLY)[0] == B.ERR_ARG
    assert B.recover_init(2, 2, [0, 8, 4], None, None, 0, 0, 0, 0, flags=B.FLAG_HOST_ONLY)[0] == B.ERR_ARG
    assert B.recover_init(2, 2, [0, (1 << 38) + 1], None, None, 0, 0, 0, 0, flags=B.FLAG_HOST_ONLY)[0] == B.ERR_ARG
    assert "RECOVER_MAX_ELEMS" in B.recover_last_error(None)
    code, big = B.recover_init(2, 2, [0, 5, 1 << 38], None, None, 0, 0, 0, 0, flags=B.FLAG_HOST_ONLY)
    assert code == B.OK and B.recover_destroy(big) == B.OK
    assert B.recover_init(2, 2, [0, 8], [16, 24 + 4], None, 16, 16, 16, 16)[0] == B.ERR_ALIGN
    s = B.Shard(2, 2, [0, 8, 16], host_only=True)
    assert B.recover_accumulate(s.ctx, 2, 0, 0, B.F32, 0, 2) == B.ERR_ARG
    assert B.recover_accumulate(s.ctx, 0, 0, 0, 7, 0, 2) == B.ERR_ARG
    assert B.recover_accumulate(s.ctx, 0, 0, 0, B.F32, 1, 3) == B.ERR_ARG
    assert B.recover_reduce(s.ctx, 0, 2, 8) == B.ERR_ARG
    assert B.recover_adamw_step(s.ctx, 1e-3, 1.5, 0.95, 1e-8, 0.1) == B.ERR_ARG
    assert B.recover_policy_adjust(s.ctx, [0, 1], 2)[0] == B.ERR_NO_SURVIVOR
    assert B.recover_policy_adjust(s.ctx, [5], 2)[0] == B.ERR_ARG
    key = B.TUNE_VECS + B.KERNEL_ADAMW
    before = B.recover_get_tuning(key)
    assert before[0] == B.OK
    assert B.recover_set_tuning(key, 3) == B.ERR_ARG and B.recover_get_tuning(key) == before
    assert B.recover_set_tuning(key, 4) == B.OK and B.recover_get_tuning(key) == (B.OK, 4)
    assert B.recover_set_tuning(key, before[1]) == B.OK
    assert B.recover_set_tuning(B.TUNE_WAVES + B.KERNEL_CLASSES, 8) == B.ERR_ARG        # no such kernel class
    assert B.recover_set_tuning(B.TUNE_WAVES + B.KERNEL_COPY, 1) == B.ERR_ARG
    assert B.recover_set_tuning(0, 1) == B.ERR_ARG
    assert B.recover_get_tuning(B.TUNE_ONE_PASS_MAX) == (B.OK, 32)
    assert B.recover_set_tuning(B.TUNE_ONE_PASS_MAX, 65) == B.ERR_ARG and B.recover_set_tuning(B.TUNE_ONE_PASS_MAX, -1) == B.ERR_ARG
    assert B.recover_set_tuning(B.TUNE_ONE_PASS_MAX, 0) == B.OK and B.recover_get_tuning(B.TUNE_ONE_PASS_MAX) == (B.OK, 0)
    assert B.recover_set_tuning(B.TUNE_ONE_PASS_MAX, 32) == B.OK
    assert B.recover_query(s.ctx, 2)[1]["target"] == [2, 2]        # unchanged by the failed calls


INT_KEYS = ("at_boundary", "restore_mode", "epoch", "W_cur", "C_cur", "G_ext", "n_bdry", "G_cur", "R_cur",
            "loop_bound", "n_maj", "n_min", "n_ms", "n_mi", "n_bm", "role", "target", "contributed",
            "is_boundary_minor")


def same_decision(a, b):
    for k in INT_KEYS:
        assert a[k] == b[k], (k, a[k], b[k])


def view_hip(s):
    q = s.query()
    return dict(alive=[r for r in range(s.W) if q["role"][r] != B.ROLE_DEAD], target=q["target"],
                contributed=q["contributed"], loop_bound=q["loop_bound"], role=q["role"], epoch=q["epoch"])


def test_policy_bit_exact_against_oracle_on_sweeps():
    """Every (W <= 6, G <= 3) and every sequence of three failure sets of size <= 2, plus the
    64-replica attrition: each decision record equals the oracle's field by field."""
    n = 0
    for W in range(1, 7):
        for G in range(1, 4):
            sets = [()] + [(a,) for a in range(W)] + list(itertools.combinations(range(W), 2))
            for seq in itertools.product(sets, repeat=3):
                o = OP.World(W, G)
                s = B.Shard(W, G, [0, 4], host_only=True)
                for picks in seq:
                    for r in o.alive():                       # everybody reaches the quota
                        while o.contributed[r] < o.target[r]:
                            o.contributed[r] += 1
                            assert s.accumulate(r, r + W * o.contributed[r], None)
                        assert not s.accumulate(r, 10 ** 6, None)
                    alive = o.alive()
                    failed = sorted({alive[k % len(alive)] for k in picks})
                    if len(failed) == len(alive):
                        assert B.recover_policy_adjust(s.ctx, failed, W)[0] == B.ERR_NO_SURVIVOR
                        break
                    if failed:
                        same_decision(s.on_failure(failed), o.on_failure(failed))
                        s.restore()
                        for r in o.alive():
                            while o.contributed[r] < o.target[r]:
                                o.contributed[r] += 1
                                assert s.accumulate(r, r + W * o.contributed[r], None)
                    assert s.reduce()
                    s.adamw_step(**HP)
                    o.commit()
                    same_decision(s.advance(), o.advance())
                    n += 1
                s.close()
    assert n > 3000


@pytest.mark.parametrize("static", [True, False])
def test_protocol_bookkeeping_matches_oracle_call_by_call(static):
    """Random schedules (failures at random offsets, partial in-place synchronisation, snapshots
    at every boundary) through the shared driver: same decisions, same committed ids."""
    rng = np.random.default_rng(5)
    off = [0, 3, 8, 8, 20]
    g = np.zeros(off[-1], np.float32)
    for trial in range(60):
        W, G = int(rng.integers(2, 9)), int(rng.integers(1, 5))
        o = Proto(W, G, off, dtype=np.float32, static=static)
        o.set_state(g)
        s = B.Shard(W, G, off, host_only=True, flags=0 if static else B.FLAG_ADAPTIVE)

        class HostOnly:                                    # adapter: the driver passes arrays
            def __getattr__(self, k):
                return getattr(s, k)

            def accumulate(self, r, mb, grad, tb=0, te=None, snapshot=False):
                return s.accumulate(r, mb, None, tb, te, snapshot=snapshot)

            def accumulate_many(self, replicas, ids, grads):
                return s.accumulate_many(replicas, ids, None)

        h = HostOnly()
        for t in range(5):
            alive = o.world.alive()
            if len(alive) == 1:
                break
            nf = int(rng.integers(0, min(3, len(alive))))
            dying = {int(r): int(rng.integers(0, max(1, o.world.target[r]) + 1))
                     for r in rng.choice(alive, nf, replace=False)}
            kw = dict(dying=dying, fidelity_k=int(rng.integers(0, 5)), snapshot_every=bool(rng.integers(0, 2)))
            a = run_iteration(o, view_oracle, t, lambda t, mb: g, W, **kw)
            b = run_iteration(h, view_hip, t, lambda t, mb: None, W, fuse=bool(trial % 2), batch=bool(trial % 3 == 0), **kw)
            assert a["ids"] == b["ids"]
            assert len(a["decisions"]) == len(b["decisions"])
            for x, y in zip(a["decisions"], b["decisions"]):
                same_decision(y, x)
        s.close()


def test_state_errors_match_the_oracle():
    off = [0, 4, 8]
    g = np.zeros(8, np.float32)
    o = Proto(4, 2, off, dtype=np.float32)
    o.set_state(g)
    s = B.Shard(4, 2, off, host_only=True)

    def both(name, *args, **kw):
        """Call on both; return (oracle raised?, library code)."""
        try:
            getattr(o, name)(*args, **kw)
            raised = False
        except ProtocolError:
            raised = True
        return raised

    for r in range(4):
        o.accumulate(r, r, g)
        assert s.accumulate(r, r, None)
    o.reduce()
    s.reduce()
    assert both("adamw_step", **HP) and B.recover_adamw_step(s.ctx, 1e-3, 0.9, 0.95, 1e-8, 0.1) == B.ERR_STATE
    # partial microbatch, then a different id
    o.accumulate(0, 4, g, 0, 1)
    assert s.accumulate(0, 4, None, 0, 1)
    assert both("accumulate", 0, 8, g, 1, 2) and B.recover_accumulate(s.ctx, 0, 8, 0, 0, 1, 2) == B.ERR_STATE
    assert both("accumulate", 0, 4, g, 0, 1) and B.recover_accumulate(s.ctx, 0, 4, 0, 0, 0, 1) == B.ERR_STATE
    o.accumulate(0, 4, g, 1, 2)
    assert s.accumulate(0, 4, None, 1, 2)
    assert both("accumulate", 1, 0, g) and B.recover_accumulate(s.ctx, 1, 0, 0, 0, 0, 2) == B.ERR_ARG
    # in-place sum blocks snapshot, accumulate and a second reduction until the rewind
    o.snapshot(None)
    s.snapshot()
    o.reduce(0, 1, inplace=True)
    s.reduce(0, 1, inplace=True)
    assert both("snapshot", 1, 0, 1) and B.recover_snapshot(s.ctx, 1, 0, 1) == B.ERR_STATE
    assert both("reduce", 0, 2) and B.recover_reduce(s.ctx, 0, 2, 0) == B.ERR_STATE
    assert both("accumulate", 1, 5, g) and B.recover_accumulate(s.ctx, 1, 5, 0, 0, 0, 2) == B.ERR_STATE
    o.on_failure([3])
    s.on_failure([3])
    assert o.reduce(1, 2) is False and B.recover_reduce(s.ctx, 1, 2, 0) == B.SKIPPED
    assert both("accumulate", 3, 7, g) and B.recover_accumulate(s.ctx, 3, 7, 0, 0, 0, 2) == B.ERR_STATE
    assert both("adamw_step", **HP) and B.recover_adamw_step(s.ctx, 1e-3, 0.9, 0.95, 1e-8, 0.1) == B.ERR_STATE
    o.restore(None)
    s.restore()
    assert view_hip(s)["contributed"] == list(o.world.contributed)
    assert view_hip(s)["target"] == list(o.world.target)
    # rewind that would split a replica across two microbatch counts
    o2 = Proto(2, 3, off, dtype=np.float32)
    s2 = B.Shard(2, 3, off, host_only=True)
    o2.accumulate(0, 0, g)
    s2.accumulate(0, 0, None)
    o2.snapshot(0, 0, 1)
    s2.snapshot(0, 0, 1)
    o2.accumulate(0, 2, g)
    s2.accumulate(0, 2, None)
    with pytest.raises(ProtocolError):
        o2.restore(0, stale_only=False)
    assert B.recover_restore(s2.ctx, 0, 0) == B.ERR_STATE
    # accumulate_many: a bad pair leaves everything untouched; a met quota is skipped per pair
    s3 = B.Shard(4, 1, off, host_only=True)
    assert s3.accumulate(2, 2, None)
    assert B.recover_accumulate_many(s3.ctx, [0, 0], [0, 4], [0, 0], B.F32)[0] == B.ERR_ARG      # repeated replica
    assert B.recover_accumulate_many(s3.ctx, [0, 9], [0, 4], [0, 0], B.F32)[0] == B.ERR_ARG
    assert s3.query()["contributed"] == [0, 0, 1, 0]
    assert s3.accumulate_many([0, 1, 2], [0, 1, 6], None) == [True, True, False]
    assert s3.query()["contributed"] == [1, 1, 1, 0]
    assert B.recover_accumulate_many(s3.ctx, [0, 1], [4, 5], [0, 0], B.F32)[0] == B.SKIPPED


def test_random_call_sequences_agree_with_the_oracle_host_only():
    """Differential test of the host logic: thousands of random calls (valid and invalid) leave the
    library's bookkeeping equal to the oracle's after every call."""
    from tests import differential

    class HostOnly:
        def __init__(self, s):
            self.s = s

        def __getattr__(self, k):
            return getattr(self.s, k)

        def accumulate(self, r, mb, g, tb=0, te=None, snapshot=False):
            return self.s.accumulate(r, mb, None, tb, te, snapshot=snapshot)

        def accumulate_many(self, replicas, ids, grads):
            return self.s.accumulate_many(replicas, ids, None)

    total = {"ok": 0, "err": 0, "steps": 0, "failures": 0}
    for seed in range(60):
        W, G = [(4, 2), (8, 1), (3, 3), (6, 2), (2, 4), (16, 1), (5, 2)][seed % 7]
        off = [0, 3, 8, 8, 20, 21, 40]
        s = B.Shard(W, G, off, host_only=True, flags=B.FLAG_ADAPTIVE if seed % 8 == 7 else 0)
        st = differential.run(seed, 400, W, G, off, HostOnly(s), adaptive=(seed % 8 == 7))
        for k in total:
            total[k] += st[k]
        s.close()
    assert total["ok"] > 12000 and total["err"] > 500 and total["steps"] > 300 and total["failures"] > 60, total


def test_stale_reduction_and_rewound_audit_in_the_library():
    """The library refuses to commit a reduction from before a repair even when the totals are B, and a
    rewind drops completed microbatches from its audit (same scenarios as the oracle's pins)."""
    s = B.Shard(6, 2, [0, 2, 4], host_only=True)
    for k in range(2):
        for r in range(6):
            if not (r == 5 and k == 1):
                assert s.accumulate(r, r + 6 * k, None)
    d = s.on_failure([5])
    s.restore()
    assert d["at_boundary"] and d["G_ext"] == 1 and d["n_bdry"] == 3
    for r in range(5):
        while s.accumulate(r, 100 + r + 6 * s.query()["contributed"][r], None):
            pass
    s.reduce()
    s.adamw_step(**HP)
    assert s.advance()["role"] == [0, 0, 0, 0, 2, 4]
    for k in range(3):
        for r in range(5):
            assert s.accumulate(r, r + 6 * k, None)
    s.reduce()
    d = s.on_failure([1])
    assert not d["at_boundary"] and d["role"][4] == B.ROLE_MAJOR and d["C_cur"] == 12
    s.restore()
    assert B.recover_adamw_step(s.ctx, 1e-3, 0.9, 0.95, 1e-8, 0.1) == B.ERR_STATE
    s.reduce()
    s.adamw_step(**HP)
    # rewind drops a completed microbatch
    s2 = B.Shard(2, 3, [0, 4, 8], host_only=True)
    s2.accumulate(0, 0, None)
    s2.snapshot(0)
    s2.accumulate(0, 2, None)
    assert B.recover_committed_ids(s2.ctx, 0)[1] == [0, 2]
    s2.restore(0, stale_only=False)
    assert B.recover_committed_ids(s2.ctx, 0)[1] == [0] and s2.query()["contributed"][0] == 1
    assert s2.accumulate(0, 2, None)


def test_snapshot_taken_between_commit_and_advancement_survives_the_advancement():
    """Advancement installs the next role layout; it does not reopen the iteration the commit opened
    (found by the random-call test: the oracle kept such a snapshot record, the library dropped it)."""
    off = [0, 4, 8]
    g = np.zeros(8, np.float32)
    o = Proto(3, 2, off, dtype=np.float32)
    o.set_state(g)
    s = B.Shard(3, 2, off, host_only=True)

    class E:
        def __getattr__(self, k):
            return getattr(s, k)

        def accumulate(self, r, mb, grad, tb=0, te=None, snapshot=False):
            return s.accumulate(r, mb, None, tb, te)

    e = E()
    # an iteration that crosses a boundary, stopped before the advancement
    for eng in (o, e):
        for k in range(2):
            for r in range(3):
                if not (r == 2 and k == 1):
                    eng.accumulate(r, r + 3 * k, g)
        eng.on_failure([2])
        eng.restore(None)
        for r in (0, 1):
            v = view_oracle(o) if eng is o else view_hip(s)
            while v["contributed"][r] < v["target"][r]:
                eng.accumulate(r, 100 + r + 3 * v["contributed"][r], g)
                v = view_oracle(o) if eng is o else view_hip(s)
        eng.reduce()
        eng.adamw_step(**HP)
        eng.snapshot(None, 0, 1)              # between the commit and the advancement
        eng.advance()
        eng.accumulate(0, 0, g)
    # a rewind of replica 0 now goes back to the empty bucket 0 but bucket 1 holds a microbatch: refused by both
    with pytest.raises(ProtocolError):
        o.restore(0, stale_only=False)
    assert B.recover_restore(s.ctx, 0, 0) == B.ERR_STATE


def test_context_without_snapshot_buffers_gets_past_a_failure():
    """A context created without snapshot buffers has never snapshotted anything, so after a failure the
    stale set of Alg. 5 is empty: the rewind only lifts the quiesce and the iteration goes on.  Only an
    in-place sum of the old membership cannot be taken back."""
    off = [0, 4, 8]
    s = B.Shard(4, 2, off, host_only=True, snapshots=False)
    o = Proto(4, 2, off, dtype=np.float32)
    o.set_state(np.zeros(8, np.float32))
    g = np.ones(8, np.float32)
    for eng in (s, o):
        for r in range(4):
            assert eng.accumulate(r, r, g)
        for r in (0, 1, 3):                              # replica 2 is gone after one microbatch
            assert eng.accumulate(r, r + 4, g)
    assert B.recover_snapshot(s.ctx, -1, 0, 2) == B.ERR_NO_SNAPSHOT
    assert B.recover_accumulate_snapshot(s.ctx, 0, 99, 0, B.F32, 0, 2) == B.ERR_NO_SNAPSHOT
    a, b = o.on_failure([2]), s.on_failure([2])
    for k in INT_KEYS:
        assert a[k] == b[k], k
    assert b["at_boundary"] == 1 and b["restore_mode"] == B.RESTORE_NONBLOCKING
    assert s.reduce() is False                            # quiesced
    assert B.recover_adamw_step(s.ctx, 1e-3, 0.9, 0.95, 1e-8, 0.1) == B.ERR_STATE
    assert o.restore(None) == 0
    s.restore(None)                                       # no error: nothing to rewind
    assert s.query()["restore_mode"] == B.RESTORE_SKIP
    for eng in (s, o):
        for r in (0, 1):
            assert eng.accumulate(r, r + 8, g)            # the extended pass: quotas 3, 3, 2
        assert not eng.accumulate(3, 3 + 8, g)
        eng.reduce()
        eng.adamw_step(**HP)
    assert s.advance()["G_cur"] == o.advance()["G_cur"] == 3
    # a bucket that already holds the old membership's in-place sum cannot be repaired without a snapshot
    for r in (0, 1, 3):
        assert s.accumulate(r, r, g)
    s.reduce(0, 1, inplace=True)
    s.on_failure([3])
    assert B.recover_restore(s.ctx, -1, 1) == B.ERR_NO_SNAPSHOT
    assert B.recover_restore(s.ctx, 3, 1) == B.ERR_STATE   # dead replica
    s.close()


def test_slab_layout_on_the_cpu():
    """alloc_slab's carving (alignment, padding, dtypes, zero fill) with CPU memory; no device call."""
    import torch
    owner, bufs = B.alloc_slab([(torch.float32, 1000), (torch.bfloat16, 77), (torch.float32, 5)], device="cpu",
                               pad_bytes=4096, align=4096)
    assert [b.dtype for b in bufs] == [torch.float32, torch.bfloat16, torch.float32]
    assert [b.numel() for b in bufs] == [1000, 77, 5]
    assert all(b.data_ptr() % 4096 == 0 for b in bufs)
    assert bufs[1].data_ptr() - bufs[0].data_ptr() == 4096 + 4096 and bufs[2].data_ptr() - bufs[1].data_ptr() == 4096 + 4096
    assert all(float(b.float().abs().sum()) == 0 for b in bufs)
    bufs[0].fill_(1.0)
    assert float(bufs[1].float().abs().sum()) == 0
    # groups and windows: a group that fits into a window does not straddle a multiple of the window
    specs = [(torch.float32, 3000)] * 9                                  # 12,000 bytes each -> 12 KiB + 4 KiB of room
    groups = [[0, 1, 2], [3, 4], [5], [6, 7, 8]]
    owner, bufs = B.alloc_slab(specs, device="cpu", pad_bytes=4096, align=4096, groups=groups, window=65536)
    base = bufs[0].data_ptr()
    rel = [b.data_ptr() - base for b in bufs]
    assert rel[:3] == [0, 16384, 32768]                                  # 48 KiB, fits before 64 KiB
    assert rel[3:5] == [65536, 81920]                                    # 32 KiB would cross 64 KiB: next window
    assert rel[5] == 98304                                               # 16 KiB fits up to 112 KiB
    assert rel[6:] == [131072, 147456, 163840]                           # 48 KiB from 112 KiB would cross 128 KiB
    assert all(float(b.abs().sum()) == 0 for b in bufs)
    owner, bufs = B.alloc_slab(specs, device="cpu", pad_bytes=4096, align=4096, groups=[list(range(9))], window=65536)
    assert [b.data_ptr() - bufs[0].data_ptr() for b in bufs] == [16384 * i for i in range(9)]   # too big for a window: plain sequence
    # the groups Shard builds: gradients with their replicas' accumulators, state, snapshots cut like the accumulators
    assert B.stream_groups(4, 2, True, False) == [[0, 2, 3], [1, 4, 5], [6, 7, 8, 9], [10, 11], [12, 13]]
    assert B.stream_groups(3, 2, False, True) == [[0, 1, 2, 3, 4], [5, 6, 7, 8, 9]]
    assert B.stream_groups(2, 0, True, False) == [[0, 1], [2, 3, 4, 5], [6, 7]]
