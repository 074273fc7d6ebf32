"""The two statements of Alg. 1 — the oracle's own loop (oracle/loop.py) and the library's caller loop
(paper_2605_11215_amd/loop.py) — share no code; here they are checked against each other and the
oracle is driven without either of them.

  * both loops issue the same sequence of calls on the failure schedules of the five workloads
    (the library side on a host-only context, so this runs without a GPU);
  * the oracle's Proto under hand-written call sequences, no loop at all: a failure during
    synchronisation that is absorbed by a spare (BLOCKING rewind and re-reduce) and a failure that
    crosses a policy boundary (NON-BLOCKING rewind, extended pass), each checked against the exactly
    rounded mean over the committed ids;
  * the state of the snapshot bookkeeping after a rewind in both modes (Alg. 5).
"""
import numpy as np
import pytest

from oracle import brute
from oracle.loop import run_iteration as oracle_iteration
from oracle.policy import RESTORE_BLOCKING, RESTORE_NONBLOCKING, RESTORE_SKIP, MAJOR, MAJOR_SPARE, DEAD
from oracle.proto import Proto, ProtocolError
from paper_2605_11215_amd import binding as B
from paper_2605_11215_amd.loop import run_iteration as library_iteration, view_shard
from tests.configs import CONFIGS, schedule_of

HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


class Recorder:
    """Forwards to an engine and keeps the state-changing calls, with defaults written out."""

    def __init__(self, eng, T):
        self._e, self._T, self.calls = eng, T, []

    def __getattr__(self, k):
        return getattr(self._e, k)

    def _te(self, te):
        return self._T if te is None else te

    def accumulate(self, r, mb, g, tb=0, te=None, **kw):
        self.calls.append(("accumulate", r, mb, tb, self._te(te)))
        return self._e.accumulate(r, mb, g, tb, te, **kw)

    def snapshot(self, r=None, tb=0, te=None):
        self.calls.append(("snapshot", r, tb, self._te(te)))
        return self._e.snapshot(r, tb, te)

    def reduce(self, tb=0, te=None, inplace=False):
        self.calls.append(("reduce", tb, self._te(te), bool(inplace)))
        return self._e.reduce(tb, te, inplace=inplace)

    def on_failure(self, failed):
        self.calls.append(("on_failure", tuple(failed)))
        return self._e.on_failure(failed)

    def restore(self, r=None, stale_only=True):
        self.calls.append(("restore", r, bool(stale_only)))
        return self._e.restore(r, stale_only=stale_only)

    def adamw_step(self, **hp):
        self.calls.append(("adamw_step",))
        return self._e.adamw_step(**hp)

    def advance(self):
        self.calls.append(("advance",))
        return self._e.advance()


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_both_loops_issue_the_same_calls_on_the_workload_schedules(cid):
    c = CONFIGS[cid]
    W, G = c["W"], c["G"]
    T = len(c["off"]) - 1
    off = list(range(T + 1))                            # the real tensor count, one element each
    sched = schedule_of(c)
    o = Recorder(Proto(W, G, off, dtype=np.float32), T)
    o.set_state(np.zeros(T, np.float32))
    s = B.Shard(W, G, off, host_only=True)
    lib = Recorder(s, T)
    g = np.ones(T, np.float32)
    for t in range(c["iters"]):
        dying = sched.get(t)
        k = T // 2 if c.get("fidelity") and dying else 0
        a = oracle_iteration(o, t, lambda t_, mb: g, dying=dying, reduced_before_failure=k,
                             snapshot_every=c.get("snapshot_every", False), hp=HP)
        b = library_iteration(lib, view_shard, t, lambda t_, mb: None, W, dying=dying, fidelity_k=k,
                              snapshot_every=c.get("snapshot_every", False), hp=HP)
        assert o.calls == lib.calls, (cid, t)
        assert a["ids"] == b["ids"]
        assert sum(len(v) for v in a["ids"].values()) == W * G          # Eq. 1
        o.calls.clear()
        lib.calls.clear()
    s.close()


def grads(n, seed):
    rng = np.random.default_rng(seed)
    cache = {}

    def g(mb):
        if mb not in cache:
            cache[mb] = rng.standard_normal(n) * 1e-3
        return cache[mb]
    return g


def test_hand_written_boundary_sequence():
    """W = 3, G = 2 (B = 6), two buckets.  Replica 1 crashes after one microbatch; the survivors learn of
    it while bucket 0 is already all-reduced in place.  No spare exists, so this is a policy boundary:
    G_ext = 1 with no boundary minor (C_cur = 4, 2 survivors: 4 + 2 = 6), NON-BLOCKING rewind, one extra
    slot, fresh snapshots.  Every call is written out; no loop code is involved."""
    off = [0, 3, 8]
    g = grads(8, 5)
    p = Proto(3, 2, off, dtype=np.float64)
    p.set_state(np.zeros(8))
    for mb in (0, 1, 2):                                   # slot 1: ids r + 3 * 0
        assert p.accumulate(mb, mb, g(mb))
    assert p.accumulate(0, 3, g(3)) and p.accumulate(2, 5, g(5))     # slot 2; replica 1 is gone
    p.snapshot(None, 0, 1)
    p.reduce(0, 1, inplace=True)                           # bucket 0 under the old membership (includes replica 1)
    d = p.on_failure([1])
    assert (d["at_boundary"], d["G_ext"], d["n_bdry"], d["restore_mode"]) == (1, 1, 0, RESTORE_NONBLOCKING)
    assert d["C_cur"] == 4 and d["loop_bound"] == 3 and d["target"][0] == 3 and d["target"][2] == 3
    assert p.reduce(1, 2) is False                         # quiesced until the rewind
    assert p.restore(None, stale_only=True) == 2           # bucket 0 of replicas 0 and 2
    assert not any(p.snap_valid[0]) and not any(p.snap_valid[2])       # bookkeeping cleared (Alg. 5, NON-BLOCKING)
    assert p.accumulate(0, 6, g(6)) and p.accumulate(2, 8, g(8))       # the extended pass
    assert p.accumulate(0, 9, g(9)) is False               # quota met
    p.snapshot(None)
    p.reduce()
    ids = p.committed_ids()
    assert sorted(ids) == [0, 2, 3, 5, 6, 8]
    want = brute.exact_mean([g(j) for j in ids], 6)
    assert np.max(np.abs(p.grad_out - want)) <= 1e-15 * np.max(np.abs(want))
    p.adamw_step(**HP)
    d = p.advance()
    assert (d["G_cur"], d["n_maj"], d["R_cur"]) == (3, 2, 0)


def test_hand_written_failure_during_synchronisation_absorbed_by_a_spare():
    """W = 5, G = 1 first loses replica 4 (boundary; then 4 survivors with B = 5: G_cur = 2, two majors, one
    minor at 1, one major-spare).  In the next iteration major 0 crashes during synchronisation with bucket 0
    already all-reduced: the major-spare (replica 3) is promoted, no boundary, BLOCKING mode: stale buckets
    are rewound and re-reduced, and the snapshots stay valid under the new epoch."""
    off = [0, 2, 5]
    g = grads(5, 9)
    p = Proto(5, 1, off, dtype=np.float64)
    p.set_state(np.zeros(5))
    out = oracle_iteration(p, 0, lambda t, mb: g(mb), dying={4: 0}, hp=HP)       # sets the stage
    w = p.world
    assert [w.role[r] for r in range(5)] == [MAJOR, MAJOR, 1, MAJOR_SPARE, DEAD] and w.target[:4] == [2, 2, 1, 2]
    for r, mb in ((0, 0), (1, 1), (2, 2), (3, 3), (0, 5), (1, 6), (3, 8)):       # the spare shadows a major
        assert p.accumulate(r, mb, g(10 + mb))
    p.snapshot(None, 0, 1)
    p.reduce(0, 1, inplace=True)
    before = p.acc[3].copy()
    d = p.on_failure([0])
    assert (d["at_boundary"], d["restore_mode"], d["G_ext"]) == (0, RESTORE_BLOCKING, 0)
    assert w.role[3] == MAJOR and d["loop_bound"] == 2
    assert p.restore(None, stale_only=True) == 3                      # bucket 0 of replicas 1, 2, 3
    assert w.restore_mode == RESTORE_SKIP
    for r in (1, 2, 3):                                               # BLOCKING: records kept, tag moved to eps_cur
        assert p.snap_valid[r][0] and p.snap_eps[r][0] == w.eps and not p.snap_valid[r][1]
        assert p.restore(r, stale_only=True) == 0                     # nothing is stale any more
    assert np.array_equal(p.acc[3][2:], before[2:]) and not np.array_equal(p.acc[3][:2], before[:2])
    p.snapshot(None)
    p.reduce()
    ids = p.committed_ids()
    assert sorted(ids) == [1, 2, 3, 6, 8]
    want = brute.exact_mean([g(10 + j) for j in ids], 5)
    assert np.max(np.abs(p.grad_out - want)) <= 1e-15 * np.max(np.abs(want))
    assert p.ready_to_commit()


def test_rewind_of_everything_after_a_blocking_restore_uses_the_kept_snapshots():
    """After a BLOCKING rewind the snapshot still describes the pre-reduce state under the new membership:
    a later full rewind (stale_only = False) brings back exactly that state, microbatch counts included."""
    off = [0, 4]
    g = grads(4, 3)
    p = Proto(3, 2, off, dtype=np.float64, static=False)              # Alg. 8 world: every failure is BLOCKING
    p.set_state(np.zeros(4))
    for r in range(3):
        p.accumulate(r, r, g(r))
    p.snapshot(None)
    held = [a.copy() for a in p.acc]
    p.reduce(inplace=True)
    d = p.on_failure([2])
    assert d["restore_mode"] == RESTORE_BLOCKING
    p.restore(None, stale_only=True)
    assert all(np.array_equal(p.acc[r], held[r]) for r in (0, 1)) and p.world.contributed[:2] == [1, 1]
    p.accumulate(0, 3, g(3))
    p.accumulate(1, 4, g(4))
    assert p.world.contributed[:2] == [2, 2]
    assert p.restore(None, stale_only=True) == 0 and p.world.contributed[:2] == [2, 2]
    assert p.restore(None, stale_only=False) == 2                     # back to the kept snapshots
    assert all(np.array_equal(p.acc[r], held[r]) for r in (0, 1)) and p.world.contributed[:2] == [1, 1]
    assert p.ids[0] == [0] and p.ids[1] == [1]
    with pytest.raises(ProtocolError):
        p.accumulate(2, 5, g(5))                                      # dead
