"""Oracle: step-by-step simulator of the gradient path on NumPy arrays (test infrastructure only).

One `Proto` object holds what W_init data-parallel replicas hold for one parameter shard:
a gradient accumulator per replica, a snapshot per replica, and the bookkeeping of
Sec. 4.2 (snapshot + world-epoch tag per bucket; here a bucket is one tensor of the
shard).  The steps are those of Alg. 1 in the paper's order:

  accumulate   Alg. 1, local accumulation: skipped once the quota is met
  snapshot     Alg. 1, snapshot step: S(b) <- b, tag eps(b) <- eps_cur
  reduce       Alg. 2, Reduce: sum over non-spare survivors; `inplace` leaves the sum in every
               survivor's bucket as an all-reduce does
  on_failure   Alg. 2 Record, Alg. 4, Alg. 6
  restore      Alg. 5: stale = {b : eps(b) < eps_cur}; copy S(b) -> b
  commit       Alg. 1, commit step: divide by the constant B, optimiser step
  advance      Alg. 7

`dtype` is the arithmetic type of accumulate and reduce: float64 is the reference value,
float32 is the precision the paper trains in (fp32 accumulation and synchronisation,
evaluation appendix), evaluated in the canonical order
    acc_r = ((0 + g_a) + g_b) + ...   (ids in the order they were accumulated)
    sum   = ((acc_r0 + acc_r1) + ...) (ascending replica index),  grad = sum / B.
Adds and one divide only, so a float32 run of this file is reproducible bit for bit by
any IEEE implementation that keeps the order.
"""
import numpy as np

from . import adamw as _adamw
from .policy import (World, MAJOR, MINOR, MAJOR_SPARE, MINOR_SPARE, DEAD,
                     RESTORE_SKIP, RESTORE_BLOCKING, RESTORE_NONBLOCKING)


class ProtocolError(Exception):
    pass


class Proto:
    def __init__(self, W_init, G_init, tensor_offsets, dtype=np.float64, static=True,
                 state_dtype=np.float32, fixed_order=True):
        self.world = World(W_init, G_init, static=static)
        self.off = [int(x) for x in tensor_offsets]
        assert self.off[0] == 0 and all(a <= b for a, b in zip(self.off, self.off[1:]))
        self.T = len(self.off) - 1
        self.N = self.off[-1]
        self.dtype = np.dtype(dtype)
        self.state_dtype = np.dtype(state_dtype)
        self.fixed_order = fixed_order
        W = W_init
        self.acc = [np.zeros(self.N, self.dtype) for _ in range(W)]
        self.snap = [np.zeros(self.N, self.dtype) for _ in range(W)]
        self.grad_out = np.zeros(self.N, self.dtype)
        self.param = self.m = self.v = None
        self.t = 0                                   # optimiser steps taken
        self._begin_iteration_buffers()

    # ------------------------------------------------------------------ helpers
    def _begin_iteration_buffers(self):
        W, T = self.world.W_init, self.T
        self.cnt = [[0] * T for _ in range(W)]       # microbatches summed into acc[r][b]
        self.cur_id = [None] * W                     # id of a partly accumulated microbatch
        self.ids = [[] for _ in range(W)]            # audit: ids fully accumulated, in order
        self.snap_valid = [[False] * T for _ in range(W)]
        self.snap_eps = [[0] * T for _ in range(W)]
        self.snap_cnt = [[0] * T for _ in range(W)]
        self.inplace_sum = [[False] * T for _ in range(W)]   # acc[r][b] holds a reduced sum
        self.red_eps = [-1] * T                      # epoch of the last reduction of b
        self.red_total = [0] * T                     # microbatches inside that reduction
        self.red_dirty = [True] * T                  # bucket changed since that reduction
        self.quiesced = False

    def _rng(self, tb, te):
        te = self.T if te is None else te
        if not (0 <= tb <= te <= self.T):
            raise ProtocolError("tensor range")
        return tb, te

    def set_state(self, param, m=None, v=None):
        """Optimiser state (parameters and the two moments), kept in `state_dtype` between steps."""
        self.param = np.array(param, self.state_dtype)
        self.m = np.zeros(self.N, self.state_dtype) if m is None else np.array(m, self.state_dtype)
        self.v = np.zeros(self.N, self.state_dtype) if v is None else np.array(v, self.state_dtype)

    # ------------------------------------------------------------------ Alg. 1, local accumulation
    def accumulate(self, r, mb_id, g, tb=0, te=None):
        """Add microbatch `mb_id`'s gradient `g` (flat, length N, any float type) into
        replica r's accumulator over tensors [tb, te).  Returns False when the replica
        has met its quota and the gradient is dropped."""
        w = self.world
        tb, te = self._rng(tb, te)
        if w.pending_advance:
            raise ProtocolError("advance the policy first")
        if w.role[r] == DEAD:
            raise ProtocolError("dead replica")
        if not w.should_contribute(r):
            return False
        k = w.contributed[r]
        if self.cur_id[r] is not None:
            if self.cur_id[r] != mb_id:
                raise ProtocolError("previous microbatch is incomplete")
        elif self.fixed_order and self.ids[r] and mb_id <= self.ids[r][-1]:
            raise ProtocolError("microbatch ids must ascend within a replica")
        for b in range(tb, te):
            if self.cnt[r][b] != k or self.inplace_sum[r][b]:
                raise ProtocolError("tensor %d of replica %d cannot take this microbatch" % (b, r))
        self.cur_id[r] = mb_id
        for b in range(tb, te):
            lo, hi = self.off[b], self.off[b + 1]
            gb = np.asarray(g[lo:hi]).astype(self.dtype)       # widening is exact
            if k == 0:                                         # zeroed buffer + g
                self.acc[r][lo:hi] = self.dtype.type(0) + gb
            else:
                self.acc[r][lo:hi] = self.acc[r][lo:hi] + gb
            self.cnt[r][b] = k + 1
            self.red_dirty[b] = True
        if min(self.cnt[r]) == k + 1:
            self.ids[r].append(mb_id)
            self.cur_id[r] = None
            w.contributed[r] = k + 1
        return True

    # ------------------------------------------------------------------ Alg. 1, snapshot step
    def snapshot(self, r=None, tb=0, te=None):
        w = self.world
        tb, te = self._rng(tb, te)
        who = w.alive() if r is None else [r]
        for q in who:
            if w.role[q] == DEAD:
                raise ProtocolError("dead replica")
            if any(self.inplace_sum[q][b] for b in range(tb, te)):
                raise ProtocolError("bucket already holds a reduced sum")
        for q in who:
            for b in range(tb, te):
                lo, hi = self.off[b], self.off[b + 1]
                self.snap[q][lo:hi] = self.acc[q][lo:hi]
                self.snap_valid[q][b] = True
                self.snap_eps[q][b] = w.eps
                self.snap_cnt[q][b] = self.cnt[q][b]

    # ------------------------------------------------------------------ Alg. 2, Reduce
    def reduce(self, tb=0, te=None, inplace=False):
        """Sum the contributors' buckets in ascending replica order and divide by B.
        Returns False (no-op) while the group is quiesced (Alg. 2, quiesce test)."""
        w = self.world
        tb, te = self._rng(tb, te)
        if self.quiesced:
            return False
        divisor = w.B if w.static else sum(w.contributed[r] for r in w.contributors())
        for b in range(tb, te):
            if any(self.inplace_sum[r][b] for r in w.alive()):
                raise ProtocolError("bucket %d was already reduced in place" % b)
        if divisor <= 0:
            raise ProtocolError("nothing has been contributed")
        for b in range(tb, te):
            lo, hi = self.off[b], self.off[b + 1]
            members = [r for r in w.contributors() if self.cnt[r][b] > 0]
            total = np.zeros(hi - lo, self.dtype)
            first = True
            for r in members:
                total = self.acc[r][lo:hi].copy() if first else total + self.acc[r][lo:hi]
                first = False
            self.grad_out[lo:hi] = total / self.dtype.type(divisor)
            self.red_eps[b] = w.eps
            self.red_total[b] = sum(self.cnt[r][b] for r in members)
            self.red_dirty[b] = False
            if inplace:
                for r in w.alive():
                    self.acc[r][lo:hi] = total
                    self.inplace_sum[r][b] = True
        return True

    # ------------------------------------------------------------------ Alg. 2 Record, Alg. 4, Alg. 6
    def on_failure(self, failed):
        d = self.world.on_failure(failed)
        self.quiesced = True                         # later bucket reductions are no-ops
        return d

    # ------------------------------------------------------------------ Alg. 5
    def restore(self, r=None, stale_only=True):
        """Rewind buckets from their snapshots.  stale_only: those tagged with an older
        epoch.  Counts return to the snapshot's, so microbatches accumulated after the
        snapshot (complete or partial) are as if never accumulated.  A rewind must leave
        every tensor of a replica at the same microbatch count, else nothing is copied."""
        w = self.world
        mode = w.restore_mode
        plan = []
        for q in (w.alive() if r is None else [r]):
            if w.role[q] == DEAD:
                raise ProtocolError("dead replica")
            pick = [b for b in range(self.T) if self.snap_valid[q][b]
                    and (not stale_only or self.snap_eps[q][b] < w.eps)]
            after = list(self.cnt[q])
            for b in pick:
                after[b] = self.snap_cnt[q][b]
            if pick and any(c != after[0] for c in after):
                raise ProtocolError("rewind would leave replica %d between microbatches" % q)
            plan.append((q, pick))
        n = 0
        for q, pick in plan:
            for b in pick:
                lo, hi = self.off[b], self.off[b + 1]
                self.acc[q][lo:hi] = self.snap[q][lo:hi]
                self.cnt[q][b] = self.snap_cnt[q][b]
                self.inplace_sum[q][b] = False
                self.snap_eps[q][b] = w.eps
                self.red_dirty[b] = True
                n += 1
            if pick:
                done = self.cnt[q][0]
                del self.ids[q][done:]               # microbatches the rewind dropped
                self.cur_id[q] = None
                w.contributed[q] = done
            if mode == RESTORE_NONBLOCKING:          # clear the bookkeeping: the extended
                for b in range(self.T):              # pass takes fresh snapshots
                    self.snap_valid[q][b] = False
        self.quiesced = False
        if r is None:
            w.restore_mode = RESTORE_SKIP
        return n

    # ------------------------------------------------------------------ Alg. 1, commit step
    def ready_to_commit(self):
        """Every bucket reduced once under the current membership, unchanged since, and
        holding exactly B microbatches (Eq. 1; Sec. 4.2 restoration invariant)."""
        w = self.world
        want = w.B if w.static else w.C_cur()
        for b in range(self.T):
            if self.red_eps[b] != w.eps or self.red_dirty[b] or self.red_total[b] != want:
                return False
        return not self.quiesced

    def committed_ids(self):
        """The multiset A(t) of the proof-sketch appendix: ids inside the contributors' buffers."""
        out = []
        for r in self.world.contributors():
            out.extend(self.ids[r])
        return out

    def committed_ids_by_replica(self):
        """phi_t of the proof-sketch appendix: replica -> the microbatches it contributes."""
        return {r: list(self.ids[r]) for r in self.world.contributors()}

    def adamw_step(self, lr, beta1, beta2, eps, weight_decay):
        if not self.ready_to_commit():
            raise ProtocolError("reduction incomplete or Eq. 1 violated")
        self.t += 1
        p, m, v = _adamw.adamw_step(self.param, self.m, self.v, self.grad_out, self.t,
                                    lr, beta1, beta2, eps, weight_decay)
        self.param = p.astype(self.state_dtype)
        self.m = m.astype(self.state_dtype)
        self.v = v.astype(self.state_dtype)
        self.world.commit()
        self._begin_iteration_buffers()

    def advance(self):
        """Alg. 7, after an iteration that crossed a policy boundary."""
        return self.world.advance()
