"""Pins for oracle/proto.py and oracle/brute.py (CPU only).

What fixes the oracle from outside: the definition of the iteration gradient (brute-force
exactly rounded sums over the committed ids), power-of-two coded gradients whose sum shows
which microbatches are inside and how often, constant gradients (closed form), and the
restoration invariants of Sec. 4.2 (a rewound bucket equals one that never took the lost
work)."""
import numpy as np
import pytest

from oracle import brute
from oracle.policy import RESTORE_NONBLOCKING
from oracle.proto import Proto, ProtocolError
from paper_2605_11215_amd.synth import reference_np as S
from tests.driver import run_iteration, view_oracle, HP

OFF_RAGGED = [0, 1, 4, 9, 1032, 1037, 1100]          # tensor lengths 1, 3, 5, 1023, 5, 63


def grads(seed, scale=1e-3, n=OFF_RAGGED[-1], bf16=False):
    cache = {}

    def grad_of(t, mb):
        if (t, mb) not in cache:
            g = S.fill(n, seed, S.TAG_GRAD, mb, t, scale)
            cache[(t, mb)] = S.bf16_bits_to_f32(S.f32_to_bf16_bits(g)) if bf16 else g
        return cache[(t, mb)]
    return grad_of


def new_proto(W, G, off=OFF_RAGGED, dtype=np.float64, seed=1, **kw):
    p = Proto(W, G, off, dtype=dtype, **kw)
    p.set_state(S.fill(off[-1], seed, S.TAG_PARAM, 0, 0, 0.02))
    return p


def test_tiny_schedule_quotas_and_ids():
    """R=4, G=2, replica 2 dies after one microbatch of iteration 1: survivors end at
    quotas 3, 3, 2 (sum 8) and the committed ids are the survivors' own slices."""
    p = new_proto(4, 2)
    g = grads(1)
    out = run_iteration(p, view_oracle, 0, g, 4)
    assert sorted(sum(out["ids"].values(), [])) == list(range(8))
    out = run_iteration(p, view_oracle, 1, g, 4, dying={2: 1})
    d = out["decisions"][0]
    assert d["at_boundary"] and d["C_cur"] == 6 and d["G_ext"] == 1 and d["n_bdry"] == 1
    assert out["ids"] == {0: [0, 4, 8], 1: [1, 5, 9], 3: [3, 7]}
    adv = out["decisions"][-1]
    assert (adv["G_cur"], adv["n_maj"], adv["R_cur"]) == (3, 2, 2)
    out = run_iteration(p, view_oracle, 2, g, 4)
    assert out["ids"] == {0: [0, 4, 8], 1: [1, 5, 9], 3: [3, 7]}


@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-15), (np.float32, 2e-6)])
def test_iteration_gradient_is_the_mean_over_committed_ids(dtype, tol):
    """proto's grad_out against the exactly rounded sum over A(t), failure-free and not."""
    p = new_proto(4, 2, dtype=dtype)
    g = grads(3)
    for t, dying in enumerate([None, {2: 1}, None, {0: 0, 3: 2}]):
        captured = {}
        out = run_iteration(p, view_oracle, t, g, 4, dying=dying)
        ids = sum(out["ids"].values(), [])
        assert len(ids) == 8 == len(set(ids))
        want = brute.exact_mean([g(t, j) for j in ids], 8)
        # grad_out of iteration t is still in the buffer after the step
        got = p.grad_out.astype(np.float64)
        assert np.max(np.abs(got - want)) <= tol * np.max(np.abs(want))
        assert np.allclose(brute.mean64([g(t, j) for j in ids], 8), want, rtol=0, atol=1e-18)


def coded(n=8):
    """Microbatch j's gradient is 2**j in every element: a sum shows its terms as bits."""
    def grad_of(t, mb):
        return np.full(n, 2.0 ** mb, np.float64)
    return grad_of


def terms_of(x):
    x = int(x)
    return [j for j in range(x.bit_length()) if (x >> j) & 1]


@pytest.mark.parametrize("fidelity_k", [0, 1, 2])
def test_each_committed_microbatch_enters_exactly_once(fidelity_k):
    """Sec. 4.2 invariant: every bucket is reduced once under one membership and nothing of
    the failed replica is retained, also when part of the buckets had already been
    all-reduced under the old membership (failure during synchronisation)."""
    off = [0, 3, 5, 8]
    p = new_proto(4, 2, off=off)
    out = run_iteration(p, view_oracle, 0, coded(), 4, dying={2: 1}, fidelity_k=fidelity_k)
    total = p.grad_out * 8
    assert np.all(total == total[0])
    assert terms_of(total[0]) == [0, 1, 3, 4, 5, 7, 8, 9]        # no id 2, none twice
    assert out["ids"] == {0: [0, 4, 8], 1: [1, 5, 9], 3: [3, 7]}


def test_promoted_spare_contributes_its_own_microbatches_after_rewind():
    """Non-boundary failure with in-place partial sync: the spare's buckets were overwritten
    by the all-reduce, the rewind brings its own gradients back (boundary walk-through,
    last paragraph)."""
    off = [0, 2, 4]
    p = new_proto(3, 2, off=off)                     # B = 6
    run_iteration(p, view_oracle, 0, coded(4), 3, dying={2: 0})   # boundary: 2 survivors x 3
    w = p.world
    assert w.G_cur == 3 and w.alive() == [0, 1]
    # make a world with a spare: 5 replicas, B = 10, lose one -> G_cur 3, 3 majors + minor(1)
    p = new_proto(5, 2, off=off)
    run_iteration(p, view_oracle, 0, coded(4), 5, dying={4: 1})
    w = p.world
    assert (w.G_cur, w.R_cur) == (3, 1) and w.role[:4] == [0, 0, 0, 1]
    # 6 replicas, B = 12: lose one -> 5 survivors, G_cur 3, 4 majors, no minor, 1 major-spare
    p = new_proto(6, 2, off=off)
    run_iteration(p, view_oracle, 0, coded(4), 6, dying={5: 2})
    w = p.world
    assert w.role == [0, 0, 0, 0, 2, 4]
    out = run_iteration(p, view_oracle, 1, coded(4), 6, dying={1: 2}, fidelity_k=1)
    d = out["decisions"][0]
    assert not d["at_boundary"] and d["role"][4] == 0
    total = p.grad_out * 12
    assert np.all(total == total[0])
    # ids: r0 {0,6,12}, r2 {2,8,14}, r3 {3,9,15}, promoted r4 {4,10,16}; nothing of r1
    assert terms_of(total[0]) == [0, 2, 3, 4, 6, 8, 9, 10, 12, 14, 15, 16]


def test_spare_is_masked_out_of_the_sum():
    """Sec. 4.3: a spare runs the same microbatches as its counterpart but does not enter the global
    batch.  Six replicas, one lost: four majors at 3 and one major-spare; the next, failure-free
    iteration commits the majors' twelve ids and none of the spare's (4, 10, 16)."""
    off = [0, 2, 4]
    p = new_proto(6, 2, off=off)
    run_iteration(p, view_oracle, 0, coded(4), 6, dying={5: 2})
    assert p.world.role == [0, 0, 0, 0, 2, 4]
    out = run_iteration(p, view_oracle, 1, coded(4), 6)
    total = p.grad_out * 12
    assert np.all(total == total[0])
    assert terms_of(total[0]) == [0, 1, 2, 3, 6, 7, 8, 9, 12, 13, 14, 15]
    assert p.ids[4] == [] and 4 not in out["ids"]            # the iteration is over; the spare never counted
    assert len(p.world.alive()) == 5


def test_constant_gradient_closed_form_and_constant_divisor():
    """If every microbatch gradient equals c the committed mean is c whatever failed: the
    divisor stays B = W_init * G_init (Sec. 4.3, Eq. 1; implementation appendix)."""
    c = np.float32(0.375)
    g = lambda t, mb: np.full(OFF_RAGGED[-1], c, np.float32)
    for dtype in (np.float32, np.float64):
        p = new_proto(8, 4, dtype=dtype)
        for t, dying in enumerate([None, {3: 2, 6: 2}, None, {0: 1}]):
            run_iteration(p, view_oracle, t, g, 8, dying=dying)
            assert np.all(p.grad_out == c)


def test_adaptive_policy_commits_fewer_than_B():
    p = new_proto(4, 2, static=False)
    out = run_iteration(p, view_oracle, 0, grads(1), 4, dying={2: 1})
    assert sum(len(v) for v in out["ids"].values()) == 6 < 8


def test_restore_after_partial_microbatch_equals_never_started():
    """Survivors have begun the next microbatch on some tensors when the failure is
    handled; the rewind to the boundary snapshot leaves no trace of it."""
    g = grads(5)
    a = new_proto(4, 2, dtype=np.float32)
    b = new_proto(4, 2, dtype=np.float32)
    for p in (a, b):
        for r in range(4):
            p.accumulate(r, r, g(0, r))
        p.snapshot(None)
    for r in (0, 1, 3):
        a.accumulate(r, r + 4, g(0, r + 4), 0, 3)     # tensors [0,3) only
        assert a.world.contributed[r] == 1
    for p in (a, b):
        p.on_failure([2])
        p.restore(None, stale_only=True)
    for r in (0, 1, 3):
        assert np.array_equal(a.acc[r].view(np.uint32), b.acc[r].view(np.uint32))
        assert a.cnt[r] == b.cnt[r] and a.ids[r] == b.ids[r] == [r]
    for p in (a, b):
        for r in (0, 1, 3):
            while p.world.should_contribute(r):
                k = p.world.contributed[r]
                p.accumulate(r, r + 4 * k, g(0, r + 4 * k))
        p.snapshot(None)
        p.reduce()
    assert np.array_equal(a.grad_out.view(np.uint32), b.grad_out.view(np.uint32))
    a.adamw_step(**HP)


def test_failure_run_equals_clean_replay_bit_for_bit():
    """fp32: the committed gradient depends only on the ordered ids inside each
    contributor's buffer, not on failures, snapshots, in-place reductions or rewinds."""
    g = grads(7)
    p = new_proto(8, 4, dtype=np.float32)
    run_iteration(p, view_oracle, 0, g, 8)
    out = run_iteration(p, view_oracle, 1, g, 8, dying={3: 2, 6: 2}, fidelity_k=3)
    got = p.grad_out.copy()
    assert out["decisions"][0]["restore_mode"] == RESTORE_NONBLOCKING
    acc = {}
    for r, ids in out["ids"].items():
        a = np.float32(0) + g(1, ids[0])
        for j in ids[1:]:
            a = a + g(1, j)
        acc[r] = a
    rs = sorted(acc)
    tot = acc[rs[0]].copy()
    for r in rs[1:]:
        tot = tot + acc[r]
    want = tot / np.float32(32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # another partition of the same ids agrees to rounding only
    ids = sum(out["ids"].values(), [])
    one = brute.mean64([g(1, j) for j in ids], 32)
    assert np.max(np.abs(got - one)) <= 2e-6 * np.max(np.abs(one))


def test_bf16_inputs_widen_exactly():
    g = grads(9, scale=5e-4, bf16=True)
    p32 = new_proto(4, 2, dtype=np.float32)
    p64 = new_proto(4, 2, dtype=np.float64)
    for p in (p32, p64):
        run_iteration(p, view_oracle, 0, g, 4, dying={1: 1})
    ref = p64.grad_out
    assert np.max(np.abs(p32.grad_out - ref)) <= 1e-6 * np.max(np.abs(ref))
    x = g(0, 0)
    assert np.all((x.view(np.uint32) & 0xFFFF) == 0)


def test_first_microbatch_overwrites_like_zero_then_add():
    p = new_proto(1, 2, off=[0, 4], dtype=np.float32)
    p.acc[0][:] = 123.0                                # stale content of the previous iteration
    g0 = np.array([-0.0, 1.0, -2.0, 0.0], np.float32)
    p.accumulate(0, 0, g0)
    assert np.array_equal(p.acc[0], np.array([0.0, 1.0, -2.0, 0.0], np.float32))
    assert not np.signbit(p.acc[0][0])                 # (+0) + (-0) = +0


def test_protocol_violations_are_errors():
    g = grads(1)
    p = new_proto(4, 2)
    for r in range(4):
        p.accumulate(r, r, g(0, r))
    p.reduce()
    with pytest.raises(ProtocolError):                 # only 4 of 8 microbatches inside
        p.adamw_step(**HP)
    for r in range(4):
        p.accumulate(r, r + 4, g(0, r + 4))
        assert p.accumulate(r, r + 8, g(0, r + 8)) is False     # quota met: dropped
    with pytest.raises(ProtocolError):                 # reduction predates the last adds
        p.adamw_step(**HP)
    p.reduce()
    p.on_failure([1])
    with pytest.raises(ProtocolError):                 # epoch moved: everything is stale
        p.adamw_step(**HP)
    assert p.reduce() is False                         # quiesced until the restore
    with pytest.raises(ProtocolError):
        p.accumulate(1, 99, g(0, 0))                   # dead replica
    with pytest.raises(ProtocolError):
        p.accumulate(0, 2, g(0, 0))                    # ids must ascend within a replica


def test_rewind_drops_completed_microbatches_from_the_audit():
    """A snapshot at a microbatch boundary, one more complete microbatch, then a rewind of the
    whole replica: count, audit and committed set are those of the boundary, and the same
    microbatch can be accumulated again (Sec. 4.2: rewound work is as if never done)."""
    g = grads(11)
    p = new_proto(2, 3, dtype=np.float32)
    p.accumulate(0, 0, g(0, 0))
    p.snapshot(0)
    at_boundary = p.acc[0].copy()
    p.accumulate(0, 2, g(0, 2))
    assert p.ids[0] == [0, 2] and p.world.contributed[0] == 2
    p.restore(0, stale_only=False)
    assert p.ids[0] == [0] and p.world.contributed[0] == 1 and p.cnt[0] == [1] * p.T
    assert np.array_equal(p.acc[0], at_boundary)
    assert p.accumulate(0, 2, g(0, 2)) and p.ids[0] == [0, 2]


def test_inplace_reduction_leaves_the_sum_in_every_survivor():
    """Alg. 2 Reduce is an in-place all-reduce: afterwards every member of the group, spares
    included, holds the sum; a spare's own gradients come back only through the rewind."""
    off = [0, 2, 4]
    p = new_proto(6, 2, off=off)
    run_iteration(p, view_oracle, 0, coded(4), 6, dying={5: 2})       # leaves r4 a major-spare
    for k in range(3):
        for r in range(5):
            p.accumulate(r, r + 6 * k, coded(4)(1, r + 6 * k))
    own = p.acc[4].copy()
    p.snapshot(None)
    p.reduce(0, 1, inplace=True)
    want = sum(2.0 ** j for j in (0, 1, 2, 3, 6, 7, 8, 9, 12, 13, 14, 15))
    for r in range(5):
        assert np.all(p.acc[r][0:2] == want), r                       # the spare's bucket too
        assert np.array_equal(p.acc[r][2:4], (own if r == 4 else p.acc[r])[2:4])
    p.restore(4, stale_only=False)
    assert np.array_equal(p.acc[4], own)


def test_reduction_under_an_older_epoch_cannot_be_committed():
    """Sec. 4.2: everything admitted must be reduced under one membership.  A failure absorbed by a
    spare leaves the totals at B, yet a reduction from before the repair holds the dead replica's
    gradients and lacks the promoted spare's: the step is refused until it is redone."""
    off = [0, 2, 4]
    p = new_proto(6, 2, off=off)
    run_iteration(p, view_oracle, 0, coded(4), 6, dying={5: 2})       # r4 becomes a major-spare
    for k in range(3):
        for r in range(5):
            p.accumulate(r, r + 6 * k, coded(4)(1, r + 6 * k))
    p.reduce()                                                        # no snapshots taken
    d = p.on_failure([1])
    assert not d["at_boundary"] and d["role"][4] == 0
    p.restore(None)                                                   # nothing to rewind
    assert p.world.C_cur() == 12
    with pytest.raises(ProtocolError):
        p.adamw_step(**HP)
    p.reduce()
    assert terms_of((p.grad_out * 12)[0]) == [0, 2, 3, 4, 6, 8, 9, 10, 12, 14, 15, 16]
    p.adamw_step(**HP)


def test_failure_after_synchronisation_is_handled_in_the_next_iteration():
    """Sec. 4.2 case (b): every bucket was reduced in the original world, so the iteration commits
    with the lost replica's microbatches inside; the failure is declared at the start of the next
    iteration, which then runs an extended loop from its first slot."""
    off = [0, 3, 5]
    p = new_proto(4, 2, off=off)
    out = run_iteration(p, view_oracle, 0, coded(5), 4)
    assert terms_of((p.grad_out * 8)[0]) == list(range(8))          # replica 2's ids 2 and 6 included
    d = p.on_failure([2])                                           # learnt after the step
    assert d["at_boundary"] and d["C_cur"] == 0 and d["G_ext"] == 1 and d["n_bdry"] == 1
    p.restore(None)
    out = run_iteration(p, view_oracle, 1, coded(5), 4)
    assert out["ids"] == {0: [0, 4, 8], 1: [1, 5, 9], 3: [3, 7]}
    assert terms_of((p.grad_out * 8)[0]) == [0, 1, 3, 4, 5, 7, 8, 9]
    assert p.world.G_cur == 3 and p.world.role == [0, 0, 4, 1]


def test_random_call_sequences_commit_each_audited_microbatch_exactly_once():
    """The restoration invariant under random (not scripted) call sequences: partial ranges, partial
    microbatches, snapshots, in-place reductions, failures, rewinds.  Microbatch j carries 2**(j mod 52)
    scaled per round of 52, so at every commit the reduced gradient, read as an integer, must be
    exactly the sum over the audited ids: each once, nothing of a dead replica, nothing rewound."""
    from tests import differential

    class Mirror:
        """A second oracle behind the library-side interface (the harness needs two engines)."""

        def __init__(self, W, G, off):
            self.p = Proto(W, G, off, dtype=np.float64)
            self.p.set_state(np.zeros(off[-1], np.float32))
            self.W = W

        def query(self):
            w = self.p.world
            return dict(role=list(w.role), target=list(w.target), contributed=list(w.contributed),
                        loop_bound=w.loop_bound, epoch=w.eps)

        def _replica(self, r):
            if r is not None and not 0 <= r < self.W:
                raise ProtocolError("replica index")
            return r

        def accumulate(self, r, mb, g, tb=0, te=None, snapshot=False):
            return self.p.accumulate(self._replica(r), mb, g, tb, te)

        def snapshot(self, r=None, tb=0, te=None):
            return self.p.snapshot(self._replica(r), tb, te)

        def restore(self, r=None, stale_only=True):
            return self.p.restore(self._replica(r), stale_only)

        def __getattr__(self, k):
            return getattr(self.p, k)

    off = [0, 2, 3, 3, 7]
    checked = 0
    for seed in range(30):
        W, G = [(4, 2), (2, 4), (8, 1), (4, 4)][seed % 4]        # B a power of two: the division is exact

        def code(mb):
            return np.full(off[-1], float(2 ** (mb % 52)) * (1 + (mb // 52)), np.float64)

        def check(o):
            nonlocal checked
            want = sum(float(2 ** (j % 52)) * (1 + j // 52) for j in o.committed_ids())
            assert len(o.committed_ids()) == o.world.B
            assert np.all(o.grad_out * o.world.B == want), (seed, o.committed_ids())
            checked += 1

        differential.run(700 + seed, 300, W, G, off, Mirror(W, G, off), grad_of_id=code, oracle_dtype=np.float64,
                         before_commit=check)
    assert checked > 100
