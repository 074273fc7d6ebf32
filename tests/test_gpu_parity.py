"""GPU parity tests proper: the HIP library, called through the C ABI, against the CPU
oracle element by element on the same seeded inputs.

Bars: integers (quotas, roles, ids) bit-exact; the iteration gradient bit-exact against the
oracle evaluated in fp32 (the precision the paper accumulates and synchronises in: adds and
one divide, same order) and within 1e-6 max-norm relative error of the fp64 oracle (1e-2
when bf16 gradients are compared with the unrounded fp32 samples); AdamW state within 1e-6
max-norm relative error of the fp64 oracle fed the same fp32 gradient."""
import numpy as np
import pytest

from oracle.proto import Proto
from oracle import adamw as oracle_adamw
from paper_2605_11215_amd import binding as B
from paper_2605_11215_amd import synth
from paper_2605_11215_amd.synth import reference_np as S
from tests.driver import run_iteration, view_oracle, HP
from tests.gpu_harness import HipEngine, view_hip, max_rel, bits_equal, assert_adamw_elementwise

pytestmark = pytest.mark.gpu

# lengths 1, 3, 5, 1023, 0, 4099, 20000, 7: ragged ends, an empty tensor, several 4096-element tiles
OFF = [0, 1, 4, 9, 1032, 1032, 5131, 25131, 25138]


def torch_():
    import torch
    return torch


def hp32():
    return {k: float(np.float32(v)) for k, v in HP.items()}


def test_synth_device_stream_equals_numpy_bits():
    torch = torch_()
    n, start = 300003, 5
    for kind, bf16 in [(S.KIND_NORMAL, False), (S.KIND_NORMAL, True), (S.KIND_STUDENT_T3, False),
                       (S.KIND_STUDENT_T3, True)]:
        out = torch.empty(n, dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda")
        synth.fill_device(out, 1, S.TAG_GRAD, 9, 2, 1e-3, kind, start=start)
        want = S.fill(n, 1, S.TAG_GRAD, 9, 2, 1e-3, kind, start=start)
        if bf16:
            got = out.view(torch.int16).cpu().numpy().view(np.uint16)
            assert np.array_equal(got, S.f32_to_bf16_bits(want))
        else:
            assert bits_equal(out.cpu().numpy(), want)
    far = torch.empty(1000, dtype=torch.float32, device="cuda")
    synth.fill_device(far, 1, S.TAG_GRAD, 63, 3, 1e-3, start=1978662912 - 1000)
    assert bits_equal(far.cpu().numpy(), S.fill(1000, 1, S.TAG_GRAD, 63, 3, 1e-3, start=1978662912 - 1000))


def make_pair(W, G, off, bf16, seed, flags=0):
    torch = torch_()
    p0 = S.fill(off[-1], seed, S.TAG_PARAM, 0, 0, 0.02)
    o32 = Proto(W, G, off, dtype=np.float32, static=not (flags & B.FLAG_ADAPTIVE))
    o32.set_state(p0)
    s = B.Shard(W, G, off, flags=flags, param_bf16=True)
    s.param[:off[-1]].copy_(torch.from_numpy(p0))
    return o32, s, HipEngine(s, bf16)


def grads_np(seed, n, scale, bf16, kind=S.KIND_NORMAL):
    cache = {}

    def grad_of(t, mb):
        if (t, mb) not in cache:
            g = S.fill(n, seed, S.TAG_GRAD, mb, t, scale, kind)
            cache[(t, mb)] = S.bf16_bits_to_f32(S.f32_to_bf16_bits(g)) if bf16 else g
        return cache[(t, mb)]
    return grad_of


def compare_iteration(o32, s, N, before):
    """grad_out bit-exact; AdamW state against the fp64 step from the same gradient and state."""
    g_gpu = s.grad_out[:N].cpu().numpy()
    assert bits_equal(g_gpu, o32.grad_out), "iteration gradient differs from the fp32 oracle"
    p, m, v = oracle_adamw.adamw_step(before[0], before[1], before[2], g_gpu, o32.t, **hp32())
    assert_adamw_elementwise(before, g_gpu, o32.t, hp32(), [x[:N].cpu().numpy() for x in (s.param, s.exp_avg, s.exp_avg_sq)],
                             (p, m, v))
    assert max_rel(s.param[:N].cpu().numpy(), p) <= 1e-6
    assert max_rel(s.exp_avg[:N].cpu().numpy(), m) <= 1e-6
    assert max_rel(s.exp_avg_sq[:N].cpu().numpy(), v) <= 1e-6
    # against the oracle's own running state (fp32 storage on both sides)
    assert max_rel(s.param[:N].cpu().numpy(), o32.param) <= 1e-6
    assert max_rel(s.exp_avg[:N].cpu().numpy(), o32.m) <= 1e-6
    assert max_rel(s.exp_avg_sq[:N].cpu().numpy(), o32.v) <= 1e-6
    torch = torch_()
    pb = s.param_bf16[:N].view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(pb, S.f32_to_bf16_bits(s.param[:N].cpu().numpy()))


def state_of(s, N):
    return [x[:N].cpu().numpy().copy() for x in (s.param, s.exp_avg, s.exp_avg_sq)]


@pytest.mark.parametrize("bf16", [False, True])
def test_ragged_shard_with_failures_matches_oracle(bf16):
    """W=8, G=4 on a ragged tensor list: failure-free, two failures with partial in-place
    synchronisation, promotion-free boundary, then steady state; every iteration compared."""
    N = OFF[-1]
    o32, s, eng = make_pair(8, 4, OFF, bf16, seed=3)
    o64 = Proto(8, 4, OFF, dtype=np.float64)
    o64.set_state(o32.param)
    g = grads_np(3, N, 1e-3, bf16)
    plan = [dict(), dict(dying={3: 2, 6: 2}, fidelity_k=4), dict(), dict(dying={0: 0}, snapshot_every=True), dict()]
    for t, kw in enumerate(plan):
        before = state_of(s, N)
        a = run_iteration(o32, view_oracle, t, g, 8, hp=hp32(), **kw)
        run_iteration(o64, view_oracle, t, g, 8, hp=hp32(), **kw)
        b = run_iteration(eng, view_hip, t, g, 8, hp=hp32(), **kw)
        assert a["ids"] == b["ids"]
        for x, y in zip(a["decisions"], b["decisions"]):
            for k in x:
                assert x[k] == y[k], k
        compare_iteration(o32, s, N, before)
        assert max_rel(s.grad_out[:N].cpu().numpy(), o64.grad_out) <= 1e-6
    if bf16:                                                   # against the unrounded samples
        o_raw = Proto(8, 4, OFF, dtype=np.float64)
        o_raw.set_state(o32.param)
        g_raw = grads_np(3, N, 1e-3, False)
        o_hip, s2, eng2 = make_pair(8, 4, OFF, True, seed=3)
        run_iteration(o_raw, view_oracle, 0, g_raw, 8, hp=hp32())
        run_iteration(eng2, view_hip, 0, g_raw, 8, hp=hp32())   # the adapter rounds to bf16 on upload
        assert max_rel(s2.grad_out[:N].cpu().numpy(), o_raw.grad_out) <= 1e-2


def test_tiny_config_full_comparison():
    """Config 1: R=4, 1,048,576 elements, M=8, replica 2 fails after its first microbatch of
    iteration 1, three iterations; the whole shard is compared."""
    from tests.configs import CONFIGS
    c = CONFIGS[1]
    N = c["off"][-1]
    o32, s, eng = make_pair(c["W"], c["G"], c["off"], False, seed=c["seed"])
    g = grads_np(c["seed"], N, c["scale"], False)
    for t in range(c["iters"]):
        before = state_of(s, N)
        kw = dict(dying=c["schedule"].get(t))
        a = run_iteration(o32, view_oracle, t, g, c["W"], hp=hp32(), **kw)
        b = run_iteration(eng, view_hip, t, g, c["W"], hp=hp32(), **kw)
        assert a["ids"] == b["ids"]
        if t == 1:
            assert a["ids"] == {0: [0, 4, 8], 1: [1, 5, 9], 3: [3, 7]}
        compare_iteration(o32, s, N, before)


def test_failure_run_equals_clean_replay_bit_for_bit():
    """Fixed-order mode: a run with failures, snapshots, in-place reductions and rewinds gives
    the same bits (gradient and AdamW state) as a failure-free run that accumulates the same
    ordered ids into the same replicas with the dead replicas absent from the start."""
    torch = torch_()
    N = OFF[-1]
    _, s, eng = make_pair(8, 4, OFF, False, seed=5)
    g = grads_np(5, N, 1e-3, False)
    run_iteration(eng, view_hip, 0, g, 8, hp=hp32())
    out = run_iteration(eng, view_hip, 1, g, 8, hp=hp32(), dying={3: 2, 6: 2}, fidelity_k=3, snapshot_every=True)
    _, s2, eng2 = make_pair(8, 4, OFF, False, seed=5)
    run_iteration(eng2, view_hip, 0, g, 8, hp=hp32())
    # replay: feed exactly the audited ids; replicas 3 and 6 never accumulate
    s2.on_failure([3, 6])
    s2.restore()
    for r, ids in out["ids"].items():
        for mb in ids:
            assert eng2.accumulate(r, mb, g(1, mb))
    s2.reduce()
    assert torch.equal(s.grad_out, s2.grad_out)
    s2.adamw_step(**hp32())
    s2.advance()
    for x, y in [(s.param, s2.param), (s.exp_avg, s2.exp_avg), (s.exp_avg_sq, s2.exp_avg_sq)]:
        assert torch.equal(x, y)


def test_restore_equals_never_accumulated():
    """Partial microbatch on the survivors at failure time, then rewind: buffers equal those of
    a run that never started that microbatch (bit-exact copies)."""
    torch = torch_()
    N = OFF[-1]
    g = grads_np(7, N, 1e-3, False)
    runs = []
    for partial in (True, False):
        o, s, eng = make_pair(4, 2, OFF, False, seed=7)
        for e, gg in ((o, g), (eng, g)):
            for r in range(4):
                e.accumulate(r, r, gg(0, r))
            e.snapshot(None)
            if partial:
                for r in (0, 1, 3):
                    e.accumulate(r, r + 4, gg(0, r + 4), 0, 6)
            e.on_failure([2])
            e.restore(None, stale_only=True)
        for r in (0, 1, 3):
            assert bits_equal(s.acc[r][:N].cpu().numpy(), o.acc[r])
        assert view_hip(s)["contributed"] == list(o.world.contributed)
        runs.append(s)
    for r in (0, 1, 3):
        assert torch.equal(runs[0].acc[r], runs[1].acc[r])


def test_negative_zero_and_stale_buffers():
    torch = torch_()
    s = B.Shard(1, 2, [0, 7])
    s.acc[0].fill_(123.0)
    g0 = torch.tensor([-0.0, 1.0, -2.0, 0.0, -0.0, 5.0, -0.0, 0.0], device="cuda")
    s.accumulate(0, 0, g0)
    got = s.acc[0][:7].cpu().numpy()
    assert np.array_equal(got, np.array([0, 1, -2, 0, 0, 5, 0], np.float32))
    assert list(np.signbit(got)) == [False, False, True, False, False, False, False]   # (+0) + (-0) = +0


def test_launch_shapes_do_not_change_the_bits():
    """Vectors per lane, resident wavefronts per CU, lanes per workgroup, cache hints and the contributor walk
    of every kernel class, and the contributor count up to which reduce+AdamW is one kernel (0: never, 2: for
    some tensors of the failure iteration, 64: always): the results are the same bits under all of them, through
    the separate and through the one-pass calls."""
    torch = torch_()
    N = OFF[-1]
    g = grads_np(11, N, 1e-3, False)
    ref = None
    keys = [B.TUNE_NONTEMPORAL, B.TUNE_THREADS, B.TUNE_ONE_PASS_MAX, B.TUNE_DEPTH + B.KERNEL_REDUCE,
            B.TUNE_DEPTH + B.KERNEL_REDUCE_ADAMW] + \
           [B.TUNE_VECS + k for k in range(B.KERNEL_CLASSES)] + [B.TUNE_WAVES + k for k in range(B.KERNEL_CLASSES)]
    defaults = {k: B.recover_get_tuning(k) for k in keys}
    assert all(code == 0 for code, _ in defaults.values())
    try:
        for U, waves in ((1, 0), (2, 8), (4, 2), (1, 32), (2, 13)):
            for nt, depth, T, one_pass in ((1, 1, 64, 0), (0, 2, 256, 64), (1, 2, 64, 2), (0, 1, 256, 32)):
                for key, val in ((B.TUNE_NONTEMPORAL, nt), (B.TUNE_THREADS, T), (B.TUNE_DEPTH + B.KERNEL_REDUCE, depth),
                                 (B.TUNE_DEPTH + B.KERNEL_REDUCE_ADAMW, depth), (B.TUNE_ONE_PASS_MAX, one_pass)):
                    assert B.recover_set_tuning(key, val) == 0
                for k in range(B.KERNEL_CLASSES):
                    assert B.recover_set_tuning(B.TUNE_VECS + k, U) == 0
                    assert B.recover_set_tuning(B.TUNE_WAVES + k, waves) == 0
                for fuse in (False, True):
                    _, s, eng = make_pair(4, 2, OFF, False, seed=11)
                    run_iteration(eng, view_hip, 0, g, 4, hp=hp32(), dying={1: 1}, fidelity_k=2, fuse=fuse,
                                  snapshot_every=fuse)
                    cur = [x.clone() for x in (s.grad_out, s.param, s.exp_avg, s.exp_avg_sq)]
                    if ref is None:
                        ref = cur
                    for x, y in zip(ref, cur):
                        assert torch.equal(x, y), (U, waves, nt, depth, T, one_pass, fuse)
    finally:
        for k, (_, v) in defaults.items():
            assert B.recover_set_tuning(k, v) == 0


def test_promoted_spare_and_inplace_sum_on_gpu():
    """Six replicas, one lost (boundary), then a major lost while a major-spare exists: the
    spare's buffer, overwritten by the in-place sum, is rewound and admitted."""
    N = OFF[-1]
    o32, s, eng = make_pair(6, 2, OFF, False, seed=13)
    g = grads_np(13, N, 1e-3, False)
    for t, kw in enumerate([dict(dying={5: 2}), dict(dying={1: 2}, fidelity_k=5), dict()]):
        before = state_of(s, N)
        a = run_iteration(o32, view_oracle, t, g, 6, hp=hp32(), **kw)
        b = run_iteration(eng, view_hip, t, g, 6, hp=hp32(), **kw)
        assert a["ids"] == b["ids"]
        if t == 1:
            assert not b["decisions"][0]["at_boundary"] and b["decisions"][0]["role"][4] == B.ROLE_MAJOR
        compare_iteration(o32, s, N, before)


def test_adaptive_policy_divides_by_the_committed_count():
    N = OFF[-1]
    o32, s, eng = make_pair(4, 2, OFF, False, seed=17, flags=B.FLAG_ADAPTIVE)
    g = grads_np(17, N, 1e-3, False)
    before = state_of(s, N)
    a = run_iteration(o32, view_oracle, 0, g, 4, hp=hp32(), dying={2: 1})
    b = run_iteration(eng, view_hip, 0, g, 4, hp=hp32(), dying={2: 1})
    assert a["ids"] == b["ids"] and sum(len(v) for v in b["ids"].values()) == 6
    compare_iteration(o32, s, N, before)


def test_nonblocking_restore_on_a_side_stream_is_ordered_by_the_library():
    """Sec. 4.2 non-blocking restoration: the rewind runs on a side stream, snapshots on another,
    while the main stream is held busy; the context orders its own calls with events, so the
    result equals the single-stream run bit for bit."""
    torch = torch_()
    off = [0, 3000001, 3000004, 8388611]
    N = off[-1]
    g = grads_np(19, N, 1e-3, False)

    class Streamed(HipEngine):
        def __init__(self, shard):
            super().__init__(shard)
            self.side, self.side2 = torch.cuda.Stream(), torch.cuda.Stream()

        def reduce(self, tb=0, te=None, inplace=False):
            if inplace:
                torch.cuda._sleep(100_000_000)              # hold the main stream: ~50 ms
            return self.s.reduce(tb, te, inplace)

        def restore(self, r=None, stale_only=True):
            with torch.cuda.stream(self.side):
                self.s.restore(r, stale_only)

        def snapshot(self, r=None, tb=0, te=None):
            with torch.cuda.stream(self.side2):
                self.s.snapshot(r, tb, te)

    results = []
    for cls in (HipEngine, Streamed):
        _, s, _ = make_pair(6, 2, off, False, seed=19)
        eng = cls(s)
        run_iteration(eng, view_hip, 0, g, 6, hp=hp32(), dying={5: 2}, fidelity_k=2)
        run_iteration(eng, view_hip, 1, g, 6, hp=hp32(), dying={1: 1}, fidelity_k=3, snapshot_every=True)
        torch.cuda.synchronize()
        results.append([x.clone() for x in (s.grad_out, s.param, s.exp_avg, s.exp_avg_sq)] + [a.clone() for a in s.acc])
    for x, y in zip(*results):
        assert torch.equal(x, y)


@pytest.mark.parametrize("bf16", [False, True])
def test_fused_calls_give_the_bits_of_the_separate_calls(bf16):
    """recover_accumulate_snapshot and recover_reduce_adamw_step against accumulate + snapshot and
    reduce + adamw_step: every buffer identical, through failures, rewinds and an extended pass;
    and the fused run against the oracle."""
    torch = torch_()
    N = OFF[-1]
    g = grads_np(23, N, 1e-3, bf16)
    o32, s_f, eng_f = make_pair(8, 2, OFF, bf16, seed=23)
    _, s_u, eng_u = make_pair(8, 2, OFF, bf16, seed=23)
    plan = [dict(), dict(dying={2: 1, 5: 0}, fidelity_k=3), dict(dying={0: 2}), dict()]
    for t, kw in enumerate(plan):
        before = state_of(s_f, N)
        a = run_iteration(o32, view_oracle, t, g, 8, hp=hp32(), snapshot_every=True, **kw)
        b = run_iteration(eng_f, view_hip, t, g, 8, hp=hp32(), snapshot_every=True, fuse=True, **kw)
        c = run_iteration(eng_u, view_hip, t, g, 8, hp=hp32(), snapshot_every=True, fuse=False, **kw)
        assert a["ids"] == b["ids"] == c["ids"]
        for x, y in [(s_f.grad_out, s_u.grad_out), (s_f.param, s_u.param), (s_f.exp_avg, s_u.exp_avg),
                     (s_f.exp_avg_sq, s_u.exp_avg_sq), (s_f.param_bf16, s_u.param_bf16)]:
            assert torch.equal(x, y)
        for r in b["ids"]:
            assert torch.equal(s_f.acc[r], s_u.acc[r]) and torch.equal(s_f.snap[r], s_u.snap[r])
        compare_iteration(o32, s_f, N, before)
    # without the flag the gradient buffer is left alone
    s_f.grad_out.fill_(7.0)
    for r in view_hip(s_f)["alive"]:
        while s_f.accumulate(r, 1000 + r + 8 * view_hip(s_f)["contributed"][r], torch.from_numpy(g(9, r)).cuda()
                             if not bf16 else torch.from_numpy(g(9, r)).cuda().bfloat16()):
            pass
    s_f.reduce_adamw_step(**hp32())
    assert float(s_f.grad_out.min()) == 7.0 == float(s_f.grad_out.max())


def test_accumulate_many_gives_the_bits_of_separate_calls():
    torch = torch_()
    N = OFF[-1]
    for bf16 in (False, True):
        g = grads_np(29, N, 1e-3, bf16)
        o32, s_b, eng_b = make_pair(8, 2, OFF, bf16, seed=29)
        _, s_u, eng_u = make_pair(8, 2, OFF, bf16, seed=29)
        for t, kw in enumerate([dict(), dict(dying={2: 1, 5: 0}, fidelity_k=3), dict()]):
            before = state_of(s_b, N)
            a = run_iteration(o32, view_oracle, t, g, 8, hp=hp32(), **kw)
            b = run_iteration(eng_b, view_hip, t, g, 8, hp=hp32(), batch=True, fuse=True, **kw)
            c = run_iteration(eng_u, view_hip, t, g, 8, hp=hp32(), **kw)
            assert a["ids"] == b["ids"] == c["ids"]
            for x, y in [(s_b.grad_out, s_u.grad_out), (s_b.param, s_u.param), (s_b.exp_avg_sq, s_u.exp_avg_sq)]:
                assert torch.equal(x, y)
            compare_iteration(o32, s_b, N, before)


def test_degenerate_shapes_and_special_values():
    """Empty shard, one replica, one microbatch; infinities, NaNs and subnormal numbers go through the
    adds and the divide as IEEE arithmetic says (the oracle is NumPy on the CPU)."""
    torch = torch_()
    # an empty shard: every call is a no-op that still keeps the books
    s = B.Shard(2, 1, [0, 0])
    z = torch.zeros(8, device="cuda")
    assert s.accumulate(0, 0, z) and s.accumulate(1, 1, z)
    s.snapshot()
    s.reduce()
    s.adamw_step(**hp32())
    s.advance()
    # W = 1, G = 1 with special values
    vals = np.array([np.inf, -np.inf, np.nan, 1e-40, -1e-45, 3e-39, 1.0, -0.0, 2e-38, 1.17549435e-38, 0.0, 5e-41, 7.0],
                    np.float32)
    off = [0, len(vals)]
    for W, G in ((1, 1), (2, 2), (3, 1)):
        o = Proto(W, G, off, dtype=np.float32)
        o.set_state(np.zeros(len(vals), np.float32))
        s = B.Shard(W, G, off)
        eng = HipEngine(s)
        with np.errstate(all="ignore"):
            for k in range(G):
                for r in range(W):
                    gk = (vals * np.float32(1 + r + k)).astype(np.float32)
                    o.accumulate(r, r + W * k, gk)
                    eng.accumulate(r, r + W * k, gk)
            o.reduce()
            s.reduce()
        got = s.grad_out[:len(vals)].cpu().numpy()
        assert np.array_equal(np.isnan(got), np.isnan(o.grad_out))
        ok = ~np.isnan(got)
        assert bits_equal(got[ok], o.grad_out[ok]), (W, G, got, o.grad_out)
        assert got[3] != 0 and got[4] != 0                      # subnormals are kept, not flushed
    # the bf16 copy of the parameters keeps a NaN a NaN whatever its payload (the rounding increment would
    # otherwise carry 0x7F800001 into Inf and 0x7FFFFFFF / 0xFFFFFFFF into zero)
    bits = np.array([0x7F800001, 0x7FFFFFFF, 0xFFFFFFFF, 0x7FC00000, 0x7F7FFFFF, 0x3F80FFFF, 0x7F800000, 0xFF800000],
                    np.uint32)
    s = B.Shard(1, 1, [0, len(bits)], param_bf16=True)
    s.param[:len(bits)].copy_(torch.from_numpy(bits.view(np.float32)))
    s.accumulate(0, 0, torch.zeros(8, device="cuda"))
    s.reduce()
    s.adamw_step(lr=0.0, beta1=0.0, beta2=0.0, eps=1.0, weight_decay=0.0)      # leaves finite parameters unchanged
    pb = s.param_bf16[:len(bits)].view(torch.int16).cpu().numpy().view(np.uint16)
    pf = s.param[:len(bits)].cpu().numpy()
    assert np.array_equal(pb, S.f32_to_bf16_bits(pf))
    back = S.bf16_bits_to_f32(pb)
    assert np.all(np.isnan(back[:4])) and np.isinf(back[4]) and back[5] == np.float32(1.0078125)
    assert back[6] == np.inf and back[7] == -np.inf


@pytest.mark.parametrize("random_streams", [False, True])
def test_random_call_sequences_agree_with_the_oracle_on_the_gpu(random_streams):
    """The differential test with real buffers: after random calls (partial tensor ranges, partial
    microbatches, snapshots, in-place reductions, failures, rewinds, steps, one-pass forms) the
    accumulators of every live replica, the snapshots, the gradient and the AdamW state equal the
    fp32 oracle's.  random_streams: every call goes to one of four streams picked at random; the
    context's event ordering must make that invisible."""
    torch = torch_()
    import random
    from tests import differential
    off = [0, 3, 8, 8, 4107, 4200]
    N = off[-1]
    total = {"ok": 0, "err": 0, "steps": 0, "failures": 0}
    streams = [torch.cuda.Stream() for _ in range(3)] + [torch.cuda.default_stream()]
    for seed in range(8):
        W, G = [(4, 2), (8, 1), (3, 3), (6, 2)][seed % 4]
        s = B.Shard(W, G, off)
        eng = HipEngine(s)
        if random_streams:
            rs = random.Random(seed)

            def on_random_stream(f):
                def g(*a, **k):
                    with torch.cuda.stream(rs.choice(streams)):
                        return f(*a, **k)
                return g
            for name in ("accumulate", "accumulate_many"):
                setattr(eng, name, on_random_stream(getattr(eng, name)))
            for name in ("snapshot", "restore", "reduce", "adamw_step", "reduce_adamw_step"):
                setattr(eng, name, on_random_stream(getattr(s, name)))
        pool = [S.fill(N, 31 + seed, S.TAG_GRAD, j, 0, 1e-3) for j in range(16)]

        def compare(o, lib, where):
            torch.cuda.synchronize()
            for r in o.world.alive():
                a = s.acc[r][:N].cpu().numpy()
                sn = s.snap[r][:N].cpu().numpy()
                for b in range(len(off) - 1):
                    lo, hi = off[b], off[b + 1]
                    if o.cnt[r][b] > 0 or o.inplace_sum[r][b]:
                        assert bits_equal(a[lo:hi], o.acc[r][lo:hi]), (where, "acc", r, b)
                    if o.snap_valid[r][b] and o.snap_cnt[r][b] > 0:
                        assert bits_equal(sn[lo:hi], o.snap[r][lo:hi]), (where, "snap", r, b)
            g = s.grad_out[:N].cpu().numpy()
            for b in range(len(off) - 1):
                if o.red_eps[b] >= 0:
                    assert bits_equal(g[off[b]:off[b + 1]], o.grad_out[off[b]:off[b + 1]]), (where, "grad", b)
            if o.t > 0:
                assert max_rel(s.exp_avg[:N].cpu().numpy(), o.m) <= 1e-6, where
                assert max_rel(s.exp_avg_sq[:N].cpu().numpy(), o.v) <= 1e-6, where

        st = differential.run(100 + seed, 250, W, G, off, eng, grads=lambda i: pool[i % 16], compare_buffers=compare)
        for k in total:
            total[k] += st[k]
        s.close()
    assert total["steps"] > 20 and total["failures"] > 5, total


def test_bucketed_arrival_in_reverse_order_with_failure_during_the_bucket_loop():
    """The paper's bucket loop (Alg. 1; walk-through appendix): gradients arrive bucket by
    bucket in reverse order, each bucket is snapshotted and all-reduced in place as soon as the last
    microbatch has produced it; a replica fails after some buckets were reduced.  300 tensors of
    0..40 elements in 13 buckets: every bucket boundary is ragged."""
    rng = np.random.default_rng(3)
    off = [0] + [int(x) for x in np.cumsum(rng.integers(0, 41, 300))]
    N, T = off[-1], 300
    cuts = sorted(set([0, T] + [int(x) for x in rng.integers(1, T, 12)]))
    buckets = list(zip(cuts[:-1], cuts[1:]))[::-1]
    W, G = 4, 2
    o, s, eng = make_pair(W, G, off, False, seed=37)
    g = grads_np(37, N, 1e-3, False)
    before = state_of(s, N)
    for e in (o, eng):
        def feed(r):
            k = (view_oracle(e) if e is o else view_hip(s))["contributed"][r]
            mb = r + W * k
            for tb, te in buckets:
                e.accumulate(r, mb, g(0, mb), tb, te)
        for k in range(G):
            for r in range(W):
                if not (r == 2 and k == 1):                  # replica 2 crashes after one microbatch
                    feed(r)
        for tb, te in buckets[:5]:                           # five buckets go through before the failure shows
            e.snapshot(None, tb, te)
            e.reduce(tb, te, inplace=True)
        d = e.on_failure([2])
        assert d["at_boundary"] and d["G_ext"] == 1 and d["n_bdry"] == 1
        e.restore(None, stale_only=True)
        for r in (0, 1):                                     # the extended pass (replica 3 is the boundary minor)
            feed(r)
        for tb, te in buckets:
            e.snapshot(None, tb, te)
            e.reduce(tb, te, inplace=True)
        e.adamw_step(**hp32())
        e.advance()
    compare_iteration(o, s, N, before)
    assert view_hip(s)["target"] == list(o.world.target)


def test_device_compare_matches_numpy():
    torch = torch_()
    rng = np.random.default_rng(41)
    for n in (0, 1, 63, 64, 1000003):
        x = rng.normal(0, 1, max(n, 1)).astype(np.float32)[:n]
        y = x.copy()
        if n > 10:
            y[[3, n // 2, n - 1]] += np.float32(0.5)
            y[7] = np.nan
            x[9] = -0.0
            y[9] = 0.0                                            # equal as numbers, different bits
            x[11] = y[11] = np.inf                                # equal infinities differ by nothing
            x[12] = y[12] = -np.inf
        got = B.compare_tensors(torch.from_numpy(np.append(x, 0).astype(np.float32)).cuda(),
                                torch.from_numpy(np.append(y, 0).astype(np.float32)).cuda(), n)
        xb, yb = x.view(np.uint32).astype(np.uint64), y.view(np.uint32).astype(np.uint64)
        w = 2 * np.arange(n, dtype=np.uint64) + np.uint64(1)
        assert got["n_mismatch"] == int(np.sum(xb != yb))
        assert got["n_nan"] == int(np.sum(np.isnan(x) | np.isnan(y)))
        assert got["checksum_x"] == int(np.sum(xb * w, dtype=np.uint64))
        assert got["checksum_ref"] == int(np.sum(yb * w, dtype=np.uint64))
        ok = ~(np.isnan(x) | np.isnan(y))
        with np.errstate(invalid="ignore"):
            d = np.where(xb == yb, np.float32(0), np.abs(x - y))
        assert got["max_abs_diff"] == (np.max(d[ok]) if ok.any() else 0.0)
        assert got["max_abs_ref"] == (np.max(np.abs(y[ok])) if ok.any() else 0.0)
    # opposite infinities are infinitely far apart, and a NaN payload survives the bf16 rounding of the parameters
    a = torch.tensor([np.inf, 1.0, 2.0, 3.0, 4.0], device="cuda")
    b = torch.tensor([-np.inf, 1.0, 2.0, 3.0, 4.0], device="cuda")
    got = B.compare_tensors(a, b, 5)
    assert got["max_abs_diff"] == np.inf and got["n_mismatch"] == 1 and got["n_nan"] == 0


def test_device_step_state_gives_the_same_bits_as_host_constants():
    torch = torch_()
    N = OFF[-1]
    g = grads_np(43, N, 1e-3, False)
    res = []
    for dev in (False, True):
        p0 = S.fill(N, 43, S.TAG_PARAM, 0, 0, 0.02)
        s = B.Shard(4, 2, OFF, device_step=dev)
        s.param[:N].copy_(torch.from_numpy(p0))
        eng = HipEngine(s)
        for t in range(4):
            run_iteration(eng, view_hip, t, g, 4, hp=hp32(), fuse=bool(t % 2))
        res.append([x.clone() for x in (s.param, s.exp_avg, s.exp_avg_sq)])
        if dev:
            st = s.step_state.cpu().numpy()
            assert st[0] == 4                                            # four steps counted on the device
            assert abs(st[1:3].view(np.float64)[0] - 0.9 ** 4) < 1e-7    # running product of beta1 (as fp32 0.9)
    for x, y in zip(*res):
        assert torch.equal(x, y)


def test_hip_graph_replay_of_a_whole_iteration():
    """A launch-bound shard: one iteration (accumulate_many per microbatch slot, snapshot, one-pass
    reduce+AdamW) captured into a HIP graph and replayed with new gradient contents, with eager work of
    a twin context and synchronisation between the replays; every replay equals the eager twin."""
    torch = torch_()
    off = [0, 1000, 4099, 4100]
    N, W, G = off[-1], 4, 2
    p0 = S.fill(N, 47, S.TAG_PARAM, 0, 0, 0.02)
    twins = []
    for dev in (True, False):
        s = B.Shard(W, G, off, device_step=dev)
        s.param[:N].copy_(torch.from_numpy(p0))
        twins.append(s)
    s_graph, s_eager = twins
    bufs = [[torch.zeros(N + 4, device="cuda") for _ in range(W)] for _ in range(G)]

    def iteration(s):
        for k in range(G):
            s.accumulate_many(list(range(W)), [r + W * k for r in range(W)], bufs[k])
        s.snapshot()
        s.reduce_adamw_step(write_grad=True, **hp32())
        s.advance()

    def load(t):
        for k in range(G):
            for r in range(W):
                bufs[k][r][:N].copy_(torch.from_numpy(S.fill(N, 47, S.TAG_GRAD, r + W * k, t, 1e-3)))

    load(0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        iteration(s_graph)
    for t in range(5):
        load(t)
        graph.replay()
        iteration(s_eager)
        torch.cuda.synchronize()
        for x, y in ((s_graph.grad_out, s_eager.grad_out), (s_graph.param, s_eager.param),
                     (s_graph.exp_avg, s_eager.exp_avg), (s_graph.exp_avg_sq, s_eager.exp_avg_sq)):
            assert torch.equal(x, y), t
    assert int(s_graph.step_state.cpu()[0]) == 5
    # the context is still usable eagerly after the capture (its books are at an iteration start)
    load(5)
    iteration(s_graph)
    iteration(s_eager)
    torch.cuda.synchronize()
    assert torch.equal(s_graph.param, s_eager.param)


def test_failure_reported_between_iterations_case_b():
    """Failure after a complete synchronisation (Sec. 4.2 case (b)): the step commits with the lost
    replica's gradients, the failure is declared before the next iteration's first microbatch."""
    N = OFF[-1]
    o, s, eng = make_pair(4, 2, OFF, False, seed=53)
    g = grads_np(53, N, 1e-3, False)
    for t in range(2):
        before = state_of(s, N)
        a = run_iteration(o, view_oracle, t, g, 4, hp=hp32())
        b = run_iteration(eng, view_hip, t, g, 4, hp=hp32())
        assert a["ids"] == b["ids"]
        compare_iteration(o, s, N, before)
        if t == 0:
            assert sorted(sum(b["ids"].values(), [])) == list(range(8))
            da, db = o.on_failure([2]), eng.on_failure([2])
            for k in da:
                assert da[k] == db[k], k
            o.restore(None)
            eng.restore(None)
    assert b["ids"] == {0: [0, 4, 8], 1: [1, 5, 9], 3: [3, 7]}


def test_cpp_program_on_the_c_abi_without_python():
    """The prebuilt C++ example (hipMalloc'd buffers, no PyTorch): two iterations with a failure,
    checked inside the program against the constant-gradient closed form."""
    import os
    import subprocess
    from paper_2605_11215_amd import build
    assert os.path.exists(build.EXAMPLE), "run python -m paper_2605_11215_amd.build first"
    r = subprocess.run([build.EXAMPLE], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("ok"), (r.returncode, r.stdout, r.stderr)
