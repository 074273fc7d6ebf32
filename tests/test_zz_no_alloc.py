"""The optimiser step for callers that cannot allocate device memory: recover_adamw_step_static keeps the
device-resident step state in a slot of the library's own device array.  Checked against
recover_adamw_step on a context whose step state is a caller buffer: same bits in param, exp_avg,
exp_avg_sq (and the bf16 copy), on two runs in a row, the second on a smaller shard, each over several
steps; then slots do not leak into each other and a restart begins at step 1 again."""
import numpy as np
import pytest

from paper_2605_11215_amd import binding as B
from paper_2605_11215_amd.synth import reference_np as S

pytestmark = pytest.mark.gpu
HP = (1e-3, 0.9, 0.95, 1e-8, 0.1)


def one_iteration(s, t, grads, step):
    """W x G accumulates and a reduce, then `step(ctx, stream)`, then the advancement no-op."""
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    for k in range(s.G):
        for r in range(s.W):
            assert s.accumulate(r, r + s.W * k, grads[(t * 7 + k * s.W + r) % len(grads)])
    s.reduce()
    assert step(s.ctx, stream) == B.OK, B.recover_last_error(s.ctx)
    s.advance()


def run_pair(off, slot, steps, seed):
    import torch
    N = off[-1]
    grads = [torch.from_numpy(S.fill(max(N, 8), seed, S.TAG_GRAD, j, 0, 1e-3)).cuda() for j in range(5)]
    p0 = torch.from_numpy(S.fill(max(N, 8), seed, S.TAG_PARAM, 0, 0, 0.02)).cuda()
    ref = B.Shard(3, 2, off, snapshots=False, param_bf16=True, device_step=True)      # caller-owned step state
    new = B.Shard(3, 2, off, snapshots=False, param_bf16=True)                          # library-owned slot
    for s in (ref, new):
        s.param[:N].copy_(p0[:N])
    for t in range(steps):
        one_iteration(ref, t, grads, lambda ctx, st: B.recover_adamw_step(ctx, *HP, st))
        one_iteration(new, t, grads, lambda ctx, st: B.recover_adamw_step_static(ctx, slot, t == 0, *HP, st))
        for a, b in ((ref.param, new.param), (ref.exp_avg, new.exp_avg), (ref.exp_avg_sq, new.exp_avg_sq)):
            assert torch.equal(a[:N].view(torch.int32), b[:N].view(torch.int32)), (N, t)
        assert torch.equal(ref.param_bf16[:N].view(torch.int16), new.param_bf16[:N].view(torch.int16))
        assert float(new.exp_avg_sq[:N].max()) > 0
    return ref, new, grads


def test_static_step_state_matches_the_caller_owned_one_on_two_runs_the_second_smaller():
    import torch
    big = [0, 3, 1000, 70001]                        # ragged: several tiles and a scalar tail
    small = [0, 5, 1031]
    r1, n1, _ = run_pair(big, 5, 3, seed=41)
    r2, n2, g2 = run_pair(small, 5, 3, seed=42)      # same slot again: the restart clears what the first run left
    # another slot is untouched by all of that: its first step without a restart is step 1 of a zeroed state ...
    n3 = B.Shard(3, 2, small, snapshots=False, param_bf16=True)
    r3 = B.Shard(3, 2, small, snapshots=False, param_bf16=True, device_step=True)
    for s in (n3, r3):
        s.param[:1031].copy_(n2.param[:1031])
    one_iteration(r3, 0, g2, lambda ctx, st: B.recover_adamw_step(ctx, *HP, st))
    one_iteration(n3, 0, g2, lambda ctx, st: B.recover_adamw_step_static(ctx, 6, 1, *HP, st))
    assert torch.equal(r3.param[:1031].view(torch.int32), n3.param[:1031].view(torch.int32))
    # ... and slot 5 goes on counting where the second run left it (step 4), whichever context calls
    one_iteration(r2, 3, g2, lambda ctx, st: B.recover_adamw_step(ctx, *HP, st))
    one_iteration(n2, 3, g2, lambda ctx, st: B.recover_adamw_step_static(ctx, 5, 0, *HP, st))
    assert torch.equal(r2.param[:1031].view(torch.int32), n2.param[:1031].view(torch.int32))
    # errors: slot outside the array, context with a step state of its own
    assert B.recover_adamw_step_static(n2.ctx, B.STATIC_STEP_SLOTS, 0, *HP) == B.ERR_ARG
    assert "64 step states" in B.recover_last_error(n2.ctx)
    assert B.recover_adamw_step_static(n2.ctx, -1, 0, *HP) == B.ERR_ARG
    assert B.recover_adamw_step_static(r2.ctx, 0, 0, *HP) == B.ERR_STATE
    for s in (r1, n1, r2, n2, r3, n3):
        s.close()
