"""Random call sequences applied to the CPU oracle and to the HIP library side by side.  Every call
must succeed or fail on both, return the same value, and leave the same bookkeeping; on a GPU the
buffers are compared too.  Used by test_abi.py (host-only contexts, CPU) and test_gpu_parity.py."""
import numpy as np

from oracle.policy import NoSurvivor
from oracle.proto import Proto, ProtocolError
from paper_2605_11215_amd import binding as B
from tests.driver import HP, view_oracle

HP32 = {k: float(np.float32(v)) for k, v in HP.items()}


def call(fn, *a, **k):
    try:
        return ("ok", fn(*a, **k))
    except (ProtocolError, NoSurvivor, AssertionError, B.RecoverError):
        return ("err", None)


def view_lib(s):
    q = s.query()
    return dict(alive=[r for r in range(s.W) if q["role"][r] != B.ROLE_DEAD], target=q["target"],
                contributed=q["contributed"], loop_bound=q["loop_bound"], role=q["role"], epoch=q["epoch"])


def sensible_next(o, rng):
    """The call a well-behaved training loop would make next, from the oracle's state."""
    w = o.world
    if w.pending_advance:
        return "advance"
    if o.quiesced or any(o.inplace_sum[r][b] for r in w.alive() for b in range(o.T)
                         if w.contributed[r] < w.target[r]):
        return "restore"
    todo = [r for r in w.alive() if w.contributed[r] < w.target[r]]
    if todo:
        return "acc"
    if not o.ready_to_commit():
        return "snap" if rng.random() < 0.3 else "reduce"
    return "step"


def run(seed, n_ops, W, G, off, lib_engine, grads=None, compare_buffers=None, adaptive=False,
        grad_of_id=None, oracle_dtype=np.float32, before_commit=None):
    """lib_engine: object with Shard's methods (accumulate takes the NumPy gradient or None).
    grads(i) -> float32 array for the i-th accumulate, or None on host-only contexts;
    grad_of_id(mb) -> the gradient of microbatch mb (then used instead of grads);
    before_commit(o) is called when a step is about to succeed (the reduction is complete)."""
    rng = np.random.default_rng(seed)
    T = len(off) - 1
    o = Proto(W, G, off, dtype=oracle_dtype, static=not adaptive)
    o.set_state(np.zeros(off[-1], np.float32))
    zero = np.zeros(off[-1], np.float32)
    stats = {"ok": 0, "err": 0, "steps": 0, "failures": 0}
    n_acc = 0
    kinds = ["acc", "snap", "restore", "reduce", "fail", "step", "advance", "bad"]
    one_pass = hasattr(lib_engine, "reduce_adamw_step")      # also exercise the one-pass forms of the library
    for i in range(n_ops):
        w = o.world
        alive = w.alive()
        if rng.random() < 0.75:
            kind = sensible_next(o, rng)
        else:
            kind = str(rng.choice(kinds, p=[0.3, 0.15, 0.1, 0.15, 0.08, 0.1, 0.05, 0.07]))
        r = int(rng.choice(alive)) if rng.random() < 0.95 else int(rng.integers(0, W))
        tb = int(rng.integers(0, T + 1))
        te = int(rng.integers(tb, T + 1))
        if rng.random() < 0.6:
            tb, te = 0, T
        if kind == "acc" and one_pass and not w.pending_advance and rng.random() < 0.12:
            # one accumulate_many call against separate accumulates (only pairs the oracle will accept)
            free = [q for q in alive if o.cur_id[q] is None and not any(o.inplace_sum[q])]
            if len(free) >= 2:
                pick = [int(x) for x in rng.choice(free, size=int(rng.integers(2, len(free) + 1)), replace=False)]
                ids = [(o.ids[q][-1] + W) if o.ids[q] else q for q in pick]
                gs = [grad_of_id(mb) if grad_of_id else (grads(n_acc + j) if grads else None)
                      for j, mb in enumerate(ids)]
                n_acc += len(pick)
                ra = [o.accumulate(q, mb, zero if g is None else g) for q, mb, g in zip(pick, ids, gs)]
                rb = lib_engine.accumulate_many(pick, ids, gs if grads else None) if any(ra) else None
                if rb is None:                               # every pair skipped: the library says SKIPPED
                    code, _ = B.recover_accumulate_many(lib_engine.ctx, pick, ids, [0] * len(pick), B.F32) \
                        if not grads else (B.SKIPPED, None)
                    assert code == B.SKIPPED
                    rb = [False] * len(pick)
                assert [bool(x) for x in ra] == [bool(x) for x in rb], (seed, i, "many", ra, rb)
                a = b = ("ok", None)
                kind = "many"
        if kind == "many":
            pass
        elif kind == "acc":
            todo = [q for q in alive if w.contributed[q] < w.target[q]]
            if todo and rng.random() < 0.9:
                r = int(rng.choice(todo))
            if o.cur_id[r] is not None and rng.random() < 0.9:        # finish the open microbatch
                mb = o.cur_id[r]
                missing = [b for b in range(T) if o.cnt[r][b] == w.contributed[r]]
                if missing and rng.random() < 0.8:
                    tb, te = missing[0], missing[-1] + 1 if rng.random() < 0.7 else missing[0] + 1
            else:
                mb = (o.ids[r][-1] + W) if o.ids[r] else r
                if rng.random() < 0.04:
                    mb = max(0, mb - W)
            g = grad_of_id(mb) if grad_of_id else (grads(n_acc) if grads else None)
            n_acc += 1
            a = call(o.accumulate, r, mb, zero if g is None else g, tb, te)
            if one_pass and rng.random() < 0.15:             # accumulate+snapshot in one pass
                b = call(lib_engine.accumulate, r, mb, g, tb, te, snapshot=True)
                if a[0] == "ok" and a[1]:
                    o.snapshot(r, tb, te)
            else:
                b = call(lib_engine.accumulate, r, mb, g, tb, te)
        elif kind == "snap":
            rr = None if rng.random() < 0.5 else r
            a, b = call(o.snapshot, rr, tb, te), call(lib_engine.snapshot, rr, tb, te)
        elif kind == "restore":
            rr = None if rng.random() < 0.7 else r
            so = bool(rng.random() < 0.7)
            a, b = call(o.restore, rr, so), call(lib_engine.restore, rr, so)
            a = (a[0], None)
        elif kind == "reduce":
            covered = all(o.snap_valid[q][b_] and o.snap_cnt[q][b_] == o.cnt[q][b_]
                          for q in alive for b_ in range(tb, te))
            inplace = bool(rng.random() < 0.25) and (covered or rng.random() < 0.05)
            a, b = call(o.reduce, tb, te, inplace), call(lib_engine.reduce, tb, te, inplace)
        elif kind == "fail":
            k = int(rng.integers(1, 3))
            failed = [int(x) for x in rng.choice(W, size=min(k, W), replace=False)]
            if len(alive) <= 2 and rng.random() < 0.8:
                failed = [W + 1]                                      # keep the world alive a little longer
            a, b = call(o.on_failure, failed), call(lib_engine.on_failure, failed)
            if a[0] == "ok" and b[0] == "ok":
                stats["failures"] += 1
                for key in a[1]:
                    assert a[1][key] == b[1][key], (seed, i, key)
                a = b = ("ok", None)
        elif kind == "step" and one_pass and rng.random() < 0.4 and not o.quiesced and not w.pending_advance \
                and all(w.contributed[q] == w.target[q] for q in w.contributors()) \
                and not any(o.inplace_sum[q][b_] for q in alive for b_ in range(T)) \
                and all(o.cur_id[q] is None for q in w.contributors()):
            # reduce + AdamW in one pass against the two calls (a state in which both succeed)
            o.reduce()
            if before_commit and o.ready_to_commit():
                before_commit(o)
            a, b = call(o.adamw_step, **HP32), call(lib_engine.reduce_adamw_step, write_grad=True, **HP32)
            if a[0] == "ok":
                stats["steps"] += 1
        elif kind == "step":
            if before_commit and o.ready_to_commit():
                before_commit(o)
            a, b = call(o.adamw_step, **HP32), call(lib_engine.adamw_step, **HP32)
            if a[0] == "ok":
                stats["steps"] += 1
        elif kind == "advance":
            a, b = call(o.advance), call(lib_engine.advance)
            if a[0] == "ok" and b[0] == "ok":
                for key in a[1]:
                    assert a[1][key] == b[1][key], (seed, i, key)
                a = b = ("ok", None)
        else:                                                        # malformed calls
            a = ("err", None)
            which = int(rng.integers(0, 4))
            if which == 0:
                b = call(lib_engine.accumulate, W + 3, 0, grads(0) if grads else None, 0, T)
            elif which == 1:
                b = call(lib_engine.reduce, T, T + 2, False)
            elif which == 2:
                b = call(lib_engine.snapshot, -5, 0, T)
            else:
                b = call(lib_engine.on_failure, [W])
        assert a[0] == b[0], (seed, i, kind, a, b, B.recover_last_error(getattr(lib_engine, "ctx", None)))
        if a[0] == "ok" and kind in ("acc", "reduce"):
            assert bool(a[1]) == bool(b[1]), (seed, i, kind, a, b)
        stats[a[0]] += 1
        va, vb = view_oracle(o), view_lib(lib_engine)
        assert va == vb, (seed, i, kind, va, vb)
        assert o.committed_ids_by_replica() == lib_engine.committed_ids_by_replica(), (seed, i, kind)
        if compare_buffers and (i % 7 == 0 or i == n_ops - 1):
            compare_buffers(o, lib_engine, (seed, i, kind))
    return stats
