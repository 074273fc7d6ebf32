"""The caller's side of Alg. 1 for the HIP library: the microbatch loop of a training step with the
forward/backward pass replaced by a gradient source.  It drives a `binding.Shard` (or any object
with its method names) through whole iterations and stands in for the training loop: it decides
nothing the method decides; quotas, roles, loop bound and restore mode are read back from the
context after every call.  The benchmark's failure iteration and the attrition report use it.

Microbatch ids: replica r's k-th microbatch of an iteration has global id r + W_init * k
(each replica advances through its own slice of the stream; a failed replica's slice drops
out), so a failure-free iteration commits ids 0 .. B-1 and extra microbatches get ids >= B.
"""

HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def view_shard(s):
    """State view of a binding.Shard."""
    q = s.query()
    return dict(alive=[r for r in range(s.W) if q["role"][r] != 4], target=q["target"],
                contributed=q["contributed"], loop_bound=q["loop_bound"], role=q["role"], epoch=q["epoch"])


def run_iteration(eng, view, t, grad_of, W_init, dying=None, fidelity_k=0,
                  snapshot_every=False, hp=HP, on_sync=None, fuse=False, batch=False):
    """One iteration of Alg. 1.

    dying        {replica: n}: the replica crashes having accumulated n microbatches; the
                 survivors learn of it at the synchronisation point (Sec. 3, iteration anatomy)
    fidelity_k   > 0: before the failure is detected, the first k tensors are snapshotted
                 and all-reduced in place under the old membership (failure case (c), Sec. 4.2)
    fuse         use the engine's one-pass calls where it has them: accumulate+snapshot for
                 snapshot_every, reduce+AdamW for the commit (same results as the separate calls)
    batch        one accumulate_many call per microbatch slot instead of one accumulate per replica
    Returns dict(decisions=[...], ids={replica: [ids]}).
    """
    fuse = fuse and hasattr(eng, "reduce_adamw_step")
    batch = batch and hasattr(eng, "accumulate_many") and not (fuse and snapshot_every)
    dying = dict(dying or {})
    crashed = set()
    decisions = []
    m = 0
    while True:
        while m < view(eng)["loop_bound"]:
            m += 1
            v = view(eng)
            pairs = []
            for r in v["alive"]:
                if r in dying and v["contributed"][r] >= dying[r]:
                    crashed.add(r)
                if r in crashed:
                    continue
                if v["contributed"][r] < v["target"][r]:
                    mb = r + W_init * v["contributed"][r]
                    if batch:
                        pairs.append((r, mb, grad_of(t, mb)))
                    elif fuse and snapshot_every:
                        eng.accumulate(r, mb, grad_of(t, mb), snapshot=True)
                    else:
                        eng.accumulate(r, mb, grad_of(t, mb))
            if pairs:
                eng.accumulate_many([p[0] for p in pairs], [p[1] for p in pairs], [p[2] for p in pairs])
            if snapshot_every and not fuse:
                for r in view(eng)["alive"]:
                    if r not in crashed:
                        eng.snapshot(r)
        if dying:
            if fidelity_k:
                eng.snapshot(None, 0, fidelity_k)
                eng.reduce(0, fidelity_k, inplace=True)
            d = eng.on_failure(sorted(dying))
            decisions.append(d)
            dying, crashed = {}, set()
            eng.restore(None, stale_only=True)
            if d["at_boundary"]:
                continue                               # extended pass (Alg. 1 outer while)
        eng.snapshot(None)
        if on_sync:
            on_sync(eng)
        if not fuse:
            eng.reduce()
        break
    ids = eng_committed_ids(eng)
    if fuse:
        eng.reduce_adamw_step(write_grad=True, **hp)
    else:
        eng.adamw_step(**hp)
    decisions.append(eng.advance())
    return dict(decisions=decisions, ids=ids)


def eng_committed_ids(eng):
    return eng.committed_ids_by_replica()
