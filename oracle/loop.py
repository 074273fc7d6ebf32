"""Oracle: one iteration of the protocol (Alg. 1) driven on a `Proto` (test infrastructure only).

This is the oracle's own statement of the iteration loop, written from Alg. 1 and the boundary-step
walk-through appendix; it imports nothing from the HIP library's package.  The forward/backward pass
is replaced by a gradient source `grad_of(t, id)`; failures are injected by the caller, as the paper's
failure simulator does (implementation appendix): a replica crashes at a microbatch boundary and the
survivors learn of it at the synchronisation point, where the guarded all-reduce reports it
(Sec. 3, iteration anatomy; Sec. 4.2 cases (a)-(c)).

Microbatch ids.  The data stream is partitioned across replicas (Sec. 4.3 (ii), proof-sketch
appendix): replica r's k-th microbatch of an iteration is item r + W_init * k of that iteration's
stream, so survivors that take extra microbatches advance through their own slices and the slices
of failed replicas drop out.
"""

HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def run_iteration(p, t, grad_of, dying=None, reduced_before_failure=0, snapshot_every=False, hp=HP):
    """Alg. 1 on the Proto `p` for iteration t.

    dying                   {replica: n}: the replica crashes once it has accumulated n microbatches
    reduced_before_failure  k > 0: the failure shows during synchronisation, after the first k buckets
                            were snapshotted and all-reduced in place under the old membership
                            (Sec. 4.2 case (c)); 0: it shows before any bucket is reduced (case (a))
    snapshot_every          also snapshot every live replica after every microbatch slot
    Returns dict(decisions=[failure records..., advancement], ids={replica: [ids]}).
    """
    w = p.world
    W_init = w.W_init
    pending = dict(dying or {})        # crashes the survivors have not learnt of yet
    gone = set()                       # crashed processes: their buffers no longer move
    decisions = []
    m = 0                              # Alg. 1: microbatch index
    while m < w.loop_bound:            # while m < P(major)
        m += 1
        for r in w.alive():
            if r in pending and w.contributed[r] >= pending[r]:
                gone.add(r)
            if r in gone:
                continue
            if w.contributed[r] < w.target[r]:             # m <= P(rho): accumulate; else the gradient is dropped
                mb = r + W_init * w.contributed[r]
                p.accumulate(r, mb, grad_of(t, mb))
        if snapshot_every:
            for r in w.alive():
                if r not in gone:
                    p.snapshot(r)
        if m < w.loop_bound:
            continue
        # m = P(major): synchronisation
        if pending:
            if reduced_before_failure:
                k = reduced_before_failure
                p.snapshot(None, 0, k)                     # S(b) <- b, eps(b) <- eps_cur for the buckets already produced
                p.reduce(0, k, inplace=True)               # ... and all-reduced before the failure shows
            d = p.on_failure(sorted(pending))              # the guarded collective reports the failure:
            decisions.append(d)                            # handle_work_failure + policy_adjustment
            pending, gone = {}, set()
            p.restore(None, stale_only=True)               # gradient_restoration
            if m < w.loop_bound:                           # P(major) grew: the while loop goes on (extended pass)
                continue
        p.snapshot(None)                                   # every bucket: snapshot, tag, all-reduce
        p.reduce()
    ids = p.committed_ids_by_replica()
    p.adamw_step(**hp)                                     # divide by B (inside reduce), optimiser step
    decisions.append(p.advance())                          # policy_advancement if a boundary was crossed
    return dict(decisions=decisions, ids=ids)
