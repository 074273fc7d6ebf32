"""Workload table for the tests: the package's five configs plus the failure schedule of
config 5, which is drawn from the seeded schedule stream and needs the quotas in force."""
from paper_2605_11215_amd.synth import reference_np as S
from paper_2605_11215_amd.workloads import CONFIGS  # noqa: F401


def schedule_seed7(W_init, G_init, iters):
    """Config 5: one failure per iteration while more than one replica survives; replica and
    offset drawn from the schedule stream (seed 7)."""
    import oracle.policy as OP          # integer bookkeeping only, to know who is alive and the quotas
    w = OP.World(W_init, G_init)
    sched = {}
    for t in range(iters):
        alive = w.alive()
        if len(alive) > 1:
            x = S.schedule_words(7, t)
            r = alive[x[0] % len(alive)]
            n = x[1] % (w.target[r] + 1)
            sched[t] = {r: n}
            for q in alive:
                w.contributed[q] = w.target[q]
            d = w.on_failure([r])
            for q in w.alive():
                w.contributed[q] = w.target[q]
        w.commit()
        w.advance()
    return sched


def schedule_of(cfg):
    if cfg["schedule"] is None:
        return schedule_seed7(cfg["W"], cfg["G"], cfg["iters"])
    return cfg["schedule"]


