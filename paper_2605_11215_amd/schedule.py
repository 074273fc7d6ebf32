"""Deterministic failure schedules in the form of the paper's failure simulator (implementation
appendix, "Failure simulator"): a list of (step, replica id, local rank, location) entries that
is a pure function of (parallelism spec, seed, count, step range, location weights), so every
rank can generate the same schedule without a broadcast, and that can be written to and read
from YAML.

Locations (points of the microbatch loop at which a rank checks its schedule):
  "mb:<k>"    the replica crashes at the microbatch boundary after k microbatches of the step
              (k is clamped to the replica's quota when the schedule is consumed)
  "sync:<p>"  the replica crashes during gradient synchronisation, after p percent of the
              buckets have been all-reduced under the old membership (failure case (c), Sec. 4.2)

This module only decides WHEN WHO fails; it holds none of the method's arithmetic.  Random
words come from the seeded schedule stream of paper_2605_11215_amd.synth (Philox4x32-10,
key (seed, TAG_SCHEDULE), counter (entry index, 0, 0, 0)).
"""
import math

from .synth import reference_np as S


def generate(n_replicas, ranks_per_replica, seed, count, step_range, location_weights=None, max_microbatch=8):
    """`count` entries, sorted by step.  step_range = (first, last) inclusive; location_weights =
    {"mb": w1, "sync": w2} (default all "sync", the paper's hardest setting)."""
    lo, hi = step_range
    assert hi >= lo and count >= 0 and n_replicas >= 1 and ranks_per_replica >= 1
    w = dict(location_weights or {"sync": 1.0})
    total = float(sum(w.values()))
    p_mb = float(w.get("mb", 0.0)) / total
    out = []
    for i in range(count):
        x = S.schedule_words(seed, i)
        gpu = x[1] % (n_replicas * ranks_per_replica)            # a uniformly chosen device
        u = (x[2] >> 8) / float(1 << 24)
        if u < p_mb:
            loc = "mb:%d" % (x[3] % (max_microbatch + 1))
        else:
            loc = "sync:%d" % (x[3] % 101)
        out.append(dict(step=lo + x[0] % (hi - lo + 1), replica=gpu // ranks_per_replica,
                        local_rank=gpu % ranks_per_replica, location=loc))
    out.sort(key=lambda e: (e["step"], e["replica"], e["local_rank"], e["location"]))
    return out


def to_yaml(entries):
    import yaml
    return yaml.safe_dump({"failures": [dict(e) for e in entries]}, sort_keys=True)


def from_yaml(text):
    import yaml
    doc = yaml.safe_load(text) or {}
    out = []
    for e in doc.get("failures", []):
        out.append(dict(step=int(e["step"]), replica=int(e["replica"]), local_rank=int(e.get("local_rank", 0)),
                        location=str(e["location"])))
    return out


def for_step(entries, step, alive, target, n_tensors):
    """What the microbatch loop of `step` has to inject: ({replica: microbatches before the crash},
    fidelity_k).  Entries naming a replica that is already dead are dropped, as are entries that
    would leave no survivor (the guarantee needs one, Sec. 4 Claim); losing any rank loses the
    replica (Sec. 4.4), so the local rank does not matter here."""
    dying, fidelity_k = {}, 0
    for e in entries:
        r = e["replica"]
        if e["step"] != step or r not in alive or r in dying:
            continue
        if len(dying) + 1 >= len(alive):
            continue
        kind, val = e["location"].split(":")
        if kind == "mb":
            dying[r] = min(int(val), target[r])
        else:
            dying[r] = target[r]
            fidelity_k = max(fidelity_k, min(n_tensors, int(math.ceil(int(val) / 100.0 * n_tensors))))
    return dying, fidelity_k
