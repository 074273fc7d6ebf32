"""Attrition report: drive one workload through a generated failure schedule on the GPU and print,
per iteration, the survivors, the quotas in force and the paper's effective-throughput measure
(Sec. 5 / evaluation appendix: processed work / (runtime x alive replicas)), here in
microbatches per second per alive replica for the gradient path alone (gradient generation,
the stand-in for forward/backward, is excluded from the clock).

  python -m paper_2605_11215_amd.attrition --workload 4 --failures 12 --iters 16 [--yaml schedule.yaml]
"""
import argparse
import json
import sys
import time


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=4, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--iters", type=int, default=16)
    ap.add_argument("--failures", type=int, default=12)
    ap.add_argument("--seed", type=int, default=7)
    ap.add_argument("--mb-weight", type=float, default=0.5, help="share of failures at microbatch boundaries")
    ap.add_argument("--yaml", default="", help="read the schedule from this file instead of generating it")
    ap.add_argument("--dump-yaml", default="", help="write the schedule used to this file")
    a = ap.parse_args(argv)

    import torch
    from . import binding as B
    from . import schedule, synth
    from .loop import HP, run_iteration, view_shard
    from .synth import reference_np as S
    from .workloads import CONFIGS

    c = CONFIGS[a.workload]
    W, G, off = c["W"], c["G"], c["off"]
    N, T = off[-1], len(off) - 1
    if a.yaml:
        entries = schedule.from_yaml(open(a.yaml).read())
    else:
        entries = schedule.generate(W, 1, a.seed, a.failures, (0, a.iters - 1),
                                    {"mb": a.mb_weight, "sync": 1.0 - a.mb_weight}, max_microbatch=G)
    if a.dump_yaml:
        open(a.dump_yaml, "w").write(schedule.to_yaml(entries))

    # one allocation; gradient buffer j next to the accumulators of the replicas it feeds (binding.stream_groups)
    n_pool = 4 if W % 4 == 0 else 1
    sh = B.Shard(W, G, off, device="cuda:0", slab=True, contiguous=True,
                 extra=[(torch.bfloat16 if c["bf16"] else torch.float32, N)] * n_pool)
    synth.fill_device(sh.param, c["seed"], S.TAG_PARAM, 0, 0, 0.02, n=N)
    pool = [synth.fill_device(g, c["seed"], S.TAG_GRAD, j, 0, c["scale"], c["kind"]) for j, g in enumerate(sh.extra)]
    hp = dict(HP)
    rows = []
    for t in range(a.iters):
        v = view_shard(sh)
        dying, fid = schedule.for_step(entries, t, v["alive"], v["target"], T)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = run_iteration(sh, view_shard, t, lambda it, mb: pool[(mb % W) * n_pool // W], W, dying=dying, fidelity_k=fid, hp=hp)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        committed = sum(len(x) for x in out["ids"].values())
        assert committed == W * G, "Eq. 1 violated"
        after = view_shard(sh)
        rows.append(dict(iteration=t, failed=sorted(dying), alive_before=len(v["alive"]), alive_after=len(after["alive"]),
                         boundary=int(any(d.get("at_boundary") for d in out["decisions"])),
                         loop_bound=max(d["loop_bound"] for d in out["decisions"]), committed=committed,
                         ms=dt * 1e3, microbatches_per_s_per_alive_replica=committed / dt / len(v["alive"])))
        print("iter %2d  failed %-12s alive %2d -> %2d  boundary %d  slots %2d  %7.2f ms  %8.1f mb/s/replica" %
              (t, sorted(dying), len(v["alive"]), len(after["alive"]), rows[-1]["boundary"], rows[-1]["loop_bound"],
               dt * 1e3, rows[-1]["microbatches_per_s_per_alive_replica"]), flush=True)
    print(json.dumps(dict(workload=c["name"], schedule=entries, iterations=rows)))
    sh.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
